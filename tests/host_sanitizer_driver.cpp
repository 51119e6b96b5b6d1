// Exercises the host-side entry points of the library (no GPU needed) so that a build with AddressSanitizer /
// UndefinedBehaviorSanitizer or ThreadSanitizer can watch them: the host producers with several workers, the
// walk tables of a weighted graph, the redistribution into orthogonal blocks, the rank statistic, and the
// argument-error paths of the context calls.  Exit code 0 = every check passed (the sanitizers abort on a finding).
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <vector>

#include "gvhot.h"

#define CHECK(cond)                                                          \
    do {                                                                     \
        if (!(cond)) {                                                       \
            fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            return 1;                                                        \
        }                                                                    \
    } while (0)

static uint64_t next_random(uint64_t *state) {  // xorshift: test input only
    *state ^= *state << 13;
    *state ^= *state >> 7;
    *state ^= *state << 17;
    return *state;
}

int main() {
    // a ring with chords, n nodes of degree 4, plus edge weights
    const uint32_t n = 5000;
    std::vector<uint64_t> offsets(n + 1);
    std::vector<uint32_t> adj(4 * (size_t)n);
    std::vector<float> weights(4 * (size_t)n);
    uint64_t state = 88172645463325252ull;
    for (uint32_t i = 0; i < n; ++i) {
        offsets[i] = 4ull * i;
        const uint32_t to[4] = {(i + 1) % n, (i + 2) % n, (i + n - 1) % n, (i + n - 2) % n};
        for (int k = 0; k < 4; ++k) {
            adj[4 * (size_t)i + k] = to[k];
            weights[4 * (size_t)i + k] = (float)(1 + next_random(&state) % 9);
        }
    }
    offsets[n] = 4ull * n;

    const uint64_t count = 190 * 700 + 13;
    std::vector<uint32_t> one(2 * count), many(2 * count);
    uint64_t walks1 = 0, walks8 = 0;
    CHECK(gv_augment(n, offsets.data(), adj.data(), 7, 40, 5, 1ull << 40, count, GV_SHUFFLE_PSEUDO, 1, one.data(), &walks1) == GV_OK);
    CHECK(gv_augment(n, offsets.data(), adj.data(), 7, 40, 5, 1ull << 40, count, GV_SHUFFLE_PSEUDO, 8, many.data(), &walks8) == GV_OK);
    CHECK(walks1 == 701 && walks8 == 701 && one == many);
    CHECK(gv_augment(n, offsets.data(), adj.data(), 7, 3, 0xFFFFFFFFu, 0, 100, GV_SHUFFLE_NONE, 2, many.data(), nullptr) == GV_EINVAL);
    CHECK(gv_augment(n, offsets.data(), adj.data(), 7, 3, GV_MAX_WINDOW, 0, 100, GV_SHUFFLE_NONE, 2, many.data(), nullptr) == GV_OK);
    std::vector<uint32_t> broken(adj);
    for (size_t e = 0; e < broken.size(); e += 3) broken[e] = n + 5;  // entries beyond the node range
    CHECK(gv_augment(n, offsets.data(), broken.data(), 7, 40, 5, 0, count, GV_SHUFFLE_PSEUDO, 4, many.data(), nullptr) == GV_EINVAL);

    std::vector<double> wdeg(n);
    std::vector<uint32_t> node_thresh(n), node_alias(n), nbr_thresh(adj.size()), nbr_alias(adj.size());
    CHECK(gv_build_walk_tables(n, offsets.data(), weights.data(), wdeg.data(), node_thresh.data(), node_alias.data(),
                               nbr_thresh.data(), nbr_alias.data()) == GV_OK);
    CHECK(gv_augment_weighted(n, offsets.data(), adj.data(), node_thresh.data(), node_alias.data(), nbr_thresh.data(),
                              nbr_alias.data(), 9, 40, 5, 3, count, GV_SHUFFLE_PSEUDO, 1, one.data(), &walks1) == GV_OK);
    CHECK(gv_augment_weighted(n, offsets.data(), adj.data(), node_thresh.data(), node_alias.data(), nbr_thresh.data(),
                              nbr_alias.data(), 9, 40, 5, 3, count, GV_SHUFFLE_PSEUDO, 6, many.data(), &walks8) == GV_OK);
    CHECK(walks1 == walks8 && one == many);
    std::vector<float> no_weight(weights.size(), 0.0f);
    CHECK(gv_build_walk_tables(n, offsets.data(), no_weight.data(), nullptr, node_thresh.data(), node_alias.data(),
                               nbr_thresh.data(), nbr_alias.data()) == GV_EINVAL);

    const uint32_t B = 8;
    std::vector<uint32_t> part(n);
    for (uint32_t i = 0; i < n; ++i) part[i] = (uint32_t)(next_random(&state) % B);
    std::vector<uint32_t> sorted1(2 * count), sorted8(2 * count), order1(count), order8(count);
    std::vector<uint64_t> blocks1(B * B + 1), blocks8(B * B + 1);
    CHECK(gv_redistribute_pool(n, part.data(), B, one.data(), count, 1, sorted1.data(), order1.data(), blocks1.data()) == GV_OK);
    CHECK(gv_redistribute_pool(n, part.data(), B, one.data(), count, 8, sorted8.data(), order8.data(), blocks8.data()) == GV_OK);
    CHECK(sorted1 == sorted8 && order1 == order8 && blocks1 == blocks8 && blocks1[B * B] == count);
    for (uint64_t b = 0; b < (uint64_t)B * B; ++b)
        for (uint64_t k = blocks1[b]; k < blocks1[b + 1]; ++k) {
            const uint32_t pi = part[sorted1[2 * k]], pj = part[sorted1[2 * k + 1]];
            CHECK(((pj + B - pi) % B) * B + pi == b);
            CHECK(k == blocks1[b] || order1[k] > order1[k - 1]);
        }
    part[17] = B;  // a partition number out of range
    one[0] = 17;
    CHECK(gv_redistribute_pool(n, part.data(), B, one.data(), count, 3, sorted1.data(), order1.data(), blocks1.data()) == GV_EINVAL);

    const float pos[5] = {0.9f, 0.5f, 0.5f, 0.1f, 0.7f}, neg[4] = {0.5f, 0.2f, 0.8f, 0.5f};
    double auc = -1.0;
    CHECK(gv_auc(pos, 5, neg, 4, &auc) == GV_OK);
    double wins = 0.0;
    for (float p : pos)
        for (float q : neg) wins += p > q ? 1.0 : (p == q ? 0.5 : 0.0);
    CHECK(auc == wins / 20.0);
    CHECK(gv_auc(pos, 0, neg, 4, &auc) == GV_EINVAL);

    // context calls: argument errors before any device is touched, and a clean refusal without a device
    gv_config cfg{};
    cfg.dim = 100;
    gv_ctx *ctx = nullptr;
    CHECK(gv_create(&cfg, &ctx) == GV_EINVAL && ctx == nullptr && gv_last_error(nullptr)[0] != 0);
    cfg.dim = 128;
    cfg.num_neg = 1;
    cfg.lr0 = 0.025f;
    cfg.neg_weight = GV_NEG_WEIGHT_DEFAULT;
    cfg.total_samples = 1000;
    cfg.pool_capacity = 1000;
    cfg.pool_slots = 4;
    const int rc = gv_create(&cfg, &ctx);
    CHECK(rc == GV_OK || rc == GV_EHIP);  // GV_EHIP: no GPU in this machine
    if (rc == GV_OK) gv_destroy(ctx);
    CHECK(gv_sync(nullptr) == GV_EINVAL && gv_train_pool(nullptr) == GV_EINVAL);
    gv_destroy(nullptr);
    printf("host sanitizer driver: all checks passed\n");
    return 0;
}
