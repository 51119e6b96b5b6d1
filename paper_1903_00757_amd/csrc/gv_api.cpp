// Host runtime behind the C boundary declared in include/gvhot.h: context,
// alias-table builder, pinned double-buffered pool ring with asynchronous
// host-to-device copies, launch sequencing, deterministic batch cutting.
#include "gvhot.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <exception>
#include <mutex>
#include <new>
#include <string>
#include <utility>
#include <vector>

#include "gv_host.hpp"
#include "gv_internal.hpp"

namespace {

thread_local std::string g_create_error;

enum SlotState { kFree = 0, kFilling = 1, kQueued = 2, kTraining = 3 };

struct PoolSlot {
    uint32_t *host = nullptr;    // pinned, pool_capacity samples
    uint32_t *dev = nullptr;     // device twin
    hipEvent_t copied = nullptr; // host-to-device copy finished (copy stream)
    hipEvent_t trained = nullptr;// training launch that read `dev` finished (compute stream)
    uint64_t count = 0;
    SlotState state = kFree;
};

struct TimedSpan {
    hipEvent_t start, stop;
    int kind;  // 0 training launch, 1 host-to-device copy
};

}  // namespace

// Scratch of the entry point that must not allocate (gv_train_device_pool_static): the per-sample records
// of the tiled kernel, in a device array that is part of the loaded code object.  Every GPU holds its own
// copy at its own address; the name below is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) uint32_t scratch[GV_STATIC_SCRATCH_WORDS];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
uint32_t *g_scratch_address[kMaxDevices];  // device address of `scratch` on each GPU, looked up once per GPU
}  // namespace

struct gv_ctx {
    gv_config cfg{};
    uint32_t n = 0;
    std::vector<uint32_t> degree;
    std::vector<double> wdegree;          // weighted graph: sum of the edge weights of every node (else empty)
    uint2 *dev_node_table = nullptr;      // weighted graph: alias table of the departure nodes {threshold, alias}
    uint2 *dev_nbr_table = nullptr;       // weighted graph: one alias table per adjacency row {threshold, alias in row}
    float *vertex = nullptr;
    float *context = nullptr;
    uint4 *alias = nullptr;
    bool alias_ready = false;
    uint16_t *dev_rank = nullptr;         // device, per node: hot rank (see gv::TrainArgs)
    uint32_t *dev_ranked = nullptr;       // device, bitmap of the nodes that have a hot rank
    uint32_t warm_ranks = 0;              // number of warm rows
    // orthogonal blocks (cfg.partitions > 0): partition of every node, and one alias table per partition
    std::vector<uint32_t> part;           // host, per node
    std::vector<uint64_t> part_offsets;   // host, partitions + 1: partition j owns table buckets [j] .. [j + 1] - 1
    std::vector<uint32_t> part_members, part_thresh, part_alias;  // host copies of the concatenated tables
    uint4 *dev_part_tables = nullptr;     // device, n buckets
    uint64_t *dev_part_offsets = nullptr; // device
    uint8_t *dev_part = nullptr;          // device, per node
    uint64_t *dev_offsets = nullptr;      // device CSR of the graph (gv_set_adjacency), for the device producer
    uint32_t *dev_adj = nullptr;
    uint64_t half_edges = 0;
    uint32_t *error_flag = nullptr;       // device
    double *dev_loss = nullptr;           // device, cfg.track_loss: gv::kLossSlots running sums of the training loss
    uint32_t *negatives = nullptr;        // device scratch, deterministic mode / gv_draw_negatives
    uint64_t negatives_capacity = 0;      // in uint32 elements
    uint32_t *records = nullptr;          // device scratch of the tiled kernel: K + 3 words per sample of a launch
    uint64_t records_capacity = 0;        // in uint32 elements
    uint32_t *static_records = nullptr;   // this GPU's copy of the `scratch` array (GV_STATIC_SCRATCH_WORDS words)
    void *eval_scratch = nullptr;         // device scratch of gv_eval_loss / gv_cosine / gv_auc, grown on demand
    uint64_t eval_capacity = 0;           // in bytes
    hipStream_t compute = nullptr;
    hipStream_t copy = nullptr;
    std::vector<PoolSlot> slot;           // ring of cfg.pool_slots pinned slots, each with a device twin
    std::vector<int> queue;               // FIFO of queued slot indices (front = oldest)
    int next_slot = 0;                    // slots are handed out in ring order
    uint64_t next_g = 0;
    gv_stats stats{};
    std::vector<TimedSpan> spans;         // recorded, not yet folded into stats
    std::vector<hipEvent_t> spare_events;
    std::vector<uint32_t> stamp_vertex, stamp_context;  // deterministic batch cutting
    uint32_t stamp = 0;
    std::string error;
};

namespace {

int fail(gv_ctx *ctx, int code, const char *fmt, ...) noexcept {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    try {
        if (ctx) ctx->error = buf; else g_create_error = buf;
    } catch (...) {  // no memory even for the text: the code alone is returned
    }
    return code;
}

// Every entry point runs its body through this: an exception of the C++ runtime (a container that
// cannot grow, a thread that cannot start) becomes an error code instead of crossing the C boundary.
template <class Body>
int guarded(gv_ctx *ctx, Body &&body) noexcept {
    try {
        return body();
    } catch (const std::bad_alloc &) {
        return fail(ctx, GV_ENOMEM, "out of host memory");
    } catch (const std::exception &e) {
        return fail(ctx, GV_EHIP, "host runtime error: %s", e.what());
    } catch (...) {
        return fail(ctx, GV_EHIP, "unknown host runtime error");
    }
}

#define GV_HIP(ctx, expr)                                                                          \
    do {                                                                                           \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess)                                                                      \
            return fail(ctx, e_ == hipErrorOutOfMemory ? GV_ENOMEM : GV_EHIP, "%s: %s", #expr,     \
                        hipGetErrorString(e_));                                                    \
    } while (0)

int bind_device(gv_ctx *ctx) {
    GV_HIP(ctx, hipSetDevice(ctx->cfg.device));
    return GV_OK;
}

hipEvent_t take_event(gv_ctx *ctx) {
    if (!ctx->spare_events.empty()) {
        hipEvent_t e = ctx->spare_events.back();
        ctx->spare_events.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

// Fold finished event pairs into the statistics (called with the device idle).
void fold_spans(gv_ctx *ctx) {
    for (const TimedSpan &s : ctx->spans) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, s.start, s.stop) == hipSuccess) {
            if (s.kind == 0) {
                ctx->stats.train_kernel_ms += ms;
                ctx->stats.timed_launches += 1;
            } else {
                ctx->stats.h2d_ms += ms;
            }
        }
        ctx->spare_events.push_back(s.start);
        ctx->spare_events.push_back(s.stop);
    }
    ctx->spans.clear();
}

int sync_all(gv_ctx *ctx) {
    GV_HIP(ctx, hipStreamSynchronize(ctx->copy));
    GV_HIP(ctx, hipStreamSynchronize(ctx->compute));
    fold_spans(ctx);
    for (PoolSlot &s : ctx->slot)
        if (s.state == kTraining) s.state = kFree;
    if (ctx->dev_loss) {
        double slots[gv::kLossSlots];
        GV_HIP(ctx, hipMemcpy(slots, ctx->dev_loss, sizeof slots, hipMemcpyDeviceToHost));
        double total = 0.0;
        for (double x : slots) total += x;
        ctx->stats.train_loss_sum = total;
    }
    uint32_t flag[2] = {0, 0};
    GV_HIP(ctx, hipMemcpy(flag, ctx->error_flag, sizeof flag, hipMemcpyDeviceToHost));
    if (flag[0] || flag[1]) {
        GV_HIP(ctx, hipMemset(ctx->error_flag, 0, sizeof flag));
        if (flag[0])
            return fail(ctx, GV_EINVAL, "a trained pool named a node id >= n (%u); those samples were skipped", ctx->n);
        return fail(ctx, GV_ESTATE, "training has diverged: an embedding row holds NaN (asynchronous mode on a graph "
                    "where one node takes part in a large share of all samples? see GV_MODE_HOGWILD)");
    }
    return GV_OK;
}

void free_matrices(gv_ctx *ctx) {
    if (ctx->vertex) (void)hipFree(ctx->vertex);
    if (ctx->context) (void)hipFree(ctx->context);
    if (ctx->alias) (void)hipFree(ctx->alias);
    if (ctx->dev_rank) (void)hipFree(ctx->dev_rank);
    if (ctx->dev_ranked) (void)hipFree(ctx->dev_ranked);
    ctx->dev_ranked = nullptr;
    if (ctx->dev_offsets) (void)hipFree(ctx->dev_offsets);
    if (ctx->dev_adj) (void)hipFree(ctx->dev_adj);
    if (ctx->dev_node_table) (void)hipFree(ctx->dev_node_table);
    if (ctx->dev_nbr_table) (void)hipFree(ctx->dev_nbr_table);
    ctx->dev_node_table = nullptr;
    ctx->dev_nbr_table = nullptr;
    if (ctx->dev_part_tables) (void)hipFree(ctx->dev_part_tables);
    if (ctx->dev_part_offsets) (void)hipFree(ctx->dev_part_offsets);
    if (ctx->dev_part) (void)hipFree(ctx->dev_part);
    ctx->dev_part_tables = nullptr;
    ctx->dev_part_offsets = nullptr;
    ctx->dev_part = nullptr;
    ctx->dev_offsets = nullptr;
    ctx->dev_adj = nullptr;
    ctx->half_edges = 0;
    ctx->vertex = ctx->context = nullptr;
    ctx->alias = nullptr;
    ctx->dev_rank = nullptr;
    ctx->alias_ready = false;
}

// Takes over the degrees of a new graph: allocates the matrices (cleared) and the per-node tables.
int adopt_degrees(gv_ctx *ctx, uint32_t n, std::vector<uint32_t> &&deg) {
    int rc = sync_all(ctx);
    if (rc != GV_OK && rc != GV_EINVAL && rc != GV_ESTATE) return rc;  // reports about pools already trained do not stop this call
    free_matrices(ctx);
    ctx->n = 0;
    const size_t bytes = (size_t)n * ctx->cfg.dim * sizeof(float);
    GV_HIP(ctx, hipMalloc((void **)&ctx->vertex, bytes));
    GV_HIP(ctx, hipMalloc((void **)&ctx->context, bytes));
    GV_HIP(ctx, hipMalloc((void **)&ctx->alias, (size_t)n * sizeof(uint4)));
    GV_HIP(ctx, hipMalloc((void **)&ctx->dev_rank, (size_t)n * sizeof(uint16_t)));  // filled by gv_build_alias
    GV_HIP(ctx, hipMalloc((void **)&ctx->dev_ranked, ((size_t)n + 31) / 32 * sizeof(uint32_t)));
    GV_HIP(ctx, hipMemsetAsync(ctx->vertex, 0, bytes, ctx->compute));
    GV_HIP(ctx, hipMemsetAsync(ctx->context, 0, bytes, ctx->compute));
    GV_HIP(ctx, hipStreamSynchronize(ctx->compute));
    ctx->degree = std::move(deg);
    ctx->wdegree.clear();
    ctx->part.clear();
    ctx->n = n;
    ctx->stamp_vertex.clear();
    ctx->stamp_context.clear();
    return GV_OK;
}

int need_graph(gv_ctx *ctx) {
    if (!ctx) return GV_EINVAL;
    if (ctx->n == 0) return fail(ctx, GV_ESTATE, "no graph: call gv_set_graph or gv_set_degrees first");
    return bind_device(ctx);
}

int need_trainable(gv_ctx *ctx) {
    int rc = need_graph(ctx);
    if (rc) return rc;
    if (!ctx->alias_ready) return fail(ctx, GV_ESTATE, "no alias table: call gv_build_alias first");
    return GV_OK;
}

int ensure_negatives(gv_ctx *ctx, uint64_t elements) {
    if (elements <= ctx->negatives_capacity) return GV_OK;
    if (ctx->negatives) {
        GV_HIP(ctx, hipStreamSynchronize(ctx->compute));
        (void)hipFree(ctx->negatives);
        ctx->negatives = nullptr;
        ctx->negatives_capacity = 0;
    }
    GV_HIP(ctx, hipMalloc((void **)&ctx->negatives, elements * sizeof(uint32_t)));
    ctx->negatives_capacity = elements;
    return GV_OK;
}

int ensure_records(gv_ctx *ctx, uint64_t elements) {
    if (elements <= ctx->records_capacity) return GV_OK;
    if (ctx->records) {
        GV_HIP(ctx, hipStreamSynchronize(ctx->compute));
        (void)hipFree(ctx->records);
        ctx->records = nullptr;
        ctx->records_capacity = 0;
    }
    GV_HIP(ctx, hipMalloc((void **)&ctx->records, elements * sizeof(uint32_t)));
    ctx->records_capacity = elements;
    return GV_OK;
}

gv::TrainArgs train_args(gv_ctx *ctx, const uint32_t *dev_pairs, uint64_t first_g, uint32_t count) {
    gv::TrainArgs a{};
    a.vertex = ctx->vertex;
    a.context = ctx->context;
    a.alias = ctx->alias;
    a.alias_n = ctx->n;
    a.pairs = dev_pairs;
    a.negatives = nullptr;
    a.order = nullptr;
    a.rank = ctx->dev_rank;
    a.ranked = ctx->n > 20u * 0xFFFFu ? ctx->dev_ranked : nullptr;  // under 5 % of the nodes ranked
    a.warm_ranks = ctx->warm_ranks;
    a.error_flag = ctx->error_flag;
    a.loss_slots = ctx->dev_loss;
    a.first_g = first_g;
    a.total = ctx->cfg.total_samples;
    a.seed = ctx->cfg.seed;
    a.count = count;
    a.n = ctx->n;
    a.dim = ctx->cfg.dim;
    a.lr0 = ctx->cfg.lr0;
    a.lr_min_ratio = ctx->cfg.lr_min_ratio;
    a.neg_weight = ctx->cfg.neg_weight;
    return a;
}

int begin_span(gv_ctx *ctx, int kind, hipStream_t stream, TimedSpan *span) {
    span->kind = kind;
    span->start = take_event(ctx);
    span->stop = take_event(ctx);
    if (!span->start || !span->stop) return fail(ctx, GV_EHIP, "hipEventCreate failed");
    GV_HIP(ctx, hipEventRecord(span->start, stream));
    return GV_OK;
}

int end_span(gv_ctx *ctx, hipStream_t stream, const TimedSpan &span) {
    GV_HIP(ctx, hipEventRecord(span.stop, stream));
    ctx->spans.push_back(span);
    if (ctx->spans.size() >= 8192) {  // bound the number of live events: all of them must have completed
        GV_HIP(ctx, hipStreamSynchronize(ctx->copy));
        GV_HIP(ctx, hipStreamSynchronize(ctx->compute));
        fold_spans(ctx);
    }
    return GV_OK;
}

// Asynchronous training of `count` samples at dev_pairs: one launch of the tiled
// stationary-row kernel, or of the plain pool-order kernel.
// `fixed_records`: null, or the static scratch of the entry point that must not allocate: then nothing is
// allocated on the way (no scratch growth, no events: the launch is not timed).
// `block`: null, or the part of a redistributed pool that one orthogonal block covers: its samples' pool indices
// and the context partition whose alias table its negatives come from.
struct BlockOfPool {
    const uint32_t *dev_order;
    uint32_t partition;
};
int train_hogwild(gv_ctx *ctx, const uint32_t *dev_pairs, uint64_t count, uint32_t *fixed_records = nullptr,
                  const BlockOfPool *block = nullptr) {
    // GV_SCHEDULE_AUTO: the tiled schedule exists for rows that many samples of a tile share.  A graph
    // without a single warm row has none, and there the sort, the records and the rank reads are pure
    // cost: such a graph is trained in pool order (with the mixed policy all of its rows are cold, i.e.
    // updated with device-scope stores).
    const bool wants_tiled = ctx->cfg.schedule == GV_SCHEDULE_TILED ||
                             (ctx->cfg.schedule == GV_SCHEDULE_AUTO && ctx->warm_ranks > 0);
    const bool tiled = wants_tiled && ctx->n <= 0x80000000u;
    uint32_t coherence = ctx->cfg.coherence;
    if (!tiled && ctx->cfg.schedule == GV_SCHEDULE_AUTO && coherence == GV_COHERENCE_MIXED && ctx->warm_ranks == 0)
        coherence = GV_COHERENCE_AGENT;
    if (tiled && fixed_records) {
        const uint64_t words = count * (ctx->cfg.num_neg + 3);
        if (words > GV_STATIC_SCRATCH_WORDS)
            return fail(ctx, GV_EINVAL, "pool of %llu samples needs %llu words of scratch, the static scratch holds %llu "
                        "(at most %llu samples at K = %u)", (unsigned long long)count, (unsigned long long)words,
                        (unsigned long long)GV_STATIC_SCRATCH_WORDS,
                        (unsigned long long)(GV_STATIC_SCRATCH_WORDS / (ctx->cfg.num_neg + 3)), ctx->cfg.num_neg);
    } else if (tiled) {  // before the timed span: an allocation must not count as kernel time
        int rc = ensure_records(ctx, count * (ctx->cfg.num_neg + 3));
        if (rc) return rc;
    }
    TimedSpan span{};
    const bool timed = ctx->cfg.profile != 0 && !fixed_records;
    if (timed) {
        int rc = begin_span(ctx, 0, ctx->compute, &span);
        if (rc) return rc;
    }
    gv::TrainArgs a = train_args(ctx, dev_pairs, ctx->next_g, (uint32_t)count);
    if (block) {
        a.order = block->dev_order;
        a.alias = ctx->dev_part_tables + ctx->part_offsets[block->partition];
        a.alias_n = (uint32_t)(ctx->part_offsets[block->partition + 1] - ctx->part_offsets[block->partition]);
    }
    if (tiled) {
        a.records = fixed_records ? fixed_records : ctx->records;
        GV_HIP(ctx, (a.loss_slots ? gv::launch_train_tiled_tracked : gv::launch_train_tiled)(
                        a, ctx->cfg.dim, ctx->cfg.num_neg, coherence, ctx->compute));
    } else {
        GV_HIP(ctx, (a.loss_slots ? gv::launch_train_hogwild_tracked : gv::launch_train_hogwild)(
                        a, ctx->cfg.dim, ctx->cfg.num_neg, coherence, ctx->compute));
    }
    ctx->stats.train_launches += 1;
    ctx->stats.tiled_launches += tiled ? 1 : 0;
    if (ctx->dev_loss) ctx->stats.train_loss_samples += count;
    if (timed) return end_span(ctx, ctx->compute, span);
    return GV_OK;
}

// Deterministic training: draw the pool's negatives on the device, bring them
// and the pairs to the host, cut the sample sequence greedily into maximal runs
// in which no vertex row and no context row (positive or negative) repeats, and
// launch one conflict-free batch per run, in order.  Samples inside a run commute
// exactly (Def. 1, Sec. 3.2), so the result is the sequential one up to fp32
// rounding inside a sample.
int train_deterministic(gv_ctx *ctx, const uint32_t *dev_pairs, const uint32_t *host_pairs, uint64_t count) {
    const uint32_t K = ctx->cfg.num_neg;
    int rc = ensure_negatives(ctx, count * K);
    if (rc) return rc;
    GV_HIP(ctx, gv::launch_draw_negatives(ctx->alias, ctx->n, ctx->cfg.seed, ctx->next_g, count, K, ctx->negatives,
                                          ctx->compute));
    std::vector<uint32_t> neg(count * K);
    std::vector<uint32_t> pairs_copy;
    GV_HIP(ctx, hipMemcpyAsync(neg.data(), ctx->negatives, neg.size() * sizeof(uint32_t), hipMemcpyDeviceToHost,
                               ctx->compute));
    if (!host_pairs) {
        pairs_copy.resize(count * 2);
        GV_HIP(ctx, hipMemcpyAsync(pairs_copy.data(), dev_pairs, pairs_copy.size() * sizeof(uint32_t),
                                   hipMemcpyDeviceToHost, ctx->compute));
        host_pairs = pairs_copy.data();
    }
    GV_HIP(ctx, hipStreamSynchronize(ctx->compute));

    if (ctx->stamp_vertex.size() != ctx->n) {
        ctx->stamp_vertex.assign(ctx->n, 0);
        ctx->stamp_context.assign(ctx->n, 0);
        ctx->stamp = 0;
    }
    std::vector<uint64_t> starts;
    auto open_batch = [&](uint64_t at) {
        starts.push_back(at);
        if (++ctx->stamp == 0) {  // stamp wrapped: clear and restart numbering
            std::fill(ctx->stamp_vertex.begin(), ctx->stamp_vertex.end(), 0u);
            std::fill(ctx->stamp_context.begin(), ctx->stamp_context.end(), 0u);
            ctx->stamp = 1;
        }
    };
    open_batch(0);
    for (uint64_t i = 0; i < count; ++i) {
        const uint32_t u = host_pairs[2 * i], v = host_pairs[2 * i + 1];
        if (u >= ctx->n || v >= ctx->n)
            return fail(ctx, GV_EINVAL, "sample %llu names node id >= n (%u)", (unsigned long long)i, ctx->n);
        bool clash = ctx->stamp_vertex[u] == ctx->stamp || ctx->stamp_context[v] == ctx->stamp;
        for (uint32_t k = 0; k < K && !clash; ++k) clash = ctx->stamp_context[neg[i * K + k]] == ctx->stamp;
        if (clash) open_batch(i);
        ctx->stamp_vertex[u] = ctx->stamp;
        ctx->stamp_context[v] = ctx->stamp;
        for (uint32_t k = 0; k < K; ++k) ctx->stamp_context[neg[i * K + k]] = ctx->stamp;
    }
    starts.push_back(count);

    TimedSpan span{};
    const bool timed = ctx->cfg.profile != 0;
    if (timed) {
        rc = begin_span(ctx, 0, ctx->compute, &span);
        if (rc) return rc;
    }
    for (size_t b = 0; b + 1 < starts.size(); ++b) {
        const uint64_t lo = starts[b], hi = starts[b + 1];
        gv::TrainArgs a = train_args(ctx, dev_pairs + 2 * lo, ctx->next_g + lo, (uint32_t)(hi - lo));
        a.negatives = ctx->negatives + lo * K;
        GV_HIP(ctx, (a.loss_slots ? gv::launch_train_batch_tracked : gv::launch_train_batch)(a, ctx->cfg.dim, K, ctx->compute));
    }
    ctx->stats.train_launches += starts.size() - 1;
    ctx->stats.batches += starts.size() - 1;
    if (ctx->dev_loss) ctx->stats.train_loss_samples += count;
    if (timed) return end_span(ctx, ctx->compute, span);
    return GV_OK;
}

int train_any(gv_ctx *ctx, const uint32_t *dev_pairs, const uint32_t *host_pairs, uint64_t count) {
    if (count == 0) return GV_OK;
    int rc = ctx->cfg.mode == GV_MODE_DETERMINISTIC ? train_deterministic(ctx, dev_pairs, host_pairs, count)
                                                    : train_hogwild(ctx, dev_pairs, count);
    if (rc) return rc;
    ctx->next_g += count;
    ctx->stats.samples_trained = ctx->next_g;
    ctx->stats.pools_trained += 1;
    return GV_OK;
}

// Wait until a slot no longer feeds a running launch, then mark it free.
int release_slot(gv_ctx *ctx, PoolSlot &s) {
    if (s.state == kTraining) {
        GV_HIP(ctx, hipEventSynchronize(s.trained));
        s.state = kFree;
    }
    return GV_OK;
}

// Next slot of the ring that is not being filled and not waiting to be trained (ring order =
// oldest first, so a slot still feeding a launch is the one whose launch ends soonest).
int pick_free_slot(gv_ctx *ctx, int *index) {
    const int slots = (int)ctx->slot.size();
    for (int t = 0; t < slots; ++t) {
        const int i = (ctx->next_slot + t) % slots;
        PoolSlot &s = ctx->slot[i];
        if (s.state == kFree || s.state == kTraining) {
            int rc = release_slot(ctx, s);
            if (rc) return rc;
            *index = i;
            ctx->next_slot = (i + 1) % slots;
            return GV_OK;
        }
    }
    return fail(ctx, GV_ESTATE, "all %d pool slots are filling or queued: train a pool first", slots);
}

// Device scratch shared by the evaluation calls: grown when a call needs more, kept otherwise.
int ensure_eval_scratch(gv_ctx *ctx, uint64_t bytes) {
    if (bytes <= ctx->eval_capacity) return GV_OK;
    if (ctx->eval_scratch) {
        (void)hipFree(ctx->eval_scratch);
        ctx->eval_scratch = nullptr;
        ctx->eval_capacity = 0;
    }
    GV_HIP(ctx, hipMalloc(&ctx->eval_scratch, bytes));
    ctx->eval_capacity = bytes;
    return GV_OK;
}

// Area under the ROC curve of `pos` against `neg` as the rank statistic
// (sum of the positives' ranks - P (P + 1) / 2) / (P N), equal scores sharing their mean rank.
double rank_auc(const float *pos, uint64_t num_pos, const float *neg, uint64_t num_neg) {
    std::vector<std::pair<float, uint8_t>> all;
    all.reserve(num_pos + num_neg);
    for (uint64_t i = 0; i < num_pos; ++i) all.emplace_back(pos[i], (uint8_t)1);
    for (uint64_t i = 0; i < num_neg; ++i) all.emplace_back(neg[i], (uint8_t)0);
    std::sort(all.begin(), all.end(), [](const auto &a, const auto &b) { return a.first < b.first; });
    double positive_ranks = 0.0;
    for (size_t lo = 0; lo < all.size();) {
        size_t hi = lo;
        uint64_t positives = 0;
        while (hi < all.size() && all[hi].first == all[lo].first) positives += all[hi++].second;
        positive_ranks += (double)positives * (0.5 * ((double)(lo + 1) + (double)hi));  // ranks lo+1 .. hi share their mean
        lo = hi;
    }
    const double P = (double)num_pos, N = (double)num_neg;
    return (positive_ranks - P * (P + 1.0) / 2.0) / (P * N);
}

}  // namespace

extern "C" {

const char *gv_last_error(const gv_ctx *ctx) { return ctx ? ctx->error.c_str() : g_create_error.c_str(); }

int gv_create(const gv_config *cfg, gv_ctx **out) {
    if (out) *out = nullptr;
    if (!cfg || !out) return fail(nullptr, GV_EINVAL, "null argument");
    return guarded(nullptr, [&]() -> int {
        if (!gv::supported_shape(cfg->dim, cfg->num_neg))
            return fail(nullptr, GV_EINVAL, "unsupported shape: dim %u (a multiple of 32 in 32..512), num_neg %u (1..5)",
                        cfg->dim, cfg->num_neg);
        if (cfg->total_samples == 0) return fail(nullptr, GV_EINVAL, "total_samples must be > 0");
        if (cfg->pool_capacity == 0 || cfg->pool_capacity > (1ull << 31))
            return fail(nullptr, GV_EINVAL, "pool_capacity must be in 1..2^31 samples");
        if (cfg->partitions == 1 || cfg->partitions > GV_MAX_PARTITIONS)
            return fail(nullptr, GV_EINVAL, "partitions must be 0 (none) or in 2..%d", GV_MAX_PARTITIONS);
        if (cfg->pool_slots == 1 || cfg->pool_slots > GV_MAX_POOL_SLOTS)
            return fail(nullptr, GV_EINVAL, "pool_slots must be 0 (= 2) or in 2..%d", GV_MAX_POOL_SLOTS);
        if (cfg->mode > GV_MODE_DETERMINISTIC || cfg->coherence > GV_COHERENCE_MIXED ||
            cfg->schedule > GV_SCHEDULE_AUTO)
            return fail(nullptr, GV_EINVAL, "bad mode / coherence / schedule field");
        const bool default_weight = cfg->neg_weight == GV_NEG_WEIGHT_DEFAULT;
        if (!(cfg->lr0 >= 0.0f) || !(cfg->lr_min_ratio >= 0.0f) || !(default_weight || cfg->neg_weight >= 0.0f) ||
            !isfinite(cfg->lr0) || !isfinite(cfg->neg_weight))
            return fail(nullptr, GV_EINVAL,
                        "lr0, lr_min_ratio and neg_weight must be finite and >= 0 (neg_weight may be GV_NEG_WEIGHT_DEFAULT)");
        int devices = 0;
        if (hipGetDeviceCount(&devices) != hipSuccess || devices <= 0)
            return fail(nullptr, GV_EHIP, "no HIP device available");
        if (cfg->device < 0 || cfg->device >= devices)
            return fail(nullptr, GV_EINVAL, "device %d out of range (%d present)", cfg->device, devices);
        gv_ctx *ctx = new (std::nothrow) gv_ctx;
        if (!ctx) return fail(nullptr, GV_ENOMEM, "out of host memory");
        ctx->cfg = *cfg;
        // Sec. 4.3: one negative whose gradient is scaled by 5, to match the gradient scale of 5 negatives
        if (default_weight) ctx->cfg.neg_weight = 5.0f / (float)cfg->num_neg;
        if (ctx->cfg.pool_slots == 0) ctx->cfg.pool_slots = 2;
        auto bail = [&](int code) {
            g_create_error = ctx->error;
            gv_destroy(ctx);
            return code;
        };
#define GV_TRY(expr)                                                                                       \
    do {                                                                                                   \
        hipError_t e_ = (expr);                                                                            \
        if (e_ != hipSuccess) {                                                                            \
            fail(ctx, e_ == hipErrorOutOfMemory ? GV_ENOMEM : GV_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
            return bail(e_ == hipErrorOutOfMemory ? GV_ENOMEM : GV_EHIP);                                  \
        }                                                                                                  \
    } while (0)
        try {
            ctx->slot.resize(ctx->cfg.pool_slots);
            ctx->queue.reserve(ctx->cfg.pool_slots);
        } catch (...) {
            fail(ctx, GV_ENOMEM, "out of host memory");
            return bail(GV_ENOMEM);
        }
        GV_TRY(hipSetDevice(cfg->device));
        if (cfg->device < kMaxDevices) {  // once per GPU, with that GPU current: where its copy of `scratch` lies
            std::lock_guard<std::mutex> lock(g_scratch_mutex);
            if (!g_scratch_address[cfg->device]) {
                void *address = nullptr;
                GV_TRY(hipGetSymbolAddress(&address, HIP_SYMBOL(scratch)));
                g_scratch_address[cfg->device] = (uint32_t *)address;
            }
            ctx->static_records = g_scratch_address[cfg->device];
        }
        GV_TRY(hipStreamCreateWithFlags(&ctx->compute, hipStreamNonBlocking));
        GV_TRY(hipStreamCreateWithFlags(&ctx->copy, hipStreamNonBlocking));
        GV_TRY(hipMalloc((void **)&ctx->error_flag, 2 * sizeof(uint32_t)));
        GV_TRY(hipMemset(ctx->error_flag, 0, 2 * sizeof(uint32_t)));
        if (cfg->track_loss) {
            GV_TRY(hipMalloc((void **)&ctx->dev_loss, gv::kLossSlots * sizeof(double)));
            GV_TRY(hipMemset(ctx->dev_loss, 0, gv::kLossSlots * sizeof(double)));
        }
        const size_t pool_bytes = (size_t)cfg->pool_capacity * 2 * sizeof(uint32_t);
        for (PoolSlot &s : ctx->slot) {
            GV_TRY(hipHostMalloc((void **)&s.host, pool_bytes, hipHostMallocDefault));
            GV_TRY(hipMalloc((void **)&s.dev, pool_bytes));
            GV_TRY(hipEventCreateWithFlags(&s.copied, hipEventDisableTiming));
            GV_TRY(hipEventCreateWithFlags(&s.trained, hipEventDisableTiming));
        }
#undef GV_TRY
        *out = ctx;
        return GV_OK;
    });
}

void gv_destroy(gv_ctx *ctx) {
    if (!ctx) return;
    (void)hipSetDevice(ctx->cfg.device);
    if (ctx->copy) (void)hipStreamSynchronize(ctx->copy);
    if (ctx->compute) (void)hipStreamSynchronize(ctx->compute);
    try {
        fold_spans(ctx);
    } catch (...) {
    }
    for (const TimedSpan &s : ctx->spans) {  // left over only if folding failed
        (void)hipEventDestroy(s.start);
        (void)hipEventDestroy(s.stop);
    }
    for (hipEvent_t e : ctx->spare_events) (void)hipEventDestroy(e);
    for (PoolSlot &s : ctx->slot) {
        if (s.host) (void)hipHostFree(s.host);
        if (s.dev) (void)hipFree(s.dev);
        if (s.copied) (void)hipEventDestroy(s.copied);
        if (s.trained) (void)hipEventDestroy(s.trained);
    }
    free_matrices(ctx);
    if (ctx->negatives) (void)hipFree(ctx->negatives);
    if (ctx->records) (void)hipFree(ctx->records);
    if (ctx->eval_scratch) (void)hipFree(ctx->eval_scratch);
    if (ctx->error_flag) (void)hipFree(ctx->error_flag);
    if (ctx->dev_loss) (void)hipFree(ctx->dev_loss);
    if (ctx->copy) (void)hipStreamDestroy(ctx->copy);
    if (ctx->compute) (void)hipStreamDestroy(ctx->compute);
    delete ctx;
}

int gv_set_graph(gv_ctx *ctx, uint32_t n, uint64_t m, const uint32_t *host_src, const uint32_t *host_dst) {
    if (!ctx) return GV_EINVAL;
    return guarded(ctx, [&]() -> int {
        if (n == 0 || (m > 0 && (!host_src || !host_dst)))
            return fail(ctx, GV_EINVAL, "empty graph or null edge arrays");
        int rc = bind_device(ctx);
        if (rc) return rc;
        std::vector<uint32_t> deg(n, 0u);
        for (uint64_t i = 0; i < m; ++i) {
            const uint32_t a = host_src[i], b = host_dst[i];
            if (a >= n || b >= n)
                return fail(ctx, GV_EINVAL, "edge %llu names node id >= n (%u)", (unsigned long long)i, n);
            if (deg[a] == UINT32_MAX || deg[b] == UINT32_MAX) return fail(ctx, GV_EINVAL, "degree overflow");
            ++deg[a];
            ++deg[b];
        }
        return adopt_degrees(ctx, n, std::move(deg));
    });
}

int gv_set_degrees(gv_ctx *ctx, uint32_t n, const uint32_t *host_deg) {
    if (!ctx) return GV_EINVAL;
    return guarded(ctx, [&]() -> int {
        if (n == 0 || !host_deg) return fail(ctx, GV_EINVAL, "empty graph or null degree array");
        int rc = bind_device(ctx);
        if (rc) return rc;
        return adopt_degrees(ctx, n, std::vector<uint32_t>(host_deg, host_deg + n));
    });
}

int gv_set_weighted_graph(gv_ctx *ctx, uint32_t n, const uint64_t *host_offsets, const uint32_t *host_adj,
                          const float *host_weights) {
    if (!ctx) return GV_EINVAL;
    return guarded(ctx, [&]() -> int {
        if (n == 0 || !host_offsets || !host_adj || !host_weights) return fail(ctx, GV_EINVAL, "empty graph or null arrays");
        int rc = bind_device(ctx);
        if (rc) return rc;
        if (host_offsets[0] != 0) return fail(ctx, GV_EINVAL, "offsets[0] must be 0");
        std::vector<uint32_t> counts(n);
        for (uint32_t i = 0; i < n; ++i) {
            if (host_offsets[i + 1] < host_offsets[i] || host_offsets[i + 1] - host_offsets[i] > 0xFFFFFFFFull)
                return fail(ctx, GV_EINVAL, "offsets must ascend (row %u)", i);
            counts[i] = (uint32_t)(host_offsets[i + 1] - host_offsets[i]);
        }
        const uint64_t half_edges = host_offsets[n];
        if (half_edges == 0) return fail(ctx, GV_EINVAL, "graph without edges");
        for (uint64_t e = 0; e < half_edges; ++e) {
            if (host_adj[e] >= n) return fail(ctx, GV_EINVAL, "adjacency entry %llu names node id >= n", (unsigned long long)e);
            if (!(host_weights[e] >= 0.0f) || !isfinite(host_weights[e]))
                return fail(ctx, GV_EINVAL, "weight %llu is negative or not finite", (unsigned long long)e);
        }
        std::vector<double> wdeg(n);
        std::vector<uint32_t> node_thresh(n), node_alias(n), nbr_thresh(half_edges), nbr_alias(half_edges);
        rc = gv_build_walk_tables(n, host_offsets, host_weights, wdeg.data(), node_thresh.data(), node_alias.data(),
                                  nbr_thresh.data(), nbr_alias.data());
        if (rc == GV_ENOMEM) return fail(ctx, GV_ENOMEM, "out of host memory");
        if (rc) return fail(ctx, GV_EINVAL, "a node has edges but no weight, or the graph has no weight at all");
        rc = adopt_degrees(ctx, n, std::move(counts));
        if (rc) return rc;
        std::vector<uint2> node_table(n), nbr_table(half_edges);
        for (uint32_t i = 0; i < n; ++i) node_table[i] = make_uint2(node_thresh[i], node_alias[i]);
        for (uint64_t e = 0; e < half_edges; ++e) nbr_table[e] = make_uint2(nbr_thresh[e], nbr_alias[e]);
        GV_HIP(ctx, hipMalloc((void **)&ctx->dev_offsets, ((size_t)n + 1) * sizeof(uint64_t)));
        GV_HIP(ctx, hipMalloc((void **)&ctx->dev_adj, (size_t)half_edges * sizeof(uint32_t)));
        GV_HIP(ctx, hipMalloc((void **)&ctx->dev_node_table, (size_t)n * sizeof(uint2)));
        GV_HIP(ctx, hipMalloc((void **)&ctx->dev_nbr_table, (size_t)half_edges * sizeof(uint2)));
        GV_HIP(ctx, hipMemcpy(ctx->dev_offsets, host_offsets, ((size_t)n + 1) * sizeof(uint64_t), hipMemcpyHostToDevice));
        GV_HIP(ctx, hipMemcpy(ctx->dev_adj, host_adj, (size_t)half_edges * sizeof(uint32_t), hipMemcpyHostToDevice));
        GV_HIP(ctx, hipMemcpy(ctx->dev_node_table, node_table.data(), (size_t)n * sizeof(uint2), hipMemcpyHostToDevice));
        GV_HIP(ctx, hipMemcpy(ctx->dev_nbr_table, nbr_table.data(), (size_t)half_edges * sizeof(uint2), hipMemcpyHostToDevice));
        ctx->half_edges = half_edges;
        ctx->wdegree = std::move(wdeg);
        return GV_OK;
    });
}

int gv_build_alias(gv_ctx *ctx, double power) {
    return guarded(ctx, [&]() -> int {
        int rc = need_graph(ctx);
        if (rc) return rc;
        if (power != 0.75 && power != 1.0 && power != 0.0)
            return fail(ctx, GV_EINVAL, "power must be 0.75, 1.0 or 0.0");
        const uint32_t n = ctx->n;
        // the degree of a node, or on a weighted graph the sum of the weights of its edges
        const bool weighted = ctx->wdegree.size() == n;
        auto degree_of = [&](uint32_t node) { return weighted ? ctx->wdegree[node] : (double)ctx->degree[node]; };
        auto weight = [&](uint32_t node) {
            const double d = degree_of(node);
            if (power == 0.75) {
                const double root = sqrt(d);
                return root * sqrt(root);
            }
            return power == 1.0 ? d : 1.0;
        };
        std::vector<double> q(n);
        double degree_sum = 0.0;
        for (uint32_t i = 0; i < n; ++i) {
            degree_sum += degree_of(i);
            q[i] = weight(i);
        }
        std::vector<uint32_t> thresh(n), alias(n);
        double sum = 0.0;
        if (!gv::vose_table(q.data(), n, thresh.data(), alias.data(), &sum))
            return fail(ctx, GV_EINVAL, "all weights are zero (graph without edges)");
        // Hot ranks: the 65535 nodes of highest degree in falling order (ties by id); the rest share
        // the value 0xFFFF.  The tiled kernel keeps the row of lowest rank of a sample in registers.
        // A row is warm when, with kInFlight samples being processed at once (the order of magnitude of
        // a full launch: 2048 waves at a time, each with the samples of one batch), the expected number
        // of other in-flight samples naming the same row (as a walk endpoint, share deg/sum(deg),
        // or as one of the K negatives, share q/sum(q) each) exceeds kWarmThreshold: the mixed policy then updates it with
        // atomic adds.  Colder rows are updated with plain device-scope stores, which can drop an
        // update only when two of the few samples naming such a row are in flight together.  The
        // share grows with the degree, so the warm rows are the first warm_ranks of the ranking.
        // Under the orthogonal-block schedule the samples in flight all come from one block, where a
        // row's share is `partitions` times its share of the pool.
        const uint32_t B = ctx->cfg.partitions;
        // Where rows are so long that a wave gathers fewer than four samples at once, a sample's rows stay between
        // their load and their store for longer (it moves several times the bytes): half the threshold.
        const uint32_t per_batch = gv::samples_per_batch(ctx->cfg.dim, ctx->cfg.num_neg);
        const double kInFlight = 2048.0 * per_batch * (B > 0 ? (double)B : 1.0), kWarmThreshold = per_batch >= 4 ? 0.1 : 0.05;
        const uint32_t kRanked = 0xFFFFu;
        auto hotter = [&](uint32_t x, uint32_t y) {
            const double dx = degree_of(x), dy = degree_of(y);
            return dx != dy ? dx > dy : x < y;
        };
        std::vector<uint32_t> order(n);
        for (uint32_t i = 0; i < n; ++i) order[i] = i;
        const uint32_t ranked = n < kRanked ? n : kRanked;
        if (B > 0)
            std::sort(order.begin(), order.end(), hotter);  // the partition needs the whole order
        else
            std::partial_sort(order.begin(), order.begin() + ranked, order.end(), hotter);
        std::vector<uint16_t> rank(n, (uint16_t)kRanked);
        std::vector<uint32_t> ranked_bits(((size_t)n + 31) / 32, 0u);
        uint32_t warm_ranks = 0;
        for (uint32_t r = 0; r < ranked; ++r) {
            const uint32_t i = order[r];
            rank[i] = (uint16_t)r;
            ranked_bits[i >> 5] |= 1u << (i & 31u);
            const double share = (degree_sum > 0.0 ? degree_of(i) / degree_sum : 0.0) + (double)ctx->cfg.num_neg * q[i] / sum;
            if (share * kInFlight > kWarmThreshold) warm_ranks = r + 1;
        }
        std::vector<uint4> table(n);
        for (uint32_t i = 0; i < n; ++i)  // ranks of both candidates and the bucket's node save the kernel gathers
            table[i] = make_uint4(thresh[i], alias[i], (uint32_t)rank[i] | (uint32_t)rank[alias[i]] << 16, i);

        // Orthogonal blocks (Sec. 3.2, Alg. 3): degree-guided partition (Sec. 4.3: nodes by falling degree dealt
        // back and forth over the partitions) and one alias table per partition, over its nodes in increasing id.
        std::vector<uint32_t> part, members, part_thresh, part_alias;
        std::vector<uint64_t> part_offsets;
        std::vector<uint4> part_tables;
        std::vector<uint8_t> part_bytes;
        if (B > 0) {
            part.resize(n);
            for (uint32_t r = 0; r < n; ++r) {
                const uint32_t round = r / B, k = r % B;
                part[order[r]] = round % 2 == 0 ? k : B - 1 - k;
            }
            part_offsets.assign(B + 1, 0);
            for (uint32_t i = 0; i < n; ++i) part_offsets[part[i] + 1] += 1;
            for (uint32_t j = 0; j < B; ++j) part_offsets[j + 1] += part_offsets[j];
            members.resize(n);
            std::vector<uint64_t> fill(part_offsets.begin(), part_offsets.end() - 1);
            for (uint32_t i = 0; i < n; ++i) members[fill[part[i]]++] = i;
            part_thresh.resize(n);
            part_alias.resize(n);
            part_tables.resize(n);
            for (uint32_t j = 0; j < B; ++j) {
                const uint64_t lo = part_offsets[j], size = part_offsets[j + 1] - lo;
                std::vector<double> qj(size);
                for (uint64_t l = 0; l < size; ++l) qj[l] = weight(members[lo + l]);
                std::vector<uint32_t> tj(size), aj(size);
                if (size == 0 || !gv::vose_table(qj.data(), size, tj.data(), aj.data(), nullptr))
                    return fail(ctx, GV_EINVAL, "partition %u of %u has no node with a positive weight", j, B);
                for (uint64_t l = 0; l < size; ++l) {
                    const uint32_t self = members[lo + l], other = members[lo + aj[l]];
                    part_thresh[lo + l] = tj[l];
                    part_alias[lo + l] = other;
                    part_tables[lo + l] = make_uint4(tj[l], other, (uint32_t)rank[self] | (uint32_t)rank[other] << 16, self);
                }
            }
            part_bytes.resize(n);
            for (uint32_t i = 0; i < n; ++i) part_bytes[i] = (uint8_t)part[i];
        }
        order.clear();
        order.shrink_to_fit();

        rc = sync_all(ctx);
        if (rc != GV_OK && rc != GV_EINVAL && rc != GV_ESTATE) return rc;  // reports about pools already trained do not stop this call
        GV_HIP(ctx, hipMemcpy(ctx->alias, table.data(), (size_t)n * sizeof(uint4), hipMemcpyHostToDevice));
        GV_HIP(ctx, hipMemcpy(ctx->dev_rank, rank.data(), (size_t)n * sizeof(uint16_t), hipMemcpyHostToDevice));
        GV_HIP(ctx, hipMemcpy(ctx->dev_ranked, ranked_bits.data(), ranked_bits.size() * sizeof(uint32_t),
                              hipMemcpyHostToDevice));
        if (B > 0) {
            if (!ctx->dev_part_tables) {
                GV_HIP(ctx, hipMalloc((void **)&ctx->dev_part_tables, (size_t)n * sizeof(uint4)));
                GV_HIP(ctx, hipMalloc((void **)&ctx->dev_part_offsets, ((size_t)B + 1) * sizeof(uint64_t)));
                GV_HIP(ctx, hipMalloc((void **)&ctx->dev_part, (size_t)n));
            }
            GV_HIP(ctx, hipMemcpy(ctx->dev_part_tables, part_tables.data(), (size_t)n * sizeof(uint4), hipMemcpyHostToDevice));
            GV_HIP(ctx, hipMemcpy(ctx->dev_part_offsets, part_offsets.data(), ((size_t)B + 1) * sizeof(uint64_t),
                                  hipMemcpyHostToDevice));
            GV_HIP(ctx, hipMemcpy(ctx->dev_part, part_bytes.data(), (size_t)n, hipMemcpyHostToDevice));
            ctx->part = std::move(part);
            ctx->part_offsets = std::move(part_offsets);
            ctx->part_members = std::move(members);
            ctx->part_thresh = std::move(part_thresh);
            ctx->part_alias = std::move(part_alias);
        }
        ctx->warm_ranks = warm_ranks;
        ctx->stats.warm_rows = warm_ranks;
        ctx->alias_ready = true;
        return GV_OK;
    });
}

int gv_get_alias(gv_ctx *ctx, uint32_t *host_thresh, uint32_t *host_alias) {
    return guarded(ctx, [&]() -> int {
        int rc = need_trainable(ctx);
        if (rc) return rc;
        if (!host_thresh || !host_alias) return fail(ctx, GV_EINVAL, "null output");
        std::vector<uint4> table(ctx->n);
        GV_HIP(ctx, hipMemcpy(table.data(), ctx->alias, (size_t)ctx->n * sizeof(uint4), hipMemcpyDeviceToHost));
        for (uint32_t i = 0; i < ctx->n; ++i) {
            host_thresh[i] = table[i].x;
            host_alias[i] = table[i].y;
        }
        return GV_OK;
    });
}

int gv_init_embeddings(gv_ctx *ctx, uint64_t seed) {
    return guarded(ctx, [&]() -> int {
        int rc = need_graph(ctx);
        if (rc) return rc;
        rc = sync_all(ctx);
        if (rc != GV_OK && rc != GV_EINVAL && rc != GV_ESTATE) return rc;  // reports about pools already trained do not stop this call
        GV_HIP(ctx, gv::launch_init_vertex(ctx->vertex, ctx->n, ctx->cfg.dim, seed, ctx->compute));
        GV_HIP(ctx, hipMemsetAsync(ctx->context, 0, (size_t)ctx->n * ctx->cfg.dim * sizeof(float), ctx->compute));
        GV_HIP(ctx, hipStreamSynchronize(ctx->compute));
        return GV_OK;
    });
}

static int matrix_window(gv_ctx *ctx, int which, uint64_t row0, uint64_t rows, float **base) {
    if (which != GV_VERTEX && which != GV_CONTEXT) return fail(ctx, GV_EINVAL, "which must be GV_VERTEX or GV_CONTEXT");
    if (row0 > ctx->n || rows > ctx->n - row0)
        return fail(ctx, GV_EINVAL, "rows [%llu, %llu) outside the matrix (%u rows)", (unsigned long long)row0,
                    (unsigned long long)(row0 + rows), ctx->n);
    *base = (which == GV_VERTEX ? ctx->vertex : ctx->context) + row0 * ctx->cfg.dim;
    return GV_OK;
}

int gv_set_embeddings(gv_ctx *ctx, int which, const float *host_rows, uint64_t row0, uint64_t rows) {
    return guarded(ctx, [&]() -> int {
        int rc = need_graph(ctx);
        if (rc) return rc;
        float *base = nullptr;
        rc = matrix_window(ctx, which, row0, rows, &base);
        if (rc) return rc;
        if (rows == 0) return GV_OK;
        if (!host_rows) return fail(ctx, GV_EINVAL, "null input");
        rc = sync_all(ctx);
        if (rc != GV_OK && rc != GV_EINVAL && rc != GV_ESTATE) return rc;  // reports about pools already trained do not stop this call
        GV_HIP(ctx, hipMemcpy(base, host_rows, rows * ctx->cfg.dim * sizeof(float), hipMemcpyHostToDevice));
        return GV_OK;
    });
}

int gv_read_embeddings(gv_ctx *ctx, int which, float *host_rows, uint64_t row0, uint64_t rows) {
    return guarded(ctx, [&]() -> int {
        int rc = need_graph(ctx);
        if (rc) return rc;
        float *base = nullptr;
        rc = matrix_window(ctx, which, row0, rows, &base);
        if (rc) return rc;
        if (rows == 0) return GV_OK;
        if (!host_rows) return fail(ctx, GV_EINVAL, "null output");
        rc = sync_all(ctx);
        if (rc) return rc;
        GV_HIP(ctx, hipMemcpy(host_rows, base, rows * ctx->cfg.dim * sizeof(float), hipMemcpyDeviceToHost));
        return GV_OK;
    });
}

int gv_device_embeddings(gv_ctx *ctx, int which, float **dev_rows) {
    return guarded(ctx, [&]() -> int {
        int rc = need_graph(ctx);
        if (rc) return rc;
        if (!dev_rows) return fail(ctx, GV_EINVAL, "null output");
        return matrix_window(ctx, which, 0, 0, dev_rows);
    });
}

int gv_acquire_pool_slot(gv_ctx *ctx, uint32_t **host_pairs) {
    if (!ctx || !host_pairs) return ctx ? fail(ctx, GV_EINVAL, "null output") : GV_EINVAL;
    return guarded(ctx, [&]() -> int {
        int rc = bind_device(ctx);
        if (rc) return rc;
        int i = -1;
        rc = pick_free_slot(ctx, &i);
        if (rc) return rc;
        ctx->slot[i].state = kFilling;
        *host_pairs = ctx->slot[i].host;
        return GV_OK;
    });
}

int gv_push_pool(gv_ctx *ctx, const uint32_t *host_pairs, uint64_t count) {
    return guarded(ctx, [&]() -> int {
        if (!ctx) return GV_EINVAL;
        int i = -1;  // the acquired slot this push refers to, if any
        for (size_t t = 0; t < ctx->slot.size(); ++t)
            if (ctx->slot[t].state == kFilling && ctx->slot[t].host == host_pairs) i = (int)t;
        // a push that fails gives an acquired slot back: it would otherwise stay out of the ring for good
        auto give_back = [&](int rc) -> int {
            if (i >= 0) ctx->slot[i].state = kFree;
            return rc;
        };
        int rc = need_trainable(ctx);
        if (rc) return give_back(rc);
        if (count > ctx->cfg.pool_capacity)
            return give_back(fail(ctx, GV_EINVAL, "pool of %llu samples exceeds pool_capacity %llu",
                                  (unsigned long long)count, (unsigned long long)ctx->cfg.pool_capacity));
        if (count > 0 && !host_pairs) return fail(ctx, GV_EINVAL, "null pool");
        if (i < 0) {
            rc = pick_free_slot(ctx, &i);
            if (rc) return rc;
            memcpy(ctx->slot[i].host, host_pairs, count * 2 * sizeof(uint32_t));
            ctx->slot[i].state = kFilling;
        }
        PoolSlot &s = ctx->slot[i];
        s.count = count;
        auto hip_step = [&](hipError_t e, const char *what) -> int {
            if (e == hipSuccess) return GV_OK;
            return give_back(fail(ctx, e == hipErrorOutOfMemory ? GV_ENOMEM : GV_EHIP, "%s: %s", what, hipGetErrorString(e)));
        };
        TimedSpan span{};
        const bool timed = ctx->cfg.profile != 0 && count > 0;
        if (timed) {
            rc = begin_span(ctx, 1, ctx->copy, &span);
            if (rc) return give_back(rc);
        }
        if (count > 0) {
            rc = hip_step(hipMemcpyAsync(s.dev, s.host, count * 2 * sizeof(uint32_t), hipMemcpyHostToDevice, ctx->copy),
                          "hipMemcpyAsync of the pool");
            if (rc) return rc;
        }
        if (timed) {
            rc = end_span(ctx, ctx->copy, span);
            if (rc) return give_back(rc);
        }
        rc = hip_step(hipEventRecord(s.copied, ctx->copy), "hipEventRecord");
        if (rc) return rc;
        ctx->stats.h2d_bytes += count * 2 * sizeof(uint32_t);
        s.state = kQueued;
        ctx->queue.push_back(i);
        return GV_OK;
    });
}

int gv_train_pool(gv_ctx *ctx) {
    return guarded(ctx, [&]() -> int {
        int rc = need_trainable(ctx);
        if (rc) return rc;
        if (ctx->queue.empty()) return fail(ctx, GV_ESTATE, "no pool queued: call gv_push_pool first");
        const int i = ctx->queue.front();
        ctx->queue.erase(ctx->queue.begin());
        PoolSlot &s = ctx->slot[i];
        // Whatever goes wrong from here on, the slot returns to the ring only after the copy into its
        // device twin and every launch that may read it have ended.
        auto drop_slot = [&](int rc) -> int {
            (void)hipStreamSynchronize(ctx->copy);
            (void)hipStreamSynchronize(ctx->compute);
            s.state = kFree;
            return rc;
        };
        hipError_t e = hipStreamWaitEvent(ctx->compute, s.copied, 0);
        if (e != hipSuccess) return drop_slot(fail(ctx, GV_EHIP, "hipStreamWaitEvent: %s", hipGetErrorString(e)));
        rc = train_any(ctx, s.dev, s.host, s.count);
        if (rc) return drop_slot(rc);
        e = hipEventRecord(s.trained, ctx->compute);
        if (e != hipSuccess) return drop_slot(fail(ctx, GV_EHIP, "hipEventRecord: %s", hipGetErrorString(e)));
        s.state = kTraining;
        return GV_OK;
    });
}

int gv_train_device_pool(gv_ctx *ctx, const uint32_t *dev_pairs, uint64_t count) {
    return guarded(ctx, [&]() -> int {
        int rc = need_trainable(ctx);
        if (rc) return rc;
        if (count > (1ull << 31)) return fail(ctx, GV_EINVAL, "at most 2^31 samples per call");
        if (count > 0 && !dev_pairs) return fail(ctx, GV_EINVAL, "null pool");
        return train_any(ctx, dev_pairs, nullptr, count);
    });
}

int gv_train_device_pool_static(gv_ctx *ctx, const uint32_t *dev_pairs, uint64_t count) {
    return guarded(ctx, [&]() -> int {
        int rc = need_trainable(ctx);
        if (rc) return rc;
        if (ctx->cfg.mode != GV_MODE_HOGWILD)
            return fail(ctx, GV_ESTATE, "gv_train_device_pool_static trains asynchronously only (GV_MODE_HOGWILD)");
        if (!ctx->static_records) return fail(ctx, GV_ESTATE, "no static scratch on device %d", ctx->cfg.device);
        if (count > (1ull << 31)) return fail(ctx, GV_EINVAL, "at most 2^31 samples per call");
        if (count == 0) return GV_OK;
        if (!dev_pairs) return fail(ctx, GV_EINVAL, "null pool");
        rc = train_hogwild(ctx, dev_pairs, count, ctx->static_records);
        if (rc) return rc;
        ctx->next_g += count;
        ctx->stats.samples_trained = ctx->next_g;
        ctx->stats.pools_trained += 1;
        return GV_OK;
    });
}

int gv_get_partitions(gv_ctx *ctx, uint32_t *host_part, uint64_t *host_offsets, uint32_t *host_members,
                      uint32_t *host_thresh, uint32_t *host_alias) {
    return guarded(ctx, [&]() -> int {
        int rc = need_trainable(ctx);
        if (rc) return rc;
        if (ctx->cfg.partitions == 0 || ctx->part.size() != ctx->n)
            return fail(ctx, GV_ESTATE, "the context was created without partitions");
        if (!host_part || !host_offsets || !host_members || !host_thresh || !host_alias)
            return fail(ctx, GV_EINVAL, "null output");
        std::copy(ctx->part.begin(), ctx->part.end(), host_part);
        std::copy(ctx->part_offsets.begin(), ctx->part_offsets.end(), host_offsets);
        std::copy(ctx->part_members.begin(), ctx->part_members.end(), host_members);
        std::copy(ctx->part_thresh.begin(), ctx->part_thresh.end(), host_thresh);
        std::copy(ctx->part_alias.begin(), ctx->part_alias.end(), host_alias);
        return GV_OK;
    });
}

int gv_train_device_blocks(gv_ctx *ctx, const uint32_t *dev_pairs, const uint32_t *dev_order,
                           const uint64_t *host_block_offsets, uint64_t count) {
    return guarded(ctx, [&]() -> int {
        int rc = need_trainable(ctx);
        if (rc) return rc;
        const uint32_t B = ctx->cfg.partitions;
        if (B == 0 || ctx->part.size() != ctx->n) return fail(ctx, GV_ESTATE, "the context was created without partitions");
        if (ctx->cfg.mode != GV_MODE_HOGWILD)
            return fail(ctx, GV_ESTATE, "orthogonal blocks are trained asynchronously only (GV_MODE_HOGWILD)");
        if (count > (1ull << 32)) return fail(ctx, GV_EINVAL, "at most 2^32 samples per call");
        if (!host_block_offsets) return fail(ctx, GV_EINVAL, "null block offsets");
        const uint64_t blocks = (uint64_t)B * B;
        if (host_block_offsets[0] != 0 || host_block_offsets[blocks] != count)
            return fail(ctx, GV_EINVAL, "block offsets must run from 0 to count");
        for (uint64_t b = 0; b < blocks; ++b)
            if (host_block_offsets[b] > host_block_offsets[b + 1] ||
                host_block_offsets[b + 1] - host_block_offsets[b] > (1ull << 31))
                return fail(ctx, GV_EINVAL, "block offsets must ascend, at most 2^31 samples per block");
        if (count == 0) return GV_OK;
        if (!dev_pairs || !dev_order) return fail(ctx, GV_EINVAL, "null pool");
        // sub-episode o = b / B trains the blocks (i, (i + o) mod B), i = b mod B, one launch each, in order
        for (uint64_t b = 0; b < blocks; ++b) {
            const uint64_t lo = host_block_offsets[b], size = host_block_offsets[b + 1] - lo;
            if (size == 0) continue;
            const uint32_t o = (uint32_t)(b / B), i = (uint32_t)(b % B);
            const BlockOfPool block{dev_order + lo, (i + o) % B};
            rc = train_hogwild(ctx, dev_pairs + 2 * lo, size, nullptr, &block);
            if (rc) return rc;
        }
        ctx->next_g += count;
        ctx->stats.samples_trained = ctx->next_g;
        ctx->stats.pools_trained += 1;
        return GV_OK;
    });
}

int gv_draw_negatives_partitioned(gv_ctx *ctx, uint64_t first_g, uint64_t count, const uint32_t *host_v,
                                  uint32_t *host_out) {
    return guarded(ctx, [&]() -> int {
        int rc = need_trainable(ctx);
        if (rc) return rc;
        if (ctx->cfg.partitions == 0 || ctx->part.size() != ctx->n)
            return fail(ctx, GV_ESTATE, "the context was created without partitions");
        if (count == 0) return GV_OK;
        if (!host_v || !host_out) return fail(ctx, GV_EINVAL, "null argument");
        if (count > (1ull << 31)) return fail(ctx, GV_EINVAL, "at most 2^31 samples per call");
        for (uint64_t i = 0; i < count; ++i)
            if (host_v[i] >= ctx->n) return fail(ctx, GV_EINVAL, "sample %llu names node id >= n", (unsigned long long)i);
        const uint32_t K = ctx->cfg.num_neg;
        rc = sync_all(ctx);
        if (rc) return rc;
        rc = ensure_negatives(ctx, count * K);
        if (rc) return rc;
        rc = ensure_eval_scratch(ctx, count * sizeof(uint32_t));
        if (rc) return rc;
        uint32_t *dev_v = (uint32_t *)ctx->eval_scratch;
        GV_HIP(ctx, hipMemcpyAsync(dev_v, host_v, count * sizeof(uint32_t), hipMemcpyHostToDevice, ctx->compute));
        GV_HIP(ctx, gv::launch_draw_negatives_partitioned(ctx->dev_part_tables, ctx->dev_part_offsets, ctx->dev_part, dev_v,
                                                          ctx->cfg.seed, first_g, count, K, ctx->negatives, ctx->compute));
        GV_HIP(ctx, hipMemcpyAsync(host_out, ctx->negatives, count * K * sizeof(uint32_t), hipMemcpyDeviceToHost,
                                   ctx->compute));
        GV_HIP(ctx, hipStreamSynchronize(ctx->compute));
        return GV_OK;
    });
}

int gv_set_adjacency(gv_ctx *ctx, const uint64_t *host_offsets, const uint32_t *host_adj) {
    return guarded(ctx, [&]() -> int {
        int rc = need_graph(ctx);
        if (rc) return rc;
        if (!host_offsets || !host_adj) return fail(ctx, GV_EINVAL, "null adjacency");
        const uint32_t n = ctx->n;
        if (host_offsets[0] != 0) return fail(ctx, GV_EINVAL, "offsets[0] must be 0");
        for (uint32_t i = 0; i < n; ++i)
            if (host_offsets[i + 1] - host_offsets[i] != (uint64_t)ctx->degree[i])
                return fail(ctx, GV_EINVAL, "row %u of the adjacency has %llu entries, the graph gives node %u degree %u",
                            i, (unsigned long long)(host_offsets[i + 1] - host_offsets[i]), i, ctx->degree[i]);
        const uint64_t half_edges = host_offsets[n];
        if (half_edges == 0) return fail(ctx, GV_EINVAL, "graph without edges");
        for (uint64_t e = 0; e < half_edges; ++e)
            if (host_adj[e] >= n)
                return fail(ctx, GV_EINVAL, "adjacency entry %llu names node id >= n", (unsigned long long)e);
        rc = sync_all(ctx);
        if (rc != GV_OK && rc != GV_EINVAL && rc != GV_ESTATE) return rc;  // reports about pools already trained do not stop this call
        if (ctx->wdegree.size() == n)
            return fail(ctx, GV_ESTATE, "the graph is weighted: gv_set_weighted_graph has uploaded its adjacency already");
        if (ctx->dev_offsets) (void)hipFree(ctx->dev_offsets);
        if (ctx->dev_adj) (void)hipFree(ctx->dev_adj);
        ctx->dev_offsets = nullptr;
        ctx->dev_adj = nullptr;
        ctx->half_edges = 0;
        GV_HIP(ctx, hipMalloc((void **)&ctx->dev_offsets, ((size_t)n + 1) * sizeof(uint64_t)));
        GV_HIP(ctx, hipMalloc((void **)&ctx->dev_adj, (size_t)half_edges * sizeof(uint32_t)));
        GV_HIP(ctx, hipMemcpy(ctx->dev_offsets, host_offsets, ((size_t)n + 1) * sizeof(uint64_t), hipMemcpyHostToDevice));
        GV_HIP(ctx, hipMemcpy(ctx->dev_adj, host_adj, (size_t)half_edges * sizeof(uint32_t), hipMemcpyHostToDevice));
        ctx->half_edges = half_edges;
        return GV_OK;
    });
}

int gv_augment_device(gv_ctx *ctx, uint64_t seed, uint32_t walk_length, uint32_t window, uint64_t first_walk,
                      uint64_t count, uint32_t shuffle, uint32_t *dev_pairs, uint64_t *walks_used) {
    if (walks_used) *walks_used = 0;
    return guarded(ctx, [&]() -> int {
        int rc = need_graph(ctx);
        if (rc) return rc;
        if (!ctx->dev_offsets) return fail(ctx, GV_ESTATE, "no adjacency: call gv_set_adjacency first");
        if (walk_length == 0 || walk_length > 64 || window == 0 || window > GV_MAX_WINDOW || shuffle > GV_SHUFFLE_PSEUDO)
            return fail(ctx, GV_EINVAL, "walk_length must be in 1..64, window in 1..GV_MAX_WINDOW, shuffle GV_SHUFFLE_*");
        if (count == 0) return GV_OK;
        if (!dev_pairs) return fail(ctx, GV_EINVAL, "null output");
        gv::AugmentArgs a{};
        a.offsets = ctx->dev_offsets;
        a.adj = ctx->dev_adj;
        a.pairs = (uint2 *)dev_pairs;
        a.half_edges = ctx->half_edges;
        a.seed = seed;
        a.first_walk = first_walk;
        a.count = count;
        a.per_walk = 0;  // pairs (i, j), i < j <= min(i + window, walk_length)
        for (uint32_t d = 1; d <= window && d <= walk_length; ++d) a.per_walk += walk_length + 1 - d;
        a.walks = (count + a.per_walk - 1) / a.per_walk;
        a.n = ctx->n;
        a.length = walk_length;
        a.window = window;
        a.pseudo_shuffle = shuffle == GV_SHUFFLE_PSEUDO ? 1u : 0u;
        a.node_table = ctx->dev_node_table;
        a.nbr_table = ctx->dev_nbr_table;
        if (walks_used) *walks_used = a.walks;
        GV_HIP(ctx, gv::launch_augment(a, ctx->compute));
        return GV_OK;
    });
}

int gv_draw_negatives(gv_ctx *ctx, uint64_t first_g, uint64_t count, uint32_t *host_out) {
    return guarded(ctx, [&]() -> int {
        int rc = need_trainable(ctx);
        if (rc) return rc;
        if (count == 0) return GV_OK;
        if (!host_out) return fail(ctx, GV_EINVAL, "null output");
        if (count > (1ull << 32)) return fail(ctx, GV_EINVAL, "at most 2^32 samples per call");
        const uint32_t K = ctx->cfg.num_neg;
        rc = ensure_negatives(ctx, count * K);
        if (rc) return rc;
        GV_HIP(ctx, gv::launch_draw_negatives(ctx->alias, ctx->n, ctx->cfg.seed, first_g, count, K, ctx->negatives,
                                              ctx->compute));
        GV_HIP(ctx, hipMemcpyAsync(host_out, ctx->negatives, count * K * sizeof(uint32_t), hipMemcpyDeviceToHost,
                                   ctx->compute));
        GV_HIP(ctx, hipStreamSynchronize(ctx->compute));
        return GV_OK;
    });
}

int gv_eval_loss(gv_ctx *ctx, const uint32_t *host_pairs, uint64_t count, uint64_t eval_seed, double *mean_loss) {
    return guarded(ctx, [&]() -> int {
        int rc = need_trainable(ctx);
        if (rc) return rc;
        if (!mean_loss || (count > 0 && !host_pairs)) return fail(ctx, GV_EINVAL, "null argument");
        if (count == 0 || count > (1ull << 32) - 1) return fail(ctx, GV_EINVAL, "count must be in 1 .. 2^32-1");
        rc = sync_all(ctx);
        if (rc) return rc;
        // scratch layout: the running total (a double, 256 bytes reserved), then the pairs
        rc = ensure_eval_scratch(ctx, 256 + count * 2 * sizeof(uint32_t));
        if (rc) return rc;
        double *dev_total = (double *)ctx->eval_scratch;
        uint32_t *dev_pairs = (uint32_t *)((char *)ctx->eval_scratch + 256);
        GV_HIP(ctx, hipMemcpyAsync(dev_pairs, host_pairs, count * 2 * sizeof(uint32_t), hipMemcpyHostToDevice, ctx->compute));
        GV_HIP(ctx, hipMemsetAsync(dev_total, 0, sizeof(double), ctx->compute));
        gv::TrainArgs a = train_args(ctx, dev_pairs, 0, (uint32_t)count);
        a.seed = eval_seed;
        GV_HIP(ctx, gv::launch_eval_loss(a, ctx->cfg.dim, ctx->cfg.num_neg, dev_total, ctx->compute));
        double total = 0.0;
        GV_HIP(ctx, hipMemcpyAsync(&total, dev_total, sizeof(double), hipMemcpyDeviceToHost, ctx->compute));
        GV_HIP(ctx, hipStreamSynchronize(ctx->compute));
        *mean_loss = total / (double)count;
        return sync_all(ctx);  // reports ids >= n
    });
}

// cosines of `count` node pairs into host_out, through the evaluation scratch
static int cosine_scores(gv_ctx *ctx, const uint32_t *host_first, const uint32_t *host_second, uint64_t count,
                         float *host_out) {
    int rc = ensure_eval_scratch(ctx, count * (2 * sizeof(uint32_t) + sizeof(float)));
    if (rc) return rc;
    uint32_t *dev_ids = (uint32_t *)ctx->eval_scratch;
    float *dev_out = (float *)(dev_ids + 2 * count);
    GV_HIP(ctx, hipMemcpyAsync(dev_ids, host_first, count * sizeof(uint32_t), hipMemcpyHostToDevice, ctx->compute));
    GV_HIP(ctx, hipMemcpyAsync(dev_ids + count, host_second, count * sizeof(uint32_t), hipMemcpyHostToDevice, ctx->compute));
    GV_HIP(ctx, gv::launch_cosine(ctx->vertex, ctx->n, ctx->cfg.dim, dev_ids, dev_ids + count, (uint32_t)count, dev_out,
                                  ctx->error_flag, ctx->compute));
    GV_HIP(ctx, hipMemcpyAsync(host_out, dev_out, count * sizeof(float), hipMemcpyDeviceToHost, ctx->compute));
    GV_HIP(ctx, hipStreamSynchronize(ctx->compute));
    return GV_OK;
}

int gv_cosine(gv_ctx *ctx, const uint32_t *host_first, const uint32_t *host_second, uint64_t count, float *host_out) {
    return guarded(ctx, [&]() -> int {
        int rc = need_graph(ctx);
        if (rc) return rc;
        if (count == 0) return GV_OK;
        if (!host_first || !host_second || !host_out) return fail(ctx, GV_EINVAL, "null argument");
        if (count > (1ull << 32) - 1) return fail(ctx, GV_EINVAL, "at most 2^32-1 pairs per call");
        rc = sync_all(ctx);
        if (rc) return rc;
        rc = cosine_scores(ctx, host_first, host_second, count, host_out);
        if (rc) return rc;
        return sync_all(ctx);
    });
}

int gv_auc(const float *host_pos, uint64_t num_pos, const float *host_neg, uint64_t num_neg, double *auc) {
    if (!auc) return GV_EINVAL;
    *auc = 0.0;
    if (num_pos == 0 || num_neg == 0 || !host_pos || !host_neg) return GV_EINVAL;
    return guarded(nullptr, [&]() -> int {
        for (uint64_t i = 0; i < num_pos; ++i)
            if (!isfinite(host_pos[i])) return fail(nullptr, GV_EINVAL, "positive score %llu is not finite", (unsigned long long)i);
        for (uint64_t i = 0; i < num_neg; ++i)
            if (!isfinite(host_neg[i])) return fail(nullptr, GV_EINVAL, "negative score %llu is not finite", (unsigned long long)i);
        *auc = rank_auc(host_pos, num_pos, host_neg, num_neg);
        return GV_OK;
    });
}

int gv_link_prediction_auc(gv_ctx *ctx, const uint32_t *host_edge_first, const uint32_t *host_edge_second,
                           uint64_t num_edges, const uint32_t *host_other_first, const uint32_t *host_other_second,
                           uint64_t num_others, double *auc) {
    return guarded(ctx, [&]() -> int {
        int rc = need_graph(ctx);
        if (rc) return rc;
        if (!auc || !host_edge_first || !host_edge_second || !host_other_first || !host_other_second)
            return fail(ctx, GV_EINVAL, "null argument");
        if (num_edges == 0 || num_others == 0 || num_edges + num_others > (1ull << 31))
            return fail(ctx, GV_EINVAL, "both pair sets must be non-empty and hold at most 2^31 pairs together");
        rc = sync_all(ctx);
        if (rc) return rc;
        std::vector<float> scores(num_edges + num_others);
        rc = cosine_scores(ctx, host_edge_first, host_edge_second, num_edges, scores.data());
        if (rc) return rc;
        rc = cosine_scores(ctx, host_other_first, host_other_second, num_others, scores.data() + num_edges);
        if (rc) return rc;
        rc = sync_all(ctx);  // ids >= n
        if (rc) return rc;
        for (float x : scores)
            if (!isfinite(x)) return fail(ctx, GV_EINVAL, "an embedding row is not finite");
        *auc = rank_auc(scores.data(), num_edges, scores.data() + num_edges, num_others);
        return GV_OK;
    });
}

int gv_sync(gv_ctx *ctx) {
    if (!ctx) return GV_EINVAL;
    return guarded(ctx, [&]() -> int {
        int rc = bind_device(ctx);
        if (rc) return rc;
        return sync_all(ctx);
    });
}

int gv_get_stats(gv_ctx *ctx, gv_stats *out) {
    if (!ctx || !out) return ctx ? fail(ctx, GV_EINVAL, "null output") : GV_EINVAL;
    *out = ctx->stats;
    return GV_OK;
}

int gv_set_position(gv_ctx *ctx, uint64_t next_g) {
    if (!ctx) return GV_EINVAL;
    ctx->next_g = next_g;
    ctx->stats.samples_trained = next_g;
    return GV_OK;
}

}  // extern "C"
