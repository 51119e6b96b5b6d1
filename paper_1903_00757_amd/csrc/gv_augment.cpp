// Host producer of sample pools: parallel online augmentation (Sec. 3.1, Alg. 2) with the
// cache-friendly pseudo shuffle of the same section.  Pure host code: it writes into any
// caller buffer, in particular into the pinned pool slots of a context.
#include <stdint.h>

#include <math.h>

#include <algorithm>
#include <atomic>
#include <exception>
#include <new>
#include <thread>
#include <vector>

#include "gv_host.hpp"
#include "gvhot.h"

namespace {

struct Words {
    uint32_t w[4];
};

// Philox4x32-10 (Salmon et al., SC'11), counter (index lo, index hi, sub-index, stream).
inline Words philox(uint64_t seed, uint64_t index, uint32_t sub, uint32_t stream) {
    uint32_t c0 = (uint32_t)index, c1 = (uint32_t)(index >> 32), c2 = sub, c3 = stream;
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    for (int round = 0; round < 10; ++round) {
        const uint64_t a = 0xD2511F53ull * c0, b = 0xCD9E8D57ull * c2;
        const uint32_t n0 = (uint32_t)(b >> 32) ^ c1 ^ k0, n2 = (uint32_t)(a >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)b;
        c3 = (uint32_t)a;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Words{{c0, c1, c2, c3}};
}

// uniform integer in [0, range) from the first two words
inline uint64_t pick(const Words &r, uint64_t range) {
    const unsigned __int128 wide = (unsigned __int128)(((uint64_t)r.w[0] << 32) | r.w[1]) * range;
    return (uint64_t)(wide >> 64);
}

constexpr uint32_t kWalkStream = 4;

}  // namespace

// Tables of a weighted graph's walk (null for an unweighted graph): alias table over the nodes for the
// departure, one alias table per adjacency row for the steps (Sec. 4.3).
struct WalkTables {
    const uint32_t *node_thresh, *node_alias, *nbr_thresh, *nbr_alias;
};

static int augment(uint32_t n, const uint64_t *host_offsets, const uint32_t *host_adj, const WalkTables *tables,
                   uint64_t seed, uint32_t walk_length, uint32_t window, uint64_t first_walk, uint64_t count,
                   uint32_t shuffle, uint32_t threads, uint32_t *host_pairs, uint64_t *walks_used) {
    if (walks_used) *walks_used = 0;
    if (count == 0) return GV_OK;
    if (!host_offsets || !host_adj || !host_pairs || n == 0 || walk_length == 0 || window == 0 ||
        window > GV_MAX_WINDOW || shuffle > GV_SHUFFLE_PSEUDO)
        return GV_EINVAL;
    const uint64_t half_edges = host_offsets[n];
    if (half_edges == 0 || host_offsets[0] != 0) return GV_EINVAL;
    const uint32_t L = walk_length, s = window;
    uint64_t per_walk = 0;  // pairs (i, j), i < j <= min(i + s, L)
    for (uint32_t d = 1; d <= s && d <= L; ++d) per_walk += L + 1 - d;
    const uint64_t walks = (count + per_walk - 1) / per_walk;
    if (walks_used) *walks_used = walks;

    // Pseudo shuffle: the pool is cut into `s` consecutive blocks and sample number t (in
    // generation order) is appended to block t mod s, so the s samples that follow each other
    // inside a walk (and share a node) end up a block apart while every block is written
    // sequentially.  Block b holds the samples t = b, b + s, b + 2s, ...
    std::vector<uint64_t> block_start(s + 1, 0);
    for (uint32_t b = 0; b < s; ++b) block_start[b + 1] = block_start[b] + (count > b ? (count - b + s - 1) / s : 0);

    const uint32_t workers = (uint32_t)std::max<uint64_t>(1, std::min<uint64_t>(threads ? threads : 1, walks));
    // The adjacency is checked where a walk touches it (a full scan per pool would cost as much as
    // the walks): a row that is empty, runs backwards or past the end, or an entry >= n stops the
    // walk's worker and the call reports GV_EINVAL.
    std::atomic<bool> broken{false};
    // A worker advances kGroup walks together, step by step: every step of a walk waits for the memory
    // access of the step before it, and the chains of different walks overlap.
    constexpr uint32_t kGroup = 32;
    std::vector<std::vector<uint32_t>> paths(workers);
    for (auto &path : paths) path.resize((size_t)kGroup * (L + 1));
    auto work = [&](uint32_t worker) {
        uint32_t *const path = paths[worker].data();  // walk k of the group: path[k * (L + 1) + t]
        const uint64_t lo = walks * worker / workers, hi = walks * (worker + 1) / workers;
        for (uint64_t w0 = lo; w0 < hi; w0 += kGroup) {
            const uint32_t group = (uint32_t)std::min<uint64_t>(kGroup, hi - w0);
            if (tables) {
                for (uint32_t k = 0; k < group; ++k) {
                    // weighted graph: alias draw over the nodes, weights = weighted degrees
                    const Words r0 = philox(seed, first_walk + w0 + k, 0, kWalkStream);
                    const uint64_t j = pick(r0, n);
                    const uint32_t start = r0.w[2] < tables->node_thresh[j] ? (uint32_t)j : tables->node_alias[j];
                    if (start >= n) {
                        broken.store(true, std::memory_order_relaxed);
                        return;
                    }
                    path[(size_t)k * (L + 1)] = start;
                }
            } else {
                // departure: owner of a uniformly chosen half-edge = probability proportional to degree; the
                // last node x with offsets[x] <= e, found by the group's binary searches side by side
                uint64_t e[kGroup];
                uint32_t first[kGroup], length[kGroup];  // the answer lies in first .. first + length - 1
                for (uint32_t k = 0; k < group; ++k) {
                    e[k] = pick(philox(seed, first_walk + w0 + k, 0, kWalkStream), half_edges);
                    first[k] = 0;
                    length[k] = n;
                }
                for (uint32_t span = n; span > 1; span -= span / 2)  // the longest search decides the number of turns
                    for (uint32_t k = 0; k < group; ++k) {
                        const uint32_t half = length[k] / 2;
                        const bool right = half > 0 && host_offsets[first[k] + half] <= e[k];
                        first[k] += right ? half : 0u;
                        length[k] = half == 0 ? length[k] : (right ? length[k] - half : half);
                    }
                for (uint32_t k = 0; k < group; ++k) {
                    if (!(host_offsets[first[k]] <= e[k] && e[k] < host_offsets[first[k] + 1])) {  // offsets not ascending
                        broken.store(true, std::memory_order_relaxed);
                        return;
                    }
                    path[(size_t)k * (L + 1)] = first[k];
                }
            }
            for (uint32_t t = 1; t <= L; ++t) {
                // passes over the group, so that its row bounds, then (weighted graph) its table entries, then its
                // neighbours, are all requested from memory before the first of them is needed
                uint64_t begin[kGroup], degree[kGroup], at[kGroup];
                for (uint32_t k = 0; k < group; ++k) {
                    const uint32_t x = path[(size_t)k * (L + 1) + t - 1];
                    begin[k] = host_offsets[x];
                    degree[k] = host_offsets[x + 1] - begin[k];
                }
                uint32_t word[kGroup];  // weighted step: the random word that decides between an entry and its alias
                for (uint32_t k = 0; k < group; ++k) {
                    if (degree[k] == 0 || begin[k] + degree[k] > half_edges || begin[k] + degree[k] < begin[k]) {
                        broken.store(true, std::memory_order_relaxed);
                        return;
                    }
                    const Words r = philox(seed, first_walk + w0 + k, t, kWalkStream);
                    at[k] = pick(r, degree[k]);
                    word[k] = r.w[2];
                    if (tables) {
                        __builtin_prefetch(tables->nbr_thresh + begin[k] + at[k]);
                        __builtin_prefetch(tables->nbr_alias + begin[k] + at[k]);
                    } else {
                        __builtin_prefetch(host_adj + begin[k] + at[k]);
                    }
                }
                if (tables)
                    for (uint32_t k = 0; k < group; ++k) {
                        if (!(word[k] < tables->nbr_thresh[begin[k] + at[k]])) {  // weighted step: the entry or its alias
                            at[k] = tables->nbr_alias[begin[k] + at[k]];
                            if (at[k] >= degree[k]) {
                                broken.store(true, std::memory_order_relaxed);
                                return;
                            }
                        }
                        __builtin_prefetch(host_adj + begin[k] + at[k]);
                    }
                for (uint32_t k = 0; k < group; ++k) {
                    const uint32_t next = host_adj[begin[k] + at[k]];
                    if (next >= n) {
                        broken.store(true, std::memory_order_relaxed);
                        return;
                    }
                    path[(size_t)k * (L + 1) + t] = next;
                    __builtin_prefetch(host_offsets + next);
                }
            }
            for (uint32_t k = 0; k < group; ++k) {
                const uint32_t *const mine = path + (size_t)k * (L + 1);
                uint64_t t_global = (w0 + k) * per_walk;
                // sample t goes to block t mod s at offset t / s: both kept up to date by counting
                uint64_t block = t_global % s, offset = t_global / s;
                for (uint32_t i = 0; i <= L; ++i)
                    for (uint32_t j = i + 1; j <= L && j - i <= s; ++j, ++t_global) {
                        if (t_global >= count) return;
                        const uint64_t at = shuffle == GV_SHUFFLE_PSEUDO ? block_start[block] + offset : t_global;
                        host_pairs[2 * at] = mine[i];
                        host_pairs[2 * at + 1] = mine[j];
                        if (++block == s) {
                            block = 0;
                            ++offset;
                        }
                    }
            }
        }
    };
    if (workers == 1) {
        work(0);
    } else {
        std::vector<std::thread> pool;
        pool.reserve(workers);
        try {
            for (uint32_t i = 0; i < workers; ++i) pool.emplace_back(work, i);
        } catch (...) {  // a thread could not start: finish the ones that did, then report
            for (std::thread &t : pool) t.join();
            throw;
        }
        for (std::thread &t : pool) t.join();
    }
    return broken.load() ? GV_EINVAL : GV_OK;
}

extern "C" int gv_augment(uint32_t n, const uint64_t *host_offsets, const uint32_t *host_adj, uint64_t seed,
                          uint32_t walk_length, uint32_t window, uint64_t first_walk, uint64_t count,
                          uint32_t shuffle, uint32_t threads, uint32_t *host_pairs, uint64_t *walks_used) {
    try {
        return augment(n, host_offsets, host_adj, nullptr, seed, walk_length, window, first_walk, count, shuffle, threads,
                       host_pairs, walks_used);
    } catch (const std::bad_alloc &) {
        return GV_ENOMEM;
    } catch (...) {  // std::system_error of a thread that could not start, and anything else
        return GV_EHIP;
    }
}

extern "C" int gv_augment_weighted(uint32_t n, const uint64_t *host_offsets, const uint32_t *host_adj,
                                   const uint32_t *host_node_thresh, const uint32_t *host_node_alias,
                                   const uint32_t *host_nbr_thresh, const uint32_t *host_nbr_alias, uint64_t seed,
                                   uint32_t walk_length, uint32_t window, uint64_t first_walk, uint64_t count,
                                   uint32_t shuffle, uint32_t threads, uint32_t *host_pairs, uint64_t *walks_used) {
    if (walks_used) *walks_used = 0;
    if (!host_node_thresh || !host_node_alias || !host_nbr_thresh || !host_nbr_alias) return GV_EINVAL;
    const WalkTables tables{host_node_thresh, host_node_alias, host_nbr_thresh, host_nbr_alias};
    try {
        return augment(n, host_offsets, host_adj, &tables, seed, walk_length, window, first_walk, count, shuffle, threads,
                       host_pairs, walks_used);
    } catch (const std::bad_alloc &) {
        return GV_ENOMEM;
    } catch (...) {
        return GV_EHIP;
    }
}

bool gv::vose_table(const double *q, uint64_t size, uint32_t *thresh, uint32_t *alias, double *sum_out) {
    double sum = 0.0;
    for (uint64_t i = 0; i < size; ++i) sum += q[i];
    if (sum_out) *sum_out = sum;
    if (size == 0 || size > 0xFFFFFFFFull || !(sum > 0.0)) return false;
    std::vector<double> p(size), keep(size, 1.0);
    std::vector<uint32_t> below, above;  // stacks of entries under / at-or-over the mean
    below.reserve(size);
    above.reserve(size);
    for (uint64_t i = 0; i < size; ++i) {
        p[i] = q[i] * (double)size / sum;
        (p[i] < 1.0 ? below : above).push_back((uint32_t)i);
        alias[i] = (uint32_t)i;
    }
    while (!below.empty() && !above.empty()) {
        const uint32_t poor = below.back();
        below.pop_back();
        const uint32_t rich = above.back();
        above.pop_back();
        keep[poor] = p[poor];
        alias[poor] = rich;
        p[rich] = (p[rich] + p[poor]) - 1.0;
        (p[rich] < 1.0 ? below : above).push_back(rich);
    }
    for (uint64_t i = 0; i < size; ++i) {
        const double scaled = floor(keep[i] * 4294967296.0);
        thresh[i] = scaled >= 4294967295.0 ? 0xFFFFFFFFu : (uint32_t)scaled;
    }
    return true;
}

// Everything a walk on a weighted graph draws from (Sec. 4.3): weighted degrees (edge weights of a row summed
// left to right in fp64), the alias table over the nodes with those weights, and one alias table per adjacency
// row over its edge weights.
static int build_walk_tables(uint32_t n, const uint64_t *host_offsets, const float *host_weights, double *host_wdeg,
                             uint32_t *node_thresh, uint32_t *node_alias, uint32_t *nbr_thresh, uint32_t *nbr_alias) {
    if (n == 0 || !host_offsets || !host_weights || !node_thresh || !node_alias || !nbr_thresh || !nbr_alias)
        return GV_EINVAL;
    std::vector<double> wdeg(n), row;
    for (uint32_t x = 0; x < n; ++x) {
        const uint64_t begin = host_offsets[x], end = host_offsets[x + 1];
        if (end < begin) return GV_EINVAL;
        double total = 0.0;
        row.resize(end - begin);
        for (uint64_t e = begin; e < end; ++e) {
            if (!(host_weights[e] >= 0.0f)) return GV_EINVAL;
            row[e - begin] = (double)host_weights[e];
            total += (double)host_weights[e];
        }
        wdeg[x] = total;
        if (end > begin && !gv::vose_table(row.data(), end - begin, nbr_thresh + begin, nbr_alias + begin, nullptr))
            return GV_EINVAL;  // a row with entries but no weight
    }
    if (!gv::vose_table(wdeg.data(), n, node_thresh, node_alias, nullptr)) return GV_EINVAL;
    if (host_wdeg) std::copy(wdeg.begin(), wdeg.end(), host_wdeg);
    return GV_OK;
}

extern "C" int gv_build_walk_tables(uint32_t n, const uint64_t *host_offsets, const float *host_weights,
                                    double *host_wdeg, uint32_t *host_node_thresh, uint32_t *host_node_alias,
                                    uint32_t *host_nbr_thresh, uint32_t *host_nbr_alias) {
    try {
        return build_walk_tables(n, host_offsets, host_weights, host_wdeg, host_node_thresh, host_node_alias,
                                 host_nbr_thresh, host_nbr_alias);
    } catch (const std::bad_alloc &) {
        return GV_ENOMEM;
    } catch (...) {
        return GV_EHIP;
    }
}


// Redistribution of a pool into the grid of orthogonal blocks (Sec. 3.2, Alg. 3, the Redistribute step, done on
// the host as in the paper): a stable counting sort of the samples by block, blocks in training order.
static int redistribute(uint32_t n, const uint32_t *host_part, uint32_t partitions, const uint32_t *host_pairs,
                        uint64_t count, uint32_t threads, uint32_t *host_pairs_out, uint32_t *host_order,
                        uint64_t *host_block_offsets) {
    if (!host_block_offsets || partitions == 0 || partitions > GV_MAX_PARTITIONS) return GV_EINVAL;
    const uint32_t B = partitions;
    const uint64_t blocks = (uint64_t)B * B;
    for (uint64_t b = 0; b <= blocks; ++b) host_block_offsets[b] = 0;
    if (count == 0) return GV_OK;
    if (!host_part || !host_pairs || !host_pairs_out || !host_order || n == 0 || count > (1ull << 32)) return GV_EINVAL;
    const uint32_t workers = (uint32_t)std::max<uint64_t>(1, std::min<uint64_t>(threads ? threads : 1, (count + 65535) / 65536));
    // worker w owns samples [count w / workers, count (w + 1) / workers): counts per block, then its first
    // output place per block = everything of earlier blocks + that block's samples of earlier workers
    std::vector<std::vector<uint64_t>> place(workers, std::vector<uint64_t>(blocks, 0));
    std::atomic<bool> broken{false};
    auto block_of = [&](uint64_t i, uint64_t *b) {
        const uint32_t u = host_pairs[2 * i], v = host_pairs[2 * i + 1];
        if (u >= n || v >= n) return false;
        const uint32_t pi = host_part[u], pj = host_part[v];
        if (pi >= B || pj >= B) return false;
        *b = (uint64_t)((pj + B - pi) % B) * B + pi;  // sub-episode (pj - pi) mod B, then the vertex partition
        return true;
    };
    auto run = [&](auto &&body) {
        if (workers == 1) {
            body(0);
            return;
        }
        std::vector<std::thread> pool;
        pool.reserve(workers);
        try {
            for (uint32_t w = 0; w < workers; ++w) pool.emplace_back(body, w);
        } catch (...) {
            for (std::thread &t : pool) t.join();
            throw;
        }
        for (std::thread &t : pool) t.join();
    };
    run([&](uint32_t w) {
        for (uint64_t i = count * w / workers; i < count * (w + 1) / workers; ++i) {
            uint64_t b;
            if (!block_of(i, &b)) {
                broken.store(true, std::memory_order_relaxed);
                return;
            }
            place[w][b] += 1;
        }
    });
    if (broken.load()) return GV_EINVAL;
    uint64_t at = 0;
    for (uint64_t b = 0; b < blocks; ++b) {
        host_block_offsets[b] = at;
        for (uint32_t w = 0; w < workers; ++w) {
            const uint64_t mine = place[w][b];
            place[w][b] = at;
            at += mine;
        }
    }
    host_block_offsets[blocks] = at;
    run([&](uint32_t w) {
        for (uint64_t i = count * w / workers; i < count * (w + 1) / workers; ++i) {
            uint64_t b;
            (void)block_of(i, &b);
            const uint64_t to = place[w][b]++;
            host_pairs_out[2 * to] = host_pairs[2 * i];
            host_pairs_out[2 * to + 1] = host_pairs[2 * i + 1];
            host_order[to] = (uint32_t)i;
        }
    });
    return GV_OK;
}

extern "C" int gv_redistribute_pool(uint32_t n, const uint32_t *host_part, uint32_t partitions,
                                    const uint32_t *host_pairs, uint64_t count, uint32_t threads,
                                    uint32_t *host_pairs_out, uint32_t *host_order, uint64_t *host_block_offsets) {
    try {
        return redistribute(n, host_part, partitions, host_pairs, count, threads, host_pairs_out, host_order,
                            host_block_offsets);
    } catch (const std::bad_alloc &) {
        return GV_ENOMEM;
    } catch (...) {
        return GV_EHIP;
    }
}
