// Internal interface between the host runtime (gv_api.cpp) and the gfx950
// kernels (gv_kernels.hip).  Not part of the C boundary.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gv {

// Everything a training launch needs; passed by value as the kernel argument.
struct TrainArgs {
    float *vertex;            // |V| x d, row-major
    float *context;           // |V| x d, row-major
    const uint4 *alias;       // alias table: per bucket {threshold, alias node, hot rank of the bucket's node | hot rank
                              // of the alias << 16, the bucket's node}; the whole graph's table (bucket = node), or
                              // the table of one partition of the nodes (orthogonal blocks)
    uint32_t alias_n;         // buckets in that table
    const uint32_t *pairs;    // count x (u, v)
    const uint32_t *negatives;// deterministic mode: count x K precomputed draws (else unused)
    const uint32_t *order;    // null, or per sample its index in the pool it was redistributed from: sample i then has
                              // global position first_g + order[i] (its negatives and learning rate) instead of
                              // first_g + i
    const uint16_t *rank;     // per node: its place among the nodes by falling degree (ties by id), 0xFFFF
                              // from place 65535 on ("hot rank")
    const uint32_t *ranked;   // bit i set: node i has a hot rank below 0xFFFF (small enough to stay in cache,
                              // so the rank table is only read for the few nodes that are in it); null when
                              // so many nodes are ranked that the detour does not pay
    uint32_t warm_ranks;      // rows of hot rank below this are warm: their updates must not be lost
                              // (see gv_build_alias)
    uint32_t *records;        // tiled schedule: scratch of count x (K + 3) words, written and read by the launch
                              // (u, v, the K negatives, warm flags of the negatives)
    uint32_t *error_flag;     // two words: [0] set to 1 when a sample names a node id >= n (sample skipped), [1] set
                              // to 1 when the tiled kernel meets a row that holds NaN (training has diverged)
    double *loss_slots;       // null, or kLossSlots sums: every wave adds the losses its samples saw before their
                              // steps to slot (workgroup number mod kLossSlots)
    uint64_t first_g;         // global position of pairs[0]
    uint64_t total;           // T of the learning-rate schedule
    uint64_t seed;            // Philox key of the negative stream
    uint32_t count;           // samples in this launch
    uint32_t n;               // |V|
    uint32_t dim;             // d: row length in floats
    float lr0, lr_min_ratio, neg_weight;
};

constexpr uint32_t kLossSlots = 64;

// Launch shapes are chosen here; both return the HIP error of the launch.
hipError_t launch_train_hogwild(const TrainArgs &a, uint32_t dim, uint32_t num_neg, uint32_t coherence,
                                hipStream_t stream);
// Tiled stationary-row training (see k_train_tiled).
hipError_t launch_train_tiled(const TrainArgs &a, uint32_t dim, uint32_t num_neg, uint32_t coherence,
                              hipStream_t stream);
// One wave per sample over samples [0, a.count): the caller guarantees that no
// two of them share a vertex row or a context row (negatives included).
hipError_t launch_train_batch(const TrainArgs &a, uint32_t dim, uint32_t num_neg, hipStream_t stream);
// The same three launches with kernels that also sum the running loss into a.loss_slots (which must be set for
// these and null for the ones above).
hipError_t launch_train_hogwild_tracked(const TrainArgs &a, uint32_t dim, uint32_t num_neg, uint32_t coherence,
                                        hipStream_t stream);
hipError_t launch_train_tiled_tracked(const TrainArgs &a, uint32_t dim, uint32_t num_neg, uint32_t coherence,
                                      hipStream_t stream);
hipError_t launch_train_batch_tracked(const TrainArgs &a, uint32_t dim, uint32_t num_neg, hipStream_t stream);
// out[i*K + k] = negative k of positive sample first_g + i.
hipError_t launch_draw_negatives(const uint4 *alias, uint32_t n, uint64_t seed, uint64_t first_g, uint64_t count,
                                 uint32_t num_neg, uint32_t *out, hipStream_t stream);
// The same with one alias table per partition of the nodes: sample i draws from the table of the partition of its
// context node v[i]; tables[] holds the tables one after the other, partition j owning buckets offsets[j] ..
// offsets[j + 1] - 1.
hipError_t launch_draw_negatives_partitioned(const uint4 *tables, const uint64_t *offsets, const uint8_t *part,
                                             const uint32_t *v, uint64_t seed, uint64_t first_g, uint64_t count,
                                             uint32_t num_neg, uint32_t *out, hipStream_t stream);
// vertex ~ U(-0.5/d, 0.5/d) from Philox stream 1 (context is cleared by the caller).
hipError_t launch_init_vertex(float *vertex, uint64_t rows, uint32_t dim, uint64_t seed, hipStream_t stream);

// *total += sum of the per-sample losses of a.pairs[0 .. a.count) (a.seed = evaluation seed).
hipError_t launch_eval_loss(const TrainArgs &a, uint32_t dim, uint32_t num_neg, double *total, hipStream_t stream);
hipError_t launch_cosine(const float *vertex, uint32_t n, uint32_t dim, const uint32_t *first, const uint32_t *second,
                         uint32_t count, float *out, uint32_t *error_flag, hipStream_t stream);

// One pool of walk samples written on the device (see k_augment).
struct AugmentArgs {
    const uint64_t *offsets;  // CSR row starts, n + 1 entries
    const uint32_t *adj;      // neighbours, both directions of every edge
    const uint2 *node_table;  // weighted graph: alias table of the departure nodes {threshold, alias node}; else null
    const uint2 *nbr_table;   // weighted graph: per adjacency entry {threshold, alias entry of the same row}; else null
    uint2 *pairs;             // output, count x (u, v)
    uint64_t half_edges;      // offsets[n]
    uint64_t seed, first_walk, walks, count, per_walk;
    uint32_t n, length, window, pseudo_shuffle;
};
// walk length at most 64
hipError_t launch_augment(const AugmentArgs &a, hipStream_t stream);

bool supported_shape(uint32_t dim, uint32_t num_neg);
// samples whose rows one wave of the tiled kernel gathers together (4, or fewer where rows are long)
uint32_t samples_per_batch(uint32_t dim, uint32_t num_neg);

}  // namespace gv
