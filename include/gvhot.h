/*
 * gvhot.h -- C boundary of the GPU training hot path of GraphVite
 * (arXiv 1903.00757) on one AMD MI355X (gfx950).
 *
 * The library holds a vertex- and a context-embedding matrix (|V| x d, fp32,
 * row-major, Sec. 2.1) in device memory and trains them with pools of positive
 * edge samples (u, v): per sample, K negative context rows are drawn on the
 * device from the degree^(3/4) alias table (Sec. 4.3), the dot products
 * vertex[u].context[.] are formed, and the rows are moved in place by one
 * logistic-loss gradient step (Alg. 1, the Train calls), asynchronously and
 * without locks across samples (Sec. 4.3, asynchronous SGD).
 *
 * Conventions
 *   - Every call returns GV_OK (0) or a negative error code; nothing aborts or
 *     throws across this boundary.  gv_last_error() gives the text of the last
 *     failure of that context.
 *   - Pointers named `host_*` are host memory owned by the caller; the library
 *     has finished reading or writing them when the call returns unless stated
 *     otherwise.  Pointers named `dev_*` are device memory of the context's GPU
 *     owned by the caller.  All other device memory is owned by the library.
 *   - Node ids are uint32, sample/edge counts uint64 (Table 1: 4-byte ids,
 *     8-byte samples).  A sample pool is uint32[count][2] = (u, v) pairs.
 *   - One context must not be used from two threads at once; contexts are
 *     independent of each other.
 *   - Random numbers: Philox4x32-10, key = 64-bit seed, counter =
 *     (index low, index high, sub-index, stream); stream 0 = training
 *     negatives (index = global position of the positive sample, sub-index =
 *     k), stream 1 = initial embeddings (index = row, sub-index = column / 4).
 */
#ifndef GVHOT_H
#define GVHOT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gv_ctx gv_ctx;

enum { GV_OK = 0, GV_EINVAL = -1, GV_ENOMEM = -2, GV_ESTATE = -3, GV_EHIP = -4 };
/* HOGWILD: asynchronous SGD (Sec. 4.3), thousands of samples in flight; it relies on concurrent samples rarely
 *   sharing rows (Def. 1, Sec. 3.2) and is not meant for graphs on which a single node takes part in a large
 *   share of all samples (a star): those train in DETERMINISTIC mode.
 * DETERMINISTIC: samples in pool order, cut into batches without shared rows; equals sequential SGD up to
 *   fp32 rounding inside a sample.                                                                       */
enum { GV_MODE_HOGWILD = 0, GV_MODE_DETERMINISTIC = 1 };
enum { GV_VERTEX = 0, GV_CONTEXT = 1 };
/* How embedding rows travel between compute units and memory while an
 * asynchronous training kernel runs.
 *   PLAIN        ordinary cached loads and stores: fastest, but a compute unit keeps
 *                reading its own cached copy of a hot row, so concurrent updates of
 *                shared rows are mostly lost (kept for measurement only).
 *   AGENT        device-scope loads and stores: every wave sees the others' updates,
 *                but two waves updating one row at the same time lose one update
 *                (classic lock-free asynchronous SGD).
 *   ATOMIC_AGENT device-scope loads, updates applied as fp32 atomic adds: no update
 *                is ever lost, reads may be slightly stale.
 *   MIXED        ATOMIC_AGENT for rows likely to be shared by concurrent samples,
 *                AGENT stores for the rest (tiled schedule only; otherwise it
 *                behaves as ATOMIC_AGENT).                                            */
enum { GV_COHERENCE_PLAIN = 0, GV_COHERENCE_AGENT = 1, GV_COHERENCE_ATOMIC_AGENT = 2, GV_COHERENCE_MIXED = 3 };
/* Order in which an asynchronous launch walks a pool.
 *   POOL_ORDER   waves take chunks of 64 consecutive samples.
 *   TILED        workgroups take tiles of 8192 consecutive samples and sort each tile
 *                by the hottest row of every sample (the highest-degree one of u, v and
 *                the negatives); a wave keeps that row in registers across the run of
 *                samples sharing it, trading its change with memory every four samples
 *                and at the end of the run.  The launch still moves through the pool
 *                front to back, and each sample keeps the negatives and learning rate
 *                of its position in the pool.
 *   AUTO         TILED when the graph has rows that concurrent samples are likely to share
 *                (decided by gv_build_alias from the degrees), POOL_ORDER otherwise: on a
 *                graph without such rows the tile bookkeeping buys nothing.  With
 *                GV_COHERENCE_MIXED the pool-order launch then uses AGENT stores (all rows
 *                are cold).                                                            */
enum { GV_SCHEDULE_POOL_ORDER = 0, GV_SCHEDULE_TILED = 1, GV_SCHEDULE_AUTO = 2 };

/* gv_config.neg_weight value that asks for the paper's setting: 5 / K (Sec. 4.3: one
 * negative whose gradient is scaled by 5, i.e. the gradient scale of five negatives).  */
#define GV_NEG_WEIGHT_DEFAULT (-1.0f)
/* Largest number of pinned pool slots of a context (gv_config.pool_slots).              */
#define GV_MAX_POOL_SLOTS 16
/* Largest number of partitions of the orthogonal-block schedule (gv_config.partitions).   */
#define GV_MAX_PARTITIONS 64

typedef struct gv_config {
    uint32_t dim;            /* d: a multiple of 32 in 32..512 (128, or 96 in Sec. 4.3)       */
    uint32_t num_neg;        /* K negatives per positive sample, 1..5                         */
    float lr0;               /* initial learning rate (0.025 in Sec. 4.3)                      */
    float lr_min_ratio;      /* floor of the linear decay as a fraction of lr0 (0 = none)      */
    float neg_weight;        /* w >= 0: factor on every negative's gradient, or
                                GV_NEG_WEIGHT_DEFAULT for 5 / K (5 at K = 1, Sec. 4.3)         */
    uint32_t mode;           /* GV_MODE_*                                                      */
    uint64_t total_samples;  /* T: planned positive samples; lr(g) = lr0 * max(1 - g/T, floor) */
    uint64_t seed;           /* key of the negative-sampling stream                            */
    uint64_t pool_capacity;  /* largest pool (in samples, <= 2^31) that will be pushed; sizes the
                                pinned host slots and their device twins (8 B / sample each)   */
    int32_t device;          /* HIP device ordinal                                             */
    uint32_t coherence;      /* GV_COHERENCE_*                                                 */
    uint32_t profile;        /* nonzero: time every training launch with HIP events            */
    uint32_t schedule;       /* GV_SCHEDULE_* (asynchronous mode)                              */
    uint32_t pool_slots;     /* pinned pool slots in the ring: 0 (= 2, the two pools of Sec. 3.3)
                                or 2..GV_MAX_POOL_SLOTS                                        */
    uint32_t partitions;     /* 0, or the number B of partitions of the rows for the orthogonal-block
                                schedule of Sec. 3.2 (2..GV_MAX_PARTITIONS): gv_build_alias then also
                                partitions the nodes and builds one alias table per partition    */
    uint32_t track_loss;     /* nonzero: every training launch also sums the loss its samples see before
                                their step (gv_stats.train_loss_sum)                             */
} gv_config;

typedef struct gv_stats {
    uint64_t samples_trained;   /* positive samples consumed so far = next global position g   */
    uint64_t pools_trained;
    uint64_t train_launches;    /* training kernel launches (deterministic mode: one per batch) */
    uint64_t batches;           /* deterministic mode: conflict-free batches cut so far         */
    double train_kernel_ms;     /* sum of event-timed launch durations (profile != 0), resolved
                                   by gv_sync                                                   */
    uint64_t timed_launches;    /* launches contributing to train_kernel_ms                    */
    double h2d_ms;              /* event-timed pool copies host -> device (profile != 0)        */
    uint64_t h2d_bytes;
    uint64_t tiled_launches;    /* asynchronous launches that took the tiled schedule            */
    uint64_t warm_rows;         /* rows that gv_build_alias classed as warm (see GV_SCHEDULE_AUTO) */
    double train_loss_sum;      /* track_loss != 0: sum over the samples trained so far of the loss (Alg. 1 with
                                   the logistic loss of negative sampling, as gv_eval_loss) each of them saw
                                   at the rows it read, before its own step: the running training loss is
                                   train_loss_sum / train_loss_samples.  Resolved by gv_sync.            */
    uint64_t train_loss_samples;
} gv_stats;

/* Create a context on cfg->device (one GPU holds all rows: the single-GPU case of
 * Sec. 3.4).  Allocates the pool slots only; the graph decides the matrix sizes later.
 * *out is NULL on failure (GV_EINVAL for a bad field, GV_EHIP without a usable device,
 * GV_ENOMEM).                                                                        */
int gv_create(const gv_config *cfg, gv_ctx **out);
/* Wait for the context's device work, free everything it owns.  (Housekeeping, no passage.) */
void gv_destroy(gv_ctx *ctx);
/* Text of the context's last failure; ctx may be NULL: error of a failed gv_create or of a
 * context-free call, per thread.  (Housekeeping, no passage.)                          */
const char *gv_last_error(const gv_ctx *ctx);

/* Graph G = (V, E), undirected (Sec. 2.1, Sec. 4.3): m edges (host_src[i],
 * host_dst[i]), ids < n; only the degrees are kept.  Allocates both n x d
 * matrices (zero) and the alias table.  GV_EINVAL on an id >= n.               */
int gv_set_graph(gv_ctx *ctx, uint32_t n, uint64_t m, const uint32_t *host_src, const uint32_t *host_dst);
/* Same, from degrees alone (for graphs whose edge list the caller streams): the degrees
 * are all that negative sampling (Sec. 4.3) needs of the graph.                        */
int gv_set_degrees(gv_ctx *ctx, uint32_t n, const uint32_t *host_deg);

/* Alias table over nodes with weights degree^power (Sec. 4.3: alias table trick, power 3/4).
 * power must be 0.75 (exact, via square roots), 1.0 or 0.0.  Built on the host
 * with Vose's method in fp64 (index-ordered stacks), thresholds stored as
 * floor(p * 2^32) saturated; uploaded to the device.                           */
int gv_build_alias(gv_ctx *ctx, double power);
/* Copy the table out: host_thresh[n], host_alias[n].  (Test hook, no passage.)          */
int gv_get_alias(gv_ctx *ctx, uint32_t *host_thresh, uint32_t *host_alias);

/* Initial embeddings (Sec. 4.3 defers to earlier systems; benchmark configuration 1 fixes
 * them): vertex ~ U(-0.5/d, 0.5/d) from stream 1 of `seed`, element (row, col) from word
 * col % 4 of block (row, col / 4) as ((word + 0.5) / 2^32 - 0.5) / d; context = 0.      */
int gv_init_embeddings(gv_ctx *ctx, uint64_t seed);
/* Overwrite rows [row0, row0+rows) of one matrix (Sec. 2.1: vertex and context) from
 * host_rows[rows][d].  Waits for training first.  (Test and resume hook.)               */
int gv_set_embeddings(gv_ctx *ctx, int which, const float *host_rows, uint64_t row0, uint64_t rows);
/* Wait for all training, then copy rows [row0, row0+rows) to host_rows: the learned
 * embeddings of Sec. 2.1 (the vertex matrix is the output embedding).                   */
int gv_read_embeddings(gv_ctx *ctx, int which, float *host_rows, uint64_t row0, uint64_t rows);
/* Device address of a matrix (library-owned; valid until the next gv_set_graph /
 * gv_set_degrees / gv_destroy).  (Diagnostic hook, no passage.)                         */
int gv_device_embeddings(gv_ctx *ctx, int which, float **dev_rows);

/* Pool streaming (Sec. 3.3 collaboration strategy: producers fill one pool while the GPU
 * trains on another; Sec. 3.4 batched transfer).  The context has a ring of
 * cfg.pool_slots pinned host slots of pool_capacity samples, each paired with a device
 * buffer.  gv_acquire_pool_slot hands out the next slot of the ring that is neither being
 * filled nor queued, for the producer to fill in place; it blocks until the training launch
 * that last used that slot has finished.  A slot keeps what was last written into it: a
 * caller that filled the ring once may acquire and push the slots again without rewriting
 * them.  gv_push_pool queues `count` samples for training: if host_pairs is a pointer
 * returned by gv_acquire_pool_slot the copy to the device starts directly from it,
 * otherwise the samples are first copied into the next free slot (host_pairs may be reused
 * on return).  The copy runs on its own stream and overlaps the training of the pools
 * pushed before.  At most pool_slots pools can be acquired or queued and untrained: one
 * more gv_acquire_pool_slot / gv_push_pool returns GV_ESTATE.  A push that fails releases
 * the acquired slot it named.
 * Node ids are checked on the device while training: a sample naming an id >= n
 * is skipped, and the next gv_sync (or any call that synchronises) returns
 * GV_EINVAL once.                                                              */
int gv_acquire_pool_slot(gv_ctx *ctx, uint32_t **host_pairs);
int gv_push_pool(gv_ctx *ctx, const uint32_t *host_pairs, uint64_t count);
/* Train the oldest queued pool (Alg. 1, the loop over positive samples; Sec. 4.3
 * asynchronous SGD): positive samples g .. g+count-1 where g is the
 * number of samples trained so far.  Returns after launching (asynchronous);
 * GV_ESTATE if nothing is queued.  The training calls keep device scratch sized
 * for the largest pool seen so far (a few words per sample): the first call, and
 * a call with a larger pool than any before, allocate (GV_ENOMEM / GV_EHIP if
 * that fails) and wait for the launches in flight.                              */
int gv_train_pool(gv_ctx *ctx);
/* The same training step for a pool that already lies in device memory (dev_pairs must stay
 * valid and unchanged until gv_sync).  Ids are checked as for pushed pools.
 * count <= 2^31.                                                               */
int gv_train_device_pool(gv_ctx *ctx, const uint32_t *dev_pairs, uint64_t count);

/* gv_train_device_pool for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid it): the same training step, in
 * asynchronous mode only, with the kernels' per-sample scratch in a static device array of
 * GV_STATIC_SCRATCH_WORDS 32-bit words (16 MiB, part of the loaded library, held by every GPU
 * the library runs on until the process ends) instead of a buffer allocated on demand.  The call
 * allocates nothing, on the device or through any library, and times nothing (gv_stats'
 * train_kernel_ms does not grow).  GV_EINVAL when count * (K + 3) exceeds
 * GV_STATIC_SCRATCH_WORDS under the tiled schedule (2^20 samples at K = 1; the pool-order
 * schedule needs no scratch and takes any count <= 2^31); GV_ESTATE in deterministic mode.
 * All contexts of one GPU share that GPU's array: launches of one context are ordered on its
 * stream, but calls of two contexts that overlap on one GPU race on it.                      */
#define GV_STATIC_SCRATCH_WORDS (1u << 22)
int gv_train_device_pool_static(gv_ctx *ctx, const uint32_t *dev_pairs, uint64_t count);

/* Orthogonal blocks (Sec. 3.2, Alg. 3; degree-guided partition, Sec. 4.3), for contexts created with
 * gv_config.partitions = B > 0.  The rows of both matrices are partitioned B ways: gv_build_alias sorts the
 * nodes by falling degree (ties by id), deals them to the partitions back and forth (0, 1, .., B-1, B-1, .., 0,
 * 0, ..), and builds one alias table per partition over its nodes in increasing id, same weights and
 * construction as the whole-graph table.  A pool is redistributed into the B x B grid, sample (u, v) to block
 * (partition of u, partition of v); sub-episode o = 0..B-1 trains the blocks (i, (i + o) mod B), i = 0..B-1, which
 * share no row; the negatives of a sample are drawn from the alias table of the partition of its context node v
 * only (Sec. 3.2), so a block touches one vertex partition and one context partition.  A sample keeps the
 * position (negatives, learning rate) of its place in the pool it came from.  On one GPU the blocks are
 * trained one after the other: what this buys is a working set of 2/B of the matrices per launch.
 * gv_get_partitions (test hook): host_part[n] = partition of every node; host_offsets[B + 1], and, concatenated
 *   by partition, host_members[n] (the node of every table bucket), host_thresh[n], host_alias[n] (node ids).
 * gv_redistribute_pool (host, no context, no GPU; the Redistribute step of Alg. 3): stable counting sort of
 *   host_pairs[count][2] by block in training order (sub-episode first, then vertex partition) with `threads`
 *   workers: host_pairs_out[count][2], host_order[count] = pool index of every sorted sample,
 *   host_block_offsets[B * B + 1] = first sorted sample of block number o * B + i.  count <= 2^32.  GV_EINVAL
 *   for an id >= n or a partition number >= B.
 * gv_train_device_blocks: trains a redistributed pool that lies in device memory (dev_pairs[count][2],
 *   dev_order[count]; both must stay valid until gv_sync; host_block_offsets as written by
 *   gv_redistribute_pool, read before the call returns): one asynchronous launch per block, in training order, with the
 *   context's schedule and coherence; positions g + dev_order[k].  GV_ESTATE without partitions or in
 *   deterministic mode.
 * gv_draw_negatives_partitioned (parity hook): the K negatives of positive samples first_g .. first_g+count-1
 *   with context nodes host_v[count], as block training draws them: host_out[count][K].                  */
int gv_get_partitions(gv_ctx *ctx, uint32_t *host_part, uint64_t *host_offsets, uint32_t *host_members,
                      uint32_t *host_thresh, uint32_t *host_alias);
int gv_redistribute_pool(uint32_t n, const uint32_t *host_part, uint32_t partitions, const uint32_t *host_pairs,
                         uint64_t count, uint32_t threads, uint32_t *host_pairs_out, uint32_t *host_order,
                         uint64_t *host_block_offsets);
int gv_train_device_blocks(gv_ctx *ctx, const uint32_t *dev_pairs, const uint32_t *dev_order,
                           const uint64_t *host_block_offsets, uint64_t count);
int gv_draw_negatives_partitioned(gv_ctx *ctx, uint64_t first_g, uint64_t count, const uint32_t *host_v,
                                  uint32_t *host_out);

/* Host producer of a pool (Sec. 3.1, Alg. 2, parallel online augmentation): walk number
 * first_walk + w departs from a node drawn with probability proportional to its degree,
 * takes walk_length uniform steps over the adjacency (host_offsets[n+1], host_adj[] = CSR
 * with both directions of every edge), and yields every ordered pair (w_i, w_j),
 * i < j <= i + window, in order of i then j; walks are concatenated until `count` pairs
 * exist.  Random numbers: Philox stream 4 of `seed`, counter (walk number, step).
 * shuffle = GV_SHUFFLE_NONE keeps generation order; GV_SHUFFLE_PSEUDO applies the pseudo
 * shuffle of Sec. 3.1 (sample t goes to block t mod window of `window` consecutive blocks,
 * appended in order).  `threads` workers split the walks; the result does not depend on
 * their number.  host_pairs[count][2] may be any host memory, e.g. a slot returned by
 * gv_acquire_pool_slot.  Uses no GPU and no context.  *walks_used (may be NULL) receives
 * the number of walks consumed.  A node without neighbours must not be reachable
 * (degree-proportional departure never starts at one).  The adjacency is checked where the
 * walks touch it: an empty or ill-formed row, or an entry >= n, gives GV_EINVAL (the pool
 * is then incomplete); GV_ENOMEM / GV_EHIP when workers cannot be set up.  An adjacency of
 * gigabytes is best kept on huge pages (madvise MADV_HUGEPAGE before it is filled): every
 * step of a walk is a random access into it.                                             */
enum { GV_SHUFFLE_NONE = 0, GV_SHUFFLE_PSEUDO = 1 };
#define GV_MAX_WINDOW (1u << 20) /* largest augmentation distance `window` the producers accept */
int gv_augment(uint32_t n, const uint64_t *host_offsets, const uint32_t *host_adj, uint64_t seed,
               uint32_t walk_length, uint32_t window, uint64_t first_walk, uint64_t count, uint32_t shuffle,
               uint32_t threads, uint32_t *host_pairs, uint64_t *walks_used);

/* The same producer on the device (Sec. 3.1, Alg. 2; the paper runs it on the host CPUs: a
 * host with few cores per GPU cannot feed this trainer once the adjacency leaves its caches).
 * gv_set_adjacency uploads the CSR adjacency of the graph given to gv_set_graph /
 * gv_set_degrees: host_offsets[n + 1] (offsets[0] = 0, row i has degree(i) entries),
 * host_adj[offsets[n]] with both directions of every edge; both are copied, the caller keeps
 * its arrays; a later gv_set_graph / gv_set_degrees discards the copy.  Errors: GV_ESTATE
 * without a graph, GV_EINVAL when a row length differs from the node's degree, an entry is
 * >= n or the graph has no edge.
 * gv_augment_device writes the pool that gv_augment would write for the same arguments
 * (bit-identical: same walks, same random numbers, same order) into dev_pairs[count][2] in
 * DEVICE memory, asynchronously on the context's compute stream, i.e. ordered with
 * gv_train_device_pool calls before and after it: a buffer may be refilled right after the
 * call that trains it, and trained right after the call that fills it.  walk_length <= 64.
 * *walks_used (may be NULL) receives the number of walks consumed.                          */
int gv_set_adjacency(gv_ctx *ctx, const uint64_t *host_offsets, const uint32_t *host_adj);
int gv_augment_device(gv_ctx *ctx, uint64_t seed, uint32_t walk_length, uint32_t window, uint64_t first_walk,
                      uint64_t count, uint32_t shuffle, uint32_t *dev_pairs, uint64_t *walks_used);

/* Weighted graphs (Sec. 4.3: the alias table trick also serves online augmentation): the departure node of a walk is
 * drawn in proportion to its weighted degree (the sum of the weights of its edges) and every step goes to a
 * neighbour in proportion to the weight of the edge, both with alias tables; negatives follow the 3/4 power of
 * the weighted degree.  Weights are float >= 0 per adjacency entry (both directions of an edge carry its weight).
 * gv_build_walk_tables (host, no context): host_wdeg[n] (may be NULL) = weighted degrees, row sums left to right
 *   in fp64; host_node_thresh/alias[n] = alias table over the nodes with those weights; host_nbr_thresh/alias
 *   [offsets[n]] = one alias table per adjacency row over its weights, alias = index within the row.  Same
 *   construction as gv_build_alias.  GV_EINVAL for a negative weight, a row with entries but no weight, or a
 *   graph without weight.
 * gv_augment_weighted: gv_augment with those tables: walk w departs at the node table's draw from Philox
 *   block (w, 0) of stream 4 (bucket from words 0 and 1 over n, accepted when word 2 is below the threshold)
 *   and step t is the row table's draw from block (w, t).  With all weights 1 every step equals gv_augment's.
 * gv_set_weighted_graph: the graph of a context from its weighted adjacency (replaces gv_set_graph /
 *   gv_set_degrees + gv_set_adjacency): keeps weighted degrees, which gv_build_alias then uses in place of
 *   degrees, allocates the matrices, and uploads adjacency and walk tables, so that gv_augment_device walks the
 *   weighted graph (bit-identical to gv_augment_weighted).  GV_EINVAL as above or for an entry >= n.        */
int gv_build_walk_tables(uint32_t n, const uint64_t *host_offsets, const float *host_weights, double *host_wdeg,
                         uint32_t *host_node_thresh, uint32_t *host_node_alias, uint32_t *host_nbr_thresh,
                         uint32_t *host_nbr_alias);
int gv_augment_weighted(uint32_t n, const uint64_t *host_offsets, const uint32_t *host_adj,
                        const uint32_t *host_node_thresh, const uint32_t *host_node_alias,
                        const uint32_t *host_nbr_thresh, const uint32_t *host_nbr_alias, uint64_t seed,
                        uint32_t walk_length, uint32_t window, uint64_t first_walk, uint64_t count, uint32_t shuffle,
                        uint32_t threads, uint32_t *host_pairs, uint64_t *walks_used);
int gv_set_weighted_graph(gv_ctx *ctx, uint32_t n, const uint64_t *host_offsets, const uint32_t *host_adj,
                          const float *host_weights);

/* The K negatives of positive samples first_g .. first_g+count-1, exactly as
 * training draws them (Alg. 1, NegativeSampling; Sec. 4.3 alias table): host_out[count][K].
 * (Parity hook.)                                                                        */
int gv_draw_negatives(gv_ctx *ctx, uint64_t first_g, uint64_t count, uint32_t *host_out);

/* Evaluation on the device (after waiting for all training).
 * gv_eval_loss: mean over host_pairs[count][2] of the loss one training step descends
 *   (Alg. 1 with the logistic loss of negative sampling),
 *   -log sigmoid(x_u . c_v) - w sum_k log sigmoid(-x_u . c_k), the K negatives of sample i
 *   drawn from the alias table with Philox stream 2 of eval_seed, counter (i, k).
 * gv_cosine: host_out[i] = cosine of vertex rows host_first[i], host_second[i] (0 for a
 *   zero row): the score of a node pair in link prediction (Sec. 4.5).
 * Ids >= n give GV_EINVAL.  Both keep one device scratch buffer that grows with the largest
 * call.                                                                              */
int gv_eval_loss(gv_ctx *ctx, const uint32_t *host_pairs, uint64_t count, uint64_t eval_seed, double *mean_loss);
int gv_cosine(gv_ctx *ctx, const uint32_t *host_first, const uint32_t *host_second, uint64_t count, float *host_out);
/* Link prediction (Sec. 4.5): the held-out edges are ranked against other node pairs by the
 * cosine of their vertex rows and the result is the area under the ROC curve.
 * gv_auc: *auc = (sum of the ranks of host_pos among all scores - P (P + 1) / 2) / (P N),
 *   equal scores sharing their mean rank; P = num_pos, N = num_neg, both > 0; pure host
 *   code, no context.  GV_EINVAL for an empty set or a score that is not finite.
 * gv_link_prediction_auc: the same statistic of the cosines of num_edges pairs
 *   (host_edge_first[i], host_edge_second[i]) against num_others pairs
 *   (host_other_first[i], host_other_second[i]); waits for training first.             */
int gv_auc(const float *host_pos, uint64_t num_pos, const float *host_neg, uint64_t num_neg, double *auc);
int gv_link_prediction_auc(gv_ctx *ctx, const uint32_t *host_edge_first, const uint32_t *host_edge_second,
                           uint64_t num_edges, const uint32_t *host_other_first, const uint32_t *host_other_second,
                           uint64_t num_others, double *auc);

/* Wait for all queued device work of the context; folds event timings into the
 * statistics; reports samples that named an id >= n (GV_EINVAL, once), and training that has
 * diverged: an embedding row holding NaN met by an asynchronous tiled launch (GV_ESTATE, once).
 * (Housekeeping, no passage.)                                                   */
int gv_sync(gv_ctx *ctx);
/* Counters of the context so far.  (Diagnostic hook, no passage.)               */
int gv_get_stats(gv_ctx *ctx, gv_stats *out);
/* Set the position g of the next positive sample: g selects the negatives (stream 0,
 * counter (g, k)) and the learning rate lr0 * max(1 - g / T, floor) of Sec. 4.3, so a run
 * resumes exactly.  (Resume and test hook.)                                      */
int gv_set_position(gv_ctx *ctx, uint64_t next_g);

#ifdef __cplusplus
}
#endif
#endif /* GVHOT_H */
