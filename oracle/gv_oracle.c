/*
 * gv_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, sequential, slow CPU reference for the embedding-training hot path of
 * GraphVite (arXiv 1903.00757): counter-based random numbers, the alias table
 * for negative sampling, random-walk edge augmentation, and one-sample-at-a-time
 * skip-gram SGD with negative sampling.  fp32 storage, fp64 arithmetic.  It
 * shares no code with the HIP library and must never be called from it; only
 * tests, the smoke check and the CPU-baseline leg of the benchmark use it.
 *
 * Every function names the passage of the paper it follows.  Where the paper
 * is silent the reading taken is stated in the comment.
 *
 * Parity status: negative draws, alias table, augmentation, the SGD step, the
 * loss and the AUC are pinned by tests that do not go through this file's own
 * arithmetic (known-answer vectors, closed forms, finite differences, brute
 * force).  Final embeddings of a long run have no printed value in the paper:
 * "parity unpinned" in absolute terms, pinned only step by step.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): a keyed bijection on
 * 128-bit counters.  Ten rounds; before every round but the first the key is
 * advanced by the Weyl constants.                                            */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Random words of this reference: key = 64-bit seed, counter =
 * (index low, index high, sub-index, stream).  Streams: 0 training negatives,
 * 1 embedding initialisation, 2 evaluation negatives, 3 shuffle, 4 walks.
 * (The paper does not say how random bits are produced; a counter-based
 * generator makes every draw a pure function of its position.)              */
enum { STREAM_NEG = 0, STREAM_INIT = 1, STREAM_EVAL = 2, STREAM_SHUFFLE = 3, STREAM_WALK = 4 };

static void words(uint64_t seed, uint64_t index, uint32_t sub, uint32_t stream, uint32_t r[4])
{
    uint32_t ctr[4] = { (uint32_t)index, (uint32_t)(index >> 32), sub, stream };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    orc_philox4x32_10(ctr, key, r);
}

/* floor(R * n / 2^64) for a 64-bit R: a uniform integer in [0, n).           */
static uint64_t scale64(uint32_t hi, uint32_t lo, uint64_t n)
{
    unsigned __int128 R = ((uint64_t)hi << 32) | lo;
    return (uint64_t)((R * n) >> 64);
}

/* ------------------------------------------------------------------------- */
/* Alias table (Sec. 4.3 names the alias-table trick and the 3/4 power of the
 * degree; construction details are this reference's reading, Vose's method):
 * weights q, scaled p_i = q_i * n / S with S the left-to-right sum; nodes with
 * p < 1 and p >= 1 go on two stacks in increasing index order; while both are
 * non-empty pop a small s and a large l, s keeps probability p_s and aliases
 * to l, l loses 1 - p_s and is re-filed.  Whatever is left keeps itself with
 * certainty.  Acceptance thresholds are stored as 32-bit integers
 * floor(p * 2^32), saturated.                                                */
int orc_alias_build(uint64_t n, const double *q, uint32_t *thresh, uint32_t *alias)
{
    if (n == 0 || n > 0xFFFFFFFFull) return -1;
    double S = 0.0;
    for (uint64_t i = 0; i < n; ++i) {
        if (!(q[i] >= 0.0)) return -1;
        S += q[i];
    }
    if (!(S > 0.0)) return -1;
    double *p = (double *)malloc(n * sizeof(double));
    uint32_t *small = (uint32_t *)malloc(n * sizeof(uint32_t));
    uint32_t *large = (uint32_t *)malloc(n * sizeof(uint32_t));
    double *prob = (double *)malloc(n * sizeof(double));
    if (!p || !small || !large || !prob) { free(p); free(small); free(large); free(prob); return -2; }
    uint64_t ns = 0, nl = 0;
    for (uint64_t i = 0; i < n; ++i) {
        p[i] = q[i] * (double)n / S;
        if (p[i] < 1.0) small[ns++] = (uint32_t)i; else large[nl++] = (uint32_t)i;
    }
    for (uint64_t i = 0; i < n; ++i) { prob[i] = 1.0; alias[i] = (uint32_t)i; }
    while (ns > 0 && nl > 0) {
        uint32_t s = small[--ns];
        uint32_t l = large[--nl];
        prob[s] = p[s];
        alias[s] = l;
        p[l] = (p[l] + p[s]) - 1.0;
        if (p[l] < 1.0) small[ns++] = l; else large[nl++] = l;
    }
    for (uint64_t i = 0; i < n; ++i) {
        double t = floor(prob[i] * 4294967296.0);
        thresh[i] = t >= 4294967295.0 ? 0xFFFFFFFFu : (uint32_t)t;
    }
    free(p); free(small); free(large); free(prob);
    return 0;
}

/* Negative-sampling weights: degree to the power 3/4 (Sec. 4.3), written with
 * square roots only so that the value is correctly rounded everywhere.       */
void orc_degree_weights(uint64_t n, const uint32_t *deg, double *q)
{
    for (uint64_t i = 0; i < n; ++i) {
        double r = sqrt((double)deg[i]);
        q[i] = r * sqrt(r);
    }
}

/* One alias draw from four random words: bucket from the first two words,
 * acceptance from the third.                                                 */
static uint32_t alias_draw(const uint32_t r[4], uint64_t n, const uint32_t *thresh, const uint32_t *alias)
{
    uint64_t j = scale64(r[0], r[1], n);
    return r[2] < thresh[j] ? (uint32_t)j : alias[j];
}

/* Negatives of positive samples first_g .. first_g+count-1: K per sample,
 * out[(g-first_g)*K + k]   (Alg. 1, the NegativeSampling call).  No redraw
 * when a negative equals u or v: the paper does not ask for one.             */
void orc_draw_negatives(uint64_t seed, uint32_t stream, uint64_t first_g, uint64_t count, uint32_t K,
                        uint64_t n, const uint32_t *thresh, const uint32_t *alias, uint32_t *out)
{
    for (uint64_t i = 0; i < count; ++i)
        for (uint32_t k = 0; k < K; ++k) {
            uint32_t r[4];
            words(seed, first_g + i, k, stream, r);
            out[i * K + k] = alias_draw(r, n, thresh, alias);
        }
}

/* ------------------------------------------------------------------------- */
/* Online augmentation, sequential form (Sec. 3.1, Alg. 2): walk number w
 * departs from a node chosen with probability proportional to degree (the
 * owner of a uniformly chosen half-edge of the CSR adjacency), takes L steps,
 * each to a uniformly chosen neighbour, and contributes every ordered pair
 * (w_i, w_j), i < j <= i+s, in order of i then j.  Walks first_walk,
 * first_walk+1, ... are concatenated until `count` pairs exist (the last walk
 * is cut).  Returns the number of walks used.                                */
uint64_t orc_augment(uint64_t seed, uint64_t n, const uint64_t *offsets, const uint32_t *adj,
                     uint32_t L, uint32_t s, uint64_t first_walk, uint64_t count, uint32_t *pairs)
{
    uint32_t *path = (uint32_t *)malloc(((size_t)L + 1) * sizeof(uint32_t));
    uint64_t half_edges = offsets[n];
    uint64_t produced = 0, w = first_walk;
    while (produced < count) {
        uint32_t r[4];
        words(seed, w, 0, STREAM_WALK, r);
        uint64_t e = scale64(r[0], r[1], half_edges);
        /* owner of half-edge e: the node x with offsets[x] <= e < offsets[x+1] */
        uint64_t lo = 0, hi = n;
        while (hi - lo > 1) {
            uint64_t mid = lo + (hi - lo) / 2;
            if (offsets[mid] <= e) lo = mid; else hi = mid;
        }
        path[0] = (uint32_t)lo;
        for (uint32_t t = 1; t <= L; ++t) {
            uint32_t x = path[t - 1];
            uint64_t deg = offsets[x + 1] - offsets[x];
            words(seed, w, t, STREAM_WALK, r);
            path[t] = adj[offsets[x] + scale64(r[0], r[1], deg)];
        }
        for (uint32_t i = 0; i <= L && produced < count; ++i)
            for (uint32_t j = i + 1; j <= L && j <= i + s && produced < count; ++j) {
                pairs[2 * produced] = path[i];
                pairs[2 * produced + 1] = path[j];
                ++produced;
            }
        ++w;
    }
    free(path);
    return w - first_walk;
}

/* ------------------------------------------------------------------------- */
/* Weighted graphs.  Sec. 4.3 names the alias table trick for online augmentation too: on a graph with edge
 * weights the departure node is drawn in proportion to its weighted degree and every step goes to a
 * neighbour in proportion to the weight of the edge, each with an alias table (one over the nodes, one per
 * adjacency row); negatives follow the 3/4 power of the weighted degree.                                  */

/* Weighted degree: the edge weights of a row of the CSR adjacency, summed left to right in fp64.         */
void orc_weighted_degrees(uint64_t n, const uint64_t *offsets, const float *weights, double *wdeg)
{
    for (uint64_t i = 0; i < n; ++i) {
        double total = 0.0;
        for (uint64_t e = offsets[i]; e < offsets[i + 1]; ++e) total += (double)weights[e];
        wdeg[i] = total;
    }
}

/* The 3/4 power of a weighted degree, with square roots only (as for plain degrees).                     */
void orc_weights_pow34(uint64_t n, const double *wdeg, double *q)
{
    for (uint64_t i = 0; i < n; ++i) {
        double r = sqrt(wdeg[i]);
        q[i] = r * sqrt(r);
    }
}

/* One alias table per adjacency row over that row's edge weights: entry e of row x (offsets[x] <= e <
 * offsets[x+1]) is accepted below thresh[e], otherwise the step takes entry offsets[x] + alias[e] of the
 * same row.  Returns 0, or -1 when a row has entries but no weight.                                       */
int orc_neighbor_alias(uint64_t n, const uint64_t *offsets, const float *weights, uint32_t *thresh, uint32_t *alias)
{
    for (uint64_t x = 0; x < n; ++x) {
        uint64_t begin = offsets[x], deg = offsets[x + 1] - begin;
        if (deg == 0) continue;
        double *q = (double *)malloc(deg * sizeof(double));
        for (uint64_t e = 0; e < deg; ++e) q[e] = (double)weights[begin + e];
        int rc = orc_alias_build(deg, q, thresh + begin, alias + begin);
        free(q);
        if (rc != 0) return -1;
    }
    return 0;
}

/* Online augmentation on a weighted graph (Sec. 3.1, Alg. 2 with the tables above): as orc_augment, but walk w
 * departs from an alias draw over the nodes (weights = weighted degrees) and step t is an alias draw over the
 * current node's row; both take their random words like the unweighted walk (stream 4, counter (w, t)).   */
uint64_t orc_augment_weighted(uint64_t seed, uint64_t n, const uint64_t *offsets, const uint32_t *adj,
                              const uint32_t *node_thresh, const uint32_t *node_alias,
                              const uint32_t *nbr_thresh, const uint32_t *nbr_alias,
                              uint32_t L, uint32_t s, uint64_t first_walk, uint64_t count, uint32_t *pairs)
{
    uint32_t *path = (uint32_t *)malloc(((size_t)L + 1) * sizeof(uint32_t));
    uint64_t produced = 0, w = first_walk;
    while (produced < count) {
        uint32_t r[4];
        words(seed, w, 0, STREAM_WALK, r);
        path[0] = alias_draw(r, n, node_thresh, node_alias);
        for (uint32_t t = 1; t <= L; ++t) {
            uint32_t x = path[t - 1];
            uint64_t begin = offsets[x], deg = offsets[x + 1] - begin;
            words(seed, w, t, STREAM_WALK, r);
            path[t] = adj[begin + alias_draw(r, deg, nbr_thresh + begin, nbr_alias + begin)];
        }
        for (uint32_t i = 0; i <= L && produced < count; ++i)
            for (uint32_t j = i + 1; j <= L && j <= i + s && produced < count; ++j) {
                pairs[2 * produced] = path[i];
                pairs[2 * produced + 1] = path[j];
                ++produced;
            }
        ++w;
    }
    free(path);
    return w - first_walk;
}

/* Uniform shuffle of a pool (Alg. 2, the Shuffle call): Fisher-Yates from the
 * last position down, position i swapped with a uniform j in [0, i].         */
void orc_shuffle(uint64_t seed, uint64_t count, uint32_t *pairs)
{
    for (uint64_t i = count; i-- > 1;) {
        uint32_t r[4];
        words(seed, i, 0, STREAM_SHUFFLE, r);
        uint64_t j = scale64(r[0], r[1], i + 1);
        uint32_t a = pairs[2 * i], b = pairs[2 * i + 1];
        pairs[2 * i] = pairs[2 * j]; pairs[2 * i + 1] = pairs[2 * j + 1];
        pairs[2 * j] = a; pairs[2 * j + 1] = b;
    }
}

/* Pseudo shuffle (Sec. 3.1): the pool is divided into s consecutive blocks; going through
 * the samples in generation order, each one is appended to the next block in turn (sample t
 * to block t mod s), so that the s samples following each other in a walk, which share a
 * node, are scattered over different blocks; the blocks are then read one after the other.
 * (The paper gives the idea, not the scatter rule; round-robin is the reading taken.)       */
void orc_pseudo_shuffle(uint64_t count, uint32_t s, const uint32_t *in, uint32_t *out)
{
    uint64_t *fill = (uint64_t *)calloc(s, sizeof(uint64_t));
    uint64_t *start = (uint64_t *)calloc((size_t)s + 1, sizeof(uint64_t));
    for (uint64_t t = 0; t < count; ++t) start[t % s + 1] += 1;      /* block sizes */
    for (uint32_t b = 0; b < s; ++b) start[b + 1] += start[b];         /* block offsets */
    for (uint64_t t = 0; t < count; ++t) {
        uint32_t b = (uint32_t)(t % s);
        uint64_t at = start[b] + fill[b]++;
        out[2 * at] = in[2 * t];
        out[2 * at + 1] = in[2 * t + 1];
    }
    free(fill); free(start);
}

/* ------------------------------------------------------------------------- */
/* Initial embeddings (the paper defers to earlier work; the benchmark
 * configuration fixes it): vertex uniform in (-0.5/d, 0.5/d), context zero.
 * Element (row, col) takes word col%4 of the block (row, col/4).             */
void orc_init_vertex_rows(uint64_t seed, uint64_t row0, uint64_t rows, uint32_t d, float *vertex)
{
    for (uint64_t i = 0; i < rows; ++i)
        for (uint32_t col = 0; col < d; ++col) {
            uint32_t r[4];
            words(seed, row0 + i, col / 4, STREAM_INIT, r);
            double unit = ((double)r[col % 4] + 0.5) * (1.0 / 4294967296.0);
            vertex[i * d + col] = (float)((unit - 0.5) / (double)d);
        }
}

void orc_init_embeddings(uint64_t seed, uint64_t n, uint32_t d, float *vertex, float *context)
{
    orc_init_vertex_rows(seed, 0, n, d, vertex);
    memset(context, 0, (size_t)n * d * sizeof(float));
}

static double sigmoid(double z) { return 1.0 / (1.0 + exp(-z)); }

/* log(sigmoid(z)) without overflow */
static double log_sigmoid(double z) { return z >= 0.0 ? -log1p(exp(-z)) : z - log1p(exp(z)); }

/* Learning rate of positive sample g of T (Sec. 4.3: initial value, linear
 * decay): evaluated per sample in fp64, stored as fp32.                      */
float orc_learning_rate(float lr0, float lr_min_ratio, uint64_t g, uint64_t T)
{
    double f = 1.0 - (double)g / (double)T;
    if (f < (double)lr_min_ratio) f = (double)lr_min_ratio;
    return (float)((double)lr0 * f);
}

/* Sequential SGD over `count` positive samples (Alg. 1, the training loop):
 * for sample (u, v) with negatives u'_1..u'_K the scores are the dot products
 * of vertex[u] with context[v] and context[u'_k] (Sec. 2.1); Train(., ., label)
 * moves both rows along the gradient of the logistic loss with coefficient
 * lr * (label - sigmoid(score)), the negative's coefficient scaled by w
 * (Sec. 4.3: one negative, its gradient scaled by 5).  All scores of a sample
 * are taken before any of its rows moves, i.e. the sample performs one exact
 * gradient step of
 *     loss = -log sigmoid(x_u . c_v) - w * sum_k log sigmoid(-x_u . c_{u'_k});
 * rows named twice within a sample receive the sum of their updates.
 * `negatives` may be NULL (then they are drawn here from stream 0) or hold K
 * indices per sample.                                                        */
/* One positive sample at global position g: u, v, its K negatives in neg[1..K] (neg[0] = v).  Scratch
 * arrays of d doubles (dx, xu) and K + 1 doubles (coef) come from the caller.  `loss` (may be NULL): the
 * value of the loss above at the rows as the sample finds them is added to it.                          */
static void train_sample(float *vertex, float *context, uint32_t d, uint32_t K, uint32_t u, const uint32_t *neg,
                         uint64_t g, uint64_t T, float lr0, float lr_min_ratio, float w,
                         double *dx, double *xu, double *coef, double *loss)
{
    double lr = (double)orc_learning_rate(lr0, lr_min_ratio, g, T);
    float *x = vertex + (size_t)u * d;
    for (uint32_t k = 0; k <= K; ++k) {
        const float *c = context + (size_t)neg[k] * d;
        double score = 0.0;
        for (uint32_t j = 0; j < d; ++j) score += (double)x[j] * (double)c[j];
        coef[k] = k == 0 ? lr * (1.0 - sigmoid(score)) : -lr * (double)w * sigmoid(score);
        if (loss) *loss += k == 0 ? -log_sigmoid(score) : -(double)w * log_sigmoid(-score);
    }
    for (uint32_t j = 0; j < d; ++j) { xu[j] = (double)x[j]; dx[j] = 0.0; }
    for (uint32_t k = 0; k <= K; ++k) {
        const float *c = context + (size_t)neg[k] * d;
        for (uint32_t j = 0; j < d; ++j) dx[j] += coef[k] * (double)c[j];
    }
    /* context rows: a row named several times gets the summed coefficient once */
    for (uint32_t k = 0; k <= K; ++k) {
        int seen = 0;
        for (uint32_t k2 = 0; k2 < k; ++k2) if (neg[k2] == neg[k]) seen = 1;
        if (seen) continue;
        double total = 0.0;
        for (uint32_t k2 = k; k2 <= K; ++k2) if (neg[k2] == neg[k]) total += coef[k2];
        float *c = context + (size_t)neg[k] * d;
        for (uint32_t j = 0; j < d; ++j) c[j] = (float)((double)c[j] + total * xu[j]);
    }
    for (uint32_t j = 0; j < d; ++j) x[j] = (float)(xu[j] + dx[j]);
}

/* `order` (may be NULL = pool order): the sequence in which the samples are taken, order[k] = index into
 * pairs / negatives of the k-th sample trained; a sample keeps the position first_g + its index whatever
 * its turn (position decides its negatives and its learning rate).                                      */
/* `loss_sum` (may be NULL): receives the sum over the samples of the loss each of them saw before its step
 * (the running training loss that a trainer reports while it works).                                    */
void orc_train_tracked(float *vertex, float *context, uint64_t n, uint32_t d, uint32_t K,
                       const uint32_t *pairs, uint64_t count, uint64_t first_g, uint64_t T,
                       float lr0, float lr_min_ratio, float w, uint64_t seed,
                       const uint32_t *thresh, const uint32_t *alias, const uint32_t *negatives,
                       const uint32_t *order, double *loss_sum)
{
    double seen = 0.0;
    double *dx = (double *)malloc((size_t)d * sizeof(double));
    double *xu = (double *)malloc((size_t)d * sizeof(double));
    uint32_t *neg = (uint32_t *)malloc(((size_t)K + 1) * sizeof(uint32_t));
    double *coef = (double *)malloc(((size_t)K + 1) * sizeof(double));
    for (uint64_t turn = 0; turn < count; ++turn) {
        uint64_t i = order ? order[turn] : turn;
        uint64_t g = first_g + i;
        /* row 0 of the sample is the positive context row, rows 1..K the negatives */
        neg[0] = pairs[2 * i + 1];
        for (uint32_t k = 0; k < K; ++k) {
            if (negatives) neg[k + 1] = negatives[i * K + k];
            else {
                uint32_t r[4];
                words(seed, g, k, STREAM_NEG, r);
                neg[k + 1] = alias_draw(r, n, thresh, alias);
            }
        }
        train_sample(vertex, context, d, K, pairs[2 * i], neg, g, T, lr0, lr_min_ratio, w, dx, xu, coef,
                     loss_sum ? &seen : NULL);
    }
    if (loss_sum) *loss_sum = seen;
    free(dx); free(xu); free(neg); free(coef);
}

void orc_train_ordered(float *vertex, float *context, uint64_t n, uint32_t d, uint32_t K,
                       const uint32_t *pairs, uint64_t count, uint64_t first_g, uint64_t T,
                       float lr0, float lr_min_ratio, float w, uint64_t seed,
                       const uint32_t *thresh, const uint32_t *alias, const uint32_t *negatives,
                       const uint32_t *order)
{
    orc_train_tracked(vertex, context, n, d, K, pairs, count, first_g, T, lr0, lr_min_ratio, w, seed,
                      thresh, alias, negatives, order, NULL);
}

void orc_train(float *vertex, float *context, uint64_t n, uint32_t d, uint32_t K,
               const uint32_t *pairs, uint64_t count, uint64_t first_g, uint64_t T,
               float lr0, float lr_min_ratio, float w, uint64_t seed,
               const uint32_t *thresh, const uint32_t *alias, const uint32_t *negatives)
{
    orc_train_ordered(vertex, context, n, d, K, pairs, count, first_g, T, lr0, lr_min_ratio, w, seed,
                      thresh, alias, negatives, NULL);
}

/* ------------------------------------------------------------------------- */
/* Orthogonal blocks (Sec. 3.2, Alg. 3) on partitioned matrices.
 *
 * Degree-guided partition (Sec. 4.3; its figure is missing from the text at hand): the nodes are sorted by
 * falling degree (ties by id) and dealt to the B partitions back and forth, 0, 1, .., B-1, B-1, .., 1, 0,
 * 0, 1, ..: every partition gets the same number of nodes (up to one) and about the same degree mass.   */
struct by_degree { uint32_t degree, id; };
static int hotter_first(const void *a, const void *b)
{
    const struct by_degree *x = (const struct by_degree *)a, *y = (const struct by_degree *)b;
    if (x->degree != y->degree) return x->degree > y->degree ? -1 : 1;
    return x->id < y->id ? -1 : (x->id > y->id ? 1 : 0);
}

void orc_zigzag_partition(uint64_t n, const uint32_t *deg, uint32_t B, uint32_t *part)
{
    struct by_degree *order = (struct by_degree *)malloc(n * sizeof *order);
    for (uint64_t i = 0; i < n; ++i) { order[i].degree = deg[i]; order[i].id = (uint32_t)i; }
    qsort(order, n, sizeof *order, hotter_first);
    for (uint64_t r = 0; r < n; ++r) {
        uint64_t round = r / B;
        uint32_t k = (uint32_t)(r % B);
        part[order[r].id] = round % 2 == 0 ? k : B - 1 - k;
    }
    free(order);
}

/* One alias table per partition (Sec. 3.2: negatives are drawn only from the context rows of the partition
 * at hand), over the partition's nodes in increasing id with the same weights degree^(3/4).  Concatenated:
 * partition j owns entries offsets[j] .. offsets[j+1]-1; entry e stands for node members[e], is accepted
 * below thresh[e] and otherwise gives node alias[e].  Returns 0, or -1 when a partition has no weight.   */
int orc_partition_alias(uint64_t n, const uint32_t *deg, uint32_t B, const uint32_t *part,
                        uint64_t *offsets, uint32_t *members, uint32_t *thresh, uint32_t *alias)
{
    for (uint32_t j = 0; j <= B; ++j) offsets[j] = 0;
    for (uint64_t i = 0; i < n; ++i) offsets[part[i] + 1] += 1;
    for (uint32_t j = 0; j < B; ++j) offsets[j + 1] += offsets[j];
    uint64_t *fill = (uint64_t *)calloc(B, sizeof(uint64_t));
    for (uint64_t i = 0; i < n; ++i) members[offsets[part[i]] + fill[part[i]]++] = (uint32_t)i;
    free(fill);
    int rc = 0;
    for (uint32_t j = 0; j < B && rc == 0; ++j) {
        uint64_t nj = offsets[j + 1] - offsets[j];
        uint32_t *mine = members + offsets[j];
        uint32_t *degrees = (uint32_t *)malloc(nj * sizeof(uint32_t));
        double *q = (double *)malloc(nj * sizeof(double));
        uint32_t *local = (uint32_t *)malloc(nj * sizeof(uint32_t));
        for (uint64_t l = 0; l < nj; ++l) degrees[l] = deg[mine[l]];
        orc_degree_weights(nj, degrees, q);
        if (nj == 0 || orc_alias_build(nj, q, thresh + offsets[j], local) != 0) rc = -1;
        else for (uint64_t l = 0; l < nj; ++l) alias[offsets[j] + l] = mine[local[l]];
        free(degrees); free(q); free(local);
    }
    return rc;
}

/* Negatives restricted to the partition of the positive context node: out[i*K + k] for positive samples
 * first_g + i with context nodes v[i].                                                                  */
void orc_draw_negatives_partitioned(uint64_t seed, uint32_t stream, uint64_t first_g, uint64_t count, uint32_t K,
                                    const uint32_t *v, const uint32_t *part, const uint64_t *offsets,
                                    const uint32_t *members, const uint32_t *thresh, const uint32_t *alias,
                                    uint32_t *out)
{
    for (uint64_t i = 0; i < count; ++i) {
        uint32_t j = part[v[i]];
        uint64_t nj = offsets[j + 1] - offsets[j];
        for (uint32_t k = 0; k < K; ++k) {
            uint32_t r[4];
            words(seed, first_g + i, k, stream, r);
            uint64_t e = offsets[j] + scale64(r[0], r[1], nj);
            out[i * K + k] = r[2] < thresh[e] ? members[e] : alias[e];
        }
    }
}

/* Order of training under Alg. 3 run by one worker: the pool is redistributed into the B x B grid, sample
 * (u, v) to block (part[u], part[v]); sub-episode o = 0..B-1 takes the blocks (i, (i + o) mod B), i = 0..B-1
 * (blocks of one sub-episode share no row, Def. 1); inside a block the samples keep their pool order.
 * order[k] = pool index of the k-th sample; block_offsets[o*B + i] = first k of block (i, (i + o) mod B).  */
void orc_block_order(uint64_t count, const uint32_t *pairs, uint32_t B, const uint32_t *part,
                     uint32_t *order, uint64_t *block_offsets)
{
    uint64_t blocks = (uint64_t)B * B;
    for (uint64_t b = 0; b <= blocks; ++b) block_offsets[b] = 0;
    for (uint64_t i = 0; i < count; ++i) {
        uint32_t pi = part[pairs[2 * i]], pj = part[pairs[2 * i + 1]];
        uint32_t o = (pj + B - pi) % B;
        block_offsets[(uint64_t)o * B + pi + 1] += 1;
    }
    for (uint64_t b = 0; b < blocks; ++b) block_offsets[b + 1] += block_offsets[b];
    uint64_t *fill = (uint64_t *)calloc(blocks, sizeof(uint64_t));
    for (uint64_t i = 0; i < count; ++i) {
        uint32_t pi = part[pairs[2 * i]], pj = part[pairs[2 * i + 1]];
        uint64_t b = (uint64_t)((pj + B - pi) % B) * B + pi;
        order[block_offsets[b] + fill[b]++] = (uint32_t)i;
    }
    free(fill);
}

/* Mean per-sample loss (the objective the step above descends) over a fixed
 * evaluation pool, negatives from stream 2 with sample index i.              */
double orc_loss(const float *vertex, const float *context, uint64_t n, uint32_t d, uint32_t K,
                const uint32_t *pairs, uint64_t count, float w, uint64_t seed, uint32_t stream,
                const uint32_t *thresh, const uint32_t *alias)
{
    double total = 0.0;
    for (uint64_t i = 0; i < count; ++i) {
        const float *x = vertex + (size_t)pairs[2 * i] * d;
        const float *c = context + (size_t)pairs[2 * i + 1] * d;
        double score = 0.0;
        for (uint32_t j = 0; j < d; ++j) score += (double)x[j] * (double)c[j];
        double loss = -log_sigmoid(score);
        for (uint32_t k = 0; k < K; ++k) {
            uint32_t r[4];
            words(seed, i, k, stream, r);
            const float *cn = context + (size_t)alias_draw(r, n, thresh, alias) * d;
            double sn = 0.0;
            for (uint32_t j = 0; j < d; ++j) sn += (double)x[j] * (double)cn[j];
            loss -= (double)w * log_sigmoid(-sn);
        }
        total += loss;
    }
    return total / (double)count;
}

/* Cosine similarity of vertex rows a[i], b[i] (Sec. 4.5: an edge is scored by
 * the cosine of its two node embeddings).  A zero row scores 0.              */
void orc_cosine(const float *vertex, uint32_t d, const uint32_t *a, const uint32_t *b, uint64_t count, double *out)
{
    for (uint64_t i = 0; i < count; ++i) {
        const float *x = vertex + (size_t)a[i] * d;
        const float *y = vertex + (size_t)b[i] * d;
        double xy = 0.0, xx = 0.0, yy = 0.0;
        for (uint32_t j = 0; j < d; ++j) {
            xy += (double)x[j] * (double)y[j];
            xx += (double)x[j] * (double)x[j];
            yy += (double)y[j] * (double)y[j];
        }
        out[i] = (xx > 0.0 && yy > 0.0) ? xy / (sqrt(xx) * sqrt(yy)) : 0.0;
    }
}
