// gfx950 kernels of the embedding-training hot path (GraphVite, arXiv 1903.00757).
//
// Work decomposition: one 64-lane wavefront owns one positive sample at a time.
// A row of d floats is spread over the 64 lanes (d/64 floats per lane), so a row
// gather or scatter is one fully coalesced request per 64 x 16 B, the dot product
// is a per-lane partial followed by a cross-lane (DPP) reduction, and all node ids
// and coefficients of the sample are wave-uniform scalars.
//
// The file is compiled twice, side by side: plainly, and with GV_TRACK_LOSS=1 into a second object that holds
// nothing but the training kernels that also sum the running loss, under names ending in _tracked.
#include "gv_internal.hpp"

#ifndef GV_TRACK_LOSS
#define GV_TRACK_LOSS 0
#endif
#if GV_TRACK_LOSS
#define GV_TRAIN_NAME(name) name##_tracked
#else
#define GV_TRAIN_NAME(name) name
#endif

namespace gv {
namespace {

typedef float f2 __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kBlock = 256;  // 4 waves per workgroup
// Row traffic policies (gv_config.coherence).
constexpr int kPlain = 0;        // cached loads and stores
constexpr int kAgent = 1;        // device-scope loads and stores
constexpr int kAtomicAgent = 2;  // device-scope loads, updates as device-scope fp32 atomic adds
constexpr int kMixed = 3;        // as kAtomicAgent for rows flagged warm, plain device-scope store otherwise
constexpr bool is_atomic(int c) { return c == kAtomicAgent || c == kMixed; }
constexpr bool is_agent(int c) { return c == kAgent || c == kAtomicAgent || c == kMixed; }

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies
// and a word permutation; the key advances by the Weyl constants between rounds.
__device__ __forceinline__ uint4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                               uint32_t k1) {
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return make_uint4(c0, c1, c2, c3);
}

// Negative k of positive sample g (Alg. 1, NegativeSampling; Sec. 4.3 alias
// table): bucket = floor(R * n / 2^64) from the first two words, accepted when
// the third word is below the bucket's threshold, else the bucket's alias.
// The table entry also carries the node of the bucket (the table may cover a partition of the nodes only) and
// the hot ranks of both candidates.
struct Drawn {
    uint32_t id;
    uint32_t rank;
};
__device__ __forceinline__ Drawn draw_ranked_negative(const uint4 *__restrict__ alias, uint32_t n, uint64_t seed,
                                                      uint64_t g, uint32_t k, uint32_t stream = 0u) {
    const uint4 r =
        philox4x32_10((uint32_t)g, (uint32_t)(g >> 32), k, stream, (uint32_t)seed, (uint32_t)(seed >> 32));
    const uint64_t R = ((uint64_t)r.x << 32) | r.y;
    const uint32_t j = (uint32_t)__umul64hi(R, (uint64_t)n);
    const uint4 e = alias[j];
    const bool keep = r.z < e.x;
    return Drawn{keep ? e.w : e.y, keep ? (e.z & 0xFFFFu) : (e.z >> 16)};
}
__device__ __forceinline__ uint32_t draw_negative(const uint4 *__restrict__ alias, uint32_t n, uint64_t seed,
                                                  uint64_t g, uint32_t k, uint32_t stream = 0u) {
    return draw_ranked_negative(alias, n, seed, g, k, stream).id;
}

// Learning rate of positive sample g (Sec. 4.3: linear decay from lr0), fp64 then fp32.
__device__ __forceinline__ float learning_rate(float lr0, float lr_min_ratio, uint64_t g, uint64_t total) {
    double f = 1.0 - (double)g / (double)total;
    if (f < (double)lr_min_ratio) f = (double)lr_min_ratio;
    return (float)((double)lr0 * f);
}

// ---------------------------------------------------------------------------
// Cross-lane sum of a wave64 with DPP moves: quad butterflies, half-row and row
// mirrors give every lane its 16-lane row sum; two row broadcasts carry the sums
// to the last row; the result is read from lane 63 as a wave-uniform scalar.
template <int kCtrl, int kRowMask>
__device__ __forceinline__ float dpp_take(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), kCtrl, kRowMask, 0xF, false));
}

__device__ __forceinline__ float wave_sum(float x) {
    x += dpp_take<0xB1, 0xF>(x);   // quad_perm [1,0,3,2]
    x += dpp_take<0x4E, 0xF>(x);   // quad_perm [2,3,0,1]
    x += dpp_take<0x141, 0xF>(x);  // row_half_mirror
    x += dpp_take<0x140, 0xF>(x);  // row_mirror
    x += dpp_take<0x142, 0xA>(x);  // row_bcast15 into rows 1 and 3
    x += dpp_take<0x143, 0xC>(x);  // row_bcast31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

__device__ __forceinline__ uint32_t lane_value(uint32_t x, uint32_t lane) {
    return (uint32_t)__builtin_amdgcn_readlane((int)x, (int)lane);
}

// ---------------------------------------------------------------------------
// Row <-> registers.  A lane holds kV floats of the row in segments: plain
// accesses use 16-byte segments when the row allows, device-scope accesses use
// 8-byte segments (the widest single-copy-atomic access).  Element e of segment
// s sits at row[s * 64 * W + lane * W + e], so each segment is one contiguous
// 64 * W * 4 byte request per wave.  kFull says that the row is exactly 64 * kV floats long:
// then no lane is ever past the end and the per-lane bounds tests (and the execution-mask
// bookkeeping they cost around every memory instruction) are compiled out.
template <int kV, int kCoherence, bool kFull = false>
struct RowIo {
    static constexpr int W = is_agent(kCoherence) ? (kV >= 2 ? 2 : 1) : (kV >= 4 ? 4 : kV);
    static constexpr int S = kV / W;

    // dim (a multiple of 32, at most 64 * kV) is the row length: lanes past the end hold zeros
    static __device__ __forceinline__ void load(const float *row, int lane, uint32_t dim, float (&x)[kV]) {
#pragma unroll
        for (int s = 0; s < S; ++s) {
            if (!kFull && (uint32_t)(s * (kWave * W) + lane * W) >= dim) {
#pragma unroll
                for (int e = 0; e < W; ++e) x[s * W + e] = 0.0f;
                continue;
            }
            const float *p = row + s * (kWave * W) + lane * W;
            if constexpr (is_agent(kCoherence)) {
                if constexpr (W == 2) {
                    const uint64_t bits =
                        __hip_atomic_load((const uint64_t *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    x[s * W] = __uint_as_float((uint32_t)bits);
                    x[s * W + 1] = __uint_as_float((uint32_t)(bits >> 32));
                } else {
                    x[s] = __uint_as_float(
                        __hip_atomic_load((const uint32_t *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                }
            } else if constexpr (W == 4) {
                const f4 t = *(const f4 *)p;
                x[s * 4] = t.x; x[s * 4 + 1] = t.y; x[s * 4 + 2] = t.z; x[s * 4 + 3] = t.w;
            } else if constexpr (W == 2) {
                const f2 t = *(const f2 *)p;
                x[s * 2] = t.x; x[s * 2 + 1] = t.y;
            } else {
                x[s] = *p;
            }
        }
    }

    // row += delta without losing concurrent updates of other waves: one fp32 atomic add
    // per element.  With two floats per lane the values are first exchanged between lanes
    // (lane l takes elements l and l + 64 of the 128-float segment) so that every atomic
    // instruction covers 256 contiguous bytes instead of every other word of 512.
    static __device__ __forceinline__ void add(float *row, int lane, uint32_t dim, const float (&delta)[kV]) {
        static_assert(W <= 2, "atomic adds are used with the device-scope layouts only");
#pragma unroll
        for (int s = 0; s < S; ++s) {
            if constexpr (W == 2) {
                const int lo = (lane >> 1) * 4, hi = (32 + (lane >> 1)) * 4;  // byte addresses of the source lanes
                const int e0 = __float_as_int(delta[s * 2]), e1 = __float_as_int(delta[s * 2 + 1]);
                const int lo0 = __builtin_amdgcn_ds_bpermute(lo, e0), lo1 = __builtin_amdgcn_ds_bpermute(lo, e1);
                const int hi0 = __builtin_amdgcn_ds_bpermute(hi, e0), hi1 = __builtin_amdgcn_ds_bpermute(hi, e1);
                const float first = __int_as_float((lane & 1) ? lo1 : lo0);
                const float second = __int_as_float((lane & 1) ? hi1 : hi0);
                float *p = row + s * (kWave * 2) + lane;
                if (kFull || (uint32_t)(s * (kWave * 2) + lane) < dim)
                    (void)__hip_atomic_fetch_add(p, first, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (kFull || (uint32_t)(s * (kWave * 2) + kWave + lane) < dim)
                    (void)__hip_atomic_fetch_add(p + kWave, second, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                if (kFull || (uint32_t)(s * kWave + lane) < dim)
                    (void)__hip_atomic_fetch_add(row + s * kWave + lane, delta[s], __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }

    // row += delta with returning atomic adds, x = the row right after this wave's addition
    // (whatever other waves added before it is included), delta = 0.  Same lane exchange as
    // add(), and the inverse exchange for the values that come back.
    static __device__ __forceinline__ void exchange(float *row, int lane, uint32_t dim, float (&delta)[kV],
                                                    float (&x)[kV]) {
        static_assert(W <= 2, "atomic adds are used with the device-scope layouts only");
#pragma unroll
        for (int s = 0; s < S; ++s) {
            if constexpr (W == 2) {
                const int lo = (lane >> 1) * 4, hi = (32 + (lane >> 1)) * 4;
                const int e0 = __float_as_int(delta[s * 2]), e1 = __float_as_int(delta[s * 2 + 1]);
                const int lo0 = __builtin_amdgcn_ds_bpermute(lo, e0), lo1 = __builtin_amdgcn_ds_bpermute(lo, e1);
                const int hi0 = __builtin_amdgcn_ds_bpermute(hi, e0), hi1 = __builtin_amdgcn_ds_bpermute(hi, e1);
                float first = __int_as_float((lane & 1) ? lo1 : lo0);    // element lane of the segment
                float second = __int_as_float((lane & 1) ? hi1 : hi0);   // element 64 + lane
                float *p = row + s * (kWave * 2) + lane;
                if (kFull || (uint32_t)(s * (kWave * 2) + lane) < dim)
                    first += __hip_atomic_fetch_add(p, first, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (kFull || (uint32_t)(s * (kWave * 2) + kWave + lane) < dim)
                    second += __hip_atomic_fetch_add(p + kWave, second, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                // lane l wants elements 2l and 2l + 1: lanes 2l, 2l + 1 hold them in `first` when
                // l < 32, lanes 2l - 64, 2l - 63 in `second` otherwise
                const int even = ((2 * lane) & 63) * 4, odd = ((2 * lane + 1) & 63) * 4;
                const int f_even = __builtin_amdgcn_ds_bpermute(even, __float_as_int(first));
                const int f_odd = __builtin_amdgcn_ds_bpermute(odd, __float_as_int(first));
                const int s_even = __builtin_amdgcn_ds_bpermute(even, __float_as_int(second));
                const int s_odd = __builtin_amdgcn_ds_bpermute(odd, __float_as_int(second));
                x[s * 2] = __int_as_float(lane < 32 ? f_even : s_even);
                x[s * 2 + 1] = __int_as_float(lane < 32 ? f_odd : s_odd);
                delta[s * 2] = delta[s * 2 + 1] = 0.0f;
            } else {
                if (kFull || (uint32_t)(s * kWave + lane) < dim)
                    x[s] = delta[s] + __hip_atomic_fetch_add(row + s * kWave + lane, delta[s], __ATOMIC_RELAXED,
                                                             __HIP_MEMORY_SCOPE_AGENT);
                delta[s] = 0.0f;
            }
        }
    }

    static __device__ __forceinline__ void store(float *row, int lane, uint32_t dim, const float (&x)[kV]) {
#pragma unroll
        for (int s = 0; s < S; ++s) {
            if (!kFull && (uint32_t)(s * (kWave * W) + lane * W) >= dim) continue;
            float *p = row + s * (kWave * W) + lane * W;
            if constexpr (is_agent(kCoherence)) {
                if constexpr (W == 2) {
                    const uint64_t bits =
                        (uint64_t)__float_as_uint(x[s * W]) | ((uint64_t)__float_as_uint(x[s * W + 1]) << 32);
                    __hip_atomic_store((uint64_t *)p, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    __hip_atomic_store((uint32_t *)p, __float_as_uint(x[s]), __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                }
            } else if constexpr (W == 4) {
                f4 t = {x[s * 4], x[s * 4 + 1], x[s * 4 + 2], x[s * 4 + 3]};
                *(f4 *)p = t;
            } else if constexpr (W == 2) {
                f2 t = {x[s * 2], x[s * 2 + 1]};
                *(f2 *)p = t;
            } else {
                *p = x[s];
            }
        }
    }
};

__device__ __forceinline__ float sigmoid(float z) { return 1.0f / (1.0f + __expf(-z)); }

// Running training loss (kernels instantiated with kTrack only): -log sigmoid(z) = log(1 + e^-z) for either
// sign of z; a positive's score s contributes minus_log_sigmoid(s), a negative's w * minus_log_sigmoid(-s).
// A wave sums what its samples saw in fp32 and hands the sum over every so often as one fp64 atomic add
// (the values are wave-uniform: lane 0 adds).
__device__ __forceinline__ float minus_log_sigmoid(float z) { return fmaxf(-z, 0.0f) + log1pf(__expf(-fabsf(z))); }
__device__ __forceinline__ void hand_over_loss(double *slots, float &loss, int lane) {
    if (lane == 0)
        (void)__hip_atomic_fetch_add(slots + (blockIdx.x % kLossSlots), (double)loss, __ATOMIC_RELAXED,
                                     __HIP_MEMORY_SCOPE_AGENT);
    loss = 0.0f;
}

// One positive sample with its K negatives (Alg. 1, the Train calls; Sec. 2.1
// scores; Sec. 4.3 negative weight): rows[0] is the positive context row v,
// rows[1..K] the negatives.  All 1+K scores come from the rows as loaded, then
//   vertex[u]      += sum_k coef_k * context[rows_k]
//   context[rows_k] += coef_k * vertex[u]
// with coef_0 = lr (1 - sigmoid(s_0)), coef_k = -lr w sigmoid(s_k).  A context
// row named more than once in the sample is written once with the summed
// coefficient.  u and rows[] are wave-uniform.  kTrack: the sample's loss at the rows as loaded is added
// to `loss`.
template <int kV, int kK, int kCoherence, bool kFull, bool kTrack>
__device__ __forceinline__ void sgns_step(float *__restrict__ vertex, float *__restrict__ context, uint32_t u,
                                          const uint32_t (&rows)[kK + 1], float lr, float w, int lane, uint32_t D,
                                          float &loss) {
    using Io = RowIo<kV, kCoherence, kFull>;
    float *xp = vertex + (size_t)u * D;
    float x[kV];
    float c[kK + 1][kV];
    Io::load(xp, lane, D, x);
#pragma unroll
    for (int k = 0; k <= kK; ++k) Io::load(context + (size_t)rows[k] * D, lane, D, c[k]);

    float coef[kK + 1];
#pragma unroll
    for (int k = 0; k <= kK; ++k) {
        float partial = 0.0f;
#pragma unroll
        for (int j = 0; j < kV; ++j) partial = fmaf(x[j], c[k][j], partial);
        const float score = wave_sum(partial);
        coef[k] = k == 0 ? lr * (1.0f - sigmoid(score)) : -(lr * w) * sigmoid(score);
        if constexpr (kTrack) loss += k == 0 ? minus_log_sigmoid(score) : w * minus_log_sigmoid(-score);
    }

    float dx[kV];
#pragma unroll
    for (int j = 0; j < kV; ++j) {
        float acc = 0.0f;
#pragma unroll
        for (int k = 0; k <= kK; ++k) acc = fmaf(coef[k], c[k][j], acc);
        dx[j] = acc;
    }

#pragma unroll
    for (int k = 0; k <= kK; ++k) {
        bool repeated = false;
#pragma unroll
        for (int k2 = 0; k2 < k; ++k2) repeated |= rows[k2] == rows[k];
        if (repeated) continue;  // wave-uniform: already folded into its first occurrence
        float total = coef[k];
#pragma unroll
        for (int k2 = k + 1; k2 <= kK; ++k2) total += rows[k2] == rows[k] ? coef[k2] : 0.0f;
        if constexpr (is_atomic(kCoherence)) {
            float dc[kV];
#pragma unroll
            for (int j = 0; j < kV; ++j) dc[j] = total * x[j];
            Io::add(context + (size_t)rows[k] * D, lane, D, dc);
        } else {
#pragma unroll
            for (int j = 0; j < kV; ++j) c[k][j] = fmaf(total, x[j], c[k][j]);
            Io::store(context + (size_t)rows[k] * D, lane, D, c[k]);
        }
    }
    if constexpr (is_atomic(kCoherence)) {
        Io::add(xp, lane, D, dx);
    } else {
#pragma unroll
        for (int j = 0; j < kV; ++j) dx[j] += x[j];
        Io::store(xp, lane, D, dx);
    }
}

// ---------------------------------------------------------------------------
// Asynchronous (Hogwild) training of one pool.  A wave takes chunks of 64
// consecutive samples: lane l reads sample l of the chunk (one coalesced 512 B
// read), draws that sample's negatives and learning rate, and the wave then
// walks the 64 samples in order, fetching each one's ids from the owning lane.
template <int kV, int kK, int kCoherence, bool kFull, bool kTrack>
__global__ __launch_bounds__(kBlock) void k_train_hogwild(TrainArgs a) {
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane((blockIdx.x * kBlock + threadIdx.x) / kWave);
    const uint32_t waves = gridDim.x * (kBlock / kWave);
    const uint32_t chunks = (a.count + kWave - 1) / kWave;
    const uint2 *__restrict__ pairs = (const uint2 *)a.pairs;
    float loss = 0.0f;
    uint32_t chunks_done = 0;

    for (uint32_t chunk = wave; chunk < chunks; chunk += waves) {
        const uint32_t base = chunk * kWave;
        const uint32_t in_chunk = min((uint32_t)kWave, a.count - base);
        const bool mine = (uint32_t)lane < in_chunk;
        const uint2 p = mine ? pairs[base + lane] : make_uint2(0u, 0u);
        const uint64_t g = a.first_g + (a.order && mine ? a.order[base + lane] : base + lane);
        uint32_t neg[kK];
#pragma unroll
        for (int k = 0; k < kK; ++k) neg[k] = draw_negative(a.alias, a.alias_n, a.seed, g, k);
        const float lr = learning_rate(a.lr0, a.lr_min_ratio, g, a.total);
        if (mine && (p.x >= a.n || p.y >= a.n)) *a.error_flag = 1u;

        for (uint32_t i = 0; i < in_chunk; ++i) {
            const uint32_t u = lane_value(p.x, i);
            uint32_t rows[kK + 1];
            rows[0] = lane_value(p.y, i);
            if (u >= a.n || rows[0] >= a.n) continue;  // reported through error_flag
#pragma unroll
            for (int k = 0; k < kK; ++k) rows[k + 1] = lane_value(neg[k], i);
            const float lr_i = __uint_as_float(lane_value(__float_as_uint(lr), i));
            sgns_step<kV, kK, kCoherence, kFull, kTrack>(a.vertex, a.context, u, rows, lr_i, a.neg_weight, lane, a.dim,
                                                         loss);
        }
        if (kTrack && (++chunks_done & 15u) == 0u) hand_over_loss(a.loss_slots, loss, lane);
    }
    if constexpr (kTrack) hand_over_loss(a.loss_slots, loss, lane);
}

// Update of a row that is not held in registers: row += total * other.  Atomic adds keep
// every concurrent update; the plain variant writes back loaded + total * other and can
// lose an update that another wave makes between this wave's load and store.
template <int kV, int kCoherence, bool kFull>
__device__ __forceinline__ void remote_update(float *row, int lane, uint32_t D, bool warm, float total,
                                              const float (&other)[kV], const float (&loaded)[kV]) {
    using Io = RowIo<kV, kCoherence, kFull>;
    if (kCoherence == kAtomicAgent || (kCoherence == kMixed && warm)) {
        float d[kV];
#pragma unroll
        for (int j = 0; j < kV; ++j) d[j] = total * other[j];
        Io::add(row, lane, D, d);
    } else {
        float r[kV];
#pragma unroll
        for (int j = 0; j < kV; ++j) r[j] = fmaf(total, other[j], loaded[j]);
        Io::store(row, lane, D, r);
    }
}

// ---------------------------------------------------------------------------
// Tiled stationary-row training.  A workgroup takes a tile of kTile consecutive samples
// of the pool, tags every sample with the hottest of its rows (vertex[u], context[v] or the
// context row of a negative: the one of lowest hot rank, ties going to the earlier of the
// three) and sorts the tile by that row in LDS, so that samples sharing their hot row become
// adjacent.  Each of its four waves then walks a quarter of the sorted tile
// and keeps the hot row in registers for as long as consecutive samples name it: the row is
// read once per run, the run's updates are applied to the register copy in order, and the
// run's change is added to memory with fp32 atomic adds (nothing another wave adds meanwhile
// is lost): every four samples, taking in what memory holds by then, and at the end of the
// run.  The other rows of a sample are fetched and updated per sample with the given
// policy.  Accesses to one row are served one after the other by the memory system, so a
// row that a percent of all samples name -- as an endpoint or, drawn in proportion to
// degree^0.75, as a negative -- would otherwise set the pace of the whole launch.
// Tiles are taken in pool order (one workgroup per tile, started as earlier ones end, or a
// fixed number of workgroups striding over the tiles), so the launch still moves through
// the pool front to back and a row's samples stay spread over time.  Every sample keeps the
// negatives and the learning rate of its position in the pool.
template <int kTile>
__device__ __forceinline__ void sort_tile(uint32_t *word) {
    for (uint32_t k = 2; k <= (uint32_t)kTile; k <<= 1) {
        for (uint32_t j = k >> 1; j > 0; j >>= 1) {
            for (uint32_t t = threadIdx.x; t < (uint32_t)kTile / 2; t += kBlock) {
                const uint32_t lo = 2 * t - (t & (j - 1));  // partner pairs (lo, lo + j) of this bitonic step
                const uint32_t hi = lo + j;
                const bool ascending = (lo & k) == 0;
                const uint32_t wa = word[lo], wb = word[hi];
                if ((wa > wb) == ascending) {
                    word[lo] = wb;
                    word[hi] = wa;
                }
            }
            __syncthreads();
        }
    }
}

// samples whose gathers a wave of the tiled kernel has in flight together (V floats of a row per lane, K negatives)
__host__ __device__ constexpr int tiled_batch(int V, int K) { return V * (K + 1) <= 4 ? 4 : (V * (K + 1) <= 12 ? 2 : 1); }

// bit of the pair of context rows j1 < j2 (rows 1 .. K + 1 of a sample) in a sample's `same` word
__host__ __device__ constexpr int pair_bit(int j1, int j2) { return (j1 - 1) * 6 + (j2 - 1); }

template <int kV, int kK, int kCoherence, int kTile, bool kFull, bool kTrack>
__global__ __launch_bounds__(kBlock) void k_train_tiled(TrainArgs a) {
    const uint32_t D = a.dim;
    // One sort word per sample.  On top, 14 bits for its stationary row: the matrix, then either
    // the hot rank (the kGroupedRanks hottest rows: their samples must end up adjacent) or a
    // 12-bit hash of the row id (the others: they turn up less than once per tile, and the hash
    // puts their samples in an order unrelated to the pool's, where neighbours come from one
    // walk and often share a row).  Below, the number of that row within the sample (3 bits),
    // the sample's slot in the tile (13 bits) and the warm flags of u and v (2 bits).
    constexpr uint32_t kSkip = 0xFFFFFFFFu;  // word of a slot without a trainable sample (row number 7 is never used)
    constexpr uint32_t kSlotBits = 13, kGroupedRanks = 4096;
    constexpr uint32_t kRecord = kK + 3;  // words of a sample's record: u, v, K negatives, warm flags of the negatives
    static_assert(kTile <= (1 << kSlotBits) && kTile >= 2 * kBlock, "tile size");
    static_assert(kK + 1 < 7, "row numbers take three bits and 7 is reserved");
    constexpr uint32_t kPerWave = kTile / (kBlock / kWave);
    static_assert(kPerWave % kWave == 0, "a wave walks whole 64-sample chunks");
    // samples whose gathers are in flight together: bounded by the registers their rows take
    constexpr int kBatch = tiled_batch(kV, kK);
    // A held row trades with memory every four samples where four samples are gathered at once, every two
    // where rows are so long that one or two samples fill the registers: there an exchange is a small part of
    // a sample's traffic, and the shorter interval halves how far the run's scores lag behind the other
    // holders of the row (measured on d = 512, K = 5: distance to the sequential trajectory after 4 pools
    // -0.33 % -> -0.10 % in loss at 3 % more time).
    constexpr uint32_t kExchangeEvery = kBatch >= 4 ? 4u : 2u;
    constexpr int kRows = kK + 2;  // rows of a sample: 0 = vertex[u], 1 = context[v], 2 + k = context[negative k]
    constexpr uint32_t kNoRow = 0xFFFFFFFFu;  // never a node id (ids are below n <= 2^31)
    // layout of a sample's flag word in the walk: 3 bits stationary row number, kRows warm bits, kRows
    // register-copy bits, 2 kBatch - 1 clash bits, and (K = 1 only) the one same-row bit
    constexpr uint32_t kWarmShift = 3, kTakesShift = kWarmShift + kRows, kClashShift = kTakesShift + kRows,
                       kSameShift = kClashShift + 2 * kBatch - 1;
    static_assert(kSameShift < 32, "flag word");
    using Io = RowIo<kV, kCoherence, kFull>;
    __shared__ uint32_t s_word[kTile];
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t wave_in_group = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const uint2 *__restrict__ pairs = (const uint2 *)a.pairs;
    const uint32_t tiles = (a.count + kTile - 1) / kTile;
    float loss = 0.0f;  // kTrack: of the samples this wave has trained since it last handed its sum over

    for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const uint32_t tile_base = tile * kTile;
        // Every tile orders the rows through its own mask, so the order in which a tile reaches
        // the hot rows differs from tile to tile.  With one common order all workgroups, started
        // together, would reach the same rows at the same moment, and a row would receive its
        // updates of thousands of tiles in one burst, all computed from the same stale value.
        const uint32_t scramble = (tile * 0x9E3779B1u) >> 18;  // 14 bits
        for (uint32_t t = threadIdx.x; t < (uint32_t)kTile; t += kBlock) {
            uint32_t word = kSkip;
            if (tile_base + t < a.count) {
                const uint2 p = pairs[tile_base + t];
                if (p.x < a.n && p.y < a.n) {
                    // most nodes of a large graph have no hot rank: there a cache-resident bitmap says
                    // which do, and the rank table is read for those only
                    uint32_t ru, rv;
                    if (a.ranked) {
                        ru = (a.ranked[p.x >> 5] >> (p.x & 31u)) & 1u ? a.rank[p.x] : 0xFFFFu;
                        rv = (a.ranked[p.y >> 5] >> (p.y & 31u)) & 1u ? a.rank[p.y] : 0xFFFFu;
                    } else {
                        ru = a.rank[p.x];
                        rv = a.rank[p.y];
                    }
                    uint32_t best = ru, held = 0u, row = p.x;
                    if (rv < best) {
                        best = rv;
                        held = 1u;
                        row = p.y;
                    }
                    const uint64_t g = a.first_g + (a.order ? a.order[tile_base + t] : tile_base + t);
                    // the walk below takes the sample from this record instead of drawing it again
                    uint32_t *record = a.records + (size_t)(tile_base + t) * kRecord;
                    uint32_t warm_negatives = 0;
                    record[0] = p.x;
                    record[1] = p.y;
#pragma unroll
                    for (int k = 0; k < kK; ++k) {
                        const Drawn nk = draw_ranked_negative(a.alias, a.alias_n, a.seed, g, k);
                        record[2 + k] = nk.id;
                        warm_negatives |= (nk.rank < a.warm_ranks ? 1u : 0u) << k;
                        if (nk.rank < best) {
                            best = nk.rank;
                            held = 2u + k;
                            row = nk.id;
                        }
                    }
                    record[2 + kK] = warm_negatives;
                    const uint32_t group = (held == 0u ? 0u : 1u << 13) |
                                           (best < kGroupedRanks ? __brev(best) >> 20 : kGroupedRanks | (row * 0x9E3779B1u) >> 20);
                    const uint32_t warm_uv = (ru < a.warm_ranks ? 1u : 0u) | (rv < a.warm_ranks ? 2u : 0u);
                    word = (group ^ scramble) << 18 | held << 15 | t << 2 | warm_uv;
                } else {
                    *a.error_flag = 1u;  // the sample is skipped and reported at the next synchronisation
                }
            }
            s_word[t] = word;
        }
        __syncthreads();
        sort_tile<kTile>(s_word);

        float *held = nullptr;   // address of the row kept in y[]
        bool held_warm = true;   // its merge must not lose concurrent updates
        uint32_t since_exchange = 0;  // samples of the current run since memory last saw the held row
        // the held row as (matrix, id), for the lane-parallel clash tests of the next chunk; kNoRow: none
        uint32_t carried_id = kNoRow, carried_is_vertex = 0u;
        float y[kV], moved[kV];
#pragma unroll
        for (int j = 0; j < kV; ++j) y[j] = moved[j] = 0.0f;

        // Merge the held row back: add the run's total change atomically, or, for a row that
        // concurrent samples are unlikely to share (mixed policy) or under the plain
        // device-scope policy, store the register copy.
        auto flush = [&]() {
            if (!held) return;
            if (kCoherence == kAtomicAgent || (kCoherence == kMixed && held_warm))
                Io::add(held, lane, D, moved);
            else
                Io::store(held, lane, D, y);
        };

        for (uint32_t base = wave_in_group * kPerWave; base < (wave_in_group + 1) * kPerWave; base += kWave) {
            // ---- per chunk, lane l works out everything about sample l of the chunk, so that the walk
            // below only has to fetch ready-made scalars from the owning lane (the scalar unit of a
            // compute unit is shared by its four SIMDs and is what this kernel runs out of first).
            const uint32_t word = s_word[base + lane];
            const bool mine = word != kSkip;
            const uint32_t pos = tile_base + ((word >> 2) & ((1u << kSlotBits) - 1u));
            const uint32_t *record = a.records + (size_t)pos * kRecord;
            uint32_t id[kRows];  // u, v, negatives
            id[0] = mine ? record[0] : 0u;
            id[1] = mine ? record[1] : 0u;
#pragma unroll
            for (int k = 0; k < kK; ++k) id[2 + k] = mine ? record[2 + k] : 0u;
            // bit j: row j of the sample is warm (u and v from the sort word, the negatives from the record)
            const uint32_t warm = (word & 3u) | (mine ? record[2 + kK] << 2 : 0u);
            const float lr = learning_rate(a.lr0, a.lr_min_ratio, a.first_g + (a.order && mine ? a.order[pos] : pos), a.total);
            const uint32_t h = (word >> 15) & 7u;  // number of the stationary row
            uint32_t stationary_id = id[0];
#pragma unroll
            for (int j = 1; j < kRows; ++j)
                if (h == (uint32_t)j) stationary_id = id[j];
            const uint32_t is_vertex = h == 0u ? 1u : 0u;
            // bit j: row j is the stationary row, or the same context row again (a row can be named twice in
            // a sample: positive and negative, or two negatives): its value is the register copy
            uint32_t takes = 1u << h;
#pragma unroll
            for (int j = 1; j < kRows; ++j) takes |= (h != 0u && id[j] == stationary_id ? 1u : 0u) << j;
            // bit pair_bit(j1, j2): context rows j1 < j2 of the sample are the same row
            uint32_t same = 0u;
#pragma unroll
            for (int j1 = 1; j1 < kRows; ++j1)
#pragma unroll
                for (int j2 = j1 + 1; j2 < kRows; ++j2) same |= (id[j1] == id[j2] ? 1u : 0u) << pair_bit(j1, j2);
            // Clash bits.  The walk gathers up to kBatch samples at once.  A sample must not be gathered
            // while this wave still owes memory an update of one of its rows: a row that an earlier sample of
            // the batch names, or the row held when the batch starts -- unless that row is the held row simply
            // continuing from sample to sample.  It would read the row as it was before the wave's own
            // update, and under a store policy write the stale value back over it.
            //   bit d - 1           (d < kBatch):  a row of this sample is a row of the sample d places before
            //   bit kBatch - 1 + d - 1 (d <= kBatch): a row of this sample is the stationary row of that sample
            // The row held when the chunk starts stands in for "the sample before sample 0".
            uint32_t clash = 0u;
            if constexpr (kCoherence != kAtomicAgent) {
                // x of the lane d places down.  Every lane must take part in every exchange (a lane that is
                // switched off hands out nothing): the exchanges stand alone, selections follow them.
                auto from_before = [&](uint32_t x, int d) {
                    return (uint32_t)__builtin_amdgcn_ds_bpermute((lane - d) * 4, (int)x);
                };
                // run[d]: this sample and the d before it all have the same stationary row
                const uint32_t id_before = from_before(stationary_id, 1), is_vertex_before = from_before(is_vertex, 1);
                const uint32_t prev_id = lane >= 1 ? id_before : carried_id;
                const uint32_t prev_is_vertex = lane >= 1 ? is_vertex_before : carried_is_vertex;
                const uint32_t same_as_before = prev_id == stationary_id && prev_is_vertex == is_vertex ? 1u : 0u;
                uint32_t run[kBatch + 1];
                run[0] = 1u;
                run[1] = same_as_before;
#pragma unroll
                for (int d = 2; d <= kBatch; ++d) {
                    const uint32_t same_there = from_before(same_as_before, d - 1);
                    run[d] = run[d - 1] & (lane >= d - 1 ? same_there : 0u);
                }
#pragma unroll
                for (int d = 1; d <= kBatch; ++d) {
                    // the stationary row of the sample d before (the carried row for the sample "before sample 0")
                    const bool real = lane >= d;
                    const uint32_t stationary_there = from_before(stationary_id, d), is_vertex_there = from_before(is_vertex, d);
                    const uint32_t their_stationary = real ? stationary_there : (lane == d - 1 ? carried_id : kNoRow);
                    const uint32_t their_is_vertex = real ? is_vertex_there : carried_is_vertex;
                    bool names_their_stationary = false;
#pragma unroll
                    for (int j = 0; j < kRows; ++j)
                        names_their_stationary |= id[j] == their_stationary && (j == 0) == (their_is_vertex != 0u) &&
                                                  !(run[d] != 0u && h == (uint32_t)j);
                    clash |= (names_their_stationary && their_stationary != kNoRow ? 1u : 0u) << (kBatch - 1 + d - 1);
                    if (d < kBatch) {
                        uint32_t theirs[kRows];
#pragma unroll
                        for (int j = 0; j < kRows; ++j) theirs[j] = from_before(id[j], d);
                        const uint32_t their_h = from_before(h, d);
                        bool shares = id[0] == theirs[0] && !(run[d] != 0u && h == 0u && their_h == 0u);
#pragma unroll
                        for (int j1 = 1; j1 < kRows; ++j1)
#pragma unroll
                            for (int j2 = 1; j2 < kRows; ++j2)
                                shares |= id[j1] == theirs[j2] &&
                                          !(run[d] != 0u && h == (uint32_t)j1 && their_h == (uint32_t)j2);
                        clash |= (real && shares ? 1u : 0u) << (d - 1);
                    }
                }
            }
            // one word for the walk: stationary row number, warm bits, register-copy bits, clash bits
            const uint32_t flags = h | warm << kWarmShift | takes << kTakesShift | clash << kClashShift |
                                   (kK == 1 ? ((same >> pair_bit(1, 2)) & 1u) << kSameShift : 0u);
            // sorted order puts the skipped slots last: the first one ends this wave's work
            const uint64_t live = __ballot(mine);
            const uint32_t in_chunk = live == ~0ull ? (uint32_t)kWave : (uint32_t)__builtin_ctzll(~live);

            // ---- the walk: wave-uniform copies of one sample's scalars
            struct Sample {
                float *row[kRows];   // addresses of vertex[u], context[v], context[negative k]
                float *stationary;   // the one of them that is kept in registers
                uint32_t flags, same;
                float lr;
            };
            auto decode = [&](uint32_t i) {
                Sample s;
                s.flags = lane_value(flags, i);
                s.row[0] = a.vertex + (size_t)lane_value(id[0], i) * D;
#pragma unroll
                for (int j = 1; j < kRows; ++j) s.row[j] = a.context + (size_t)lane_value(id[j], i) * D;
                const size_t stationary_at = (size_t)lane_value(stationary_id, i) * D;
                s.stationary = (s.flags & 7u) == 0u ? a.vertex + stationary_at : a.context + stationary_at;
                s.same = kK > 1 ? lane_value(same, i) : ((s.flags >> kSameShift) & 1u) << pair_bit(1, 2);
                s.lr = __uint_as_float(lane_value(__float_as_uint(lr), i));
                return s;
            };
            // Issue the loads of a sample: every row whose value is not the register copy, and the
            // stationary row when that is not the row the wave will be holding at that point.
            auto fetch = [&](const Sample &s, const float *held_then, float (&loaded)[kRows][kV], float (&fresh)[kV]) {
#pragma unroll
                for (int j = 0; j < kRows; ++j)
                    if (!((s.flags >> (kTakesShift + j)) & 1u)) Io::load(s.row[j], lane, D, loaded[j]);
                if (s.stationary != held_then) Io::load(s.stationary, lane, D, fresh);
            };

            // One sample (same arithmetic as sgns_step): switch the held row if needed, then all
            // scores and coefficients from the rows as they are before the sample, then the updates:
            // into the register copy for the held row, to memory for the others.
            auto train_one = [&](const Sample &cur, const float (&loaded)[kRows][kV], const float (&fresh)[kV]) {
                if (cur.stationary != held) {
                    flush();
#pragma unroll
                    for (int e = 0; e < kV; ++e) {
                        y[e] = fresh[e];
                        moved[e] = 0.0f;
                    }
                    held = cur.stationary;
                    held_warm = ((cur.flags >> kWarmShift >> (cur.flags & 7u)) & 1u) != 0;
                }
                const float lrw = cur.lr * a.neg_weight;
                // x = vertex[u], c[k] = context row 1 + k: the register copy where the flags say so
                float x[kV], c[kK + 1][kV];
                bool held_row[kRows];
#pragma unroll
                for (int j = 0; j < kRows; ++j) held_row[j] = ((cur.flags >> (kTakesShift + j)) & 1u) != 0;
#pragma unroll
                for (int e = 0; e < kV; ++e) x[e] = held_row[0] ? y[e] : loaded[0][e];
#pragma unroll
                for (int k = 0; k <= kK; ++k)
#pragma unroll
                    for (int e = 0; e < kV; ++e) c[k][e] = held_row[1 + k] ? y[e] : loaded[1 + k][e];
                float coef[kK + 1];
#pragma unroll
                for (int k = 0; k <= kK; ++k) {
                    float partial = 0.0f;
#pragma unroll
                    for (int e = 0; e < kV; ++e) partial = fmaf(x[e], c[k][e], partial);
                    const float score = wave_sum(partial);
                    coef[k] = k == 0 ? cur.lr * (1.0f - sigmoid(score)) : -lrw * sigmoid(score);
                    if constexpr (kTrack)
                        loss += k == 0 ? minus_log_sigmoid(score) : a.neg_weight * minus_log_sigmoid(-score);
                }
                // context rows first (they take the vertex row as it was), each distinct row once
#pragma unroll
                for (int k = 0; k <= kK; ++k) {
                    bool repeated = false;
#pragma unroll
                    for (int k2 = 0; k2 < k; ++k2) repeated |= ((cur.same >> pair_bit(1 + k2, 1 + k)) & 1u) != 0;
                    if (repeated) continue;
                    float total = coef[k];
#pragma unroll
                    for (int k2 = k + 1; k2 <= kK; ++k2)
                        total += (cur.same >> pair_bit(1 + k, 1 + k2)) & 1u ? coef[k2] : 0.0f;
                    if (held_row[1 + k]) {
#pragma unroll
                        for (int e = 0; e < kV; ++e) {
                            const float d = total * x[e];
                            y[e] += d;
                            moved[e] += d;
                        }
                    } else {
                        remote_update<kV, kCoherence, kFull>(cur.row[1 + k], lane, D,
                                                             (cur.flags >> (kWarmShift + 1 + k)) & 1u, total, x, c[k]);
                    }
                }
                float dx[kV];
#pragma unroll
                for (int e = 0; e < kV; ++e) {
                    float acc = 0.0f;
#pragma unroll
                    for (int k = 0; k <= kK; ++k) acc = fmaf(coef[k], c[k][e], acc);
                    dx[e] = acc;
                }
                if (held_row[0]) {
#pragma unroll
                    for (int e = 0; e < kV; ++e) {
                        y[e] += dx[e];
                        moved[e] += dx[e];
                    }
                } else {
                    remote_update<kV, kCoherence, kFull>(cur.row[0], lane, D, (cur.flags >> kWarmShift) & 1u, 1.0f, dx, x);
                }
            };

            // Samples go through in batches of up to kBatch: all gathers of a batch are issued first,
            // then the samples are computed one after the other (a later sample of the batch sees
            // the held row as the earlier ones left it), so one memory round trip serves kBatch
            // samples instead of one.  A sample whose clash bits name a sample of the batch, or the row
            // held when the batch starts, is left for the next batch (and that held row is merged first).
            for (uint32_t i0 = 0; i0 < in_chunk;) {
                Sample batch[kBatch];
                float loaded[kBatch][kRows][kV], fresh[kBatch][kV];
                batch[0] = decode(i0);
                // A run that goes on trades with memory before its staleness would pass kExchangeEvery
                // samples: its change so far is added and the register copy takes in what other waves
                // added meanwhile, so a held row is never more than that many samples behind the other
                // holders of that row.
                if (held && held == batch[0].stationary && since_exchange > 0u &&
                    since_exchange + kBatch > kExchangeEvery &&
                    (kCoherence == kAtomicAgent || (kCoherence == kMixed && held_warm))) {
                    Io::exchange(held, lane, D, moved, y);
                    since_exchange = 0;
                }
                if constexpr (kCoherence != kAtomicAgent) {
                    if (held && ((batch[0].flags >> (kClashShift + kBatch - 1)) & 1u)) {
                        flush();
                        held = nullptr;
                    }
                }
                const float *then = held;
                uint32_t taken = 0;
#pragma unroll
                for (int b = 0; b < kBatch; ++b) {
#pragma unroll
                    for (int e = 0; e < kV; ++e) fresh[b][e] = 0.0f;
                    if (taken == (uint32_t)b && i0 + b < in_chunk) {
                        if (b > 0) {
                            batch[b] = decode(i0 + b);
                            // earlier samples of the batch (b places at most), and the row held at its start
                            const uint32_t kEarlier = ((1u << b) - 1u) | 1u << (kBatch - 1 + b);
                            if (kCoherence != kAtomicAgent && ((batch[b].flags >> kClashShift) & kEarlier)) continue;
                        }
                        fetch(batch[b], then, loaded[b], fresh[b]);
                        then = batch[b].stationary;
                        taken = b + 1;
                    }
                }
                // All gathers of the batch are awaited here, once, whichever of them were issued: the
                // counter of outstanding vector memory operations also counts stores and atomic adds, so a
                // wait placed between the samples would sit out the previous sample's updates as well.
                __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), the other counters untouched
#pragma unroll
                for (int b = 0; b < kBatch; ++b)
                    if ((uint32_t)b < taken) {
                        since_exchange = batch[b].stationary == held ? since_exchange + 1u : 1u;
                        train_one(batch[b], loaded[b], fresh[b]);
                    }
                i0 += taken;
            }
            // what the next chunk's clash tests compare with: the row held now
            if (in_chunk > 0u) {
                carried_id = lane_value(stationary_id, in_chunk - 1u);
                carried_is_vertex = lane_value(is_vertex, in_chunk - 1u);
            }
            if (in_chunk < (uint32_t)kWave) break;
        }
        // a row that is no number any more: training has diverged (reported by the next synchronising call)
        if (held && !(y[0] == y[0])) a.error_flag[1] = 1u;
        flush();
        if constexpr (kTrack) hand_over_loss(a.loss_slots, loss, lane);
        __syncthreads();  // the next tile overwrites the LDS arrays
    }
}

// Deterministic mode: wave i trains sample i of a batch whose samples share no
// vertex row and no context row (Def. 1, Sec. 3.2: such samples commute), so the
// result equals the sequential order up to fp32 rounding inside a sample.
template <int kV, int kK, bool kFull, bool kTrack>
__global__ __launch_bounds__(kBlock) void k_train_batch(TrainArgs a) {
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t i = __builtin_amdgcn_readfirstlane((blockIdx.x * kBlock + threadIdx.x) / kWave);
    if (i >= a.count) return;
    const uint32_t u = a.pairs[2 * (size_t)i];
    uint32_t rows[kK + 1];
    rows[0] = a.pairs[2 * (size_t)i + 1];
    if (u >= a.n || rows[0] >= a.n) {
        *a.error_flag = 1u;
        return;
    }
#pragma unroll
    for (int k = 0; k < kK; ++k) rows[k + 1] = a.negatives[(size_t)i * kK + k];
    const float lr = learning_rate(a.lr0, a.lr_min_ratio, a.first_g + i, a.total);
    float loss = 0.0f;
    sgns_step<kV, kK, kPlain, kFull, kTrack>(a.vertex, a.context, u, rows, lr, a.neg_weight, lane, a.dim, loss);
    if constexpr (kTrack) hand_over_loss(a.loss_slots, loss, lane);
}

#if !GV_TRACK_LOSS
// ---------------------------------------------------------------------------
// Evaluation (no training runs meanwhile, so plain cached loads are fine).
//
// Mean of the per-sample loss  -log sigmoid(x_u . c_v) - w sum_k log sigmoid(-x_u . c_k)
// over an evaluation pool; the negatives of sample i come from Philox stream 2, counter
// (i, k).  Dot products in fp32, the logarithms and the sum in fp64.
__device__ __forceinline__ double log_sigmoid(double z) { return z >= 0.0 ? -log1p(exp(-z)) : z - log1p(exp(z)); }

template <int kV, int kK>
__global__ __launch_bounds__(kBlock) void k_eval_loss(TrainArgs a, double *__restrict__ total) {
    using Io = RowIo<kV, kPlain>;
    const uint32_t D = a.dim;
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane((blockIdx.x * kBlock + threadIdx.x) / kWave);
    const uint32_t waves = gridDim.x * (kBlock / kWave);
    const uint32_t chunks = (a.count + kWave - 1) / kWave;
    const uint2 *__restrict__ pairs = (const uint2 *)a.pairs;
    double sum = 0.0;
    for (uint32_t chunk = wave; chunk < chunks; chunk += waves) {
        const uint32_t base = chunk * kWave;
        const uint32_t in_chunk = min((uint32_t)kWave, a.count - base);
        const bool mine = (uint32_t)lane < in_chunk;
        const uint2 p = mine ? pairs[base + lane] : make_uint2(0u, 0u);
        uint32_t neg[kK];
#pragma unroll
        for (int k = 0; k < kK; ++k) neg[k] = draw_negative(a.alias, a.alias_n, a.seed, (uint64_t)base + lane, k, 2u);
        if (mine && (p.x >= a.n || p.y >= a.n)) *a.error_flag = 1u;
        for (uint32_t i = 0; i < in_chunk; ++i) {
            const uint32_t u = lane_value(p.x, i), v = lane_value(p.y, i);
            if (u >= a.n || v >= a.n) continue;
            float x[kV], c[kV];
            Io::load(a.vertex + (size_t)u * D, lane, D, x);
            double loss = 0.0;
#pragma unroll
            for (int k = 0; k <= kK; ++k) {
                const uint32_t row = k == 0 ? v : lane_value(neg[k > 0 ? k - 1 : 0], i);
                Io::load(a.context + (size_t)row * D, lane, D, c);
                float partial = 0.0f;
#pragma unroll
                for (int j = 0; j < kV; ++j) partial = fmaf(x[j], c[j], partial);
                const double score = (double)wave_sum(partial);
                loss -= k == 0 ? log_sigmoid(score) : (double)a.neg_weight * log_sigmoid(-score);
            }
            sum += loss;
        }
    }
    if (lane == 0) atomicAdd(total, sum);
}

// out[i] = cosine of vertex rows first[i], second[i] (0 when a row is zero), the score of
// an edge in link prediction (Sec. 4.5).
template <int kV>
__global__ __launch_bounds__(kBlock) void k_cosine(const float *__restrict__ vertex, uint32_t n, uint32_t dim,
                                                   const uint32_t *__restrict__ first,
                                                   const uint32_t *__restrict__ second, uint32_t count,
                                                   float *__restrict__ out, uint32_t *error_flag) {
    using Io = RowIo<kV, kPlain>;
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t waves = gridDim.x * (kBlock / kWave);
    for (uint32_t i = __builtin_amdgcn_readfirstlane((blockIdx.x * kBlock + threadIdx.x) / kWave); i < count;
         i += waves) {
        const uint32_t ra = first[i], rb = second[i];
        if (ra >= n || rb >= n) {
            *error_flag = 1u;
            if (lane == 0) out[i] = 0.0f;
            continue;
        }
        float x[kV], y[kV];
        Io::load(vertex + (size_t)ra * dim, lane, dim, x);
        Io::load(vertex + (size_t)rb * dim, lane, dim, y);
        float xy = 0.0f, xx = 0.0f, yy = 0.0f;
#pragma unroll
        for (int j = 0; j < kV; ++j) {
            xy = fmaf(x[j], y[j], xy);
            xx = fmaf(x[j], x[j], xx);
            yy = fmaf(y[j], y[j], yy);
        }
        xy = wave_sum(xy);
        xx = wave_sum(xx);
        yy = wave_sum(yy);
        if (lane == 0) out[i] = (xx > 0.0f && yy > 0.0f) ? xy / (sqrtf(xx) * sqrtf(yy)) : 0.0f;
    }
}

__global__ __launch_bounds__(kBlock) void k_draw_negatives(const uint4 *__restrict__ alias, uint32_t n, uint64_t seed,
                                                           uint64_t first_g, uint64_t count, uint32_t num_neg,
                                                           uint32_t *__restrict__ out) {
    const uint64_t total = count * num_neg;
    for (uint64_t t = (uint64_t)blockIdx.x * kBlock + threadIdx.x; t < total; t += (uint64_t)gridDim.x * kBlock) {
        const uint64_t i = t / num_neg;
        const uint32_t k = (uint32_t)(t - i * num_neg);
        out[t] = draw_negative(alias, n, seed, first_g + i, k);
    }
}

// Negatives restricted to a partition (Sec. 3.2): sample i draws from the alias table of the partition of its
// context node v[i].
__global__ __launch_bounds__(kBlock) void k_draw_negatives_partitioned(const uint4 *__restrict__ tables,
                                                                       const uint64_t *__restrict__ offsets,
                                                                       const uint8_t *__restrict__ part,
                                                                       const uint32_t *__restrict__ v, uint64_t seed,
                                                                       uint64_t first_g, uint64_t count, uint32_t num_neg,
                                                                       uint32_t *__restrict__ out) {
    const uint64_t total = count * num_neg;
    for (uint64_t t = (uint64_t)blockIdx.x * kBlock + threadIdx.x; t < total; t += (uint64_t)gridDim.x * kBlock) {
        const uint64_t i = t / num_neg;
        const uint32_t k = (uint32_t)(t - i * num_neg);
        const uint32_t j = part[v[i]];
        out[t] = draw_negative(tables + offsets[j], (uint32_t)(offsets[j + 1] - offsets[j]), seed, first_g + i, k);
    }
}

// vertex[row][4b .. 4b+3] from the four words of Philox block (row, b) of stream 1:
// ((word + 0.5) / 2^32 - 0.5) / d, evaluated in fp64.
__global__ __launch_bounds__(kBlock) void k_init_vertex(float *__restrict__ vertex, uint64_t rows, uint32_t dim,
                                                        uint64_t seed) {
    const uint32_t blocks_per_row = dim / 4;
    const uint64_t total = rows * blocks_per_row;
    for (uint64_t t = (uint64_t)blockIdx.x * kBlock + threadIdx.x; t < total; t += (uint64_t)gridDim.x * kBlock) {
        const uint64_t row = t / blocks_per_row;
        const uint32_t b = (uint32_t)(t - row * blocks_per_row);
        const uint4 r = philox4x32_10((uint32_t)row, (uint32_t)(row >> 32), b, 1u, (uint32_t)seed,
                                      (uint32_t)(seed >> 32));
        const double inv = 1.0 / 4294967296.0;
        f4 out;
        out.x = (float)((((double)r.x + 0.5) * inv - 0.5) / (double)dim);
        out.y = (float)((((double)r.y + 0.5) * inv - 0.5) / (double)dim);
        out.z = (float)((((double)r.z + 0.5) * inv - 0.5) / (double)dim);
        out.w = (float)((((double)r.w + 0.5) * inv - 0.5) / (double)dim);
        *(f4 *)(vertex + row * dim + 4 * (uint64_t)b) = out;
    }
}

// ---------------------------------------------------------------------------
// Producer on the device: online augmentation (Sec. 3.1, Alg. 2) with the pseudo shuffle of
// the same section, one thread per random walk.  Walk w departs at the owner of a uniformly
// chosen half-edge (probability proportional to degree), takes `length` uniform steps over the
// CSR adjacency (on a weighted graph both are alias draws, see below) and emits every ordered pair (w_i, w_j), i < j <= i + window, in order of i then
// j; sample number t of the pool (walks concatenated) goes to position t, or, pseudo-shuffled,
// to block t mod window at offset t / window.  Random numbers: Philox stream 4, counter
// (walk number, step): the pool depends on nothing but the seed and the walk numbers.
constexpr int kWalkBlock = 128;    // threads (= walks) per workgroup
constexpr int kMaxWalkLength = 64;

__device__ __forceinline__ uint64_t pick_below(uint4 r, uint64_t range) {
    return __umul64hi(((uint64_t)r.x << 32) | r.y, range);
}

// The pool position of sample number t (generation order): t itself, or, pseudo-shuffled, block t mod s at
// offset t / s (block b holds the samples b, b + s, b + 2s, ...: the blocks before it hold
// ceil((count - b') / s) samples each, i.e. the first count mod s blocks hold one more).
__device__ __forceinline__ uint64_t place_of(uint64_t t, uint32_t s, uint64_t count, bool pseudo_shuffle) {
    if (!pseudo_shuffle) return t;
    const uint64_t b = t % s, q = t / s, whole = count / s, extra = count % s;
    return b * whole + (b < extra ? b : extra) + q;
}

__global__ __launch_bounds__(kWalkBlock) void k_augment(AugmentArgs a) {
    // a walk's nodes, one row per thread (65 words: the rows start in different banks)
    __shared__ uint32_t s_path[kWalkBlock][kMaxWalkLength + 1];
    // the pairs of a walk in order: i << 8 | j of pair number t (i < j <= i + s, in order of i then j)
    __shared__ uint16_t s_pair[(kMaxWalkLength + 1) * kMaxWalkLength / 2];
    const uint64_t w0 = (uint64_t)blockIdx.x * kWalkBlock, w = w0 + threadIdx.x;
    const uint32_t L = a.length, s = a.window;
    for (uint32_t i = threadIdx.x; i < L; i += kWalkBlock) {
        uint32_t start = 0;  // pairs of the nodes before i
        for (uint32_t before = 0; before < i; ++before) start += min(s, L - before);
        for (uint32_t j = i + 1; j <= L && j - i <= s; ++j) s_pair[start + (j - i - 1)] = (uint16_t)(i << 8 | j);
    }
    if (w < a.walks) {
        const uint32_t k0 = (uint32_t)a.seed, k1 = (uint32_t)(a.seed >> 32);
        const uint64_t walk = a.first_walk + w;
        uint32_t x;
        const uint4 r0 = philox4x32_10((uint32_t)walk, (uint32_t)(walk >> 32), 0u, 4u, k0, k1);
        if (a.node_table) {
            // weighted graph (Sec. 4.3): departure by an alias draw over the nodes, weights = weighted degrees
            const uint32_t j = (uint32_t)pick_below(r0, a.n);
            const uint2 entry = a.node_table[j];
            x = r0.z < entry.x ? j : entry.y;
        } else {
            // departure: last node whose first half-edge is at or before the chosen one
            const uint64_t e = pick_below(r0, a.half_edges);
            uint32_t lo = 0, hi = a.n;  // offsets[lo] <= e < offsets[hi]
            while (hi - lo > 1) {
                const uint32_t mid = lo + (hi - lo) / 2;
                if (a.offsets[mid] <= e) lo = mid; else hi = mid;
            }
            x = lo;
        }
        s_path[threadIdx.x][0] = x;
        for (uint32_t t = 1; t <= L; ++t) {
            const uint64_t begin = a.offsets[x], degree = a.offsets[x + 1] - begin;
            const uint4 r = philox4x32_10((uint32_t)walk, (uint32_t)(walk >> 32), t, 4u, k0, k1);
            uint64_t at = pick_below(r, degree);
            if (a.nbr_table) {  // weighted step: alias draw over the row's edge weights
                const uint2 entry = a.nbr_table[begin + at];
                at = r.z < entry.x ? at : entry.y;
            }
            x = a.adj[begin + at];
            s_path[threadIdx.x][t] = x;
        }
    }
    __syncthreads();
    // The workgroup's walks cover the samples t_lo .. t_hi - 1 of the pool; the workgroup writes them together, a
    // thread per sample, in the order of their places in the pool, so that neighbouring threads write
    // neighbouring pairs (one thread writing its own walk's 190 pairs scatters 8-byte stores over the pool).
    const uint32_t here = (uint32_t)min((uint64_t)kWalkBlock, a.walks - w0);
    const uint64_t t_lo = w0 * a.per_walk;
    const uint64_t t_hi = min(t_lo + (uint64_t)here * a.per_walk, a.count);
    if (t_lo >= t_hi) return;
    const uint32_t per_walk = (uint32_t)a.per_walk, span = (uint32_t)(t_hi - t_lo);
    auto emit = [&](uint32_t t_rel, uint64_t place) {  // sample t_lo + t_rel goes to pairs[place]
        const uint32_t walk = t_rel / per_walk, pair = s_pair[t_rel % per_walk];
        a.pairs[place] = make_uint2(s_path[walk][pair >> 8], s_path[walk][pair & 0xFFu]);
    };
    if (!a.pseudo_shuffle) {
        for (uint32_t t_rel = threadIdx.x; t_rel < span; t_rel += kWalkBlock) emit(t_rel, t_lo + t_rel);
    } else if (s > span) {
        for (uint32_t t_rel = threadIdx.x; t_rel < span; t_rel += kWalkBlock)
            emit(t_rel, place_of(t_lo + t_rel, s, a.count, true));
    } else {
        // block after block: within block b the workgroup's samples are b + q s for consecutive q
        const uint64_t q_lo = t_lo / s, whole = a.count / s, extra = a.count % s;
        const uint32_t steps = (uint32_t)((t_hi - 1) / s - q_lo) + 1u;
        const uint32_t all = s * steps;  // s <= span here: at most span + 2 s < 2^20 places to look at
        for (uint32_t index = threadIdx.x; index < all; index += kWalkBlock) {
            const uint32_t b = index / steps, q = index % steps;
            const uint64_t t = (q_lo + q) * s + b;
            if (t >= t_lo && t < t_hi) emit((uint32_t)(t - t_lo), b * whole + (b < extra ? b : extra) + q_lo + q);
        }
    }
}

#endif  // !GV_TRACK_LOSS

// Persistent-style grid: enough workgroups to fill all 256 CUs at full occupancy; each
// wave strides over the chunks.  The number of samples in flight is also kept below
// |V|/32: every in-flight sample works on values that miss the updates of the others
// (Def. 1, Sec. 3.2: the order of updates stops mattering only while concurrent samples
// rarely share rows), and a small graph gains nothing from thousands of waves.
uint32_t hogwild_blocks(uint32_t count, uint32_t n) {
    constexpr uint32_t max_blocks = 256u * 8u;
    const uint32_t chunks = (count + kWave - 1) / kWave;
    const uint32_t wanted = (chunks + (kBlock / kWave) - 1) / (kBlock / kWave);
    const uint32_t by_rows = (n / 32u) / (kBlock / kWave);
    uint32_t blocks = wanted < max_blocks ? wanted : max_blocks;
    if (blocks > by_rows) blocks = by_rows > 64u ? by_rows : (blocks < 64u ? blocks : 64u);
    return blocks;
}

// A row that fills its lanes exactly (d = 64, 128, 256, 512) takes the kernels without per-lane bounds tests.
template <int kV, int kK, bool kFull, bool kTrack>
hipError_t launch_hogwild_vkft(const TrainArgs &a, uint32_t coherence, uint32_t blocks, hipStream_t stream) {
    switch (coherence) {
        case kAgent:
            hipLaunchKernelGGL((k_train_hogwild<kV, kK, kAgent, kFull, kTrack>), dim3(blocks), dim3(kBlock), 0, stream, a);
            break;
        case kAtomicAgent:
        case kMixed:  // the per-row choice exists in the tiled kernel only
            hipLaunchKernelGGL((k_train_hogwild<kV, kK, kAtomicAgent, kFull, kTrack>), dim3(blocks), dim3(kBlock), 0, stream, a);
            break;
        default:
            hipLaunchKernelGGL((k_train_hogwild<kV, kK, kPlain, kFull, kTrack>), dim3(blocks), dim3(kBlock), 0, stream, a);
    }
    return hipGetLastError();
}

// the kernels that also sum the running loss are separate instantiations (in an object of their own): the ones
// that do not carry none of it
template <int kV, int kK, bool kFull>
hipError_t launch_hogwild_vkf(const TrainArgs &a, uint32_t coherence, uint32_t blocks, hipStream_t stream) {
    if ((a.loss_slots != nullptr) != (GV_TRACK_LOSS != 0)) return hipErrorInvalidValue;
    return launch_hogwild_vkft<kV, kK, kFull, GV_TRACK_LOSS != 0>(a, coherence, blocks, stream);
}

template <int kV, int kK>
hipError_t launch_hogwild_vk(const TrainArgs &a, uint32_t coherence, hipStream_t stream) {
    const uint32_t blocks = hogwild_blocks(a.count, a.n);
    if (blocks == 0) return hipSuccess;
    return a.dim == (uint32_t)(kWave * kV) ? launch_hogwild_vkf<kV, kK, true>(a, coherence, blocks, stream)
                                           : launch_hogwild_vkf<kV, kK, false>(a, coherence, blocks, stream);
}

template <int kV, int kK, int kTile, bool kFull, bool kTrack>
hipError_t launch_tiled_vktt(const TrainArgs &a, uint32_t coherence, uint32_t blocks, hipStream_t stream) {
    if (coherence == kAgent)
        hipLaunchKernelGGL((k_train_tiled<kV, kK, kAgent, kTile, kFull, kTrack>), dim3(blocks), dim3(kBlock), 0, stream, a);
    else if (coherence == kMixed)
        hipLaunchKernelGGL((k_train_tiled<kV, kK, kMixed, kTile, kFull, kTrack>), dim3(blocks), dim3(kBlock), 0, stream, a);
    else
        hipLaunchKernelGGL((k_train_tiled<kV, kK, kAtomicAgent, kTile, kFull, kTrack>), dim3(blocks), dim3(kBlock), 0, stream, a);
    return hipGetLastError();
}

template <int kV, int kK, int kTile, bool kFull>
hipError_t launch_tiled_vkt(const TrainArgs &a, uint32_t coherence, uint32_t blocks, hipStream_t stream) {
    if ((a.loss_slots != nullptr) != (GV_TRACK_LOSS != 0)) return hipErrorInvalidValue;
    return launch_tiled_vktt<kV, kK, kTile, kFull, GV_TRACK_LOSS != 0>(a, coherence, blocks, stream);
}

template <int kV, int kK>
hipError_t launch_tiled_vk(const TrainArgs &a, uint32_t coherence, hipStream_t stream) {
    if (a.count == 0) return hipSuccess;
    if (a.rank == nullptr || a.records == nullptr) return hipErrorInvalidValue;
    constexpr uint32_t tile = 8192;  // samples per workgroup (2048 and 4096 were 10 % and 5 % slower on the power-law graph)
    // One workgroup per tile, started by the hardware in tile order as earlier ones end, unless the
    // graph is so small that fewer samples must be in flight: then a fixed number of workgroups
    // strides over the tiles.
    const uint32_t limit = hogwild_blocks(a.count, a.n);
    const uint32_t tiles = (a.count + tile - 1) / tile;
    const uint32_t blocks = limit >= 2048u || limit > tiles ? tiles : limit;
    return a.dim == (uint32_t)(kWave * kV) ? launch_tiled_vkt<kV, kK, (int)tile, true>(a, coherence, blocks, stream)
                                           : launch_tiled_vkt<kV, kK, (int)tile, false>(a, coherence, blocks, stream);
}

template <int kV, int kK>
hipError_t launch_batch_vk(const TrainArgs &a, hipStream_t stream) {
    if (a.count == 0) return hipSuccess;
    const uint32_t blocks = (a.count + (kBlock / kWave) - 1) / (kBlock / kWave);
    if ((a.loss_slots != nullptr) != (GV_TRACK_LOSS != 0)) return hipErrorInvalidValue;
    constexpr bool kTrack = GV_TRACK_LOSS != 0;
    if (a.dim == (uint32_t)(kWave * kV))
        hipLaunchKernelGGL((k_train_batch<kV, kK, true, kTrack>), dim3(blocks), dim3(kBlock), 0, stream, a);
    else
        hipLaunchKernelGGL((k_train_batch<kV, kK, false, kTrack>), dim3(blocks), dim3(kBlock), 0, stream, a);
    return hipGetLastError();
}

}  // namespace

#if !GV_TRACK_LOSS
uint32_t samples_per_batch(uint32_t dim, uint32_t num_neg) {
    const int V = dim <= 64 ? 1 : (dim <= 128 ? 2 : (dim <= 256 ? 4 : 8));  // as GV_DISPATCH below
    return (uint32_t)tiled_batch(V, (int)num_neg);
}

bool supported_shape(uint32_t dim, uint32_t num_neg) {
    return dim >= 32 && dim <= 512 && dim % 32 == 0 && num_neg >= 1 && num_neg <= 5;
}
#endif  // !GV_TRACK_LOSS

#define GV_DISPATCH_K(V, CALL)                 \
    switch (num_neg) {                         \
        case 1: return CALL(V, 1);             \
        case 2: return CALL(V, 2);             \
        case 3: return CALL(V, 3);             \
        case 4: return CALL(V, 4);             \
        case 5: return CALL(V, 5);             \
        default: return hipErrorInvalidValue;  \
    }
// a lane holds V floats of a row: the smallest V in {1, 2, 4, 8} with 64 V >= dim
#define GV_DISPATCH(CALL)                                                   \
    if (!supported_shape(dim, num_neg) || a.dim != dim) return hipErrorInvalidValue; \
    if (dim <= 64) { GV_DISPATCH_K(1, CALL) }                               \
    if (dim <= 128) { GV_DISPATCH_K(2, CALL) }                              \
    if (dim <= 256) { GV_DISPATCH_K(4, CALL) }                              \
    GV_DISPATCH_K(8, CALL)

hipError_t GV_TRAIN_NAME(launch_train_hogwild)(const TrainArgs &a, uint32_t dim, uint32_t num_neg, uint32_t coherence,
                                               hipStream_t stream) {
#define GV_CALL(V, K) launch_hogwild_vk<V, K>(a, coherence, stream)
    GV_DISPATCH(GV_CALL)
#undef GV_CALL
}

hipError_t GV_TRAIN_NAME(launch_train_tiled)(const TrainArgs &a, uint32_t dim, uint32_t num_neg, uint32_t coherence,
                                             hipStream_t stream) {
#define GV_CALL(V, K) launch_tiled_vk<V, K>(a, coherence, stream)
    GV_DISPATCH(GV_CALL)
#undef GV_CALL
}

hipError_t GV_TRAIN_NAME(launch_train_batch)(const TrainArgs &a, uint32_t dim, uint32_t num_neg, hipStream_t stream) {
#define GV_CALL(V, K) launch_batch_vk<V, K>(a, stream)
    GV_DISPATCH(GV_CALL)
#undef GV_CALL
}

#if !GV_TRACK_LOSS
template <int kV, int kK>
hipError_t launch_eval_vk(const TrainArgs &a, double *total, hipStream_t stream) {
    if (a.count == 0) return hipSuccess;
    const uint32_t chunks = (a.count + kWave - 1) / kWave;
    const uint32_t wanted = (chunks + (kBlock / kWave) - 1) / (kBlock / kWave);
    hipLaunchKernelGGL((k_eval_loss<kV, kK>), dim3(wanted < 2048u ? wanted : 2048u), dim3(kBlock), 0, stream, a, total);
    return hipGetLastError();
}

hipError_t launch_eval_loss(const TrainArgs &a, uint32_t dim, uint32_t num_neg, double *total, hipStream_t stream) {
#define GV_CALL(V, K) launch_eval_vk<V, K>(a, total, stream)
    GV_DISPATCH(GV_CALL)
#undef GV_CALL
}

hipError_t launch_cosine(const float *vertex, uint32_t n, uint32_t dim, const uint32_t *first, const uint32_t *second,
                         uint32_t count, float *out, uint32_t *error_flag, hipStream_t stream) {
    if (count == 0) return hipSuccess;
    const uint32_t wanted = (count + (kBlock / kWave) - 1) / (kBlock / kWave);
    const dim3 grid(wanted < 4096u ? wanted : 4096u), block(kBlock);
    if (dim <= 64)
        hipLaunchKernelGGL((k_cosine<1>), grid, block, 0, stream, vertex, n, dim, first, second, count, out, error_flag);
    else if (dim <= 128)
        hipLaunchKernelGGL((k_cosine<2>), grid, block, 0, stream, vertex, n, dim, first, second, count, out, error_flag);
    else if (dim <= 256)
        hipLaunchKernelGGL((k_cosine<4>), grid, block, 0, stream, vertex, n, dim, first, second, count, out, error_flag);
    else
        hipLaunchKernelGGL((k_cosine<8>), grid, block, 0, stream, vertex, n, dim, first, second, count, out, error_flag);
    return hipGetLastError();
}

hipError_t launch_draw_negatives(const uint4 *alias, uint32_t n, uint64_t seed, uint64_t first_g, uint64_t count,
                                 uint32_t num_neg, uint32_t *out, hipStream_t stream) {
    const uint64_t total = count * num_neg;
    if (total == 0) return hipSuccess;
    const uint64_t wanted = (total + kBlock - 1) / kBlock;
    const uint32_t blocks = (uint32_t)(wanted < 65536 ? wanted : 65536);
    hipLaunchKernelGGL(k_draw_negatives, dim3(blocks), dim3(kBlock), 0, stream, alias, n, seed, first_g, count,
                       num_neg, out);
    return hipGetLastError();
}

hipError_t launch_draw_negatives_partitioned(const uint4 *tables, const uint64_t *offsets, const uint8_t *part,
                                             const uint32_t *v, uint64_t seed, uint64_t first_g, uint64_t count,
                                             uint32_t num_neg, uint32_t *out, hipStream_t stream) {
    const uint64_t total = count * num_neg;
    if (total == 0) return hipSuccess;
    const uint64_t wanted = (total + kBlock - 1) / kBlock;
    const uint32_t blocks = (uint32_t)(wanted < 65536 ? wanted : 65536);
    hipLaunchKernelGGL(k_draw_negatives_partitioned, dim3(blocks), dim3(kBlock), 0, stream, tables, offsets, part, v, seed,
                       first_g, count, num_neg, out);
    return hipGetLastError();
}

hipError_t launch_init_vertex(float *vertex, uint64_t rows, uint32_t dim, uint64_t seed, hipStream_t stream) {
    const uint64_t total = rows * (dim / 4);
    if (total == 0) return hipSuccess;
    const uint64_t wanted = (total + kBlock - 1) / kBlock;
    const uint32_t blocks = (uint32_t)(wanted < 65536 ? wanted : 65536);
    hipLaunchKernelGGL(k_init_vertex, dim3(blocks), dim3(kBlock), 0, stream, vertex, rows, dim, seed);
    return hipGetLastError();
}

hipError_t launch_augment(const AugmentArgs &a, hipStream_t stream) {
    if (a.walks == 0) return hipSuccess;
    if (a.length == 0 || a.length > (uint32_t)kMaxWalkLength || a.window == 0) return hipErrorInvalidValue;
    const uint64_t blocks = (a.walks + kWalkBlock - 1) / kWalkBlock;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_augment, dim3((uint32_t)blocks), dim3(kWalkBlock), 0, stream, a);
    return hipGetLastError();
}

#endif  // !GV_TRACK_LOSS

}  // namespace gv
