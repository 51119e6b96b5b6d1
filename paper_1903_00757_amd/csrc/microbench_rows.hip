// Microbenchmark of the memory operations the training kernels are built from: random access to
// 512-byte rows (d = 128 fp32, one wave per row, 8 bytes per lane) under the cache policies and
// update methods the kernels choose between.  Not part of the library; its numbers are what the
// choice of policies in the training kernels rests on.
//
//   microbench_rows ops   <rows> <skew>   every operation on a table of <rows> rows, accesses drawn with
//                                         weights rank^-skew (0 = uniform), rows scattered
//   microbench_rows sizes                 device-scope read and read-modify-write against the table size
//   microbench_rows same                  2048 waves add 1 to one row 200 times with every method:
//                                         what is left in the row, and where the workgroups ran
//
// Every kernel is a bounded loop over a list of row numbers below the table size.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <random>
#include <vector>

#define CK(x)                                                                            \
    do {                                                                                 \
        hipError_t e_ = (x);                                                             \
        if (e_ != hipSuccess) {                                                          \
            printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); \
            exit(1);                                                                     \
        }                                                                                \
    } while (0)

typedef float f2 __attribute__((ext_vector_type(2)));

enum Op {
    kReadPlain,         // cached loads
    kReadAgent,         // device-scope loads
    kRmwPlain,          // cached load, plain store
    kRmwAgent,          // device-scope load, device-scope store
    kRmwGroup,          // workgroup-scope load and store (first-level cache bypassed, second level not)
    kAddAgent,          // device-scope fp32 atomic add, nothing read
    kAddGroup,          // workgroup-scope fp32 atomic add
    kReadAgentAddAgent, // device-scope load, then device-scope atomic add
    kReadPlainAddAgent, // cached load, then device-scope atomic add (same lines)
    kReadAgentNt,       // device-scope loads with the non-temporal hint
    kRmwAgentNt,        // device-scope load and store, both with the non-temporal hint
    kRmwAgentNtStore,   // device-scope load, device-scope store with the non-temporal hint
    kOps
};
static const char *kOpName[kOps] = {"read plain", "read device-scope", "rmw plain", "rmw device-scope", "rmw group-scope",
                                    "atomic add device-scope", "atomic add group-scope",
                                    "device-scope read + atomic add", "plain read + atomic add",
                                    "read device-scope, non-temporal", "rmw device-scope, non-temporal",
                                    "rmw device-scope, nt store only"};
static const double kOpBytes[kOps] = {512, 512, 1024, 1024, 1024, 512, 512, 1024, 1024, 512, 1024, 1024};

template <int kScope>
__device__ __forceinline__ f2 load_scoped(const float *p) {
    const uint64_t bits = __hip_atomic_load((const uint64_t *)p, __ATOMIC_RELAXED, kScope);
    f2 v = {__uint_as_float((uint32_t)bits), __uint_as_float((uint32_t)(bits >> 32))};
    return v;
}
template <int kScope>
__device__ __forceinline__ void store_scoped(float *p, f2 v) {
    const uint64_t bits = (uint64_t)__float_as_uint(v.x) | ((uint64_t)__float_as_uint(v.y) << 32);
    __hip_atomic_store((uint64_t *)p, bits, __ATOMIC_RELAXED, kScope);
}

// Device-scope accesses with the non-temporal hint (lines marked for early replacement in the caches): the
// compiler offers no such combination, so the instructions are written out.  A load written this way is
// invisible to the compiler's own wait counting: settle() waits for all of them and ties the registers to that
// wait, so that no use can be scheduled before it.
__device__ __forceinline__ uint64_t load_agent_nt(const float *p) {
    uint64_t bits;
    asm volatile("global_load_dwordx2 %0, %1, off sc1 nt" : "=v"(bits) : "v"(p) : "memory");
    return bits;
}
__device__ __forceinline__ void store_agent_nt(float *p, f2 v) {
    const uint64_t bits = (uint64_t)__float_as_uint(v.x) | ((uint64_t)__float_as_uint(v.y) << 32);
    asm volatile("global_store_dwordx2 %0, %1, off sc1 nt" : : "v"(p), "v"(bits) : "memory");
}
__device__ __forceinline__ void settle(uint64_t &a, uint64_t &b, uint64_t &c, uint64_t &d) {
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : : "memory");
}

// Batches of kBatch rows per wave: all loads of a batch are issued before the first update, as in the trainer.
template <int kOp, int kBatch>
__global__ __launch_bounds__(256) void k_rows(float *table, const uint32_t *ids, uint32_t count, float *sink) {
    const int lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane((blockIdx.x * 256 + threadIdx.x) >> 6);
    const uint32_t waves = gridDim.x * 4;
    float acc = 0.f;
    for (uint32_t i = wave * kBatch; i + kBatch <= count; i += waves * kBatch) {
        float *row[kBatch];
        f2 v[kBatch];
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            row[b] = table + (size_t)ids[i + b] * 128;
            if (kOp == kReadPlain || kOp == kRmwPlain || kOp == kReadPlainAddAgent) v[b] = *(const f2 *)(row[b] + lane * 2);
            if (kOp == kReadAgent || kOp == kRmwAgent || kOp == kReadAgentAddAgent)
                v[b] = load_scoped<__HIP_MEMORY_SCOPE_AGENT>(row[b] + lane * 2);
            if (kOp == kRmwGroup) v[b] = load_scoped<__HIP_MEMORY_SCOPE_WORKGROUP>(row[b] + lane * 2);
            if (kOp == kAddAgent || kOp == kAddGroup) v[b] = f2{0.f, 0.f};
            if (kOp == kRmwAgentNtStore) v[b] = load_scoped<__HIP_MEMORY_SCOPE_AGENT>(row[b] + lane * 2);
        }
        if (kOp == kReadAgentNt || kOp == kRmwAgentNt) {
            static_assert(kBatch == 4, "settle() takes four rows");
            uint64_t bits[kBatch];
#pragma unroll
            for (int b = 0; b < kBatch; ++b) bits[b] = load_agent_nt(row[b] + lane * 2);
            settle(bits[0], bits[1], bits[2], bits[3]);
#pragma unroll
            for (int b = 0; b < kBatch; ++b)
                v[b] = f2{__uint_as_float((uint32_t)bits[b]), __uint_as_float((uint32_t)(bits[b] >> 32))};
        }
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            acc += v[b].x + v[b].y;
            const f2 next = {v[b].x + 1.f, v[b].y + 1.f};
            if (kOp == kRmwPlain) *(f2 *)(row[b] + lane * 2) = next;
            if (kOp == kRmwAgent) store_scoped<__HIP_MEMORY_SCOPE_AGENT>(row[b] + lane * 2, next);
            if (kOp == kRmwGroup) store_scoped<__HIP_MEMORY_SCOPE_WORKGROUP>(row[b] + lane * 2, next);
            if (kOp == kRmwAgentNt || kOp == kRmwAgentNtStore) store_agent_nt(row[b] + lane * 2, next);
            if (kOp == kAddAgent || kOp == kReadAgentAddAgent || kOp == kReadPlainAddAgent) {
                (void)__hip_atomic_fetch_add(row[b] + lane, 1.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                (void)__hip_atomic_fetch_add(row[b] + 64 + lane, 1.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (kOp == kAddGroup) {
                (void)__hip_atomic_fetch_add(row[b] + lane, 1.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                (void)__hip_atomic_fetch_add(row[b] + 64 + lane, 1.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
    }
    if (acc == 12345.678f) sink[0] = acc;  // keeps the loads alive
}

template <int kOp>
static float time_op(float *table, const uint32_t *ids, uint32_t count, float *sink, int grid) {
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    float best = 1e30f;
    for (int rep = 0; rep < 3; ++rep) {
        CK(hipEventRecord(e0));
        hipLaunchKernelGGL((k_rows<kOp, 4>), dim3(grid), dim3(256), 0, 0, table, ids, count, sink);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        float ms;
        CK(hipEventElapsedTime(&ms, e0, e1));
        best = std::min(best, ms);
    }
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
    return best;
}

static float time_any(int op, float *table, const uint32_t *ids, uint32_t count, float *sink, int grid) {
    switch (op) {
        case kReadPlain: return time_op<kReadPlain>(table, ids, count, sink, grid);
        case kReadAgent: return time_op<kReadAgent>(table, ids, count, sink, grid);
        case kRmwPlain: return time_op<kRmwPlain>(table, ids, count, sink, grid);
        case kRmwAgent: return time_op<kRmwAgent>(table, ids, count, sink, grid);
        case kRmwGroup: return time_op<kRmwGroup>(table, ids, count, sink, grid);
        case kAddAgent: return time_op<kAddAgent>(table, ids, count, sink, grid);
        case kAddGroup: return time_op<kAddGroup>(table, ids, count, sink, grid);
        case kReadAgentAddAgent: return time_op<kReadAgentAddAgent>(table, ids, count, sink, grid);
        case kReadAgentNt: return time_op<kReadAgentNt>(table, ids, count, sink, grid);
        case kRmwAgentNt: return time_op<kRmwAgentNt>(table, ids, count, sink, grid);
        case kRmwAgentNtStore: return time_op<kRmwAgentNtStore>(table, ids, count, sink, grid);
        default: return time_op<kReadPlainAddAgent>(table, ids, count, sink, grid);
    }
}

// `count` row numbers below n with weights rank^-skew, ranks scattered over the rows
static std::vector<uint32_t> draw_rows(uint32_t n, uint32_t count, double skew, double *hottest_share) {
    std::mt19937_64 rng(42);
    std::vector<uint32_t> ids(count);
    if (skew == 0.0) {
        for (auto &x : ids) x = (uint32_t)(rng() % n);
        *hottest_share = 1.0 / n;
        return ids;
    }
    std::vector<double> cdf(n);
    double s = 0;
    for (uint32_t i = 0; i < n; ++i) cdf[i] = s += pow(i + 1.0, -skew);
    std::vector<uint32_t> perm(n);
    for (uint32_t i = 0; i < n; ++i) perm[i] = i;
    std::shuffle(perm.begin(), perm.end(), rng);
    std::uniform_real_distribution<double> U(0, s);
    for (auto &x : ids) x = perm[std::min<size_t>(n - 1, std::lower_bound(cdf.begin(), cdf.end(), U(rng)) - cdf.begin())];
    *hottest_share = 1.0 / s;
    return ids;
}

// every wave adds 1 to the 64 elements of one row `reps` times, then looks at the row
template <int kHow>
__global__ __launch_bounds__(64) void k_same_row(float *row, uint32_t reps, uint32_t *where) {
    const int lane = threadIdx.x;
    for (uint32_t i = 0; i < reps; ++i) {
        if (kHow == 0) row[lane] = row[lane] + 1.f;  // cached read-modify-write
        if (kHow == 1) {                               // device-scope read-modify-write
            const float v = __uint_as_float(__hip_atomic_load((uint32_t *)row + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            __hip_atomic_store((uint32_t *)row + lane, __float_as_uint(v + 1.f), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (kHow == 2) (void)__hip_atomic_fetch_add(row + lane, 1.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (kHow == 3) (void)__hip_atomic_fetch_add(row + lane, 1.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    if (lane == 0) {  // which of the chip's eight dies ran this workgroup (documented hardware register, read only)
        uint32_t id;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(id));
        where[blockIdx.x] = id & 0xFu;
    }
}

int main(int argc, char **argv) {
    const char *mode = argc > 1 ? argv[1] : "ops";
    const int grid = 2048;
    float *sink;
    CK(hipMalloc(&sink, 4));
    if (!strcmp(mode, "same")) {
        const int blocks = 2048;
        const uint32_t reps = 200;
        float *row;
        uint32_t *where;
        CK(hipMalloc(&row, 512));
        CK(hipMalloc(&where, blocks * 4));
        const char *names[4] = {"cached read-modify-write", "device-scope read-modify-write", "device-scope atomic add",
                                "group-scope atomic add"};
        std::vector<uint32_t> host_where(blocks);
        for (int how = 0; how < 4; ++how) {
            CK(hipMemset(row, 0, 512));
            CK(hipDeviceSynchronize());
            if (how == 0) hipLaunchKernelGGL(k_same_row<0>, dim3(blocks), dim3(64), 0, 0, row, reps, where);
            if (how == 1) hipLaunchKernelGGL(k_same_row<1>, dim3(blocks), dim3(64), 0, 0, row, reps, where);
            if (how == 2) hipLaunchKernelGGL(k_same_row<2>, dim3(blocks), dim3(64), 0, 0, row, reps, where);
            if (how == 3) hipLaunchKernelGGL(k_same_row<3>, dim3(blocks), dim3(64), 0, 0, row, reps, where);
            CK(hipDeviceSynchronize());
            float fin[64];
            CK(hipMemcpy(fin, row, 256, hipMemcpyDeviceToHost));
            printf("same row, %-32s expected %u, left in the row: %.0f (element 0) %.0f (element 63)\n", names[how],
                   blocks * reps, fin[0], fin[63]);
        }
        CK(hipMemcpy(host_where.data(), where, blocks * 4, hipMemcpyDeviceToHost));
        int round_robin = 1, per_die[16] = {0};
        for (int b = 0; b < blocks; ++b) {
            per_die[host_where[b] & 15] += 1;
            if (host_where[b] != (uint32_t)(b % 8)) round_robin = 0;
        }
        printf("workgroups per die:");
        for (int x = 0; x < 8; ++x) printf(" %d", per_die[x]);
        printf("; workgroup b ran on die b mod 8 for every b: %s\n", round_robin ? "yes" : "no");
        return 0;
    }
    if (!strcmp(mode, "sizes")) {
        const uint32_t count = 1u << 24;
        for (uint32_t mb : {16u, 64u, 128u, 192u, 256u, 512u, 1024u, 4096u}) {
            const uint32_t n = mb * 2048u;  // rows of 512 bytes
            double share;
            const std::vector<uint32_t> ids = draw_rows(n, count, 0.0, &share);
            float *table;
            uint32_t *dids;
            CK(hipMalloc(&table, (size_t)n * 512));
            CK(hipMemset(table, 0, (size_t)n * 512));
            CK(hipMalloc(&dids, (size_t)count * 4));
            CK(hipMemcpy(dids, ids.data(), (size_t)count * 4, hipMemcpyHostToDevice));
            for (int op : {(int)kReadAgent, (int)kRmwAgent, (int)kRmwPlain, (int)kRmwAgentNt}) {
                const float ms = time_any(op, table, dids, count, sink, grid);
                printf("table %5u MB  %-32s %.3f ms  %.3g rows/s  %.0f GB/s\n", mb, kOpName[op], ms, count / (ms * 1e-3),
                       count * kOpBytes[op] / (ms * 1e-3) / 1e9);
                fflush(stdout);
            }
            CK(hipFree(table));
            CK(hipFree(dids));
        }
        return 0;
    }
    // ops
    const uint32_t n = argc > 2 ? (uint32_t)atoi(argv[2]) : 2000000u;
    const double skew = argc > 3 ? atof(argv[3]) : 0.0;
    if (n < 1024u || n > 8000000u) {
        printf("rows must be in 1024 .. 8000000\n");
        return 1;
    }
    const uint32_t count = 1u << 24;
    double share;
    const std::vector<uint32_t> ids = draw_rows(n, count, skew, &share);
    float *table;
    uint32_t *dids;
    CK(hipMalloc(&table, (size_t)n * 512));
    CK(hipMemset(table, 0, (size_t)n * 512));
    CK(hipMalloc(&dids, (size_t)count * 4));
    CK(hipMemcpy(dids, ids.data(), (size_t)count * 4, hipMemcpyHostToDevice));
    printf("%u rows (%.0f MB), weights rank^-%.2f, hottest row %.4f %% of the accesses\n", n, n * 512.0 / 1e6, skew, 100.0 * share);
    for (int op = 0; op < kOps; ++op) {
        const float ms = time_any(op, table, dids, count, sink, grid);
        printf("  %-32s %8.3f ms  %.3g rows/s  %.0f GB/s\n", kOpName[op], ms, count / (ms * 1e-3),
               count * kOpBytes[op] / (ms * 1e-3) / 1e9);
        fflush(stdout);
    }
    return 0;
}
