// Grouping of a sample pool for stationary-row training: every sample is assigned the
// side whose row is hotter (higher degree) and samples are sorted, inside tiles of the
// pool, by (side, row), so that samples sharing their hot row become adjacent.
#include <stdlib.h>
#include <string.h>

#include <algorithm>

#include <rocprim/device/device_radix_sort.hpp>

#include "gv_internal.hpp"

namespace gv {
namespace {

constexpr int kBlock = 256;

// key = tile index | side | stationary row, value = position | side << 31
__global__ __launch_bounds__(kBlock) void k_group_keys(const uint2 *__restrict__ pairs, uint32_t count, uint32_t n,
                                                       const uint32_t *__restrict__ degree, uint32_t tile_shift,
                                                       uint32_t id_bits, uint32_t *__restrict__ keys,
                                                       uint32_t *__restrict__ values) {
    for (uint32_t i = blockIdx.x * kBlock + threadIdx.x; i < count; i += gridDim.x * kBlock) {
        const uint2 p = pairs[i];
        uint32_t side = 0, row = 0;
        if (p.x < n && p.y < n) {  // samples with bad ids keep key 0; the trainer reports them
            side = degree[p.x] < degree[p.y] ? 1u : 0u;
            row = side ? p.y : p.x;
        }
        const uint32_t tile = i >> tile_shift;
        keys[i] = (tile << (id_bits + 1)) | (side << id_bits) | row;
        values[i] = i | (side << 31);
    }
}

uint32_t bits_for(uint64_t values) {  // smallest b with 2^b >= values
    uint32_t b = 0;
    while ((1ull << b) < values) ++b;
    return b;
}

}  // namespace

GroupPlan plan_grouping(uint64_t count, uint32_t n) {
    GroupPlan plan{};
    if (count == 0 || count >= (1ull << 31) || n > (1u << 31)) return plan;  // not groupable: caller falls back
    const uint32_t id_bits = bits_for(n);
    // tile: a power of two, at most 2^20 samples and at most 4 samples per node.  Inside a
    // tile the samples are applied in row order instead of pool order; keeping the tile
    // small against the graph keeps that reordering local (a handful of samples per row).
    uint32_t tile_shift = 20;
    while (tile_shift > 12 && (1ull << tile_shift) > 4ull * n) --tile_shift;
    if (const char *e = getenv("GV_TILE_SHIFT")) {  // tuning sweeps
        const long v = strtol(e, nullptr, 10);
        if (v >= 6 && v <= 30) tile_shift = (uint32_t)v;
    }
    uint32_t tile_bits = bits_for((count + (1ull << tile_shift) - 1) >> tile_shift);
    while (id_bits + 1 + tile_bits > 32) {  // keys are 32 bits: fewer, larger tiles
        ++tile_shift;
        tile_bits = bits_for((count + (1ull << tile_shift) - 1) >> tile_shift);
    }
    plan.valid = true;
    plan.tile_shift = tile_shift;
    plan.id_bits = id_bits;
    plan.key_bits = id_bits + 1 + tile_bits;
    return plan;
}

hipError_t group_scratch_bytes(uint64_t count, size_t *sort_bytes) {
    size_t bytes = 0;
    uint32_t *none = nullptr;
    hipError_t e = rocprim::radix_sort_pairs(nullptr, bytes, none, none, none, none, (size_t)count, 0u, 32u, nullptr);
    *sort_bytes = bytes;
    return e;
}

hipError_t launch_group(const GroupPlan &plan, const uint32_t *pairs, uint64_t count, uint32_t n,
                        const uint32_t *degree, uint32_t *keys_in, uint32_t *values_in, uint32_t *keys_out,
                        uint32_t *values_out, void *sort_scratch, size_t sort_bytes, hipStream_t stream) {
    const uint32_t blocks = (uint32_t)std::min<uint64_t>((count + kBlock - 1) / kBlock, 8192);
    hipLaunchKernelGGL(k_group_keys, dim3(blocks), dim3(kBlock), 0, stream, (const uint2 *)pairs, (uint32_t)count, n,
                       degree, plan.tile_shift, plan.id_bits, keys_in, values_in);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return rocprim::radix_sort_pairs(sort_scratch, sort_bytes, keys_in, keys_out, values_in, values_out,
                                     (size_t)count, 0u, plan.key_bits, stream);
}

}  // namespace gv
