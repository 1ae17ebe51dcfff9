// Small kernels beside the decode kernel: workspace clearing, zero rows for all-empty batches,
// and the streaming-read probes the benchmark uses as the machine's ceiling.  Included by the
// host translation unit only.
#pragma once
#include "lean_device.h"

namespace lean {

// Clears flags and status of a fresh workspace (a fill kernel: safe under graph capture).
__global__ void lean_workspace_clear_kernel(uint32_t* words, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) words[i] = 0u;
}

// All sequences empty: only zeros to write.
__global__ void lean_zero_rows_kernel(uint32_t* out_words, float* lse, int64_t rows, int row_words) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < rows * row_words) out_words[i] = 0u;
    if (lse && i < rows) lse[i] = -INFINITY;
}

// Streaming-read probe: 16-byte loads, 8 in flight per lane, folded into one word so the
// loads cannot be dropped.  mode 0: workgroup g reads the g-th contiguous share of the
// buffer (the access pattern of contiguous stream-K spans); mode 1: the workgroups sweep
// the buffer together, 32 KiB chunks dealt round-robin (grid-stride); modes 2..4: as mode 0
// through a buffer descriptor with cache policy nt, sc1, sc0|sc1 on the loads.
template <int AUX>
__device__ __forceinline__ uint32_t probe_slab(const uint4* buf, int64_t lo, int64_t hi) {
    uint32_t acc = 0;
    const int64_t span = hi - lo;  // 16-byte units, < 2^27 per workgroup
    const buffer_rsrc r = make_slab((const uint16_t*)(buf + lo), (uint32_t)(span * 16));
    for (int64_t i = threadIdx.x; i + 7 * 256 < span; i += 8 * 256) {
        u32x4 x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = __builtin_amdgcn_raw_buffer_load_b128(r, (int)((i + u * 256) * 16), 0, AUX);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= x[u].x ^ x[u].y ^ x[u].z ^ x[u].w;
    }
    return acc;
}

// mode 5: the K access pattern of the MFMA core: per wave-wide load, lane (r = lane%16,
// g = lane/16) reads 16 bytes of row r at byte 64*c + 16*g of a 256-byte row (non-temporal).
__device__ __forceinline__ uint32_t probe_rowstrided(const uint4* buf, int64_t lo, int64_t hi) {
    uint32_t acc = 0;
    const int64_t span = hi - lo;
    const buffer_rsrc r = make_slab((const uint16_t*)(buf + lo), (uint32_t)(span * 16));
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const uint32_t lane_off = (uint32_t)(lane & 15) * 256u + (uint32_t)(lane >> 4) * 16u;
    // a workgroup step = 4 waves x 2 blocks of 16 rows x 256 B = 32 KiB
    for (int64_t i = 0; (i + 1) * 2048 <= span; ++i) {
        const uint32_t base = (uint32_t)(i * 32768) + (uint32_t)w * 8192u + lane_off;
        u32x4 x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            x[u] = __builtin_amdgcn_raw_buffer_load_b128(r, (int)(base + (u >> 2) * 4096u + (u & 3) * 64u), 0, 2);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= x[u].x ^ x[u].y ^ x[u].z ^ x[u].w;
    }
    return acc;
}

// mode 6: the K/V access pattern of the MFMA core at D = 256: per wave-wide load, lane (r, g)
// reads 16 bytes at byte 16*r of one half (256 bytes) of row g of a 4-row group; the two halves
// of the rows come from consecutive load instructions (non-temporal).
__device__ __forceinline__ uint32_t probe_halfrows(const uint4* buf, int64_t lo, int64_t hi) {
    uint32_t acc = 0;
    const int64_t span = hi - lo;
    const buffer_rsrc r = make_slab((const uint16_t*)(buf + lo), (uint32_t)(span * 16));
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const uint32_t lane_off = (uint32_t)(lane >> 4) * 512u + (uint32_t)(lane & 15) * 16u;
    // a workgroup step = 4 waves x 16 rows x 512 B = 32 KiB
    for (int64_t i = 0; (i + 1) * 2048 <= span; ++i) {
        const uint32_t base = (uint32_t)(i * 32768) + (uint32_t)w * 8192u + lane_off;
        u32x4 x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            x[u] = __builtin_amdgcn_raw_buffer_load_b128(r, (int)(base + (u >> 1) * 2048u + (u & 1) * 256u), 0, 2);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= x[u].x ^ x[u].y ^ x[u].z ^ x[u].w;
    }
    return acc;
}

__global__ __launch_bounds__(256) void lean_read_probe_kernel(const uint4* buf, int64_t n_vec, uint32_t* sink,
                                                              int mode) {
    const int G = gridDim.x;
    uint32_t acc = 0;
    int64_t lo, hi, step;
    if (mode != 1) {
        const int64_t per = (n_vec + G - 1) / G;
        lo = (int64_t)blockIdx.x * per;
        hi = lo + per < n_vec ? lo + per : n_vec;
        step = 8 * 256;
    } else {
        lo = (int64_t)blockIdx.x * (8 * 256);
        hi = n_vec;
        step = (int64_t)G * (8 * 256);
    }
    if (mode >= 2) {
        if (lo < hi)
            acc = mode == 2 ? probe_slab<2>(buf, lo, hi) : mode == 3 ? probe_slab<16>(buf, lo, hi)
                  : mode == 4 ? probe_slab<17>(buf, lo, hi)
                  : mode == 5 ? probe_rowstrided(buf, lo, hi) : probe_halfrows(buf, lo, hi);
    } else {
        int64_t i = lo + threadIdx.x;
        for (; i + 7 * 256 < hi; i += step) {
            uint4 x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = buf[i + u * 256];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc ^= x[u].x ^ x[u].y ^ x[u].z ^ x[u].w;
        }
        if (mode == 0 || i < hi) {  // ragged end: at most one partial chunk per workgroup
            for (; i < hi; i += 256) {
                const uint4 x = buf[i];
                acc ^= x.x ^ x.y ^ x.z ^ x.w;
            }
        }
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;  // practically never true: keeps the loads alive
}

}  // namespace lean
