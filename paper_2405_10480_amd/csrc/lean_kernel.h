// The persistent LeanAttention kernel: Algorithm 2, one workgroup per CTA of
// the paper.  Each workgroup walks its span of LeanTile iterations; for every
// output tile the span touches it runs the core (Algorithm 1) and then either
// publishes its un-scaled partial and signals (non-host block), or merges the
// peers' partials with the softmax re-scaling operator of Section 4.1 and
// writes the normalised output (host block).  Computation and reduction share
// one launch, as in Section 4.3.
#pragma once
#include "lean_device.h"

namespace lean {

template <class Core>
__global__ __launch_bounds__(Core::kThreads, Core::kMinWavesPerSimd) void lean_decode_kernel(const DecodeArgs a) {
    constexpr int D = Core::kD;
    constexpr int THREADS = Core::kThreads;
    constexpr int EPT = (Core::kTmMax * D + THREADS - 1) / THREADS;  // output elements per thread

    __shared__ typename Core::Smem sm;

    // CTA id.  The hardware deals consecutive workgroup ids round-robin to the
    // 8 XCDs; the optional remap makes the spans of one XCD contiguous so that
    // the partials a host block merges mostly come from its own L2.
    int g = blockIdx.x;
    const int G = a.sched.grid;
    if (a.xcd_remap && (G & 7) == 0) g = (g & 7) * (G >> 3) + (g >> 3);

    const int tid = threadIdx.x;
    const int T_m = a.T_m;
    const int n_elem = T_m * D;

    if (a.has_empty) {  // sequences with N_b = 0 own no iteration: their rows are defined as zero
        for (int row = g; row < a.sched.B * a.Hq; row += G) {
            const int b = row / a.Hq;
            if (a.table.cu_tok[b + 1] == a.table.cu_tok[b]) {
                for (int c = tid; c < D; c += THREADS) a.out[(int64_t)row * D + c] = 0.f;
                if (a.lse && tid == 0) a.lse[row] = -INFINITY;
            }
        }
    }

    int64_t cta_start, cta_end;
    span_of(a.sched, g, &cta_start, &cta_end);

    int64_t it = cta_start;
    while (it < cta_end) {
        const Segment sg = locate(a.sched, a.table, it, cta_end);
        Core::run(a, sg, sm);  // ends with a workgroup barrier

        // Host block that does not finish its tile: Wait(flags[cta]) for every peer
        // g+1 .. last_cta before touching their partials.
        const bool reduce_peers = sg.host && !sg.finishing;
        if (reduce_peers) {
            for (int cta = g + 1; cta <= sg.last_cta; ++cta) wait_arrival(a.flags + cta, a.status, a.spin_limit);
        }

        // Thread `tid` owns elements e = tid + i*THREADS of the [T_m, D] tile, one at a time:
        // fold the per-wave streams, then either publish the partial or merge the peers'
        // partials in ascending CTA order and write the normalised output.
        float* own_slot = a.partials + (int64_t)g * a.slot;
        const int64_t out_row0 = (int64_t)sg.b * a.Hq + (int64_t)sg.h * T_m;
#pragma unroll 1
        for (int i = 0; i < EPT; ++i) {
            const int e = tid + i * THREADS;
            if (e >= n_elem) break;
            const int row = e / D, col = e % D;
            float m = -INFINITY;
#pragma unroll
            for (int p = 0; p < Core::kStreams; ++p) m = fmaxf(m, sm.m[p][row]);
            const float m_fold = m == -INFINITY ? 0.f : m;
            float l = 0.f, o = 0.f;
#pragma unroll
            for (int p = 0; p < Core::kStreams; ++p) {
                const float wgt = fast_exp2(sm.m[p][row] - m_fold);
                l += wgt * sm.l[p][row];
                o += wgt * sm.o[p][row][col];
            }
            if (!sg.host) {
                // StorePartials(Op[g], mp[g], lp[g])
                own_slot[e] = o;
                if (col == 0) {
                    own_slot[n_elem + row] = m;
                    own_slot[n_elem + T_m + row] = l;
                }
            } else {
                if (reduce_peers) {
                    for (int cta = g + 1; cta <= sg.last_cta; ++cta) {
                        const float* slot = a.partials + (int64_t)cta * a.slot;
                        const float m_cta = slot[n_elem + row];
                        const float l_cta = slot[n_elem + T_m + row];
                        const float o_cta = slot[e];
                        const float m_new = fmaxf(m_cta, m);
                        const float m_ref = m_new == -INFINITY ? 0.f : m_new;
                        const float w_cta = fast_exp2(m_cta - m_ref);
                        const float w_own = fast_exp2(m - m_ref);
                        l = w_cta * l_cta + w_own * l;
                        o = w_cta * o_cta + w_own * o;
                        m = m_new;
                    }
                }
                // O = diag(l)^-1 O~ ;  L = m + log(l)  (m is kept in the base-2 domain)
                a.out[out_row0 * D + e] = o / l;
                if (a.lse && col == 0)
                    a.lse[out_row0 + row] = 0.6931471805599453f * (m + __builtin_amdgcn_logf(l));
            }
        }
        if (!sg.host) signal_arrival(a.flags + g);  // Signal(flags[g])
        it = sg.tile_iter_end;
        __syncthreads();  // the cores reuse the shared partial streams
    }
}

// Clears flags and status of a fresh workspace (a fill kernel: safe under graph capture).
__global__ void lean_workspace_clear_kernel(uint32_t* words, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) words[i] = 0u;
}

// All sequences empty: only zeros to write.
__global__ void lean_zero_rows_kernel(float* out, float* lse, int64_t rows, int D) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < rows * D) out[i] = 0.f;
    if (lse && i < rows) lse[i] = -INFINITY;
}

// Streaming-read probe: workgroup g reads the g-th contiguous share of the
// buffer with 16-byte loads, several in flight per lane, and folds them into
// one word so the loads cannot be dropped.
__global__ __launch_bounds__(256) void lean_read_probe_kernel(const uint4* buf, int64_t n_vec, uint32_t* sink) {
    const int G = gridDim.x;
    const int64_t per = (n_vec + G - 1) / G;
    const int64_t lo = (int64_t)blockIdx.x * per;
    int64_t hi = lo + per;
    if (hi > n_vec) hi = n_vec;
    uint32_t acc = 0;
    int64_t i = lo + threadIdx.x;
    for (; i + 7 * 256 < hi; i += 8 * 256) {
        uint4 x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = buf[i + u * 256];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= x[u].x ^ x[u].y ^ x[u].z ^ x[u].w;
    }
    for (; i < hi; i += 256) {
        const uint4 x = buf[i];
        acc ^= x.x ^ x.y ^ x.z ^ x.w;
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;  // practically never true: keeps the loads alive
}

}  // namespace lean
