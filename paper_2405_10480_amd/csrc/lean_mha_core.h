// LeanTile inner loop (Algorithm 1) for one query row per KV head (T_m = 1).
//
// QK^T with a single query row is a matrix-vector product at 1 flop per byte,
// far below the ridge of the vector ALUs, so it runs on VALU with DPP
// reductions; the matrix cores are not used here.
//
// Mapping.  A K or V row of D 16-bit elements is read by D/8 consecutive lanes,
// 16 bytes each, so one wave-wide global_load_dwordx4 covers 64/(D/8) whole
// rows = 1 KiB of contiguous cache.  Each group of D/8 lanes ("lane row") owns
// the tokens it loads and carries its own online-softmax state (m, l, O) over
// the span: per token, a 16-lane dot product reduced with DPP, then
// O += p * V on the 8 head-dim elements the lane holds.  The re-scaling
// operator of Section 4.1 is associative, so the lane rows of a wave, the waves
// of a workgroup and the workgroups of the grid are all merged with it.
//
// A workgroup step is one LeanTile of T_n = NW * U * 64/(D/8) tokens; wave w
// takes the w-th slice.  The default shapes use one register buffer per wave; the
// double-buffered shapes keep the next step's K and V in flight in a second one.
#pragma once
#include "lean_device.h"

namespace lean {

template <int DT, int D, int U, int NW, bool DB = true>
struct MhaCore {
    static constexpr int kD = D;
    static constexpr int kDT = DT;
    static constexpr int kLPR = D / 8;        // lanes per row
    static constexpr int kRPI = 64 / kLPR;    // rows per wave-wide load
    static constexpr int kCH = U * kRPI;      // tokens per wave per step
    static constexpr int kTn = NW * kCH;      // LeanTile
    static constexpr int kThreads = NW * 64;
    static constexpr int kTmMax = 1;
    static constexpr int kStreams = NW;       // partial streams left in LDS per segment
    static constexpr int kMinWavesPerSimd = 2;
    static_assert(D == 64 || D == 128 || D == 256, "head dim");

    struct alignas(16) Smem {
        float o[kStreams][kTmMax][D];
        float m[kStreams][kTmMax];
        float l[kStreams][kTmMax];
        __device__ const float* o_at(int stream, int row, int col) const { return &o[stream][row][col]; }
    };

    // Computes this workgroup's share of one output tile: LeanTile iterations
    // [sg.local_iter, sg.local_iter_end) of (sg.b, sg.h).  Leaves one un-scaled
    // partial (O~, m, l) per wave in `sm` (base-2 log domain) and ends with a barrier.
    __device__ static void run(const DecodeArgs& a, const Segment& sg, Smem& sm, int cta) {
        const int lane = threadIdx.x & 63;
        const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const int r = lane / kLPR;
        const int c = lane % kLPR;
        const int n_ctx = sg.n_ctx;

        const int64_t row0 = a.sched.packed
                                 ? (int64_t)sg.h * a.total_rows + a.table.cu_tok[sg.b]
                                 : ((int64_t)sg.b * a.Hkv + sg.h) * a.kv_seq_stride;
        constexpr uint32_t kRowBytes = D * 2;
        const uint32_t slab_bytes = (uint32_t)n_ctx * kRowBytes;
        const buffer_rsrc k_slab = make_slab(a.k + row0 * D, slab_bytes);
        const buffer_rsrc v_slab = make_slab(a.v + row0 * D, slab_bytes);
        const uint32_t lane_off = (uint32_t)(w * kCH + r) * kRowBytes + (uint32_t)c * 16u;
        const u32x4 q = *(reinterpret_cast<const u32x4*>(a.q + ((int64_t)sg.b * a.Hq + sg.h) * D) + c);

        float m_run = -INFINITY, l_run = 0.f;
        float o[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = 0.f;

        u32x4 kA[U], vA[U], kB[U], vB[U];

        // One wave-wide load per u: 64 lanes x 16 B = 1 KiB = kRPI whole rows.  `off` is the lane's
        // byte offset of the step in the slab (an offset past the slab loads zeros without any traffic).
        auto load_tile = [&](const buffer_rsrc& slab, u32x4(&x)[U], uint32_t off) {
#pragma unroll
            for (int u = 0; u < U; ++u) x[u] = slab_load16(slab, off + u * 1024u);
        };
        auto step_off = [&](int step) { return lane_off + (uint32_t)step * (kTn * kRowBytes); };

        // The lane's share of the U dot products q.k; frees the K registers.
        auto scores = [&](const u32x4(&kb)[U], float(&s)[U]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float acc = dot2<DT>(kb[u].x, q.x, 0.f);
                acc = dot2<DT>(kb[u].y, q.y, acc);
                acc = dot2<DT>(kb[u].z, q.z, acc);
                acc = dot2<DT>(kb[u].w, q.w, acc);
                s[u] = acc;
            }
        };

        // Row reduction of the scores, online softmax, O += p * V.
        auto attend = [&](float(&s)[U], const u32x4(&vb)[U], int step) {
            const int tok0 = step * kTn + w * kCH + r;
            float mx = -INFINITY;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                s[u] = group_allreduce_sum<kLPR>(s[u]) * a.scale_log2e;
                if (tok0 + u * kRPI >= n_ctx) s[u] = -INFINITY;  // masked tail tokens
                mx = fmaxf(mx, s[u]);
            }
            const float m_new = fmaxf(m_run, mx);
            const float m_ref = m_new == -INFINITY ? 0.f : m_new;  // no token seen yet
            const float alpha = fast_exp2(m_run - m_ref);
            float psum = 0.f;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                s[u] = fast_exp2(s[u] - m_ref);
                psum += s[u];
            }
            l_run = l_run * alpha + psum;
            m_run = m_new;
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] *= alpha;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float lo, hi;
                widen2<DT>(vb[u].x, lo, hi);
                o[0] = fmaf(s[u], lo, o[0]);
                o[1] = fmaf(s[u], hi, o[1]);
                widen2<DT>(vb[u].y, lo, hi);
                o[2] = fmaf(s[u], lo, o[2]);
                o[3] = fmaf(s[u], hi, o[3]);
                widen2<DT>(vb[u].z, lo, hi);
                o[4] = fmaf(s[u], lo, o[4]);
                o[5] = fmaf(s[u], hi, o[5]);
                widen2<DT>(vb[u].w, lo, hi);
                o[6] = fmaf(s[u], lo, o[6]);
                o[7] = fmaf(s[u], hi, o[7]);
            }
        };

        // The LeanTile iterations of the segment are visited in ascending order by every CTA.
        // (A CTA-specific rotated order was tried: it breaks the lockstep in which equally
        // aligned spans sweep memory, and on this machine that lockstep is faster.)
        const int it_first = sg.local_iter;
        const int n_it = sg.local_iter_end - sg.local_iter;
        // Loads past the segment are issued unconditionally (a branch around them would make every
        // later wait a wait for all loads) at an offset beyond the slab: zeros, no memory traffic.
        constexpr uint32_t kPastSlab = 0xF0000000u;
        auto off_at = [&](int k) { return k < n_it ? step_off(it_first + k) : kPastSlab; };
        float s[U];
        if constexpr (DB) {
            // Double-buffered walk: the loads of the next step stay in flight across the
            // arithmetic of this one.
            int k = 0;
            load_tile(k_slab, kA, off_at(0));
            load_tile(v_slab, vA, off_at(0));
            while (k < n_it) {
                load_tile(k_slab, kB, off_at(k + 1));
                load_tile(v_slab, vB, off_at(k + 1));
                scores(kA, s);
                attend(s, vA, it_first + k);
                if (a.cta_clock && k == 0 && threadIdx.x == 0) a.cta_clock[kClockWords * cta + kClkFirstStep] = wall_clock64();
                load_tile(k_slab, kA, off_at(k + 2));
                load_tile(v_slab, vA, off_at(k + 2));
                if (k + 1 < n_it) {
                    scores(kB, s);
                    attend(s, vB, it_first + k + 1);
                }
                k += 2;
            }
        } else {
            // One register buffer: a wave issues one step's loads, consumes them, then issues the
            // next; the other waves of the compute unit cover its memory latency.  (Issuing the
            // next K loads right after the dot products was tried: 2 % slower, the memory system
            // likes about 8 KiB in flight per wave best.)
            for (int k = 0; k < n_it; ++k) {
                load_tile(k_slab, kA, off_at(k));
                load_tile(v_slab, vA, off_at(k));
                scores(kA, s);
                attend(s, vA, it_first + k);
                if (a.cta_clock && k == 0 && threadIdx.x == 0) a.cta_clock[kClockWords * cta + kClkFirstStep] = wall_clock64();
            }
        }

        // Merge the lane rows of the wave with the re-scaling operator (butterfly).
#pragma unroll
        for (int off = kLPR; off < 64; off <<= 1) {
            const float m_o = xor_shuffle(m_run, off);
            const float l_o = xor_shuffle(l_run, off);
            const float m_new = fmaxf(m_run, m_o);
            const float m_ref = m_new == -INFINITY ? 0.f : m_new;
            const float w_self = fast_exp2(m_run - m_ref);
            const float w_peer = fast_exp2(m_o - m_ref);
            l_run = w_self * l_run + w_peer * l_o;
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = w_self * o[j] + w_peer * xor_shuffle(o[j], off);
            m_run = m_new;
        }
        if (lane < kLPR) {
#pragma unroll
            for (int j = 0; j < 8; ++j) sm.o[w][0][c * 8 + j] = o[j];
            if (lane == 0) {
                sm.m[w][0] = m_run;
                sm.l[w][0] = l_run;
            }
        }
        __syncthreads();
    }
};

}  // namespace lean
