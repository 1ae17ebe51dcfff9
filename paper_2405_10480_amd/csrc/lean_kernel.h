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

// One partial (O~, m, l) as the workgroup holds it in registers: thread `tid`
// owns the float4 chunks c = tid + i*THREADS of the [T_m, D] tile (row = 4c / D).
template <int CPT>
struct OwnPartial {
    f32x4 o[CPT];
    float m[CPT];
    float l[CPT];
};

// Merge up to F-1 published partials (CTAs first, first+step, ...) into `own` with the
// re-scaling operator of Section 4.1, in ascending CTA order.  All loads of a batch are
// issued before the first use, so one memory round trip covers the whole batch.
template <int CPT, int THREADS, int D, int F>
__device__ __forceinline__ void merge_children(const DecodeArgs& a, OwnPartial<CPT>& own, int first, int step,
                                               int nchild, int n_chunks, int n_elem, int T_m) {
    const int tid = threadIdx.x;
    const buffer_rsrc ws = make_slab((const uint16_t*)a.partials, (uint32_t)a.sched.grid * (uint32_t)a.slot * 4u);
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        const int c = tid + i * THREADS;
        if (c < n_chunks) {  // (no early exit: the loop must unroll so that `own` stays in registers)
            const int row = (4 * c) / D;
            f32x4 oc[F - 1];
            float mc[F - 1], lc[F - 1];
#pragma unroll
            for (int j = 0; j < F - 1; ++j) {
                const int jj = j < nchild ? j : nchild - 1;  // past the last child: re-read it, weight it zero
                const uint32_t slot = (uint32_t)(first + jj * step) * (uint32_t)a.slot * 4u;
                oc[j] = partial_load16(ws, slot + 16u * c);
                mc[j] = partial_load4(ws, slot + 4u * (n_elem + row));
                lc[j] = partial_load4(ws, slot + 4u * (n_elem + T_m + row));
            }
#pragma unroll
            for (int j = 0; j < F - 1; ++j) {
                const float m_cta = j < nchild ? mc[j] : -INFINITY;
                const float m_new = fmaxf(m_cta, own.m[i]);
                const float m_ref = m_new == -INFINITY ? 0.f : m_new;
                const float w_cta = fast_exp2(m_cta - m_ref);
                const float w_own = fast_exp2(own.m[i] - m_ref);
                own.l[i] = w_cta * lc[j] + w_own * own.l[i];
                own.o[i] = w_cta * oc[j] + w_own * own.o[i];
                own.m[i] = m_new;
            }
        }
    }
}

// The same for single-row tiles (T_m = 1: D/4 chunks, far fewer than threads), as wide as the
// workgroup: thread (slot, chunk) merges children slot, slot + SLOTS, ... of its chunk, four
// loads in flight each, the SLOTS partial results meet in LDS and the owners of `own` fold
// them in slot order.  Up to 4*SLOTS children cost one memory round trip instead of one per
// seven, which lets small problems reduce in a single tree level.  The order is fixed, so the
// result stays reproducible bit for bit.
template <int THREADS>
struct WideMergeScratch {
    f32x4 o[THREADS];
    float m[THREADS];
    float l[THREADS];
};

template <int THREADS, int D>
__device__ __forceinline__ void merge_children_wide(const DecodeArgs& a, OwnPartial<1>& own, int first, int step,
                                                    int nchild, WideMergeScratch<THREADS>& sh) {
    constexpr int NCH = D / 4;
    constexpr int SLOTS = THREADS / NCH;
    static_assert(SLOTS >= 2 && SLOTS * NCH == THREADS, "single-row tiles are much smaller than the workgroup");
    const int tid = threadIdx.x;
    const int slot = tid / NCH, c = tid % NCH;
    const buffer_rsrc ws = make_slab((const uint16_t*)a.partials, (uint32_t)a.sched.grid * (uint32_t)a.slot * 4u);
    f32x4 o = {0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f;
    for (int j0 = slot; j0 < nchild; j0 += 4 * SLOTS) {
        f32x4 oc[4];
        float mc[4], lc[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int j = j0 + u * SLOTS;
            const int jj = j < nchild ? j : j0;  // past the last child: re-read a valid one, weight it zero
            const uint32_t base = (uint32_t)(first + jj * step) * (uint32_t)a.slot * 4u;
            oc[u] = partial_load16(ws, base + 16u * c);
            mc[u] = partial_load4(ws, base + 4u * D);
            lc[u] = partial_load4(ws, base + 4u * (D + 1));
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float m_cta = j0 + u * SLOTS < nchild ? mc[u] : -INFINITY;
            const float m_new = fmaxf(m_cta, m);
            const float m_ref = m_new == -INFINITY ? 0.f : m_new;
            const float w_cta = fast_exp2(m_cta - m_ref);
            const float w_acc = fast_exp2(m - m_ref);
            l = w_cta * lc[u] + w_acc * l;
            o = w_cta * oc[u] + w_acc * o;
            m = m_new;
        }
    }
    sh.o[tid] = o;
    sh.m[tid] = m;
    sh.l[tid] = l;
    __syncthreads();
    if (tid < NCH) {
#pragma unroll
        for (int sl = 0; sl < SLOTS; ++sl) {
            const float m_s = sh.m[sl * NCH + tid];
            const float m_new = fmaxf(m_s, own.m[0]);
            const float m_ref = m_new == -INFINITY ? 0.f : m_new;
            const float w_s = fast_exp2(m_s - m_ref);
            const float w_own = fast_exp2(own.m[0] - m_ref);
            own.l[0] = w_s * sh.l[sl * NCH + tid] + w_own * own.l[0];
            own.o[0] = w_s * sh.o[sl * NCH + tid] + w_own * own.o[0];
            own.m[0] = m_new;
        }
    }
    __syncthreads();  // the scratch is reused by the next batch
}

// Reduction of one output tile across the CTAs that computed parts of it, then either the
// publication of this CTA's (merged) partial or the final write.
//
// Ranks count from the tile's END: rank 0 is the finishing block (the CTA whose span holds
// the tile's last LeanTile), the block that computed the tile's first LeanTile has the
// highest rank.  Because the re-scaling operator is associative the blocks form a tree of
// fan-in `fanin` instead of Algorithm 2's flat list: rank k merges ranks k + j*stride
// (j < fanin) while k is a multiple of stride*fanin, then publishes once; rank 0 merges
// last and writes O = diag(l)^-1 O~ and L = m + log(l).  A block therefore only ever waits
// for LOWER CTA ids, i.e. for workgroups the hardware dispatched before it, so every wait
// ends even when the grid is larger than what is resident at once.
// Threads of the LDS scratch of merge_children_wide: the workgroup for single-row cores, else a stub.
template <class Core>
constexpr int kWideThreads = Core::kTmMax == 1 ? Core::kThreads : 1;

template <class Core, int CPT, int F>
__device__ __forceinline__ void reduce_tile(const DecodeArgs& a, OwnPartial<CPT>& own, int g, int b, int h,
                                            int first_cta, int last_cta,
                                            WideMergeScratch<kWideThreads<Core>>& wide_scratch) {
    constexpr int D = Core::kD;
    constexpr int THREADS = Core::kThreads;
    const int tid = threadIdx.x;
    const int T_m = a.T_m;
    const int n_elem = T_m * D;
    const int n_chunks = n_elem / 4;
    const int rank = last_cta - g;
    const int nranks = last_cta - first_cta + 1;
    bool publish = false;
    for (int64_t stride = 1; stride < nranks; stride *= a.fanin) {
        if (rank % (stride * a.fanin) != 0) {
            publish = true;
            break;
        }
        int remaining = (int)((nranks - 1 - rank) / stride);  // children at this level
        if (remaining > a.fanin - 1) remaining = a.fanin - 1;
        int child = g - (int)stride;
        if constexpr (Core::kTmMax == 1) {
            // single-row tiles: batches as wide as four children per slot of the workgroup
            constexpr int kWide = 4 * (THREADS / (D / 4));
            while (remaining > 0) {
                const int batch = remaining < kWide ? remaining : kWide;
                wait_arrivals(a, child, -(int)stride, batch);
                stamp(a, g, kClkFlagsSeen);
                merge_children_wide<THREADS, D>(a, own, child, -(int)stride, batch, wide_scratch);
                child -= batch * (int)stride;
                remaining -= batch;
            }
        } else {
            while (remaining > 0) {  // batches of at most F-1 partials
                const int batch = remaining < F - 1 ? remaining : F - 1;
                wait_arrivals(a, child, -(int)stride, batch);
                stamp(a, g, kClkFlagsSeen);
                merge_children<CPT, THREADS, D, F>(a, own, child, -(int)stride, batch, n_chunks, n_elem, T_m);
                child -= batch * (int)stride;
                remaining -= batch;
            }
        }
        stamp(a, g, kClkMerged);
    }
    if (publish) {
        // StorePartials(Op[g], mp[g], lp[g]); Signal(flags[g])
        if (a.delay_store && debug_delayed(a, g)) debug_sleep(a.delay_store);
        const buffer_rsrc ws = make_slab((const uint16_t*)a.partials, (uint32_t)a.sched.grid * (uint32_t)a.slot * 4u);
        const uint32_t slot = (uint32_t)g * (uint32_t)a.slot * 4u;
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const int c = tid + i * THREADS;
            if (c < n_chunks) {
                partial_store16(ws, slot + 16u * c, own.o[i]);
                if ((4 * c) % D == 0) {
                    partial_store4(ws, slot + 4u * (n_elem + (4 * c) / D), own.m[i]);
                    partial_store4(ws, slot + 4u * (n_elem + T_m + (4 * c) / D), own.l[i]);
                }
            }
        }
        stamp(a, g, kClkStoresIssued);
        signal_arrival(a, g);
        stamp(a, g, kClkStoresAcked);
    } else {
        // m is kept in the base-2 domain: L = ln2 * (m + log2 l)
        const TileRows tr = tile_rows(a, b, h);
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const int c = tid + i * THREADS;
            const int row = (4 * c) / D, col = (4 * c) % D;
            if (c < n_chunks && row < tr.count) {
                int token;
                const int64_t orow = query_row(a, tr, tr.rho0 + row, &token);
                const f32x4 o = own.o[i] * (1.f / own.l[i]);
                if (a.out16) {
                    *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(a.out) + orow * D + col) =
                        u32x2{narrow2<Core::kDT>(o.x, o.y), narrow2<Core::kDT>(o.z, o.w)};
                } else {
                    *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(a.out) + orow * D + col) = o;
                }
                if (a.lse && col == 0)
                    a.lse[orow] = 0.6931471805599453f * (own.m[i] + __builtin_amdgcn_logf(own.l[i]));
            }
        }
        stamp(a, g, kClkWritten);
    }
}

template <class Core>
__device__ __forceinline__ void lean_decode_body(const DecodeArgs& a) {
    constexpr int D = Core::kD;
    constexpr int THREADS = Core::kThreads;
    constexpr int CPT = (Core::kTmMax * D / 4 + THREADS - 1) / THREADS;  // float4 chunks per thread
    constexpr int F = 8;                                                 // widest merge batch + 1

    __shared__ typename Core::Smem sm;
    // A finishing block whose span goes on to other tiles parks its partial here and
    // reduces at the end of its span, when its peers are done too (thread-private entries).
    __shared__ f32x4 parked_o[CPT * THREADS];
    __shared__ float parked_m[CPT * THREADS];
    __shared__ float parked_l[CPT * THREADS];
    __shared__ WideMergeScratch<kWideThreads<Core>> wide_scratch;  // (a 24-byte stub for the MFMA cores)

    // Touch every cache line of the argument block now, in one batch: left to itself the compiler
    // loads each field right before its first use, and the span walk below becomes a chain of
    // dependent misses to the argument segment (measured: 1.5-1.8 us before the first K/V load
    // is issued).  One field per 64-byte line is enough (later reads hit the scalar cache) and
    // keeps the scalar registers free; the first entries of the prefix tables are touched too,
    // so that the table look-ups of small batches hit as well.
    static_assert(offsetof(DecodeArgs, q) < 64 && offsetof(DecodeArgs, kv_seq_stride) / 64 == 1 &&
                      offsetof(DecodeArgs, has_empty) / 64 == 2 && offsetof(DecodeArgs, sched.grid) / 64 == 2 &&
                      offsetof(DecodeArgs, sched.iters_per_cta) / 64 == 3 && offsetof(DecodeArgs, sched.by_cn) / 64 == 3 &&
                      offsetof(DecodeArgs, table.cu_iters[1]) / 64 == 4,
                  "one touched field per line of the argument block");
    asm volatile("" ::"s"(a.q), "s"(a.kv_seq_stride), "s"(a.has_empty), "s"(a.sched.iters_per_cta),
                 "s"(a.table.cu_iters[1]), "s"(a.table.cu_tok[1]));

    // CTA id = workgroup id: the hardware dispatches workgroups in id order, and a workgroup only
    // ever waits for lower ids (reduce_tile), so every wait ends however few workgroups are
    // resident at once.  (Mapping span ids so that consecutive spans share an XCD was tried: no
    // gain in streaming rate, and a workgroup may then wait for one dispatched after it.)
    const int g = blockIdx.x;
    const int G = a.sched.grid;

    const int tid = threadIdx.x;
    const int T_m = a.T_m;
    const int n_chunks = T_m * D / 4;
    stamp(a, g, kClkEntry);

    if (a.has_empty) {  // sequences with N_b = 0 own no iteration: their rows are defined as zero
        const int row_words = a.out16 ? D / 2 : D;  // zero bits are 0.0 in every output type
        for (int b = 0; b < a.sched.B; ++b) {
            if (a.table.cu_tok[b + 1] != a.table.cu_tok[b]) continue;
            const int64_t first = (a.ragged_q ? (int64_t)a.table.cu_q[b] : (int64_t)b * a.N_q) * a.Hq;
            const int64_t last = (a.ragged_q ? (int64_t)a.table.cu_q[b + 1] : (int64_t)(b + 1) * a.N_q) * a.Hq;
            for (int64_t row = first + g; row < last; row += G) {
                for (int c = tid; c < row_words; c += THREADS)
                    reinterpret_cast<uint32_t*>(a.out)[row * row_words + c] = 0u;
                if (a.lse && tid == 0) a.lse[row] = -INFINITY;
            }
        }
    }

    int64_t cta_start, cta_end;
    span_of(a.sched, a.table, g, &cta_start, &cta_end);

    bool parked = false;
    int parked_b = 0, parked_h = 0, parked_first = 0;

    int64_t it = cta_start;
    Segment sg;
    while (it < cta_end) {
        sg = it == cta_start ? locate(a.sched, a.table, it, cta_end) : locate_next(a.sched, a.table, sg, g, cta_end);
        if (it == cta_start) stamp(a, g, kClkLocated);
        if (a.ragged_q && tile_rows(a, sg.b, sg.h).count <= 0) {
            // a sequence with fewer query tokens than the longest: this row block holds no rows.
            // Every CTA of the tile sees the same count, so none computes, publishes or waits.
            it = sg.tile_iter_end;
            continue;
        }
        Core::run(a, sg, sm, g);  // ends with a workgroup barrier
        if (it == cta_start) stamp(a, g, kClkCoreDone);

        // Fold the per-wave partial streams into the workgroup's partial.
        OwnPartial<CPT> own;
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            own.o[i] = f32x4{0.f, 0.f, 0.f, 0.f};
            own.m[i] = -INFINITY;
            own.l[i] = 0.f;
            const int c = tid + i * THREADS;
            if (c < n_chunks) {
                const int row = (4 * c) / D, col = (4 * c) % D;
                float m = -INFINITY;
#pragma unroll
                for (int p = 0; p < Core::kStreams; ++p) m = fmaxf(m, sm.m[p][row]);
                const float m_ref = m == -INFINITY ? 0.f : m;
#pragma unroll
                for (int p = 0; p < Core::kStreams; ++p) {
                    const float wgt = fast_exp2(sm.m[p][row] - m_ref);
                    own.l[i] += wgt * sm.l[p][row];
                    own.o[i] += wgt * *reinterpret_cast<const f32x4*>(sm.o_at(p, row, col));
                }
                own.m[i] = m;
            }
        }

        const bool finishing_with_peers = sg.finishing && sg.first_cta != g;
        if (finishing_with_peers && sg.tile_iter_end < cta_end) {
            // only a CTA's first segment can end a tile that began elsewhere: one parking place
#pragma unroll
            for (int i = 0; i < CPT; ++i) {
                parked_o[tid + i * THREADS] = own.o[i];
                parked_m[tid + i * THREADS] = own.m[i];
                parked_l[tid + i * THREADS] = own.l[i];
            }
            parked = true;
            parked_b = sg.b;
            parked_h = sg.h;
            parked_first = sg.first_cta;
        } else {
            reduce_tile<Core, CPT, F>(a, own, g, sg.b, sg.h, sg.first_cta, sg.last_cta, wide_scratch);
        }
        it = sg.tile_iter_end;
        __syncthreads();  // the cores reuse the shared partial streams
    }
    stamp(a, g, kClkLoopEnd);
    if (parked) {
        OwnPartial<CPT> own;
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            own.o[i] = parked_o[tid + i * THREADS];
            own.m[i] = parked_m[tid + i * THREADS];
            own.l[i] = parked_l[tid + i * THREADS];
        }
        reduce_tile<Core, CPT, F>(a, own, g, parked_b, parked_h, parked_first, g, wide_scratch);
    }
    stamp(a, g, kClkExit);
}

// The arguments travel by value in the kernel argument segment ...
template <class Core>
__global__ __launch_bounds__(Core::kThreads, Core::kMinWavesPerSimd) void lean_decode_kernel(const DecodeArgs a) {
    lean_decode_body<Core>(a);
}

// ... or are read from a block in device memory that the host rewrites between launches: the same
// captured launch then serves new sequence lengths.
template <class Core>
__global__ __launch_bounds__(Core::kThreads, Core::kMinWavesPerSimd) void lean_decode_kernel_indirect(
    const DecodeArgs* __restrict__ block) {
    lean_decode_body<Core>(*block);
}

}  // namespace lean
