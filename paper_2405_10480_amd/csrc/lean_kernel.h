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

// All partial slots of the launch as one buffer (two slots per CTA).
__device__ __forceinline__ buffer_rsrc partial_slab(const DecodeArgs& a) {
    return make_slab((const uint16_t*)a.partials, 2u * (uint32_t)a.sched.grid * (uint32_t)a.slot * 4u);
}

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
__device__ __forceinline__ void merge_children(const DecodeArgs& a, OwnPartial<CPT>& own, int tile_first, int first,
                                               int step, int nchild, int n_chunks, int n_elem, int T_m) {
    const int tid = threadIdx.x;
    const buffer_rsrc ws = partial_slab(a);
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
                const uint32_t slot = (uint32_t)slot_of(first + jj * step, tile_first) * (uint32_t)a.slot * 4u;
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
__device__ __forceinline__ void merge_children_wide(const DecodeArgs& a, OwnPartial<1>& own, int tile_first, int first,
                                                    int step, int nchild, WideMergeScratch<THREADS>& sh) {
    constexpr int NCH = D / 4;
    constexpr int SLOTS = THREADS / NCH;
    static_assert(SLOTS >= 2 && SLOTS * NCH == THREADS, "single-row tiles are much smaller than the workgroup");
    const int tid = threadIdx.x;
    const int slot = tid / NCH, c = tid % NCH;
    const buffer_rsrc ws = partial_slab(a);
    f32x4 o = {0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f;
    for (int j0 = slot; j0 < nchild; j0 += 4 * SLOTS) {
        f32x4 oc[4];
        float mc[4], lc[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int j = j0 + u * SLOTS;
            const int jj = j < nchild ? j : j0;  // past the last child: re-read a valid one, weight it zero
            const uint32_t base = (uint32_t)slot_of(first + jj * step, tile_first) * (uint32_t)a.slot * 4u;
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

// StorePartials(Op, mp, lp) into partial slot `slot`, then Signal to `readers` readers (with
// `signal` false the stores are only issued: the caller signals once they are acknowledged).
template <int CPT, int THREADS, int D>
__device__ __forceinline__ void publish_partial(const DecodeArgs& a, const OwnPartial<CPT>& own, int g, int slot,
                                                int readers, int n_chunks, int n_elem, int T_m, bool signal = true) {
    const int tid = threadIdx.x;
    if (a.delay_store && debug_delayed(a, g)) debug_sleep(a.delay_store);
    const buffer_rsrc ws = partial_slab(a);
    const uint32_t base = (uint32_t)slot * (uint32_t)a.slot * 4u;
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        const int c = tid + i * THREADS;
        if (c < n_chunks) {
            partial_store16(ws, base + 16u * c, own.o[i]);
            if ((4 * c) % D == 0) {
                partial_store4(ws, base + 4u * (n_elem + (4 * c) / D), own.m[i]);
                partial_store4(ws, base + 4u * (n_elem + T_m + (4 * c) / D), own.l[i]);
            }
        }
    }
    stamp(a, g, kClkStoresIssued);
    if (!signal) return;
    signal_arrival(a, g, slot, readers);
    stamp(a, g, kClkStoresAcked);
}

// O = diag(l)^-1 O~ and L = m + log(l) for one float4 chunk of the tile (m is kept in the base-2
// domain: L = ln2 * (m + log2 l)).
template <class Core>
__device__ __forceinline__ void write_chunk(const DecodeArgs& a, const TileRows& tr, int chunk, f32x4 o_acc, float m,
                                            float l) {
    constexpr int D = Core::kD;
    const int row = (4 * chunk) / D, col = (4 * chunk) % D;
    if (row >= tr.count) return;
    int token;
    const int64_t orow = query_row(a, tr, tr.rho0 + row, &token);
    const f32x4 o = o_acc * (1.f / l);
    if (a.out16) {
        *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(a.out) + orow * D + col) =
            u32x2{narrow2<Core::kDT>(o.x, o.y), narrow2<Core::kDT>(o.z, o.w)};
    } else {
        *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(a.out) + orow * D + col) = o;
    }
    if (a.lse && col == 0) a.lse[orow] = 0.6931471805599453f * (m + __builtin_amdgcn_logf(l));
}

// ---- Default reduction: every CTA of a shared tile publishes, a few of them reduce a slice each --------
// Algorithm 2 lets the host block merge every peer's partial in a loop.  Here every CTA that holds a
// part of a tile shared by `nranks` CTAs publishes its partial first (nobody waits before it has
// published: every wait ends whatever the residency), and the last R CTAs of the tile (ranks 0..R-1,
// counted from the tile's end) then each merge one slice of the tile's [T_m, D] floats from ALL the
// partials, their own included, and write that slice of the output.  One level whatever the number of
// CTAs, a memory round trip or two per reducer, and the partial traffic is spread over R compute
// units.  The re-scaling operator is associative and commutative (Section 4.1), so any such order is
// the same result; the order is fixed, so results are reproducible bit for bit.
constexpr int kMaxMergeSlots = 16;
constexpr int kMergeLoads = 8;  // partials a thread loads before it merges them
struct ScatterPlan {
    int R;            // reducers of the tile, 1..kMaxReducers
    int cpr;          // float4 chunks per reducer (the last reducer may have fewer)
    int slots_log2;   // 2^slots_log2 threads share a chunk of a merge: thread s takes the partials s, s + slots, ...
    int width_log2;   // 2^width_log2 chunks a reducer handles per pass: slots * width = threads
};
// Everything here is shifts and compares: the plan is computed by every CTA of a tile right before
// it polls, on the scalar unit, where a division costs some forty dependent instructions.
template <int THREADS>
__device__ __forceinline__ ScatterPlan scatter_plan(int nranks, int n_chunks) {
    static_assert((THREADS & (THREADS - 1)) == 0, "workgroup sizes are powers of two");
    constexpr int kThreadsLog2 = THREADS == 256 ? 8 : THREADS == 512 ? 9 : THREADS == 128 ? 7 : 6;
    static_assert((1 << kThreadsLog2) == THREADS, "128, 256 or 512 threads");
    // up to kMergeLoads partial loads in flight per thread, at most kMaxMergeSlots partial results to fold
    // per chunk, and as many reducers as it takes to cover the tile's chunks in one pass each
    ScatterPlan p;
    p.slots_log2 = nranks <= kMergeLoads ? 0 : nranks <= 2 * kMergeLoads ? 1 : nranks <= 4 * kMergeLoads ? 2
                   : nranks <= 8 * kMergeLoads ? 3 : 4;
    p.width_log2 = kThreadsLog2 - p.slots_log2;
    const int blocks = (n_chunks + (1 << p.width_log2) - 1) >> p.width_log2;  // passes over the whole tile
    p.R = blocks < kMaxReducers ? blocks : kMaxReducers;
    if (p.R > nranks) p.R = nranks;
    int passes = 1;  // per reducer
    while (passes * p.R < blocks) ++passes;
    p.cpr = passes << p.width_log2;
    return p;
}

// A reducer's duty for one tile, carried out at the end of the CTA's span (at most two per CTA).
struct Duty {
    int b, h, first_cta, last_cta;
    bool own_parked;      // the tile has one reducer: its own partial is not published but waits in LDS
    bool signal_pending;  // the reducer's partial stores are issued, its flags not yet set
};

// `own`: the parked partial of a sole reducer, indexed by chunk (null otherwise).
template <class Core, int THREADS>
__device__ __forceinline__ void reduce_slice(const DecodeArgs& a, const Duty& d, int g, WideMergeScratch<THREADS>& sh,
                                             const f32x4* own_o, const float* own_m, const float* own_l) {
    constexpr int D = Core::kD;
    const int tid = threadIdx.x;
    const int T_m = a.T_m;
    const int n_elem = T_m * D;
    const int n_chunks = n_elem / 4;
    const int nranks = d.last_cta - d.first_cta + 1;
    const int rank = d.last_cta - g;
    const ScatterPlan sp = scatter_plan<THREADS>(nranks, n_chunks);
    // Everything the merge and the final write read from the argument block is fetched now, under the
    // wait for the peers: by the end of a long span those lines have left the scalar cache, and a miss
    // after the flags are seen would sit on the critical path.
    const buffer_rsrc ws = partial_slab(a);
    const TileRows tr = tile_rows(a, d.b, d.h);
    asm volatile("" ::"s"(a.out), "s"(a.lse), "s"(a.out16), "s"(a.Hq), "s"(a.group), "s"(a.N_q), "s"(a.ragged_q),
                 "s"(a.slot), "s"(tr.count), "s"(tr.hk), "s"(tr.rho0), "s"(tr.q0));
    // Wait(flags): this reducer's word of every published contributor (a sole reducer does not publish)
    const int npub = d.own_parked ? nranks - 1 : nranks;
    uint32_t* const my_flag = a.flags + slot_of(d.first_cta + tid, d.first_cta) * kMaxReducers + rank;
    uint32_t seen = 0u;
    if (d.signal_pending) {
        // This reducer's own stores are still in flight: the first poll of its peers goes out behind
        // them, one wait covers both, then its own flags are set and the polling goes on.
        if (tid < npub) seen = poll_issue(my_flag);
        seen = poll_collect(seen);
        signal_acknowledged(a, g, slot_of(g, d.first_cta), sp.R);
        stamp(a, g, kClkStoresAcked);
    }
    if (tid < npub) await_flag(a, my_flag, seen);
    for (int base = THREADS; base < npub; base += THREADS) {
        const int j = base + tid;
        if (j < npub) await_flag(a, a.flags + slot_of(d.first_cta + j, d.first_cta) * kMaxReducers + rank);
    }
    __syncthreads();  // the partial loads that follow are issued after the flags were seen
    stamp(a, g, kClkFlagsSeen);
    const int c_begin = rank * sp.cpr;
    const int c_end = c_begin + sp.cpr < n_chunks ? c_begin + sp.cpr : n_chunks;
    const int width = 1 << sp.width_log2, slots = 1 << sp.slots_log2;
    const int slot = tid >> sp.width_log2, ci = tid & (width - 1);
    for (int pass = c_begin; pass < c_end; pass += width) {
        const int chunk = pass + ci;
        const bool active = chunk < c_end;
        const int row = active ? (4 * chunk) / D : 0;
        f32x4 o = {0.f, 0.f, 0.f, 0.f};
        float m = -INFINITY, l = 0.f;
        if (active) {
            for (int j0 = slot; j0 < npub; j0 += kMergeLoads * slots) {
                f32x4 oc[kMergeLoads];
                float mc[kMergeLoads], lc[kMergeLoads];
#pragma unroll
                for (int u = 0; u < kMergeLoads; ++u) {
                    const int j = j0 + u * slots;
                    const int jj = j < npub ? j : j0;  // past the last partial: re-read a valid one, weight it zero
                    const uint32_t base = (uint32_t)slot_of(d.first_cta + jj, d.first_cta) * (uint32_t)a.slot * 4u;
                    oc[u] = partial_load16(ws, base + 16u * chunk);
                    mc[u] = partial_load4(ws, base + 4u * (n_elem + row));
                    lc[u] = partial_load4(ws, base + 4u * (n_elem + T_m + row));
                }
                // the common reference first, so that the weights do not wait for each other
                float m_new = m;
#pragma unroll
                for (int u = 0; u < kMergeLoads; ++u) {
                    if (j0 + u * slots >= npub) mc[u] = -INFINITY;
                    m_new = fmaxf(m_new, mc[u]);
                }
                const float m_ref = m_new == -INFINITY ? 0.f : m_new;
                const float w_acc = fast_exp2(m - m_ref);
                l *= w_acc;
                o = o * w_acc;
#pragma unroll
                for (int u = 0; u < kMergeLoads; ++u) {
                    const float w = fast_exp2(mc[u] - m_ref);
                    l += w * lc[u];
                    o += w * oc[u];
                }
                m = m_new;
            }
        }
        if (slots > 1) {  // (workgroup-uniform) the threads of a chunk meet in LDS, folded in slot order
            sh.o[tid] = o;
            sh.m[tid] = m;
            sh.l[tid] = l;
            __syncthreads();
            if (active && slot == 0) {
                float ms[kMaxMergeSlots];
                float m_all = -INFINITY;
#pragma unroll
                for (int sl = 0; sl < kMaxMergeSlots; ++sl) {
                    ms[sl] = sl < slots ? sh.m[sl * width + ci] : -INFINITY;
                    m_all = fmaxf(m_all, ms[sl]);
                }
                const float m_ref = m_all == -INFINITY ? 0.f : m_all;
                o = f32x4{0.f, 0.f, 0.f, 0.f};
                l = 0.f;
#pragma unroll
                for (int sl = 0; sl < kMaxMergeSlots; ++sl) {
                    const int at = (sl < slots ? sl : 0) * width + ci;
                    const float w = fast_exp2(ms[sl] - m_ref);  // zero past the last slot
                    l += w * sh.l[at];
                    o += w * sh.o[at];
                }
                m = m_all;
            }
            __syncthreads();  // the scratch is reused by the next pass
        }
        if (active && slot == 0) {
            if (d.own_parked) {  // the sole reducer's own part of the tile, last
                const float m_own = own_m[chunk];
                const float m_new = fmaxf(m, m_own);
                const float m_ref = m_new == -INFINITY ? 0.f : m_new;
                const float w_acc = fast_exp2(m - m_ref), w_own = fast_exp2(m_own - m_ref);
                l = w_acc * l + w_own * own_l[chunk];
                o = w_acc * o + w_own * own_o[chunk];
                m = m_new;
            }
            write_chunk<Core>(a, tr, chunk, o, m, l);
        }
    }
    stamp(a, g, kClkWritten);
}

// ---- Alternative reduction (lean_attn_tuning.merge_fanin >= 2): a tree rooted at the finishing block ----
// Ranks count from the tile's END: rank 0 is the finishing block (the CTA whose span holds
// the tile's last LeanTile), the block that computed the tile's first LeanTile has the
// highest rank.  Because the re-scaling operator is associative the blocks form a tree of
// fan-in `fanin` instead of Algorithm 2's flat list: rank k merges ranks k + j*stride
// (j < fanin) while k is a multiple of stride*fanin, then publishes once; rank 0 merges
// last and writes O = diag(l)^-1 O~ and L = m + log(l).  A block therefore only ever waits
// for LOWER CTA ids, i.e. for workgroups the hardware dispatched before it, so every wait
// ends even when the grid is larger than what is resident at once.  A fan-in of
// LEAN_ATTN_MAX_GRID or more gives Algorithm 2's flat list (rooted at the finishing block).
template <class Core, int CPT, int F>
__device__ __forceinline__ void reduce_tile(const DecodeArgs& a, OwnPartial<CPT>& own, int g, int b, int h,
                                            int first_cta, int last_cta, int fanin,
                                            WideMergeScratch<Core::kThreads>& wide_scratch) {
    constexpr int D = Core::kD;
    constexpr int THREADS = Core::kThreads;
    const int tid = threadIdx.x;
    const int T_m = a.T_m;
    const int n_elem = T_m * D;
    const int n_chunks = n_elem / 4;
    const int rank = last_cta - g;
    const int nranks = last_cta - first_cta + 1;
    bool publish = false;
    for (int64_t stride = 1; stride < nranks; stride *= fanin) {
        if (rank % (stride * fanin) != 0) {
            publish = true;
            break;
        }
        int remaining = (int)((nranks - 1 - rank) / stride);  // children at this level
        if (remaining > fanin - 1) remaining = fanin - 1;
        int child = g - (int)stride;
        if constexpr (Core::kTmMax == 1) {
            // single-row tiles: batches as wide as four children per slot of the workgroup
            constexpr int kWide = 4 * (THREADS / (D / 4));
            while (remaining > 0) {
                const int batch = remaining < kWide ? remaining : kWide;
                wait_arrivals(a, first_cta, child, -(int)stride, batch);
                stamp(a, g, kClkFlagsSeen);
                merge_children_wide<THREADS, D>(a, own, first_cta, child, -(int)stride, batch, wide_scratch);
                child -= batch * (int)stride;
                remaining -= batch;
            }
        } else {
            while (remaining > 0) {  // batches of at most F-1 partials
                const int batch = remaining < F - 1 ? remaining : F - 1;
                wait_arrivals(a, first_cta, child, -(int)stride, batch);
                stamp(a, g, kClkFlagsSeen);
                merge_children<CPT, THREADS, D, F>(a, own, first_cta, child, -(int)stride, batch, n_chunks, n_elem, T_m);
                child -= batch * (int)stride;
                remaining -= batch;
            }
        }
        stamp(a, g, kClkMerged);
    }
    if (publish) {
        publish_partial<CPT, THREADS, D>(a, own, g, slot_of(g, first_cta), 1, n_chunks, n_elem, T_m);
    } else {
        const TileRows tr = tile_rows(a, b, h);
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const int c = tid + i * THREADS;
            if (c < n_chunks) write_chunk<Core>(a, tr, c, own.o[i], own.m[i], own.l[i]);
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
    // Tree reduction only: a finishing block whose span goes on to other tiles parks its partial here
    // and reduces at the end of its span, when its peers are done too (thread-private entries).
    struct Parked {
        f32x4 o[CPT * THREADS];
        float m[CPT * THREADS];
        float l[CPT * THREADS];
    };
    // A block that reduces a tile alone parks its own partial here (entry c: chunk c) until its span is
    // done and its peers have published.
    __shared__ Parked parked_partial;
    // Where the threads that share a chunk of a merge meet: THREADS entries of (O~ chunk, m, l).  The
    // single-row cores merge inside the span loop too (tree reduction) and own one; the multi-row cores
    // only need it once their span is done, and use the then idle partial streams of the core.
    __shared__ WideMergeScratch<Core::kTmMax == 1 ? THREADS : 1> scratch_own;
    static_assert(Core::kTmMax == 1 || sizeof(WideMergeScratch<THREADS>) <= sizeof(typename Core::Smem),
                  "the core's LDS area is large enough to lend");
    WideMergeScratch<THREADS>& merge_scratch = Core::kTmMax == 1 ? reinterpret_cast<WideMergeScratch<THREADS>&>(scratch_own)
                                                                 : reinterpret_cast<WideMergeScratch<THREADS>&>(sm);
    f32x4* const parked_o = parked_partial.o;
    float* const parked_m = parked_partial.m;
    float* const parked_l = parked_partial.l;

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

    // CTA id = workgroup id: the hardware dispatches workgroups in id order.  In the default reduction
    // nobody waits before it has published; in the tree reduction a workgroup only ever waits for lower
    // ids: either way every wait ends however few workgroups are resident at once.  (Mapping span ids
    // so that consecutive spans share an XCD was tried: no gain in streaming rate, and a workgroup may
    // then wait for one dispatched after it.)
    const int g = blockIdx.x;
    const int G = a.sched.grid;

    const int tid = threadIdx.x;
    const int T_m = a.T_m;
    const int n_elem = T_m * D;
    const int n_chunks = n_elem / 4;
    const bool tree = a.fanin >= 2;
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
    int parked_b = 0, parked_h = 0, parked_first = 0, parked_fanin = 2;
    // reducer duties of the default reduction: at most one for the tile the span starts inside and one
    // for the tile it ends inside
    Duty duty_a, duty_b;  // (two named records: an array indexed at run time would live in scratch memory)
    int n_duties = 0;

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

        const int nranks = sg.last_cta - sg.first_cta + 1;
        // A multi-row tile shared by at most F CTAs is merged by its finishing block alone, in registers,
        // as one level of the tree reduction (measured 0.4 us quicker than parking the partial in LDS).
        const bool small_tile = Core::kTmMax > 1 && nranks <= F;
        const int fanin = tree ? a.fanin : F;
        if (nranks == 1) {  // the tile is this CTA's alone: normalise and write
            const TileRows tr = tile_rows(a, sg.b, sg.h);
#pragma unroll
            for (int i = 0; i < CPT; ++i) {
                const int c = tid + i * THREADS;
                if (c < n_chunks) write_chunk<Core>(a, tr, c, own.o[i], own.m[i], own.l[i]);
            }
        } else if (!tree && !small_tile) {
            const ScatterPlan sp = scatter_plan<THREADS>(nranks, n_chunks);
            const bool reducer = sg.last_cta - g < sp.R;  // one of the tile's last R CTAs: it reduces a slice, later
            const bool sole = reducer && sp.R == 1;
            // a reducer whose span ends here starts polling at once: its stores and its first poll share a wait
            const bool overlap = reducer && !sole && sg.tile_iter_end >= cta_end && !a.delay_signal;
            if (sole) {  // nobody else reads this partial: it waits in LDS (only a CTA's first segment can
                         // end a tile that began elsewhere: one parking place)
#pragma unroll
                for (int i = 0; i < CPT; ++i) {
                    parked_o[tid + i * THREADS] = own.o[i];
                    parked_m[tid + i * THREADS] = own.m[i];
                    parked_l[tid + i * THREADS] = own.l[i];
                }
            } else {
                publish_partial<CPT, THREADS, D>(a, own, g, slot_of(g, sg.first_cta), sp.R, n_chunks, n_elem, T_m,
                                                 !overlap);
            }
            if (reducer) {
                const Duty d = {sg.b, sg.h, sg.first_cta, sg.last_cta, sole, overlap};
                if (n_duties == 0) duty_a = d;
                else duty_b = d;
                ++n_duties;
            }
        } else {
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
                parked_fanin = fanin;
            } else {
                reduce_tile<Core, CPT, F>(a, own, g, sg.b, sg.h, sg.first_cta, sg.last_cta, fanin, merge_scratch);
            }
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
        reduce_tile<Core, CPT, F>(a, own, g, parked_b, parked_h, parked_first, g, parked_fanin, merge_scratch);
    }
    if (n_duties > 0) reduce_slice<Core, THREADS>(a, duty_a, g, merge_scratch, parked_o, parked_m, parked_l);
    if (n_duties > 1) reduce_slice<Core, THREADS>(a, duty_b, g, merge_scratch, parked_o, parked_m, parked_l);
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
