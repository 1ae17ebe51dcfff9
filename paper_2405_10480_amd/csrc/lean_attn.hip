// Host side of the LeanAttention decode library: argument checks, the
// stream-K scheduler (Section 4.3), kernel selection and launch.  The C ABI is
// declared in include/lean_attn.h.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <mutex>

#include "../../include/lean_attn.h"
#include "lean_aux_kernels.h"
#include "lean_device.h"
#include "lean_sched.h"
#include "lean_variants.h"

namespace lean {

static_assert(kMaxBatch == LEAN_ATTN_MAX_BATCH, "header and scheduler disagree on the batch limit");
static_assert(kMaxGrid == LEAN_ATTN_MAX_GRID, "header and workspace layout disagree on the grid limit");

// Defaults picked by the LeanTile sweep on MI355X (the paper fixes the tile size per architecture
// after an empirical sweep, Section 4.2).
constexpr int kDefaultCtasPerCu = 1;
constexpr int kDefaultTailPermille = 60;  // share of the iterations the tail spans cover when asked for without one
constexpr int kShortContextTokens = 1536;  // mean context at or below which two workgroups share a unit
constexpr int kDefaultGridMultiple = 1;
constexpr int kMaxProbeMode = 6;

static int dim_index(int D) { return D == 64 ? 0 : D == 128 ? 1 : D == 256 ? 2 : -1; }

// Most query rows one output tile can hold: two MFMA row blocks up to D = 128, one at D = 256.
static int max_tile_rows(int D) { return D <= 128 ? LEAN_ATTN_MAX_TILE_ROWS : 16; }

// Rows-per-tile classes the defaults are keyed on: 1 | 2..8 | 9..16 | 17..32.
static int row_class(int T_m) { return T_m <= 1 ? 0 : T_m <= 8 ? 1 : T_m <= 16 ? 2 : 3; }

// Default tile shape (1..kNumShapes, see lean_kernels.hip for what each number builds) per
// [dtype f16, bf16][head dim 64, 128, 256][row class], filled from the LeanTile sweep at 1 GiB of
// K/V per call (the sweep of Section 4.2, here `bench.py --tile-sweep`).  With non-temporal loads the
// memory system runs fastest with about 32 KiB in flight per compute unit, single-buffered:
//   * one row (VALU core) and one row block at D = 128: four waves with 8 KiB each, shape 6
//     (T_n = 64 tokens at D = 128) -- 6 % ahead of every other shape at 2..16 rows;
//   * D = 64, where a 16-token block is only 4 KiB of K and V: eight waves (shape 4) up to 8 rows,
//     two blocks per wave (shape 5) for 9..16;
//   * D = 256: two token blocks per wave (shape 5);
//   * two row blocks: a step's arithmetic is about twice as long, and four waves no longer cover
//     each other's load latency: eight waves, next step's loads issued early (shape 4) at D = 128,
//     the double-buffered shape 1 at D = 64.
// Both dtypes measure alike; they keep separate rows because the table is keyed on them.
static const int8_t kDefaultShape[2][3][4] = {
    /* f16  */ {{6, 4, 5, 1}, {6, 6, 6, 4}, {6, 5, 5, 0}},
    /* bf16 */ {{6, 4, 5, 1}, {6, 6, 6, 4}, {6, 5, 5, 0}},
};

// kernel: 0 VALU single-row core, 1 MFMA query-group core; T_m: query rows per output tile;
// shape: 0 = the default of the table, 1..kNumShapes a compiled shape.  *resolved gets the shape used.
static bool pick_variant(int kernel, int dtype, int D, int shape, int T_m, Variant* v, int* resolved = nullptr) {
    if (shape < 0 || shape > kNumShapes || dim_index(D) < 0 || T_m < 1 || T_m > max_tile_rows(D)) return false;
    if (dtype != LEAN_ATTN_F16 && dtype != LEAN_ATTN_BF16) return false;
    const bool bf = dtype == LEAN_ATTN_BF16;
    // the MFMA core on a single row is served by the one-block defaults
    if (shape == 0) shape = kDefaultShape[bf][dim_index(D)][kernel == 0 ? 0 : (T_m <= 1 ? 1 : row_class(T_m))];
    if (kernel == 0) *v = bf ? variant_mha_bf16(D, shape) : variant_mha_f16(D, shape);
    else if (T_m > 16) *v = bf ? variant_gqa2_bf16(D, shape) : variant_gqa2_f16(D, shape);
    else *v = bf ? variant_gqa_bf16(D, shape) : variant_gqa_f16(D, shape);
    if (resolved) *resolved = shape;
    return v->fn != nullptr;
}

// Workspace bytes a launch of `grid` workgroups with T_m-row partials touches.
static size_t workspace_need(int64_t grid, int T_m, int D) {
    return kPartialsOffset + 2 * (size_t)grid * slot_floats(T_m, D) * sizeof(float);  // two slots per workgroup
}

// Unit count of the device and, per variant, the workgroups that fit on one unit (cached).
struct DeviceInfo {
    int cus = 0;
    int resident[3][2][3][kNumShapes + 1] = {};  // [VALU, MFMA, MFMA two row blocks][dtype][head dim][shape], 0 = not yet queried
};
static DeviceInfo g_dev[64];
static std::mutex g_dev_mutex;

static int query_device(int kernel, int dtype, int D, int shape, int T_m, int* cus, int* per_cu) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return LEAN_ATTN_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_dev_mutex);
    DeviceInfo& di = g_dev[dev];
    if (di.cus == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return LEAN_ATTN_ERR_HIP;
        di.cus = prop.multiProcessorCount;
    }
    if (dim_index(D) < 0) return LEAN_ATTN_ERR_UNSUPPORTED;
    Variant v;
    int resolved = 0;
    if (!pick_variant(kernel, dtype, D, shape, T_m, &v, &resolved)) return LEAN_ATTN_ERR_UNSUPPORTED;
    int& n = di.resident[kernel == 1 && T_m > 16 ? 2 : kernel][dtype][dim_index(D)][resolved];
    if (n == 0) {
        int blocks = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, v.fn, v.threads, 0) != hipSuccess || blocks <= 0)
            return LEAN_ATTN_ERR_HIP;
        n = blocks;
    }
    *cus = di.cus;
    *per_cu = n;
    return LEAN_ATTN_OK;
}

// any_batch: the caller splits batches beyond LEAN_ATTN_MAX_BATCH itself (lean_attn_attend)
static int check_problem(const lean_attn_problem& p, bool any_batch = false) {
    if (p.B <= 0 || p.N_q <= 0 || p.Hq <= 0 || p.Hkv <= 0 || p.Hq % p.Hkv != 0) return LEAN_ATTN_ERR_BAD_SHAPE;
    if ((int64_t)p.N_q * (p.Hq / p.Hkv) > LEAN_ATTN_MAX_QUERY_ROWS) return LEAN_ATTN_ERR_BAD_SHAPE;
    if (p.causal != 0 && p.causal != 1) return LEAN_ATTN_ERR_BAD_SHAPE;
    if (p.q_lens) {
        int longest = 0;
        for (int b = 0; b < p.B && (any_batch || b < LEAN_ATTN_MAX_BATCH); ++b) {
            if (p.q_lens[b] < 0 || p.q_lens[b] > p.N_q) return LEAN_ATTN_ERR_BAD_SHAPE;
            if (p.q_lens[b] > longest) longest = p.q_lens[b];
        }
        if (longest != p.N_q) return LEAN_ATTN_ERR_BAD_SHAPE;  // N_q is the longest query, by definition
    }
    if (p.B > LEAN_ATTN_MAX_BATCH && !any_batch) return LEAN_ATTN_ERR_BATCH_TOO_LARGE;
    if (dim_index(p.D) < 0) return LEAN_ATTN_ERR_UNSUPPORTED;
    if (p.dtype != LEAN_ATTN_F16 && p.dtype != LEAN_ATTN_BF16) return LEAN_ATTN_ERR_UNSUPPORTED;
    if (p.out_dtype != LEAN_ATTN_OUT_F32 && p.out_dtype != LEAN_ATTN_OUT_AS_INPUT) return LEAN_ATTN_ERR_UNSUPPORTED;
    if (p.kv_layout != LEAN_ATTN_KV_PADDED && p.kv_layout != LEAN_ATTN_KV_PACKED) return LEAN_ATTN_ERR_UNSUPPORTED;
    return LEAN_ATTN_OK;
}

// The R = N_q * group query rows that share a KV head, cut into C_m output tiles of T_m rows
// (Algorithm 2: C_m = ceil(N_q / T_m), with the query group folded into the rows); a tile holds
// at most 32 rows (16 at D = 256).
struct RowBlocks {
    int R, C_m, T_m;
};
static RowBlocks row_blocks(const lean_attn_problem& p) {
    RowBlocks rb;
    rb.R = p.N_q * (p.Hq / p.Hkv);
    const int cap = max_tile_rows(p.D);
    rb.C_m = (rb.R + cap - 1) / cap;
    rb.T_m = (rb.R + rb.C_m - 1) / rb.C_m;
    return rb;
}

static lean_attn_problem decode_problem(int B, int Hq, int Hkv, int D, int dtype, int kv_layout,
                                        int64_t kv_seq_stride, float scale) {
    lean_attn_problem p;
    std::memset(&p, 0, sizeof p);
    p.B = B;
    p.N_q = 1;
    p.Hq = Hq;
    p.Hkv = Hkv;
    p.D = D;
    p.dtype = dtype;
    p.out_dtype = LEAN_ATTN_OUT_F32;
    p.kv_layout = kv_layout;
    p.causal = 0;
    p.scale = scale;
    p.kv_seq_stride = kv_seq_stride;
    return p;
}

// The host scheduler: per-sequence tile counts, total iterations, grid, spans.
// O(B) integer work; nothing here touches the device unless the unit count has
// to be read.
// full_grid: the grid is units x 1 whatever the lengths are (even when that exceeds the iteration
// count: the surplus workgroups own empty spans), so that a launch captured once serves any lengths.
static int make_schedule(const lean_attn_problem& p, const int32_t* seqlens, const lean_attn_tuning* tn,
                         lean_attn_plan* plan, Sched* sched, SchedTable* table, bool full_grid = false) {
    if (!seqlens || !plan) return LEAN_ATTN_ERR_NULL_POINTER;
    int rc = check_problem(p);
    if (rc != LEAN_ATTN_OK) return rc;
    const int B = p.B, D = p.D, dtype = p.dtype, kv_layout = p.kv_layout;
    const RowBlocks rb = row_blocks(p);
    const int heads = p.Hkv * rb.C_m;  // output tiles per sequence
    lean_attn_tuning t;
    std::memset(&t, 0, sizeof t);
    if (tn) t = *tn;
    if (t.grid < 0 || t.ctas_per_cu < 0 || t.num_cus < 0 || t.kernel < 0 || t.kernel > 2 || t.tail_grid < 0 || t.tail_permille < 0 || t.tail_permille > 500 ||
        t.debug_delay_store < 0 || t.debug_delay_store > 64 ||
        t.debug_delay_signal < 0 || t.debug_delay_signal > 64 || t.debug_delay_stride < 0 || t.spin_limit < 0 || t.merge_fanin < 0 || t.merge_fanin == 1 || t.tile_shape < 0 ||
        t.tile_shape > kNumShapes || t.grid_multiple < 0 || t.fixed_split < -1)
        return LEAN_ATTN_ERR_TUNING;
    const int T_m = rb.T_m;
    // the single-row core indexes q and out by (b, head): per-sequence query lengths go to the MFMA core
    int kernel = (rb.R == 1 && !p.q_lens) ? 0 : 1;
    if (t.kernel == 1) {
        if (rb.R != 1 || p.q_lens) return LEAN_ATTN_ERR_TUNING;
        kernel = 0;
    } else if (t.kernel == 2) {
        kernel = 1;
    }
    Variant var;
    int tile_shape = 0;
    if (!pick_variant(kernel, dtype, D, t.tile_shape, T_m, &var, &tile_shape)) return LEAN_ATTN_ERR_UNSUPPORTED;
    const int T_n = var.T_n;

    int64_t iters = 0, toks = 0, q_toks = 0;
    int nonempty = 0;
    for (int b = 0; b < B; ++b) {
        nonempty += seqlens[b] > 0;
        if (seqlens[b] < 0) return LEAN_ATTN_ERR_SEQLEN;
        const int q_len = p.q_lens ? p.q_lens[b] : p.N_q;
        if (p.causal && seqlens[b] != 0 && seqlens[b] < q_len) return LEAN_ATTN_ERR_SEQLEN;
        if (table) {
            table->cu_iters[b] = (int32_t)iters;
            table->cu_tok[b] = (int32_t)toks;
            table->cu_q[b] = (int32_t)q_toks;
        }
        q_toks += q_len;
        if ((int64_t)seqlens[b] * D * 2 > INT32_MAX) return LEAN_ATTN_ERR_SEQLEN;  // one slab per buffer descriptor
        iters += ((int64_t)seqlens[b] + T_n - 1) / T_n;
        toks += seqlens[b];
        if (toks > INT32_MAX) return LEAN_ATTN_ERR_SEQLEN;
    }
    if (table) {
        table->cu_iters[B] = (int32_t)iters;
        table->cu_tok[B] = (int32_t)toks;
        table->cu_q[B] = (int32_t)q_toks;
    }
    const int64_t I = iters * heads;

    int cus = t.num_cus, per_cu = t.ctas_per_cu;
    int64_t resident;
    int hw_per_cu = 0;
    if (cus <= 0) {  // read the device: unit count and how many workgroups of this kernel fit per unit
        rc = query_device(kernel, dtype, D, t.tile_shape, T_m, &cus, &hw_per_cu);
        if (rc != LEAN_ATTN_OK) return rc;
        if (hw_per_cu <= 0) return LEAN_ATTN_ERR_HIP;
    }
    // One workgroup per unit streams fastest while its span stays inside one or two output
    // tiles.  With many short tiles (large batches of short contexts) every workgroup crosses
    // several tile boundaries, each a bubble in its K/V stream (epilogue, next Q, first load
    // round trip); a second workgroup on the unit fills those bubbles (measured: 3-5 % faster
    // at 1000 tokens per sequence, even at 2000, 1 % slower at 4000).
    int default_per_cu = kDefaultCtasPerCu;
    if (!full_grid && nonempty > 0 && toks / nonempty <= kShortContextTokens &&
        (int64_t)nonempty * heads >= 2 * (int64_t)cus)
        default_per_cu = 2;
    if (hw_per_cu > 0) {
        if (per_cu <= 0) per_cu = hw_per_cu < default_per_cu ? hw_per_cu : default_per_cu;
        if (per_cu > hw_per_cu) per_cu = hw_per_cu;
        resident = (int64_t)cus * hw_per_cu;
    } else {
        if (per_cu <= 0) per_cu = default_per_cu;
        resident = (int64_t)cus * per_cu;
    }
    // The grid may exceed what is resident at once: blocks only wait for lower CTA ids, which
    // the hardware dispatched earlier, so later blocks simply start as earlier ones retire.
    int64_t G = (int64_t)cus * per_cu * (t.grid_multiple > 0 ? t.grid_multiple : kDefaultGridMultiple);
    if (t.grid > 0) G = t.grid;
    if (G > LEAN_ATTN_MAX_GRID) G = LEAN_ATTN_MAX_GRID;
    if (G > I && !full_grid) G = I;
    if (G < 1) G = 1;

    // Baseline schedule: fixed split.  With no factor given, split so that one wave of
    // workgroups fills the device and do not split once the output tiles alone exceed it
    // (the behaviour the paper describes for FlashDecoding in Sections 3.3 and 6.1).
    int split = 0;
    if (t.fixed_split != 0) {
        const int64_t tiles = (int64_t)B * heads;
        const int64_t slots = (int64_t)cus * per_cu;
        split = t.fixed_split > 0 ? t.fixed_split : (int)(slots / tiles);
        if (split < 1) split = 1;
        if (split > 128) split = 128;
        G = tiles * split;
        if (G > 65535 || (split > 1 && G > LEAN_ATTN_MAX_GRID)) return LEAN_ATTN_ERR_TUNING;
    }

    // Tail spans: the last share of the line in short spans for `tail_grid` further workgroups, which
    // the hardware dispatches as the first G retire.  Not for the baseline schedules, and dropped when
    // the problem is too small to leave every one of the first G workgroups an iteration.
    int64_t P = 0, tail_iters = 0;
    if (split == 0 && t.tail_grid > 0) {
        if (full_grid || G + t.tail_grid > LEAN_ATTN_MAX_GRID) return LEAN_ATTN_ERR_TUNING;
        P = t.tail_grid;
        tail_iters = I * (t.tail_permille > 0 ? t.tail_permille : kDefaultTailPermille) / 1000;
        if (tail_iters < P) tail_iters = P;
        if (I - tail_iters < G) P = tail_iters = 0;
    }
    Sched spans;
    set_spans(spans, I, (int32_t)(G + P), (int32_t)P, tail_iters);

    plan->T_n = T_n;
    plan->T_m = T_m;
    plan->num_output_tiles = B * heads;
    plan->grid = spans.grid;
    plan->total_iters = I;
    plan->iters_per_cta = spans.iters_per_cta;
    plan->extra = spans.extra;
    plan->tail_grid = spans.tail_grid;
    plan->tail_iters = tail_iters;
    plan->block_threads = var.threads;
    plan->max_resident = (int32_t)resident;
    plan->kernel = kernel;
    plan->fixed_split = split;
    plan->C_m = rb.C_m;
    plan->tile_shape = tile_shape;
    if (sched) {
        sched->B = B;
        sched->Hkv = heads;
        sched->T_n = T_n;
        sched->packed = kv_layout == LEAN_ATTN_KV_PACKED;
        set_spans(*sched, I, spans.grid, spans.tail_grid, tail_iters);
        sched->fixed_split = split;
        if (table) finish_sched(*sched, *table);
    }
    return LEAN_ATTN_OK;
}

}  // namespace lean

using namespace lean;

extern "C" {

// Rows per partial slot the launches of `p` can need.  A batch beyond one launch with per-sequence
// query lengths runs chunk by chunk, each chunk cut into row blocks by ITS longest query: a chunk
// can then hold more rows per tile than the whole problem would (33 rows make two blocks of 17,
// 32 rows one block of 32), so such problems are sized for the largest tile.
static int slot_rows(const lean_attn_problem& p) {
    if (p.q_lens && p.B > LEAN_ATTN_MAX_BATCH) return max_tile_rows(p.D);
    return row_blocks(p).T_m;
}

size_t lean_attn_workspace_size_for_grid(const lean_attn_problem* problem, int max_grid) {
    if (!problem || check_problem(*problem, true) != LEAN_ATTN_OK) return 0;
    if (max_grid < 1 || max_grid > LEAN_ATTN_MAX_GRID) return 0;
    return workspace_need(max_grid, slot_rows(*problem), problem->D);
}

size_t lean_attn_problem_workspace_size(const lean_attn_problem* problem) {
    return lean_attn_workspace_size_for_grid(problem, LEAN_ATTN_MAX_GRID);
}

size_t lean_attn_workspace_size(int B, int Hq, int Hkv, int D, int dtype) {
    const lean_attn_problem p = decode_problem(B, Hq, Hkv, D, dtype, LEAN_ATTN_KV_PADDED, 0, 1.f);
    return lean_attn_problem_workspace_size(&p);
}

int lean_attn_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!workspace) return LEAN_ATTN_ERR_NULL_POINTER;
    if (workspace_bytes < kPartialsOffset || ((uintptr_t)workspace & 255) != 0) return LEAN_ATTN_ERR_WORKSPACE;
    const int n = (int)(kPartialsOffset / 4);
    hipLaunchKernelGGL(lean_workspace_clear_kernel, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)hip_stream,
                       (uint32_t*)workspace, n);
    return hipGetLastError() == hipSuccess ? LEAN_ATTN_OK : LEAN_ATTN_ERR_HIP;
}

int lean_attn_workspace_status(void* workspace, void* hip_stream) {
    if (!workspace) return LEAN_ATTN_ERR_NULL_POINTER;
    uint32_t word = 0;
    if (hipStreamSynchronize((hipStream_t)hip_stream) != hipSuccess) return LEAN_ATTN_ERR_HIP;
    if (hipMemcpy(&word, workspace, 4, hipMemcpyDeviceToHost) != hipSuccess) return LEAN_ATTN_ERR_HIP;
    if (word != 0) {
        // A peer that arrived after its host gave up left its flag set: clear them all.
        const int n = (int)(kPartialsOffset / 4);
        hipLaunchKernelGGL(lean_workspace_clear_kernel, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)hip_stream,
                           (uint32_t*)workspace, n);
        if (hipStreamSynchronize((hipStream_t)hip_stream) != hipSuccess) return LEAN_ATTN_ERR_HIP;
        return LEAN_ATTN_ERR_PEER_TIMEOUT;
    }
    return LEAN_ATTN_OK;
}

int lean_attn_schedule(const int32_t* seqlens, int B, int Hq, int Hkv, int D, int dtype, int kv_layout,
                       const lean_attn_tuning* tuning, lean_attn_plan* plan) {
    const lean_attn_problem p = decode_problem(B, Hq, Hkv, D, dtype, kv_layout, 0, 1.f);
    return make_schedule(p, seqlens, tuning, plan, nullptr, nullptr);
}

int lean_attn_problem_schedule(const lean_attn_problem* problem, const int32_t* seqlens,
                               const lean_attn_tuning* tuning, lean_attn_plan* plan) {
    if (!problem) return LEAN_ATTN_ERR_NULL_POINTER;
    return make_schedule(*problem, seqlens, tuning, plan, nullptr, nullptr);
}

int lean_attn_walk(const lean_attn_plan* plan, const int32_t* seqlens, int B, int Hkv, int kv_layout, int g,
                   int64_t* segments, int max_segments) {
    if (!plan || !seqlens || !segments) return LEAN_ATTN_ERR_NULL_POINTER;
    if (B <= 0 || B > LEAN_ATTN_MAX_BATCH || Hkv <= 0 || plan->T_n <= 0) return LEAN_ATTN_ERR_BAD_SHAPE;
    if (g < 0 || g >= plan->grid) return LEAN_ATTN_ERR_TUNING;
    const int heads = Hkv * (plan->C_m > 0 ? plan->C_m : 1);
    Sched s;
    SchedTable t;
    int64_t iters = 0, toks = 0;
    for (int b = 0; b < B; ++b) {
        if (seqlens[b] < 0) return LEAN_ATTN_ERR_SEQLEN;
        t.cu_iters[b] = (int32_t)iters;
        t.cu_tok[b] = (int32_t)toks;
        iters += ((int64_t)seqlens[b] + plan->T_n - 1) / plan->T_n;
        toks += seqlens[b];
    }
    t.cu_iters[B] = (int32_t)iters;
    t.cu_tok[B] = (int32_t)toks;
    s.B = B;
    s.Hkv = heads;
    s.T_n = plan->T_n;
    s.packed = kv_layout == LEAN_ATTN_KV_PACKED;
    if (plan->tail_grid < 0 || plan->tail_grid >= plan->grid || plan->tail_iters < 0 || plan->tail_iters > plan->total_iters)
        return LEAN_ATTN_ERR_BAD_SHAPE;
    set_spans(s, plan->total_iters, plan->grid, plan->tail_grid, plan->tail_iters);
    if (s.extra != plan->extra || s.iters_per_cta != plan->iters_per_cta) return LEAN_ATTN_ERR_BAD_SHAPE;
    s.fixed_split = plan->fixed_split;
    finish_sched(s, t);
    if (iters * heads != plan->total_iters) return LEAN_ATTN_ERR_BAD_SHAPE;
    int64_t it, end;
    span_of(s, t, g, &it, &end);
    int n = 0;
    const int64_t begin = it;
    Segment sg;
    while (it < end) {
        sg = it == begin ? locate(s, t, it, end) : locate_next(s, t, sg, g, end);  // as the kernel walks
        if (n < max_segments) {
            int64_t* rec = segments + 8 * (int64_t)n;
            rec[0] = sg.tile_idx;
            rec[1] = sg.b;
            rec[2] = sg.h;
            rec[3] = sg.local_iter;
            rec[4] = sg.local_iter_end;
            rec[5] = sg.host;
            rec[6] = sg.finishing;
            rec[7] = sg.last_cta;
        }
        ++n;
        it = sg.tile_iter_end;
    }
    return n;
}

static int check_lengths(const lean_attn_problem& p, const int32_t* seqlens, int64_t* tok_total) {
    int64_t total = 0;
    for (int b = 0; b < p.B; ++b) {
        const int64_t n = seqlens[b];
        const int q_len = p.q_lens ? p.q_lens[b] : p.N_q;
        if (n < 0 || n * p.D * 2 > INT32_MAX) return LEAN_ATTN_ERR_SEQLEN;
        if (p.causal && n != 0 && n < q_len) return LEAN_ATTN_ERR_SEQLEN;
        if (p.kv_layout == LEAN_ATTN_KV_PADDED && p.kv_seq_stride < n) return LEAN_ATTN_ERR_SEQLEN;
        total += n;
        if (total > INT32_MAX) return LEAN_ATTN_ERR_SEQLEN;
    }
    *tok_total = total;
    return LEAN_ATTN_OK;
}

// The arguments of one launch (at most LEAN_ATTN_MAX_BATCH sequences): schedule, kernel variant,
// argument block.  `tok_base` / `tok_total`: position of this batch's first token in a PACKED cache
// that holds `tok_total` tokens per head (0 and the batch's own total when the batch is the whole
// cache).
static int build_launch(const lean_attn_problem& p, const void* q, const void* k_cache, const void* v_cache,
                        const int32_t* seqlens, void* out, float* lse, void* workspace, const lean_attn_tuning* tuning,
                        int64_t tok_base, int64_t tok_total, bool full_grid, lean_attn_plan* plan, Variant* var,
                        DecodeArgs* args) {
    const int B = p.B, D = p.D;
    DecodeArgs& a = *args;
    int rc = make_schedule(p, seqlens, tuning, plan, &a.sched, &a.table, full_grid);
    if (rc != LEAN_ATTN_OK) return rc;
    int32_t has_empty = 0;
    for (int b = 0; b < B; ++b) {
        if (seqlens[b] == 0) has_empty = 1;
    }
    if (!pick_variant(plan->kernel, p.dtype, D, tuning ? tuning->tile_shape : 0, plan->T_m, var))
        return LEAN_ATTN_ERR_UNSUPPORTED;

    const RowBlocks rb = row_blocks(p);
    a.q = (const uint16_t*)q;
    a.k = (const uint16_t*)k_cache;
    a.v = (const uint16_t*)v_cache;
    a.out = out;
    a.lse = lse;
    a.status = (uint32_t*)workspace;
    a.flags = (uint32_t*)((char*)workspace + kFlagsOffset);
    a.partials = (float*)((char*)workspace + kPartialsOffset);
    a.kv_seq_stride = p.kv_seq_stride;
    if (tok_base != 0) {
        for (int b = 0; b <= B; ++b) a.table.cu_tok[b] += (int32_t)tok_base;
    }
    a.total_rows = tok_total;
    a.Hq = p.Hq;
    a.Hkv = p.Hkv;
    a.N_q = p.N_q;
    a.ragged_q = p.q_lens ? 1 : 0;
    a.group = p.Hq / p.Hkv;
    a.rows = rb.R;
    a.C_m = rb.C_m;
    a.T_m = rb.T_m;
    a.causal = p.causal;
    a.out16 = p.out_dtype == LEAN_ATTN_OUT_AS_INPUT;
    a.slot = slot_floats(rb.T_m, D);
    a.delay_store = tuning ? tuning->debug_delay_store : 0;
    a.delay_signal = tuning ? tuning->debug_delay_signal : 0;
    a.delay_stride = tuning ? tuning->debug_delay_stride : 0;
    a.spin_limit = (tuning && tuning->spin_limit > 0) ? tuning->spin_limit : (1 << 22);
    a.has_empty = has_empty;
    // 0: the default reduction (every CTA publishes, the last few of a tile reduce a slice each)
    a.fanin = (tuning && tuning->merge_fanin >= 2) ? tuning->merge_fanin : 0;
    a.cta_clock = tuning ? (unsigned long long*)tuning->cta_clock : nullptr;
    a.scale_log2e = p.scale * 1.4426950408889634f;
    return LEAN_ATTN_OK;
}

// One launch of at most LEAN_ATTN_MAX_BATCH sequences.  With `dry` every check runs (schedule, kernel
// variant, workspace need) and nothing is launched.
static int launch_one(const lean_attn_problem& p, const void* q, const void* k_cache, const void* v_cache,
                      const int32_t* seqlens, void* out, float* lse, void* workspace, size_t workspace_bytes,
                      const lean_attn_tuning* tuning, hipStream_t stream, int64_t tok_base, int64_t tok_total,
                      bool dry, int max_grid) {
    lean_attn_plan plan;
    Variant var;
    DecodeArgs a;
    int rc = build_launch(p, q, k_cache, v_cache, seqlens, out, lse, workspace, tuning, tok_base, tok_total, false,
                          &plan, &var, &a);
    if (rc != LEAN_ATTN_OK) return rc;
    // the partial stores of CTA g land at slot g: the slab of this launch must fit the caller's buffer
    if (plan.grid > max_grid || workspace_need(plan.grid, plan.T_m, p.D) > workspace_bytes)
        return LEAN_ATTN_ERR_WORKSPACE;
    if (dry) return LEAN_ATTN_OK;
    if (plan.total_iters == 0) {  // every sequence is empty
        const int64_t rows = (int64_t)a.table.cu_q[p.B] * p.Hq;
        const int row_words = a.out16 ? p.D / 2 : p.D;
        if (rows == 0) return LEAN_ATTN_OK;
        hipLaunchKernelGGL(lean_zero_rows_kernel, dim3((unsigned)((rows * row_words + 255) / 256)), dim3(256), 0,
                           stream, (uint32_t*)out, lse, rows, row_words);
        return hipGetLastError() == hipSuccess ? LEAN_ATTN_OK : LEAN_ATTN_ERR_HIP;
    }
    void* params[] = {&a};
    if (hipLaunchKernel(var.fn, dim3(plan.grid), dim3(var.threads), params, 0, stream) != hipSuccess) {
        (void)hipGetLastError();
        return LEAN_ATTN_ERR_HIP;
    }
    return LEAN_ATTN_OK;
}

// What lean_attn_attend_prepare writes into the caller's host block and lean_attn_launch reads.
struct LaunchBlock {
    uint64_t magic;
    const void* fn;  // lean_decode_kernel_indirect<...>
    uint32_t grid, threads;
    uint64_t reserved;
    alignas(16) DecodeArgs args;  // the part that is copied to the device
};
constexpr uint64_t kBlockMagic = 0x314b4c424e41454cull;  // "LEANBLK1"

// The launches of a batch beyond LEAN_ATTN_MAX_BATCH: consecutive chunks of at most that many
// sequences on the same stream (the schedule table of one launch travels in its kernel
// arguments), sharing the workspace.  With `dry` every chunk is checked and nothing is launched.
static int launch_chunks(const lean_attn_problem& p, const void* q, const void* k_cache, const void* v_cache,
                         const int32_t* seqlens, void* out, float* lse, void* workspace, size_t workspace_bytes,
                         const lean_attn_tuning* tuning, hipStream_t stream, int64_t tok_total, bool dry,
                         int max_grid) {
    const size_t out_elem = p.out_dtype == LEAN_ATTN_OUT_AS_INPUT ? 2 : 4;
    int64_t tok_base = 0, row_base = 0;  // tokens / (query token, head) rows before the chunk
    for (int b0 = 0; b0 < p.B; b0 += LEAN_ATTN_MAX_BATCH) {
        lean_attn_problem c = p;
        c.B = p.B - b0 < LEAN_ATTN_MAX_BATCH ? p.B - b0 : LEAN_ATTN_MAX_BATCH;
        int64_t chunk_toks = 0, chunk_q = 0;
        int longest_q = 0;
        for (int b = 0; b < c.B; ++b) {
            chunk_toks += seqlens[b0 + b];
            const int q_len = p.q_lens ? p.q_lens[b0 + b] : p.N_q;
            chunk_q += q_len;
            if (q_len > longest_q) longest_q = q_len;
        }
        if (longest_q > 0) {  // (a chunk without any query token has nothing to compute)
            if (p.q_lens) {
                c.q_lens = p.q_lens + b0;
                c.N_q = longest_q;
            }
            const char* kc = (const char*)k_cache;
            const char* vc = (const char*)v_cache;
            if (p.kv_layout == LEAN_ATTN_KV_PADDED) {
                const size_t skip = (size_t)b0 * p.Hkv * (size_t)p.kv_seq_stride * p.D * 2;
                kc += skip;
                vc += skip;
            }
            const int rc = launch_one(c, (const char*)q + (size_t)row_base * p.D * 2, kc, vc, seqlens + b0,
                                      (char*)out + (size_t)row_base * p.D * out_elem, lse ? lse + row_base : nullptr,
                                      workspace, workspace_bytes, tuning, stream,
                                      p.kv_layout == LEAN_ATTN_KV_PACKED ? tok_base : 0,
                                      p.kv_layout == LEAN_ATTN_KV_PACKED ? tok_total : chunk_toks, dry, max_grid);
            if (rc != LEAN_ATTN_OK) return rc;
        }
        tok_base += chunk_toks;
        row_base += chunk_q * p.Hq;
    }
    return LEAN_ATTN_OK;
}

// lean_attn_attend on a workspace the caller or the library provides.
static int attend_on(const lean_attn_problem* problem, const void* q, const void* k_cache, const void* v_cache,
                     const int32_t* seqlens, void* out, float* lse, void* workspace, size_t workspace_bytes,
                     const lean_attn_tuning* tuning, void* hip_stream, bool dry = false,
                     int max_grid = LEAN_ATTN_MAX_GRID) {
    if (!problem || !q || !k_cache || !v_cache || !seqlens || !out || !workspace) return LEAN_ATTN_ERR_NULL_POINTER;
    const lean_attn_problem& p = *problem;
    int rc = check_problem(p, true);
    if (rc != LEAN_ATTN_OK) return rc;
    if ((((uintptr_t)q | (uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)out) & 15) != 0)
        return LEAN_ATTN_ERR_BAD_SHAPE;
    if (((uintptr_t)workspace & 255) != 0 || workspace_bytes < kPartialsOffset) return LEAN_ATTN_ERR_WORKSPACE;
    // every length and every launch is checked before the first launch: on error nothing runs
    int64_t tok_total = 0;
    rc = check_lengths(p, seqlens, &tok_total);
    if (rc != LEAN_ATTN_OK) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;
    if (p.B <= LEAN_ATTN_MAX_BATCH)
        return launch_one(p, q, k_cache, v_cache, seqlens, out, lse, workspace, workspace_bytes, tuning, stream, 0,
                          tok_total, dry, max_grid);
    rc = launch_chunks(p, q, k_cache, v_cache, seqlens, out, lse, workspace, workspace_bytes, tuning, stream,
                       tok_total, true, max_grid);
    if (rc != LEAN_ATTN_OK || dry) return rc;
    return launch_chunks(p, q, k_cache, v_cache, seqlens, out, lse, workspace, workspace_bytes, tuning, stream,
                         tok_total, false, max_grid);
}

int lean_attn_attend(const lean_attn_problem* problem, const void* q, const void* k_cache, const void* v_cache,
                     const int32_t* seqlens, void* out, float* lse, void* workspace, size_t workspace_bytes,
                     const lean_attn_tuning* tuning, void* hip_stream) {
    return attend_on(problem, q, k_cache, v_cache, seqlens, out, lse, workspace, workspace_bytes, tuning, hip_stream);
}

size_t lean_attn_launch_block_size(void) { return sizeof(LaunchBlock); }

int lean_attn_attend_prepare(const lean_attn_problem* problem, const void* q, const void* k_cache,
                             const void* v_cache, const int32_t* seqlens, void* out, float* lse, void* workspace,
                             size_t workspace_bytes, const lean_attn_tuning* tuning, void* block_host) {
    if (!problem || !q || !k_cache || !v_cache || !seqlens || !out || !workspace || !block_host)
        return LEAN_ATTN_ERR_NULL_POINTER;
    const lean_attn_problem& p = *problem;
    int rc = check_problem(p);  // one launch: at most LEAN_ATTN_MAX_BATCH sequences
    if (rc != LEAN_ATTN_OK) return rc;
    if ((((uintptr_t)q | (uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)out | (uintptr_t)block_host) & 15) != 0)
        return LEAN_ATTN_ERR_BAD_SHAPE;
    if (((uintptr_t)workspace & 255) != 0 || workspace_bytes < kPartialsOffset) return LEAN_ATTN_ERR_WORKSPACE;
    if (tuning && (tuning->fixed_split != 0 || tuning->tile_shape != 0 || tuning->tail_grid != 0)) return LEAN_ATTN_ERR_TUNING;
    int64_t tok_total = 0;
    rc = check_lengths(p, seqlens, &tok_total);
    if (rc != LEAN_ATTN_OK) return rc;
    LaunchBlock blk;  // built aside: the caller's block is only touched when everything is valid
    lean_attn_plan plan;
    Variant var;
    rc = build_launch(p, q, k_cache, v_cache, seqlens, out, lse, workspace, tuning, 0, tok_total, true, &plan, &var,
                      &blk.args);
    if (rc != LEAN_ATTN_OK) return rc;
    if (workspace_need(plan.grid, plan.T_m, p.D) > workspace_bytes) return LEAN_ATTN_ERR_WORKSPACE;
    if (!var.fn_indirect) return LEAN_ATTN_ERR_UNSUPPORTED;
    blk.magic = kBlockMagic;
    blk.fn = var.fn_indirect;
    blk.grid = (uint32_t)plan.grid;
    blk.threads = (uint32_t)var.threads;
    blk.reserved = 0;
    std::memcpy(block_host, &blk, sizeof blk);
    return LEAN_ATTN_OK;
}

int lean_attn_launch(const void* block_host, void* block_device, void* hip_stream) {
    if (!block_host || !block_device) return LEAN_ATTN_ERR_NULL_POINTER;
    if ((((uintptr_t)block_host | (uintptr_t)block_device) & 15) != 0) return LEAN_ATTN_ERR_BAD_SHAPE;
    const LaunchBlock* blk = static_cast<const LaunchBlock*>(block_host);
    if (blk->magic != kBlockMagic || !blk->fn || blk->grid == 0 || blk->grid > LEAN_ATTN_MAX_GRID)
        return LEAN_ATTN_ERR_BAD_SHAPE;
    hipStream_t stream = (hipStream_t)hip_stream;
    if (hipMemcpyAsync(block_device, &blk->args, sizeof(DecodeArgs), hipMemcpyHostToDevice, stream) != hipSuccess) {
        (void)hipGetLastError();
        return LEAN_ATTN_ERR_HIP;
    }
    void* params[] = {&block_device};
    if (hipLaunchKernel(blk->fn, dim3(blk->grid), dim3(blk->threads), params, 0, stream) != hipSuccess) {
        (void)hipGetLastError();
        return LEAN_ATTN_ERR_HIP;
    }
    return LEAN_ATTN_OK;
}

int lean_attn_decode(const void* q, const void* k_cache, const void* v_cache, const int32_t* seqlens, float* out,
                     float* lse, void* workspace, size_t workspace_bytes, int B, int Hq, int Hkv, int D,
                     int kv_layout, int64_t kv_seq_stride, float scale, int dtype, const lean_attn_tuning* tuning,
                     void* hip_stream) {
    const lean_attn_problem p = decode_problem(B, Hq, Hkv, D, dtype, kv_layout, kv_seq_stride, scale);
    return lean_attn_attend(&p, q, k_cache, v_cache, seqlens, out, lse, workspace, workspace_bytes, tuning,
                            hip_stream);
}

// ---- lean_attn_decode for callers that cannot allocate: the workspace is a static device array ----
// Two partial slots of the largest tile (32 rows at D = 128, 16 at D = 256) for each of
// LEAN_ATTN_STATIC_MAX_GRID workgroups plus the flags: 17.3 MB, held by every GPU the library runs
// on until the process ends.
constexpr size_t kStaticScratchBytes =
    kPartialsOffset + 2 * (size_t)LEAN_ATTN_STATIC_MAX_GRID * 4160 * sizeof(float);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
// In host code `scratch` is only a handle for the runtime's symbol look-up, never an address a
// kernel may be given: the array's device address is read once per device and kept here.
static void* g_scratch_ptr[64];
static std::mutex g_scratch_mutex;

static int static_scratch(void** ptr) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return LEAN_ATTN_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {  // each device holds its own copy of the array at its own address
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return LEAN_ATTN_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return LEAN_ATTN_OK;
}

int lean_attn_decode_static(const void* q, const void* k_cache, const void* v_cache, const int32_t* seqlens,
                            float* out, float* lse, int B, int Hq, int Hkv, int D, int kv_layout,
                            int64_t kv_seq_stride, float scale, int dtype, const lean_attn_tuning* tuning,
                            void* hip_stream) {
    static_assert(slot_floats_max() <= 4160, "the static scratch holds the largest partial slot");
    const lean_attn_problem p = decode_problem(B, Hq, Hkv, D, dtype, kv_layout, kv_seq_stride, scale);
    void* ws = nullptr;
    int rc = static_scratch(&ws);
    if (rc != LEAN_ATTN_OK) return rc;
    // every check first, so that on error nothing is launched, not even the clearing below
    rc = attend_on(&p, q, k_cache, v_cache, seqlens, out, lse, ws, kStaticScratchBytes, tuning, hip_stream, true,
                   LEAN_ATTN_STATIC_MAX_GRID);
    if (rc == LEAN_ATTN_ERR_WORKSPACE) return LEAN_ATTN_ERR_STATIC_LIMIT;
    if (rc != LEAN_ATTN_OK) return rc;
    // The array keeps what the last call left.  A call that ran to its end left every flag cleared,
    // one that gave up waiting may not have: the status word and the flags start at zero every time
    // (a fill kernel, not a memset: the call may be under graph capture).
    // (launches from here never exceed LEAN_ATTN_STATIC_MAX_GRID workgroups: only their flag words are used)
    const int n = (int)((kFlagsOffset + 4 * kFlagWordsPerCta * LEAN_ATTN_STATIC_MAX_GRID) / 4);
    hipLaunchKernelGGL(lean_workspace_clear_kernel, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)hip_stream,
                       (uint32_t*)ws, n);
    if (hipGetLastError() != hipSuccess) return LEAN_ATTN_ERR_HIP;
    return attend_on(&p, q, k_cache, v_cache, seqlens, out, lse, ws, kStaticScratchBytes, tuning, hip_stream, false,
                     LEAN_ATTN_STATIC_MAX_GRID);
}

int lean_attn_read_probe(const void* buf, size_t bytes, void* sink, int grid, int mode, void* hip_stream) {
    if (!buf || !sink) return LEAN_ATTN_ERR_NULL_POINTER;
    if (bytes == 0 || (bytes & 15) != 0 || ((uintptr_t)buf & 15) != 0 || grid <= 0 || grid > 65535 || mode < 0 ||
        mode > kMaxProbeMode)
        return LEAN_ATTN_ERR_BAD_SHAPE;
    hipLaunchKernelGGL(lean_read_probe_kernel, dim3(grid), dim3(256), 0, (hipStream_t)hip_stream, (const uint4*)buf,
                       (int64_t)(bytes / 16), (uint32_t*)sink, mode);
    return hipGetLastError() == hipSuccess ? LEAN_ATTN_OK : LEAN_ATTN_ERR_HIP;
}

const char* lean_attn_strerror(int status) {
    switch (status) {
        case LEAN_ATTN_OK: return "ok";
        case LEAN_ATTN_ERR_NULL_POINTER: return "a required pointer is null";
        case LEAN_ATTN_ERR_BAD_SHAPE: return "bad shape: B, N_q, Hq, Hkv must be positive, Hq a multiple of Hkv, at most 256 query rows per KV head, 16-byte aligned tensors";
        case LEAN_ATTN_ERR_UNSUPPORTED: return "unsupported head dim (64, 128, 256), dtype (f16, bf16), output type, layout, or a tile shape that is not built for this core and head dim";
        case LEAN_ATTN_ERR_WORKSPACE: return "workspace missing, not 256-byte aligned, or too small for the flags and two partial slots per workgroup of the launch";
        case LEAN_ATTN_ERR_SEQLEN: return "negative sequence length, padded stride below the longest sequence, or more than 2^31 tokens";
        case LEAN_ATTN_ERR_BATCH_TOO_LARGE: return "batch larger than LEAN_ATTN_MAX_BATCH";
        case LEAN_ATTN_ERR_HIP: return "a HIP runtime call failed";
        case LEAN_ATTN_ERR_TUNING: return "tuning field out of range";
        case LEAN_ATTN_ERR_PEER_TIMEOUT: return "a host workgroup gave up waiting for a peer's partial";
        case LEAN_ATTN_ERR_STATIC_LIMIT: return "the launch needs more partial slots than the static scratch of lean_attn_decode_static holds (LEAN_ATTN_STATIC_MAX_GRID workgroups)";
        default: return "unknown status";
    }
}

}  // extern "C"
