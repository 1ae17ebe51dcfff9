/*
 * lean_attn.h -- C ABI of the MI355X (gfx950) LeanAttention decode library.
 *
 * Decode-phase attention (Section 2.1, Eq. 1 with N_q = 1; Table 1, decode
 * column): for every sequence b and query head h_q one query row attends over
 * the N_b cached K/V rows of KV head h_q / (Hq / Hkv):
 *
 *     out[b,h_q,:] = softmax(scale * q[b,h_q,:] . K[b,h,:N_b,:]^T) V[b,h,:N_b,:]
 *
 * lean_attn_attend generalises this to short query tiles (N_q > 1 rows per
 * sequence, Algorithm 2's C_m output tiles along the query dimension).
 *
 * The work is decomposed stream-K style (Section 4.3): the LeanTile iterations
 * of all (sequence, KV head) output tiles are laid on one line and cut into
 * equal contiguous spans, one per workgroup of a persistent grid; partial
 * (O~, m, l) triples are merged with the softmax re-scaling operator of
 * Section 4.1 inside the same launch (Algorithm 2).
 *
 * One deliberate difference from Algorithm 2: there the host block (the CTA
 * that computed a tile's first LeanTile) merges every peer in a flat loop.
 * Here every CTA of a shared tile publishes its partial, and the tile's last
 * 1..8 CTAs each merge one slice of the tile from all partials and write it
 * (lean_attn_tuning.merge_fanin selects a reduction tree rooted at the
 * FINISHING block instead, the CTA whose span holds the tile's last LeanTile).
 * The operator is associative and commutative (Section 4.1), so the result is
 * the same.  "host_block" in lean_attn_walk keeps Algorithm 2's meaning (first
 * LeanTile of the tile), it no longer says who reduces.
 *
 * All pointers named "device" are HIP device pointers on the current device;
 * "host" pointers are ordinary host memory.  No function takes ownership of
 * any buffer and no function allocates device memory.  Calls are asynchronous
 * on the given stream unless stated otherwise.  Every function returns
 * LEAN_ATTN_OK (0) or a negative lean_attn_status; on error nothing is
 * launched.  No exception or abort crosses this boundary.
 */
#ifndef LEAN_ATTN_H_
#define LEAN_ATTN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum lean_attn_status {
    LEAN_ATTN_OK = 0,
    LEAN_ATTN_ERR_NULL_POINTER = -1,  /* a required pointer is NULL */
    LEAN_ATTN_ERR_BAD_SHAPE = -2,     /* B, N_q, Hq, Hkv <= 0, Hq % Hkv != 0, too many query rows per KV head */
    LEAN_ATTN_ERR_UNSUPPORTED = -3,   /* head dim / dtype / layout not built */
    LEAN_ATTN_ERR_WORKSPACE = -4,     /* workspace missing, misaligned or too small */
    LEAN_ATTN_ERR_SEQLEN = -5,        /* a negative length, N_b*D*2 >= 2^31 bytes, a padded stride below the longest,
                                         or (causal) 0 < N_b < N_q */
    LEAN_ATTN_ERR_BATCH_TOO_LARGE = -6, /* B > LEAN_ATTN_MAX_BATCH in a schedule query */
    LEAN_ATTN_ERR_HIP = -7,           /* a HIP runtime call failed (no device, bad stream, ...) */
    LEAN_ATTN_ERR_TUNING = -8,        /* a lean_attn_tuning field is out of range */
    LEAN_ATTN_ERR_PEER_TIMEOUT = -9,  /* reported by lean_attn_workspace_status only */
    LEAN_ATTN_ERR_STATIC_LIMIT = -10  /* lean_attn_decode_static: the launch exceeds the static scratch */
} lean_attn_status;

/* Element type of q, k_cache and v_cache. */
typedef enum lean_attn_dtype { LEAN_ATTN_F16 = 0, LEAN_ATTN_BF16 = 1 } lean_attn_dtype;

/* Element type of out: fp32, or the 16-bit type of the inputs (rounded to nearest even). */
typedef enum lean_attn_out_dtype { LEAN_ATTN_OUT_F32 = 0, LEAN_ATTN_OUT_AS_INPUT = 1 } lean_attn_out_dtype;

/*
 * KV-cache layouts.
 * PADDED: [B, Hkv, kv_seq_stride, D]; row t of (b, h) starts at element
 *         ((b*Hkv + h)*kv_seq_stride + t)*D.  This is the constant-head-stride
 *         view Section 4.3 requires.  Rows t >= N_b are never read.
 * PACKED: [Hkv, sum_b N_b, D], no batch dimension; sequence b starts at row
 *         cu[b] = sum_{b'<b} N_b' (the ragged form of Section 4.3, "Lean Ragged
 *         Batching").  kv_seq_stride is ignored.
 */
typedef enum lean_attn_kv_layout { LEAN_ATTN_KV_PADDED = 0, LEAN_ATTN_KV_PACKED = 1 } lean_attn_kv_layout;

#define LEAN_ATTN_MAX_BATCH 256  /* sequences per launch (the schedule table travels as kernel arguments);
                                    lean_attn_decode / lean_attn_attend split larger batches into
                                    consecutive launches, the schedule queries describe one launch */
#define LEAN_ATTN_MAX_TILE_ROWS 32    /* query rows of one output tile: two MFMA row blocks (one, 16 rows, at D = 256) */
#define LEAN_ATTN_MAX_QUERY_ROWS 256  /* N_q * Hq / Hkv: query rows that share one KV head */
#define LEAN_ATTN_MAX_GRID 4096  /* upper bound on workgroups; sizes the workspace */
#define LEAN_ATTN_STATIC_MAX_GRID 512  /* workgroups per launch of lean_attn_decode_static */
#define LEAN_ATTN_NUM_TILE_SHAPES 9  /* lean_attn_tuning.tile_shape runs 1..9; not every shape exists for every core */

/*
 * The stream-K schedule of one call (Section 4.3 and the first lines of
 * Algorithm 2).  The R = N_q * Hq / Hkv query rows that share a KV head (row =
 * query token * (Hq / Hkv) + head within the group) are cut into
 * C_m = ceil(R / 32) blocks (ceil(R / 16) at D = 256) of T_m = ceil(R / C_m) rows
 * (the last may hold fewer).
 * Output tile = one (sequence, KV head, row block); it owns ceil(N_b / T_n)
 * LeanTile iterations.  CTA g owns iterations
 * [g*iters_per_cta + min(g, extra), ... + iters_per_cta + (g < extra))
 * (see tail_grid for the optional short spans at the end of the line).
 * For decode with up to 32 query heads per KV head, C_m = 1 and T_m = Hq / Hkv.
 */
typedef struct lean_attn_plan {
    int32_t T_n;              /* LeanTile size in tokens */
    int32_t T_m;              /* query rows per output tile */
    int32_t num_output_tiles; /* B * Hkv * C_m, including tiles of empty sequences */
    int32_t grid;             /* G: workgroups launched, <= total_iters */
    int64_t total_iters;      /* I: LeanTile iterations over all output tiles */
    int64_t iters_per_cta;    /* floor(I / G) */
    int32_t extra;            /* I mod G: the first `extra` CTAs take one more iteration */
    int32_t block_threads;    /* workgroup size */
    int32_t max_resident;     /* compute units x workgroups resident per unit */
    int32_t kernel;           /* 0 = VALU single-row kernel (one query row per KV head), 1 = MFMA kernel */
    int32_t fixed_split;      /* 0: stream-K spans; s >= 1: baseline schedule, s parts per output tile,
                                 CTA g = tile_idx*s + part, grid = num_output_tiles*s */
    int32_t C_m;              /* row blocks per KV head */
    int32_t tile_shape;       /* the compiled tile shape used, 1..9 (lean_attn_tuning.tile_shape, or the library's
                                 default for this head dim, dtype and T_m) */
    int32_t tail_grid;        /* P: the last P of the `grid` workgroups own short spans (0: none).  Then
                                 iters_per_cta and extra describe the first G = grid - P workgroups, which share
                                 the first total_iters - tail_iters iterations, and workgroup G + j owns
                                 floor(tail_iters / P) (+ 1 for j < tail_iters mod P) of the last tail_iters */
    int64_t tail_iters;
} lean_attn_plan;

/*
 * Optional overrides, for tests and sweeps.  A zero field means "library
 * default".  Results never depend on these (Section 4.1: any split gives the
 * same attention output); only the balance does.
 */
typedef struct lean_attn_tuning {
    int32_t grid;          /* force G (clipped to I and to LEAN_ATTN_MAX_GRID) */
    int32_t ctas_per_cu;   /* workgroups per compute unit used to size the default G */
    int32_t num_cus;       /* pretend the device has this many compute units (schedule queries) */
    int32_t kernel;        /* 0 default, 1 force VALU kernel (needs N_q * Hq == Hkv), 2 force MFMA kernel */
    int32_t tail_grid;     /* 0: none.  P > 0: the last share of the iteration line is cut into P short spans for P
                              further workgroups (grid = G + P), which the hardware starts as the first G retire:
                              a static decomposition that still lets the faster units take more of the tail.
                              Ignored when the problem is too small; not with fixed_split or lean_attn_attend_prepare */
    int32_t spin_limit;    /* polls before a waiting CTA gives up and reports PEER_TIMEOUT */
    int32_t merge_fanin;   /* 0 default: every CTA of a shared tile publishes its partial and the tile's last
                              1..8 CTAs each merge one slice of all partials and write it (one level).
                              >= 2: the reduction is a tree of this fan-in rooted at the finishing block;
                              >= LEAN_ATTN_MAX_GRID gives Algorithm 2's flat list: one block merges every
                              peer itself */
    int32_t tile_shape;    /* 0: the library's default for the head dim, dtype and rows per tile (a table filled
                              from the LeanTile sweep); 1..6: a compiled (loads or token blocks per wave, waves
                              per workgroup, buffering) shape, i.e. another LeanTile size T_n; 7..9: shapes of
                              the matrix-core kernels that stage K and V in LDS (D = 128: all three, D = 256:
                              7 and 8); a shape that is not built gives LEAN_ATTN_ERR_UNSUPPORTED.
                              lean_attn_schedule reports T_n and the shape used */
    int32_t grid_multiple; /* default G = units x ctas_per_cu x grid_multiple (0: library default) */
    int32_t fixed_split;   /* 0: LeanAttention's stream-K spans.  Baseline schedules of Sections 3.3 / 4.3:
                              s >= 1 cuts every output tile into s near-equal parts (s = 1: no split,
                              the FlashAttention-2 schedule), -1 picks s = units*ctas_per_cu / tiles */
    int32_t debug_delay_store;  /* tests: publishing workgroups sleep this many periods (about 3.4 us each, at
                                   most 64) before they store their partial ... */
    int32_t debug_delay_signal; /* ... and this many between the acknowledged stores and the flag store
                                   (widens the window between StorePartials and Signal of Algorithm 2) */
    int32_t debug_delay_stride; /* only workgroups with id % stride == stride - 1 sleep (0 or 1: all of them) */
    int32_t tail_permille;      /* share of the iterations the tail spans cover, in 1/1000 (0: library default, max 500) */
    void* cta_clock;       /* device, 16 uint64 per CTA of the grid, or NULL: 100 MHz timestamps
                              [0] kernel entry, [1] end of the span loop, [2] first segment located, [3] exit,
                              [7] first LeanTile iteration done, [8] first segment streamed, [9] partial stores
                              issued, [10] stores acknowledged, [11] peers' flags seen, [12] peers merged,
                              [13] output written; [4] HW_ID, [5] XCC_ID registers, [6] the workgroup id */
} lean_attn_tuning;

/*
 * One attention problem, for lean_attn_attend and its companions.  q, out and
 * lse are indexed [B, N_q, Hq]; the N_q query rows of a sequence are its LAST
 * N_q cached tokens (their K/V rows are already in the cache, N_b counts them).
 *   causal = 0: every query row attends to all N_b cached rows;
 *   causal = 1: query row i attends to the first N_b - N_q + i + 1 cached rows
 *               (the decoder mask, aligned to the end of the context; the paper
 *               does not discuss masks).  Needs N_b >= N_q or N_b == 0.
 * Every output tile of up to 32 query rows (16 at D = 256) streams the K/V of its
 * head once: beyond that the K/V traffic grows by C_m.  This is a decode-phase
 * path for short query tiles (speculative decoding, chunked prefill tails), not
 * a prefill kernel.  Limits: N_q * Hq / Hkv <= LEAN_ATTN_MAX_QUERY_ROWS.
 */
typedef struct lean_attn_problem {
    int32_t B;             /* sequences */
    int32_t N_q;           /* query rows per sequence, >= 1 */
    int32_t Hq;            /* query heads */
    int32_t Hkv;           /* KV heads, divides Hq */
    int32_t D;             /* head dim: 64, 128 or 256 */
    int32_t dtype;         /* lean_attn_dtype of q, k_cache, v_cache */
    int32_t out_dtype;     /* lean_attn_out_dtype */
    int32_t kv_layout;     /* lean_attn_kv_layout */
    int32_t causal;        /* 0 or 1 */
    float scale;           /* multiplies q.k before the softmax */
    int64_t kv_seq_stride; /* PADDED layout: rows between consecutive (b, h) slabs */
    const int32_t* q_lens; /* HOST, B entries, or NULL.  Per-sequence query lengths (mixed prefill and
                              decode batches): sequence b has q_lens[b] in [0, N_q] query rows, its last
                              q_lens[b] cached tokens, and N_q must equal the longest.  q, out and lse
                              are then packed: [sum_b q_lens[b], Hq, ...], sequence after sequence.
                              The schedule is that of N_q rows for every sequence; the row blocks a
                              shorter sequence does not reach are skipped (their K/V is not read),
                              which unbalances the spans once N_q * Hq / Hkv exceeds one output tile. */
} lean_attn_problem;

/*
 * Bytes of device workspace that suffice for lean_attn_decode on this problem
 * shape whatever the tuning: arrival flags plus partial (O~[T_m, D], m[T_m],
 * l[T_m]) slots as in Algorithm 2 ("Op[g], mp[g], lp[g], flags[g]"), two per CTA
 * (a span can start inside one shared tile and end inside another), for
 * LEAN_ATTN_MAX_GRID CTAs.  Host-only arithmetic; it does not depend on
 * the device.  Returns 0 for an unsupported shape.
 */
size_t lean_attn_workspace_size(int B, int Hq, int Hkv, int D, int dtype);

/* The same for the problem lean_attn_attend is given.  Returns 0 for an unsupported problem. */
size_t lean_attn_problem_workspace_size(const lean_attn_problem* problem);

/*
 * The workspace for launches of at most `max_grid` workgroups (1..LEAN_ATTN_MAX_GRID): a launch
 * needs the flags plus 2 x `grid` partial slots, and every entry point checks exactly that against
 * workspace_bytes (LEAN_ATTN_ERR_WORKSPACE otherwise, nothing launched).  The default grid is
 * compute units x 1, or x 2 for batches of many short contexts (lean_attn_plan.grid tells), so a
 * caller that never forces a larger grid can allocate for 2 x the unit count instead of
 * LEAN_ATTN_MAX_GRID (e.g. 17 MB instead of 136 MB for 32-row tiles at D = 128 on 256 units).
 * Returns 0 for an unsupported problem or grid.
 */
size_t lean_attn_workspace_size_for_grid(const lean_attn_problem* problem, int max_grid);

/*
 * Clear the flags of a freshly allocated workspace (device pointer, 256-byte
 * aligned).  Needed once per allocation: every decode call leaves the flags
 * cleared again.  A workspace must not be shared by two calls in flight.
 */
int lean_attn_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Blocking: waits for `hip_stream`, then reports LEAN_ATTN_ERR_PEER_TIMEOUT if
 * a merging CTA of an earlier call on this workspace gave up waiting for a peer
 * (after tuning->spin_limit polls or half a second; its output rows are then
 * invalid), else LEAN_ATTN_OK.  Clears the report and, after a timeout, all
 * flags, so the workspace can be used again.
 */
int lean_attn_workspace_status(void* workspace, void* hip_stream);

/*
 * Host-only: the schedule lean_attn_decode would use.  `seqlens` is a host
 * array of B context lengths (N_b counts the current token, whose K/V row is
 * already in the cache).  With tuning->num_cus > 0 no device is queried, so
 * this runs without a GPU.  `tuning` may be NULL.
 */
int lean_attn_schedule(const int32_t* seqlens, int B, int Hq, int Hkv, int D, int dtype,
                       int kv_layout, const lean_attn_tuning* tuning, lean_attn_plan* plan);

/* Host-only: the schedule lean_attn_attend would use for `problem` (see lean_attn_schedule). */
int lean_attn_problem_schedule(const lean_attn_problem* problem, const int32_t* seqlens,
                               const lean_attn_tuning* tuning, lean_attn_plan* plan);

/*
 * Host-only: the output-tile segments CTA `g` walks under `plan` (the loop of
 * Algorithm 2), computed by the same code the kernel runs.  Writes up to
 * `max_segments` records of 8 int64 each:
 *   {tile_idx, b, head, local_iter, local_iter_end, host_block, finishing_block, last_cta}
 * (head = kv_head * plan->C_m + row block; last_cta: the last CTA contributing to the
 * tile; the first one is the host block) and returns the number of segments, or a
 * negative status.
 */
int lean_attn_walk(const lean_attn_plan* plan, const int32_t* seqlens, int B, int Hkv,
                   int kv_layout, int g, int64_t* segments, int max_segments);

/*
 * Decode attention.
 *   q        device, [B, Hq, D], 16-bit elements of `dtype`, contiguous
 *   k_cache  device, layout per `kv_layout`, same element type
 *   v_cache  device, same layout as k_cache
 *   seqlens  HOST, B int32 context lengths N_b >= 0 (N_b = 0: that row's out is 0, lse -inf)
 *   out      device, [B, Hq, D] fp32
 *   lse      device, [B, Hq] fp32, or NULL: L = m + log(l) of Algorithm 2
 *   workspace, workspace_bytes  device scratch from lean_attn_workspace_size, initialised once
 *   kv_seq_stride  rows between consecutive (b, h) slabs in the PADDED layout
 *   scale    multiplies q.k before the softmax (1/sqrt(D) in Eq. 1)
 *   tuning   NULL for defaults
 * Supported: D in {64, 128, 256}, both dtypes, Hq/Hkv <= LEAN_ATTN_MAX_QUERY_ROWS,
 * any B (batches beyond LEAN_ATTN_MAX_BATCH run as consecutive launches on the stream, sharing
 * the workspace).  Same as lean_attn_attend with N_q = 1 and fp32 output.
 * q, k_cache, v_cache and out must be 16-byte aligned.
 * The first call per device and kernel variant reads the device's unit count and the
 * kernel's residency from the runtime (cached afterwards): make it outside graph capture.
 * The schedule is computed on the host from seqlens and travels in the kernel arguments, so a
 * launch captured into a HIP graph keeps the lengths it was captured with: re-capture (or
 * update the kernel node) when they change.
 */
int lean_attn_decode(const void* q, const void* k_cache, const void* v_cache,
                     const int32_t* seqlens, float* out, float* lse, void* workspace,
                     size_t workspace_bytes, int B, int Hq, int Hkv, int D, int kv_layout,
                     int64_t kv_seq_stride, float scale, int dtype, const lean_attn_tuning* tuning,
                     void* hip_stream);

/*
 * lean_attn_decode for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels and results as lean_attn_decode, without `workspace` / `workspace_bytes`: the
 * flags and partial slots live in a static device array inside the library (17.3 MB per GPU, held
 * until the process ends), enough for LEAN_ATTN_STATIC_MAX_GRID workgroups with the largest
 * partial slot.  The default grid (compute units x 1 or x 2) fits on devices of up to 256 units;
 * a launch that needs more slots (a larger device, tuning->grid, grid_multiple or fixed_split
 * beyond the limit) returns LEAN_ATTN_ERR_STATIC_LIMIT and launches nothing.  No hipMalloc,
 * hipFree or other allocating call is made.  The status word and flags are cleared by a small
 * fill kernel at the start of every call.  All calls on one GPU share the one array: calls that
 * overlap on a GPU (two streams, two threads) race; serialise them or use lean_attn_decode with
 * a workspace per stream.  A peer time-out cannot be queried here (the output rows of the tile
 * are then invalid, as for lean_attn_decode); it needs tuning->spin_limit set far below its
 * default to happen on a healthy device.  The first call on a device reads the array's address,
 * the device's unit count and the kernel's residency from the runtime: make it outside capture.
 */
int lean_attn_decode_static(const void* q, const void* k_cache, const void* v_cache,
                            const int32_t* seqlens, float* out, float* lse, int B, int Hq, int Hkv,
                            int D, int kv_layout, int64_t kv_seq_stride, float scale, int dtype,
                            const lean_attn_tuning* tuning, void* hip_stream);

/*
 * Attention of short query tiles over the KV cache (Algorithm 2 with C_m >= 1).
 *   problem  host, see lean_attn_problem
 *   q        device, [B, N_q, Hq, D] (packed [sum q_lens, Hq, D] with problem->q_lens), 16-bit
 *            elements of problem->dtype, contiguous
 *   k_cache, v_cache, seqlens, workspace, tuning, hip_stream  as for lean_attn_decode;
 *            the workspace size comes from lean_attn_problem_workspace_size
 *   out      device, shaped like q, fp32 or 16-bit per problem->out_dtype
 *   lse      device, [B, N_q, Hq] ([sum q_lens, Hq]) fp32, or NULL
 * Rows of a sequence with N_b = 0 get out = 0, lse = -inf.
 */
int lean_attn_attend(const lean_attn_problem* problem, const void* q, const void* k_cache,
                     const void* v_cache, const int32_t* seqlens, void* out, float* lse,
                     void* workspace, size_t workspace_bytes, const lean_attn_tuning* tuning,
                     void* hip_stream);

/*
 * The same attention as lean_attn_attend, split in two for callers that replay a captured HIP
 * graph while the sequence lengths change from step to step (a decode loop).
 *
 * lean_attn_attend_prepare is host-only: it validates the call, computes the schedule and writes
 * everything the kernel needs into `block_host` (lean_attn_launch_block_size() bytes, 16-byte
 * aligned; pinned host memory, e.g. hipHostMalloc, when lean_attn_launch is captured).  Nothing
 * is launched.  Limits beyond lean_attn_attend's: B <= LEAN_ATTN_MAX_BATCH, tuning->tile_shape
 * and tuning->fixed_split must be 0.  The launch shape written into the block depends only on
 * the problem shape, never on seqlens: one workgroup per compute unit, surplus workgroups own
 * empty spans.
 *
 * lean_attn_launch copies the block's arguments to `block_device` (device memory of the same
 * size, asynchronously on the stream) and launches the kernel, which reads them from there.  Both
 * steps can be captured.  To run new lengths through the same graph: wait until the previous
 * replay has started its kernel (e.g. finished), call lean_attn_attend_prepare again with the
 * same problem shape, buffers and block, replay.  On error nothing is launched and the block is
 * left as it was.
 */
size_t lean_attn_launch_block_size(void);
int lean_attn_attend_prepare(const lean_attn_problem* problem, const void* q, const void* k_cache,
                             const void* v_cache, const int32_t* seqlens, void* out, float* lse,
                             void* workspace, size_t workspace_bytes, const lean_attn_tuning* tuning,
                             void* block_host);
int lean_attn_launch(const void* block_host, void* block_device, void* hip_stream);

/*
 * Measurement helper: one pass of 16-byte loads over `bytes` of device memory
 * by `grid` workgroups of 256 threads, without any arithmetic.  mode 0: each
 * workgroup reads one contiguous share (the access pattern of contiguous
 * stream-K spans); mode 1: the workgroups sweep the buffer together in 32 KiB
 * chunks dealt round-robin; modes 2, 3, 4: as mode 0 through a buffer descriptor
 * with cache policy nt, sc1, sc0|sc1 on the loads; mode 5: non-temporal 16-byte pieces
 * strided over 16 rows of 256 bytes per wave-wide load (the operand pattern the MFMA
 * core avoids by staging K through LDS); mode 6: non-temporal half rows (256 bytes) of four
 * consecutive 512-byte rows per wave-wide load (the K/V pattern of the MFMA core at D = 256).  Used to report the streaming-read ceiling of the
 * machine next to the decode rate.  `sink` is a device pointer to at least
 * 4 bytes.  bytes must be a multiple of 16.
 */
int lean_attn_read_probe(const void* buf, size_t bytes, void* sink, int grid, int mode, void* hip_stream);

/* Static description of a status code. */
const char* lean_attn_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* LEAN_ATTN_H_ */
