// Device-side building blocks shared by the two decode cores: kernel argument
// block, workspace layout, 16-bit element handling, cross-lane reductions and
// the arrival-flag protocol of Algorithm 2 (StorePartials / Signal / Wait).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lean_sched.h"

namespace lean {

constexpr int kDtF16 = 0;
constexpr int kDtBF16 = 1;
constexpr int kMaxGrid = 4096;

// Workspace layout (bytes): [0,256) status word, then the arrival flags, then the partial slots of
// slot_floats floats each: O~[T_m][D], m[T_m], l[T_m].
// A CTA can hold parts of two output tiles that other CTAs share: the one its span starts in the
// middle of, and the one its span ends in the middle of.  It publishes a partial for each, so
// every CTA owns two slots: slot 2g for a tile that began in an earlier CTA, slot 2g + 1 for a
// tile it began itself.  Every slot has kMaxReducers flag words, one per CTA that may read it
// (each word has exactly one reader, which clears it).
constexpr int kMaxReducers = 8;
constexpr size_t kFlagsOffset = 256;
constexpr size_t kFlagWordsPerCta = 2 * kMaxReducers;
constexpr size_t kPartialsOffset = kFlagsOffset + 4 * kFlagWordsPerCta * (size_t)kMaxGrid;
__host__ __device__ inline int slot_of(int cta, int first_cta) { return 2 * cta + (cta == first_cta ? 1 : 0); }

inline __host__ __device__ int slot_floats(int T_m, int D) {
    const int n = T_m * (D + 2);
    return (n + 63) & ~63;  // 256-byte slots
}

// The largest slot any supported tile needs: 32 rows at D = 128 or 16 rows at D = 256.
constexpr int slot_floats_max() {
    constexpr int a = (32 * (128 + 2) + 63) & ~63, b = (16 * (256 + 2) + 63) & ~63, c = (32 * (64 + 2) + 63) & ~63;
    return a > b ? (a > c ? a : c) : (b > c ? b : c);
}

struct DecodeArgs {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    void* out;             // [B, N_q, Hq, D], fp32 or (out16) the element type of q
    float* lse;            // [B, N_q, Hq], may be null
    uint32_t* status;      // workspace + 0
    uint32_t* flags;       // workspace + kFlagsOffset
    float* partials;       // workspace + kPartialsOffset
    int64_t kv_seq_stride; // PADDED: rows between (b,h) slabs
    int64_t total_rows;    // PACKED: sum of N_b
    int32_t Hq;
    int32_t Hkv;           // KV heads (the schedule counts Hkv * C_m output tiles per sequence)
    int32_t N_q;           // query tokens per sequence: the last N_q cached tokens (the maximum if ragged_q)
    int32_t ragged_q;      // per-sequence query lengths: q, out, lse are packed by table.cu_q
    int32_t group;         // Hq / Hkv
    int32_t rows;          // N_q * group query rows share one KV head; row rho = token*group + head
    int32_t C_m;           // row blocks per KV head, ceil(rows / 32) (ceil(rows / 16) at D = 256)
    int32_t T_m;           // rows per block, ceil(rows / C_m); the last block may hold fewer
    int32_t causal;        // row of query token i sees the first N_b - N_q + i + 1 cached tokens
    int32_t out16;         // out holds 16-bit elements
    int32_t slot;          // floats per partial slot
    int32_t spin_limit;
    int32_t has_empty;     // some N_b == 0: those output rows must be zeroed
    int32_t fanin;         // children merged per level of the reduction tree (>= 2)
    int32_t delay_store;   // debug: a publishing workgroup sleeps this many periods before its partial stores
    int32_t delay_signal;  // debug: ... and this many between the acknowledged stores and its flag store
    int32_t delay_stride;  // debug: only workgroups with g % stride == stride - 1 sleep (0 or 1: all)
    unsigned long long* cta_clock;  // optional trace, kClockWords words per CTA, may be null
    float scale_log2e;     // scale * log2(e): scores live in the base-2 domain
    Sched sched;
    SchedTable table;
};

// The rows of output tile (b, head) where head = hk * C_m + mb: KV head hk, row block mb.
struct TileRows {
    int hk;      // KV head
    int rho0;    // first row of the block within the KV head's rows
    int count;   // rows in the block; <= 0 when the sequence has too few query tokens for this block
    int q_len;   // query tokens of the sequence
    int64_t q0;  // index of the sequence's first query token among all query tokens
};
__device__ __forceinline__ TileRows tile_rows(const DecodeArgs& a, int b, int head) {
    TileRows t;
    t.hk = a.C_m == 1 ? head : head / a.C_m;
    t.rho0 = (head - t.hk * a.C_m) * a.T_m;
    if (a.ragged_q) {
        t.q0 = a.table.cu_q[b];
        t.q_len = a.table.cu_q[b + 1] - a.table.cu_q[b];
    } else {
        t.q0 = (int64_t)b * a.N_q;
        t.q_len = a.N_q;
    }
    const int rows = a.ragged_q ? t.q_len * a.group : a.rows;
    t.count = rows - t.rho0 < a.T_m ? rows - t.rho0 : a.T_m;
    return t;
}
// Index into the q / out / lse rows (query token, query head) of row rho of the tile's KV head;
// *token gets the query token within its sequence.
__device__ __forceinline__ int64_t query_row(const DecodeArgs& a, const TileRows& t, int rho, int* token) {
    const int i = (a.N_q == 1 && !a.ragged_q) ? 0 : rho / a.group;
    *token = i;
    return (t.q0 + i) * a.Hq + (int64_t)t.hk * a.group + (rho - i * a.group);
}

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

// Two fp32 values rounded to nearest-even 16-bit elements, packed low half first.
template <int DT>
__device__ __forceinline__ uint32_t narrow2(float lo, float hi) {
    if constexpr (DT == kDtBF16) {
        const bf16x2 p = {(__bf16)lo, (__bf16)hi};
        return __builtin_bit_cast(uint32_t, p);
    } else {
        const f16x2 p = {(_Float16)lo, (_Float16)hi};
        return __builtin_bit_cast(uint32_t, p);
    }
}

// The two 16-bit elements packed in one dword, widened to fp32 (low half first).
template <int DT>
__device__ __forceinline__ void widen2(uint32_t u, float& lo, float& hi) {
    if constexpr (DT == kDtBF16) {
        lo = as_f32(u << 16);
        hi = as_f32(u & 0xffff0000u);
    } else {
        const f16x2 h = __builtin_bit_cast(f16x2, u);
        lo = (float)h.x;
        hi = (float)h.y;
    }
}

// acc + a.lo*b.lo + a.hi*b.hi on packed 16-bit pairs, fp32 accumulate.
template <int DT>
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float acc) {
    if constexpr (DT == kDtBF16) {
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), acc,
                                               false);
    } else {
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, a), __builtin_bit_cast(f16x2, b), acc, false);
    }
}

// ---- K/V streaming through buffer loads ---------------------------------------------------
// One buffer descriptor per (sequence, KV head) slab with num_records = N_b * D * 2
// bytes: a 16-byte load whose offset falls past the slab returns zeros instead of
// touching memory, so the ragged tail tile needs no address clamping.  The whole
// offset goes in the VGPR/immediate part, which is what the range check covers.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
using buffer_rsrc = __amdgpu_buffer_rsrc_t;

__device__ __forceinline__ buffer_rsrc make_slab(const uint16_t* base, uint32_t bytes) {
    // flags: raw 32-bit data format, the untyped-buffer setting for gfx9-family descriptors
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(base), 0, (int)bytes, 0x00020000);
}
// Every cached K/V byte is read exactly once per call, so the loads carry the non-temporal
// cache policy (nt): the lines are not kept in L2 / the last-level cache, which on this machine
// lifts a pure streaming read from 6.2 to 7.2 TB/s.
constexpr int kStreamOnce = 2;  // cache-policy operand of the buffer builtins: nt
__device__ __forceinline__ u32x4 slab_load16(buffer_rsrc r, uint32_t byte_off) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, kStreamOnce);
}
__device__ __forceinline__ u32x2 slab_load8(buffer_rsrc r, uint32_t byte_off) {
    return __builtin_amdgcn_raw_buffer_load_b64(r, (int)byte_off, 0, kStreamOnce);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}

// Sum over each aligned group of LANES (8 or 16) consecutive lanes; every lane
// of the group ends with the total.  Butterfly on DPP lane permutations:
// quad_perm[1,0,3,2], quad_perm[2,3,0,1], row_half_mirror, row_mirror.
template <int LANES>
__device__ __forceinline__ float group_allreduce_sum(float x) {
    static_assert(LANES == 8 || LANES == 16 || LANES == 32, "row of 8, 16 or 32 lanes");
    x += dpp_move<0xB1>(x);
    x += dpp_move<0x4E>(x);
    x += dpp_move<0x141>(x);
    if constexpr (LANES >= 16) x += dpp_move<0x140>(x);
    // lanes l and l^16: ds_swizzle in bit mode (and 0x1f, or 0, xor 0x10)
    if constexpr (LANES == 32) x += as_f32((uint32_t)__builtin_amdgcn_ds_swizzle((int)as_u32(x), 0x401F));
    return x;
}

__device__ __forceinline__ float xor_shuffle(float x, int lane_mask) { return __shfl_xor(x, lane_mask, 64); }

// ---- Algorithm 2: StorePartials / Signal / Wait / LoadPartials ---------------------------
// The workgroups of one launch run on 8 XCDs whose L2 caches are not coherent with each
// other.  Ordinary stores followed by a device-scope release fence would write the whole
// L2 back (and an acquire fence would invalidate it) once per publishing wave, stalling the
// K/V streams of every workgroup on that XCD.  Instead every access to a partial or a flag
// is itself a device-scope access (the sc1 cache-policy bit: written through to, and read
// from, the device coherence point), so no cache-wide writeback or invalidate is needed:
//   producer: sc1 stores of the partial; wait until they are acknowledged (s_waitcnt
//             vmcnt(0), then the workgroup barrier); then one sc1 store of the flag;
//   consumer: sc1 loads of the flag until set; then sc1 loads of the partial.
// (Narrower scopes were measured and dropped: a polling load with sc0 is served again and again
// from the compute unit's own cache and never sees the flag; between two workgroups of one XCD
// an sc0 store is seen by an sc1 poll after 0.3-0.4 us, an sc1 store after 0.4-0.6 us, between
// XCDs after 0.5-0.8 us: too little to pay for a second protocol.)
constexpr int kDeviceScope = 16;  // cache-policy operand of the buffer builtins: sc1
constexpr uint32_t kStatusTimeout = 1u;  // status word: a merging workgroup gave up waiting for a peer

__device__ __forceinline__ void partial_store16(buffer_rsrc r, uint32_t byte_off, f32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, (int)byte_off, 0, kDeviceScope);
}
__device__ __forceinline__ void partial_store4(buffer_rsrc r, uint32_t byte_off, float v) {
    __builtin_amdgcn_raw_buffer_store_b32(as_u32(v), r, (int)byte_off, 0, kDeviceScope);
}
__device__ __forceinline__ f32x4 partial_load16(buffer_rsrc r, uint32_t byte_off) {
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, kDeviceScope));
}
__device__ __forceinline__ float partial_load4(buffer_rsrc r, uint32_t byte_off) {
    return as_f32(__builtin_amdgcn_raw_buffer_load_b32(r, (int)byte_off, 0, kDeviceScope));
}

__device__ __forceinline__ void debug_sleep(int periods) {
    for (int i = 0; i < periods; ++i) __builtin_amdgcn_s_sleep(127);  // about 3.4 us each
}
__device__ __forceinline__ bool debug_delayed(const DecodeArgs& a, int g) {
    return a.delay_stride <= 1 || g % a.delay_stride == a.delay_stride - 1;
}

// Signal, once every thread's partial stores are acknowledged (the caller has waited for its own, the
// barrier collects the workgroup's): one flag word per reader of the slot is set (one store
// instruction of the first `readers` lanes).
__device__ __forceinline__ void signal_acknowledged(const DecodeArgs& a, int g, int slot, int readers) {
    __syncthreads();
    if (a.delay_signal && debug_delayed(a, g)) debug_sleep(a.delay_signal);
    if ((int)threadIdx.x < readers)
        __hip_atomic_store(a.flags + slot * kMaxReducers + threadIdx.x, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void signal_arrival(const DecodeArgs& a, int g, int slot, int readers) {
    __builtin_amdgcn_s_waitcnt(0);  // vmcnt(0) expcnt(0) lgkmcnt(0): stores acknowledged
    signal_acknowledged(a, g, slot, readers);
}

// Poll one flag word until it is set, then clear it (its only reader does).  Bounded twice over, by
// a poll count and by half a second of wall clock (no output tile takes that long): a peer that
// never arrives is reported, not waited for.
constexpr unsigned long long kWaitTicks = 50000000ull;  // 0.5 s of the 100 MHz wall clock
// `seen`: what an earlier load of the flag returned (0: not set then).
__device__ __forceinline__ void await_flag(const DecodeArgs& a, uint32_t* flag, uint32_t seen = 0u) {
    unsigned long long t0 = 0;  // the clock is first read after 256 polls: most waits are over by then
    int spins = 0;
    while (seen == 0u && __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) {
        __builtin_amdgcn_s_sleep(1);
        ++spins;
        bool late = false;
        if ((spins & 255) == 0) {
            const unsigned long long now = wall_clock64();
            if (t0 == 0) t0 = now;
            late = now - t0 > kWaitTicks;
        }
        if (spins >= a.spin_limit || late) {
            __hip_atomic_store(a.status, kStatusTimeout, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            break;  // peer never arrived: report, do not hang
        }
    }
    __hip_atomic_store(flag, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The first poll of a flag, issued but not waited for: the caller's pending partial stores and this
// load then share one wait (poll_collect), instead of the poll queueing behind the acknowledgements.
__device__ __forceinline__ uint32_t poll_issue(const uint32_t* flag) {
    uint32_t v;
    asm volatile("global_load_dword %0, %1, off sc1" : "=v"(v) : "v"(flag) : "memory");
    return v;
}
__device__ __forceinline__ uint32_t poll_collect(uint32_t v) {
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(v)::"memory");  // every store acknowledged, every poll back
    return v;
}

// Tree reduction: wait for `nchild` peers at once, thread j polls the flag of CTA first + j*step
// (reader 0 of its slot; the tile began in CTA `tile_first`).  The consumer clears the flags: each
// flag word has exactly one reader per launch, so the workspace is clean again when the kernel ends.
__device__ __forceinline__ void wait_arrivals(const DecodeArgs& a, int tile_first, int first, int step, int nchild) {
    if ((int)threadIdx.x < nchild) {
        const int cta = first + (int)threadIdx.x * step;
        await_flag(a, a.flags + slot_of(cta, tile_first) * kMaxReducers);
    }
    __syncthreads();  // the partial loads that follow are issued after the flags were seen
}

// Optional per-CTA trace: kClockWords uint64 per CTA: 100 MHz timestamps, the HW_ID and XCC_ID
// registers and the workgroup id.
constexpr int kClockWords = 16;
enum ClockSlot {
    kClkEntry = 0, kClkLoopEnd = 1, kClkLocated = 2, kClkExit = 3, kClkHwId = 4, kClkXccId = 5, kClkBlock = 6,
    kClkFirstStep = 7, kClkCoreDone = 8, kClkStoresIssued = 9, kClkStoresAcked = 10, kClkFlagsSeen = 11,
    kClkMerged = 12, kClkWritten = 13
};
__device__ __forceinline__ void stamp(const DecodeArgs& a, int g, int slot) {
    if (a.cta_clock && threadIdx.x == 0) {
        a.cta_clock[kClockWords * g + slot] = wall_clock64();
        if (slot == kClkEntry) {
            a.cta_clock[kClockWords * g + kClkHwId] = __builtin_amdgcn_s_getreg((31 << 11) | 4);    // HW_REG_HW_ID
            a.cta_clock[kClockWords * g + kClkXccId] = __builtin_amdgcn_s_getreg((31 << 11) | 20);  // HW_REG_XCC_ID
            a.cta_clock[kClockWords * g + kClkBlock] = blockIdx.x;
        }
    }
}

}  // namespace lean
