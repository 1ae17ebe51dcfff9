// Stream-K schedule of LeanAttention (Section 4.3; first lines and loop header
// of Algorithm 2), shared by the host scheduler and the device span walk so
// that both run literally the same index arithmetic.
//
// Output tile  = one (sequence b, head h) pair; it owns C_n[b] = ceil(N_b / T_n)
//                LeanTile iterations.  With up to 32 query rows per KV head (16 at D = 256), h is
//                the KV head; with more, the rows are cut into C_m blocks and h = kv_head*C_m + block
//                (Algorithm 2's C_m output tiles along the query dimension).
// Linearization: PADDED cache  b -> h -> context   (iter = Hkv*cuC[b] + h*C_n[b] + local)
//                PACKED cache  h -> b -> context   (iter = h*cuC[B] + cuC[b] + local)
//                (the paper's "batch -> heads -> context" and, for ragged
//                batches, "Heads -> TotalContextLength"; the result does not
//                depend on the order, each follows its layout in memory).
// Spans:         CTA g owns [g*q + min(g, r), +q + (g < r)) with q = I / G, r = I mod G
//                (the paper divides I by G and is silent on a remainder).
// Tail spans:    optionally the last `tail_iters` iterations of the line are cut into `tail_grid`
//                short spans of their own, owned by the workgroups after the first G: equal shares
//                do not finish at the same time (the units do not stream equally fast), and the
//                hardware hands the short spans, in order, to whichever units finish first.  The
//                decomposition stays a fixed function of the problem, so results stay reproducible.
// Fixed split:   the schedule LeanAttention is compared against (Section 3.3) and one of
//                its special cases (Section 4.3): every output tile is cut into `split`
//                near-equal parts, CTA g = tile_idx*split + part, G = tiles*split; split = 1
//                is the unsplit FlashAttention-2 schedule.  Kept as a built-in baseline.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define LEAN_HD __host__ __device__ inline
#else
#define LEAN_HD inline
#endif

namespace lean {

constexpr int kMaxBatch = 256;

// Prefix sums over the batch; travels to the kernel by value as kernel arguments.
struct SchedTable {
    int32_t cu_iters[kMaxBatch + 1];  // cuC[b] = sum_{b'<b} ceil(N_b' / T_n)
    int32_t cu_tok[kMaxBatch + 1];    // sum_{b'<b} N_b'
    int32_t cu_q[kMaxBatch + 1];      // sum_{b'<b} query tokens of b' (read only with per-sequence query lengths)
};

// Division of a 31-bit dividend by a divisor fixed per launch, as a multiplication: the span walk
// runs on one wave's scalar unit before the first K/V load can be issued, and a hardware-less
// 32-bit division costs it some 40 dependent instructions, four times per segment.
// For 0 <= n < 2^31 and d >= 1:  n / d == (n * mul) >> (32 + shift)  with mul = ceil(2^(31+s) / d),
// s = ceil(log2 d), shift = s - 1 (Granlund & Montgomery: an N-bit multiplier suffices for
// dividends of N-1 bits); d = 1 is encoded as mul = 0.
struct Magic {
    uint32_t mul;
    uint32_t shift;
};
inline Magic make_magic(uint32_t d) {
    Magic m = {0u, 0u};
    if (d <= 1) return m;
    uint32_t s = 0;
    while ((1ull << s) < d) ++s;
    m.mul = (uint32_t)(((1ull << (31 + s)) + d - 1) / d);
    m.shift = s - 1;
    return m;
}
LEAN_HD uint32_t magic_div(uint32_t n, Magic m) {
#if defined(__HIP_DEVICE_COMPILE__)
    const uint32_t hi = __umulhi(n, m.mul);
#else
    const uint32_t hi = (uint32_t)(((uint64_t)n * m.mul) >> 32);
#endif
    return m.mul ? hi >> m.shift : n;
}

struct Sched {
    int32_t B;
    int32_t Hkv;            // output tiles per sequence: KV heads x row blocks per KV head (C_m)
    int32_t T_n;
    int32_t packed;         // 0: PADDED order b->h->t, 1: PACKED order h->b->t
    int32_t grid;           // workgroups: the first head_grid with long spans, then tail_grid with short ones
    int32_t extra;          // head_iters mod head_grid
    int64_t total_iters;    // I
    int64_t iters_per_cta;  // head_iters / head_grid
    int32_t fixed_split;    // 0: stream-K spans; s >= 1: fixed split into s parts per output tile
    int32_t uniform_cn;     // > 0: every sequence owns this many LeanTile iterations (no table search)
    // multipliers for the divisors of the walk; valid (and used) only while I < 2^31 - 1
    Magic by_ipc;           // iters_per_cta
    Magic by_ipc1;          // iters_per_cta + 1
    Magic by_heads;         // Hkv (PADDED order: iteration -> sequence key)
    Magic by_per_head;      // cuC[B] (PACKED order: iteration -> head)
    Magic by_cn;            // uniform_cn
    // tail spans (tail_grid == 0: none; then head_grid == grid and head_iters == total_iters)
    int32_t head_grid;      // G
    int32_t tail_grid;      // workgroups with short spans
    int64_t head_iters;     // iterations [0, head_iters) belong to the first head_grid workgroups
    int32_t tail_ipc;       // (I - head_iters) / tail_grid
    int32_t tail_extra;     // (I - head_iters) mod tail_grid
    Magic by_tipc;          // tail_ipc
    Magic by_tipc1;         // tail_ipc + 1
};

// Sets the span fields of a schedule of `grid` workgroups, the last `tail_grid` of which share the
// last `tail_iters` iterations (0, 0: plain stream-K spans).  Needs grid - tail_grid >= 1.
inline void set_spans(Sched& s, int64_t total_iters, int32_t grid, int32_t tail_grid, int64_t tail_iters) {
    s.total_iters = total_iters;
    s.grid = grid;
    s.tail_grid = tail_grid;
    s.head_grid = grid - tail_grid;
    s.head_iters = total_iters - tail_iters;
    s.iters_per_cta = s.head_iters / s.head_grid;
    s.extra = (int32_t)(s.head_iters % s.head_grid);
    s.tail_ipc = tail_grid > 0 ? (int32_t)(tail_iters / tail_grid) : 0;
    s.tail_extra = tail_grid > 0 ? (int32_t)(tail_iters % tail_grid) : 0;
}

// One output-tile segment of a CTA's span (one trip of Algorithm 2's loop).
struct Segment {
    int32_t b, h;
    int32_t tile_idx;         // PADDED: b*Hkv + h, PACKED: h*B + b
    int32_t local_iter;       // first LeanTile iteration inside the tile
    int32_t local_iter_end;   // one past the last
    int32_t n_ctx;            // N_b
    int32_t host;             // this CTA computed the tile's first iteration
    int32_t finishing;        // this CTA's span reaches the tile's end
    int32_t first_cta;        // CTA that computed the tile's first iteration (the host block)
    int32_t last_cta;         // last CTA contributing to the tile
    int64_t tile_iter_end;    // global iteration index one past the tile
};

// a / b for iteration counts (0 <= a <= I, 0 < b <= I + 1).  On the device a 64-bit division is
// a long emulated sequence and the span walk needs several per segment, so iteration spaces
// below 2^31 (all realistic ones) divide in 32 bits.
LEAN_HD int64_t div_iters(const Sched& s, int64_t a, int64_t b) {
    if (s.total_iters < 0x7fffffff) return (int64_t)((uint32_t)a / (uint32_t)b);
    return a / b;
}

constexpr int64_t kMagicLimit = 0x7fffffff;  // iteration spaces below this divide by multiplication

// Fills the derived fields of a schedule whose B, Hkv and span fields (set_spans) are set.
inline void finish_sched(Sched& s, const SchedTable& t) {
    s.uniform_cn = 0;
    if (s.B >= 1) {
        const int32_t c0 = t.cu_iters[1] - t.cu_iters[0];
        bool same = c0 > 0;
        for (int b = 1; b < s.B && same; ++b) same = t.cu_iters[b + 1] - t.cu_iters[b] == c0;
        if (same) s.uniform_cn = c0;
    }
    const bool small = s.total_iters < kMagicLimit;
    s.by_ipc = make_magic(small ? (uint32_t)s.iters_per_cta : 1u);
    s.by_ipc1 = make_magic(small ? (uint32_t)s.iters_per_cta + 1u : 1u);
    s.by_heads = make_magic(small ? (uint32_t)s.Hkv : 1u);
    s.by_per_head = make_magic(small && s.B >= 1 ? (uint32_t)t.cu_iters[s.B] : 1u);
    s.by_cn = make_magic(small && s.uniform_cn > 0 ? (uint32_t)s.uniform_cn : 1u);
    s.by_tipc = make_magic(small && s.tail_ipc > 0 ? (uint32_t)s.tail_ipc : 1u);
    s.by_tipc1 = make_magic(small ? (uint32_t)s.tail_ipc + 1u : 1u);
}

// The CTA whose span holds global iteration `it` (stream-K spans).
LEAN_HD int cta_of_iter(const Sched& s, int64_t it) {
    if (it >= s.head_iters) {  // a tail span (never taken without tail spans: it < total_iters)
        const int64_t j = it - s.head_iters;
        const int64_t fat_t = (int64_t)s.tail_extra * (s.tail_ipc + 1);
        if (s.total_iters < kMagicLimit) {
            if (j < fat_t) return s.head_grid + (int)magic_div((uint32_t)j, s.by_tipc1);
            return s.head_grid + s.tail_extra + (int)magic_div((uint32_t)(j - fat_t), s.by_tipc);
        }
        if (j < fat_t) return s.head_grid + (int)(j / (s.tail_ipc + 1));
        return s.head_grid + s.tail_extra + (int)((j - fat_t) / s.tail_ipc);
    }
    const int64_t fat = (int64_t)s.extra * (s.iters_per_cta + 1);
    if (s.total_iters < kMagicLimit) {
        if (it < fat) return (int)magic_div((uint32_t)it, s.by_ipc1);
        return s.extra + (int)magic_div((uint32_t)(it - fat), s.by_ipc);
    }
    if (it < fat) return (int)(it / (s.iters_per_cta + 1));
    return s.extra + (int)((it - fat) / s.iters_per_cta);
}

// Largest b in [0, B) with cu_iters[b] <= key (key < cu_iters[B]); skips empty sequences.
LEAN_HD int find_sequence(const SchedTable& t, int B, int32_t key) {
    int lo = 0, hi = B;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (t.cu_iters[mid] <= key) lo = mid; else hi = mid;
    }
    return lo;
}

// Segment of the tile containing global iteration `it`, clipped to the CTA's span end.
LEAN_HD Segment locate(const Sched& s, const SchedTable& t, int64_t it, int64_t cta_end) {
    Segment sg;
    int64_t tile_iter;  // global index of the tile's first iteration
    int32_t c_n;
    const bool small = s.total_iters < kMagicLimit;
    // with equal lengths the sequence of a key is a quotient, otherwise a search in the prefix table
    auto sequence_of = [&](int32_t key) {
        if (s.uniform_cn > 0 && small) return (int)magic_div((uint32_t)key, s.by_cn);
        return find_sequence(t, s.B, key);
    };
    if (s.packed) {
        const int64_t per_head = t.cu_iters[s.B];
        sg.h = small ? (int32_t)magic_div((uint32_t)it, s.by_per_head) : (int32_t)(it / per_head);
        const int32_t key = (int32_t)(it - (int64_t)sg.h * per_head);
        sg.b = sequence_of(key);
        c_n = t.cu_iters[sg.b + 1] - t.cu_iters[sg.b];
        tile_iter = (int64_t)sg.h * per_head + t.cu_iters[sg.b];
        sg.tile_idx = sg.h * s.B + sg.b;
    } else {
        const int32_t key = small ? (int32_t)magic_div((uint32_t)it, s.by_heads) : (int32_t)(it / s.Hkv);
        sg.b = sequence_of(key);
        c_n = t.cu_iters[sg.b + 1] - t.cu_iters[sg.b];
        const int64_t seq_iter = (int64_t)s.Hkv * t.cu_iters[sg.b];
        if (s.uniform_cn > 0 && small) sg.h = (int32_t)magic_div((uint32_t)(it - seq_iter), s.by_cn);
        else sg.h = (int32_t)div_iters(s, it - seq_iter, c_n);
        tile_iter = seq_iter + (int64_t)sg.h * c_n;
        sg.tile_idx = sg.b * s.Hkv + sg.h;
    }
    sg.n_ctx = t.cu_tok[sg.b + 1] - t.cu_tok[sg.b];
    sg.tile_iter_end = tile_iter + c_n;
    sg.local_iter = (int32_t)(it - tile_iter);
    const int64_t stop = sg.tile_iter_end < cta_end ? sg.tile_iter_end : cta_end;
    sg.local_iter_end = (int32_t)(stop - tile_iter);
    sg.host = it == tile_iter;
    sg.finishing = cta_end >= sg.tile_iter_end;
    if (s.fixed_split) {
        const int parts = c_n < s.fixed_split ? c_n : s.fixed_split;
        sg.first_cta = sg.tile_idx * s.fixed_split;
        sg.last_cta = sg.first_cta + parts - 1;
    } else {
        sg.first_cta = cta_of_iter(s, tile_iter);
        sg.last_cta = cta_of_iter(s, sg.tile_iter_end - 1);
    }
    return sg;
}

// The segment after `prev` in the span of CTA g (stream-K spans; prev.tile_iter_end < cta_end):
// the next output tile in iteration order, from its first iteration, so this CTA is its host
// block.  Same result as locate(s, t, prev.tile_iter_end, cta_end) without the searches and
// divisions: the walk steps to the next head / next non-empty sequence.
LEAN_HD Segment locate_next(const Sched& s, const SchedTable& t, const Segment& prev, int g, int64_t cta_end) {
    Segment sg;
    sg.b = prev.b;
    sg.h = prev.h;
    if (s.packed) {
        do {
            if (++sg.b == s.B) {
                sg.b = 0;
                ++sg.h;
            }
        } while (t.cu_iters[sg.b + 1] == t.cu_iters[sg.b]);
        sg.tile_idx = sg.h * s.B + sg.b;
    } else {
        if (++sg.h == s.Hkv) {
            sg.h = 0;
            do ++sg.b; while (t.cu_iters[sg.b + 1] == t.cu_iters[sg.b]);
        }
        sg.tile_idx = sg.b * s.Hkv + sg.h;
    }
    const int32_t c_n = t.cu_iters[sg.b + 1] - t.cu_iters[sg.b];
    const int64_t tile_iter = prev.tile_iter_end;
    sg.n_ctx = t.cu_tok[sg.b + 1] - t.cu_tok[sg.b];
    sg.tile_iter_end = tile_iter + c_n;
    sg.local_iter = 0;
    const int64_t stop = sg.tile_iter_end < cta_end ? sg.tile_iter_end : cta_end;
    sg.local_iter_end = (int32_t)(stop - tile_iter);
    sg.host = 1;
    sg.finishing = cta_end >= sg.tile_iter_end;
    sg.first_cta = g;
    sg.last_cta = sg.finishing ? g : cta_of_iter(s, sg.tile_iter_end - 1);
    return sg;
}

// The range of global iterations CTA g owns (empty when begin == end).
LEAN_HD void span_of(const Sched& s, const SchedTable& t, int g, int64_t* begin, int64_t* end) {
    if (!s.fixed_split) {
        if (g >= s.head_grid) {  // a tail span
            const int j = g - s.head_grid;
            const int64_t lo = s.head_iters + (int64_t)j * s.tail_ipc + (j < s.tail_extra ? j : s.tail_extra);
            *begin = lo;
            *end = lo + s.tail_ipc + (j < s.tail_extra ? 1 : 0);
            return;
        }
        const int64_t lo = (int64_t)g * s.iters_per_cta + (g < s.extra ? g : s.extra);
        *begin = lo;
        *end = lo + s.iters_per_cta + (g < s.extra ? 1 : 0);
        return;
    }
    const int tile = g / s.fixed_split, part = g % s.fixed_split;
    const int b = s.packed ? tile % s.B : tile / s.Hkv;
    const int h = s.packed ? tile / s.B : tile % s.Hkv;
    const int32_t c_n = t.cu_iters[b + 1] - t.cu_iters[b];
    const int parts = c_n < s.fixed_split ? c_n : s.fixed_split;
    if (part >= parts) {  // more parts than LeanTiles (or an empty sequence): nothing to do
        *begin = *end = 0;
        return;
    }
    const int64_t tile_iter = s.packed ? (int64_t)h * t.cu_iters[s.B] + t.cu_iters[b]
                                       : (int64_t)s.Hkv * t.cu_iters[b] + (int64_t)h * c_n;
    *begin = tile_iter + (int64_t)part * c_n / parts;
    *end = tile_iter + (int64_t)(part + 1) * c_n / parts;
}

}  // namespace lean
