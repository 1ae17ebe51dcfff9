// LeanTile inner loop (Algorithm 1) for T_m <= 16 * MB query rows that share one KV
// head (a group of query heads, several query tokens, or both).  The rows are the T_m
// rows of Q_f, so each K/V tile is read once for all of them and QK^T / PV are small
// dense contractions: they run on the matrix cores (v_mfma_f32_16x16x32 in bf16 or
// f16), with the online softmax in fp32 on the VALU.
//
// Per wave and per block of 16 tokens (indices below are within the block):
//
//   S^T[16 tok x 16 rows] = K_blk * Q^T         A = K (m: token, k: head dim), B = Q^T
//     lane (r = lane%16, g = lane/16) supplies token 4*(r%4) + r/4, so that the
//     accumulator register i of lane (h, g) is the score of token 4*i + g for query
//     row h: the tokens a lane group needs as contraction slots of
//
//   O^T[D x 16 rows] += V_blk^T * P^T            A = V^T (m: head dim, k: token), B = P^T
//     lane (m = lane%16, g) loads, for j = 0..3, the D/16 head-dim elements
//     [m*D/16, (m+1)*D/16) of token 4*j + g: the four loads of a wave are fully
//     coalesced (one contiguous KiB each at D = 128), and the 4-token x D/16
//     sub-block a lane holds is transposed in registers (v_perm_b32) into the
//     D/16 A operands.  Accumulator e, register i of lane (h, g) is
//     O[h][ (D/16)*(4*g + i) + e ].  (At D = 256 the 16 elements of a lane are two runs
//     of 8, half a row apart, so that every load instruction stays contiguous.)
//
// P is split into a high and a low 16-bit part (P = P_hi + P_lo) so that rounding P to the
// input precision never limits accuracy.  The two parts share one MFMA: its 32 contraction
// slots hold the 16 tokens twice, once against P_hi and once against P_lo.  For S^T the 32
// slots are 32 consecutive head-dim elements.
//
// K is loaded with the same fully coalesced pattern as V (whole rows per group of 16
// lanes).  The A operand of S^T needs a different lane<->row assignment (lane r holds
// a token, lane group g a 16-byte piece of each quarter row); loading that pattern
// straight from memory reads 16-byte pieces strided over 16 rows and streams at only
// 6.0 instead of 7.1 TB/s on this machine, so the K tile of a wave takes a detour
// through a wave-private LDS area (rows padded to 272 bytes, no barrier: the LDS queue of a
// wave is in order).  The staging stores are conflict-free.  The operand reads (16 rows at
// the 272-byte stride per lane group) take twice the LDS cycles of a linear wave-wide
// 16-byte read, measured with SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE on the isolated
// patterns: store 2 units, read 1 + 1 conflict unit, i.e. the ratio 0.25 the kernel shows;
// an XOR swizzle of unpadded rows measures the same, unpadded rows 8 units.  LDS
// instructions are issued in under 4 % of the wave cycles of this HBM-bound loop, so the
// read pattern is left as it is.  V goes from global memory straight to the MFMA operand
// registers.
#pragma once
#include "lean_device.h"

namespace lean {

// D[16x16] += A[16x32] * B[32x16] on the matrix cores (v_mfma_f32_16x16x32_bf16 / _f16 of
// gfx950).  Lane (r = lane%16, g = lane/16) supplies row r of A and column r of B for the 8
// contraction slots of its lane group, in its four operand dwords (two 16-bit elements each);
// the product pairs slot (g, j) of A with slot (g, j) of B.  Accumulator register i of lane
// (r, g) is D[4*g + i][r].
template <int DT>
__device__ __forceinline__ f32x4 mfma32(u32x4 a, u32x4 b, f32x4 c) {
    if constexpr (DT == kDtBF16) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                       0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c,
                                                      0, 0, 0);
    }
}

// Split two non-negative fp32 weights into packed 16-bit high parts and packed
// 16-bit remainders: p = hi + lo up to 2^-16 (bf16, truncation) or 2^-21 (f16) relative.
template <int DT>
__device__ __forceinline__ void split_pair(float p0, float p1, uint32_t& hi, uint32_t& lo) {
    if constexpr (DT == kDtBF16) {
        hi = __builtin_amdgcn_perm(as_u32(p1), as_u32(p0), 0x07060302u);
        const float r0 = p0 - as_f32(as_u32(p0) & 0xffff0000u);
        const float r1 = p1 - as_f32(as_u32(p1) & 0xffff0000u);
        lo = __builtin_amdgcn_perm(as_u32(r1), as_u32(r0), 0x07060302u);
    } else {
        const f16x2 h = __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(p0, p1));
        hi = __builtin_bit_cast(uint32_t, h);
        const f16x2 r = __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(p0 - (float)h.x, p1 - (float)h.y));
        lo = __builtin_bit_cast(uint32_t, r);
    }
}

// What one lane loads of one K or V row: kPieces pieces of kPW dwords.  Lane r of a group
// of 16 takes bytes [256*p + r*4*kPW, +4*kPW) of the row, so that the 16 lanes of a group
// read 64*kPW contiguous bytes per piece: 8 bytes per lane at D = 64, 16 at D = 128, and
// two 16-byte pieces 256 bytes apart at D = 256.
template <int PW>
struct Piece;
template <>
struct Piece<4> {
    using type = u32x4;
};
template <>
struct Piece<2> {
    using type = u32x2;
};

// The arithmetic of one wave on its NBLK blocks of 16 tokens, common to the register-staged core
// below and the LDS-staged core (lean_gqa_lds_core.h): the query operands, the running softmax
// statistics and the output accumulators of MB blocks of 16 query rows.
template <int DT, int D, int NBLK, int MB>
struct GqaWave {
    static constexpr int kKC = D / 32;   // 16-byte K pieces per lane per block
    static constexpr int kEV = D / 16;   // head-dim elements per lane per token (V side)
    u32x4 qb[MB][kKC];  // Q^T as B operands: lane (row r, g) holds Q[r][32*c2 + 8*g .. +8), zero rows past the block
    int n_vis[MB];      // cached tokens the lane's query row may attend to (causal mask aligned to the end)
    float m_run[MB];    // row 16*mb + r, shared by the four k-group lanes
    float l_run[MB];    // this lane's share of l (tokens 4*i + g); summed over g at the end
    f32x4 acc[MB][kEV];

    __device__ __forceinline__ void load_q(const DecodeArgs& a, const TileRows& tr, int n_ctx, int r, int g) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
            for (int c2 = 0; c2 < kKC; ++c2) qb[mb][c2] = u32x4{0u, 0u, 0u, 0u};
            n_vis[mb] = n_ctx;
            if (16 * mb + r < tr.count) {
                int token;
                const int64_t qrow = query_row(a, tr, tr.rho0 + 16 * mb + r, &token);
                if (a.causal) n_vis[mb] = n_ctx - tr.q_len + token + 1;
                const u32x4* qp = reinterpret_cast<const u32x4*>(a.q + qrow * D) + g;
#pragma unroll
                for (int c2 = 0; c2 < kKC; ++c2) qb[mb][c2] = qp[4 * c2];
            }
            m_run[mb] = -INFINITY;
            l_run[mb] = 0.f;
#pragma unroll
            for (int e = 0; e < kEV; ++e) acc[mb][e] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }

    // One step: the K operands against Q, the online softmax, then O^T += V^T P^T.
    // `base`: index in the context of the wave's first token of the step.  v(blk, j, i): dword i
    // (head-dim elements 2i, 2i+1 of the lane's kEV) of token 4*j + g of block blk; the 4-token x kEV
    // sub-block of a lane is transposed here into A operands.  between(): called once the scores are
    // taken, before V is used.
    template <class V, class F>
    __device__ __forceinline__ void step(const u32x4 (&kb)[NBLK][kKC], int base, int g, float scale_log2e, V&& v, F&& between) {
        uint2 p_hi[MB][NBLK], p_lo[MB][NBLK];  // P = P_hi + P_lo, two 16-bit parts
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            f32x4 s[NBLK];
            float mx = -INFINITY;
#pragma unroll
            for (int blk = 0; blk < NBLK; ++blk) {
                // two accumulators halve the dependent MFMA chain over the head dim
                f32x4 c0 = {0.f, 0.f, 0.f, 0.f}, c1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int c2 = 0; c2 < kKC; c2 += 2) {
                    c0 = mfma32<DT>(kb[blk][c2], qb[mb][c2], c0);
                    c1 = mfma32<DT>(kb[blk][c2 + 1], qb[mb][c2 + 1], c1);
                }
                f32x4 c = c0 + c1;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float x = c[i] * scale_log2e;
                    if (base + blk * 16 + 4 * i + g >= n_vis[mb]) x = -INFINITY;  // tail and masked tokens
                    c[i] = x;
                    mx = fmaxf(mx, x);
                }
                s[blk] = c;
            }
            // The reference maximum m_run of a row is shared by its four k-group lanes.  It is
            // only raised when some score of the wave exceeds it by more than kSlack (base-2
            // units): any reference gives the same O~/l, so between updates P may reach 2^kSlack
            // and the cross-lane maximum and the re-scaling of O stay off the common path.
            constexpr float kSlack = 8.f;
            float alpha = 1.f;
            if (__any(mx > m_run[mb] + kSlack)) {
                mx = fmaxf(mx, xor_shuffle(mx, 16));
                mx = fmaxf(mx, xor_shuffle(mx, 32));
                const float m_new = fmaxf(m_run[mb], mx);
                const float m_new_ref = m_new == -INFINITY ? 0.f : m_new;
                alpha = fast_exp2(m_run[mb] - m_new_ref);
                m_run[mb] = m_new;
            }
            const float m_ref = m_run[mb] == -INFINITY ? 0.f : m_run[mb];
            float psum = 0.f;
#pragma unroll
            for (int blk = 0; blk < NBLK; ++blk) {
                float p[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    p[i] = fast_exp2(s[blk][i] - m_ref);
                    psum += p[i];
                }
                split_pair<DT>(p[0], p[1], p_hi[mb][blk].x, p_lo[mb][blk].x);
                split_pair<DT>(p[2], p[3], p_hi[mb][blk].y, p_lo[mb][blk].y);
            }
            l_run[mb] = l_run[mb] * alpha + psum;
            if (__any(alpha != 1.f)) {  // the running max moved for some row of this wave
#pragma unroll
                for (int e = 0; e < kEV; ++e) acc[mb][e] *= alpha;
            }
        }
        between();
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk) {
#pragma unroll
            for (int e = 0; e < kEV; ++e) {
                const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
                // contraction slots 0..3: the four tokens against P_hi, 4..7: the same tokens against P_lo
                const uint32_t v01 = __builtin_amdgcn_perm(v(blk, 1, e >> 1), v(blk, 0, e >> 1), sel);
                const uint32_t v23 = __builtin_amdgcn_perm(v(blk, 3, e >> 1), v(blk, 2, e >> 1), sel);
                const u32x4 va = {v01, v23, v01, v23};
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    const u32x4 pb = {p_hi[mb][blk].x, p_hi[mb][blk].y, p_lo[mb][blk].x, p_lo[mb][blk].y};
                    acc[mb][e] = mfma32<DT>(va, pb, acc[mb][e]);
                }
            }
        }
    }

    // Segment end: the wave's partial (O~ rows, m, l) into its LDS area.  COL(m, e): head-dim index of
    // element e of the lane with row index m.
    template <class Smem, class COL>
    __device__ __forceinline__ void park(Smem& sm, int w, int r, int g, COL&& col_of) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            // l over the four k-group lanes of each row; m is already common to them.
            l_run[mb] += xor_shuffle(l_run[mb], 16);
            l_run[mb] += xor_shuffle(l_run[mb], 32);
            // 16-byte stores; rows are padded by 4 floats so that the 16 rows hit different banks
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int e4 = 0; e4 < kEV; e4 += 4) {
                    const f32x4 val = {acc[mb][e4][i], acc[mb][e4 + 1][i], acc[mb][e4 + 2][i], acc[mb][e4 + 3][i]};
                    *reinterpret_cast<f32x4*>(&sm.area[w].o[16 * mb + r][col_of(4 * g + i, e4)]) = val;
                }
            }
            if (g == 0) {
                sm.m[w][16 * mb + r] = m_run[mb];
                sm.l[w][16 * mb + r] = l_run[mb];
            }
        }
    }
};

// MB: blocks of 16 query rows that share one pass over K/V (T_m <= 16 * MB).  Every K and V
// register tile feeds MB score and MB output contractions.
template <int DT, int D, int NBLK, int NW, bool DB = true, int MB = 1>
struct GqaCore {
    static constexpr int kD = D;
    static constexpr int kDT = DT;
    static constexpr int kTn = NW * NBLK * 16;  // LeanTile
    static constexpr int kCH = NBLK * 16;       // tokens per wave per step
    static constexpr int kThreads = NW * 64;
    static constexpr int kTmMax = 16 * MB;
    // With two row blocks the arithmetic phase of a step is long enough that issuing the next
    // step's loads early pays (measured +4 %); with one it only adds bytes in flight beyond the
    // 8 KiB per wave the memory system likes best (measured -1.5 %).
    static constexpr bool kPipelined = MB > 1;
    static constexpr int kStreams = NW;
    // with 256 output columns per query row block set (D = 256, or two row blocks at D = 128) a
    // four-wave workgroup needs more than half of the register file per wave; it then runs as
    // the only workgroup of its compute unit (the default launch shape anyway)
    static constexpr int kMinWavesPerSimd = (D * MB >= 256 && NW == 4) ? 1 : 2;
    static constexpr int kKC = D / 32;          // 16-byte K pieces per lane per block
    static constexpr int kEV = D / 16;          // head-dim elements per lane per token (V side)
    static constexpr int kVW = kEV / 2;         // dwords per lane per token (V side)
    static constexpr int kPieces = D == 256 ? 2 : 1;   // loads per lane per row
    static constexpr int kPW = kVW / kPieces;          // dwords per piece
    static constexpr int kPE = kEV / kPieces;          // head-dim elements per piece
    static_assert(D == 64 || D == 128 || D == 256, "head dim");
    using pvec = typename Piece<kPW>::type;
    struct vvec {
        pvec p[kPieces];
        __device__ uint32_t dword(int i) const { return p[i / kPW][i % kPW]; }
    };
    // head-dim index of element e (0..kEV) of the lane with row index m
    __device__ static constexpr int col_of(int m, int e) { return (e / kPE) * (D / kPieces) + m * kPE + e % kPE; }

    static constexpr int kRowBytes = D * 2;
    static constexpr int kStageRow = kRowBytes + 16;                 // padded K row in LDS
    static constexpr int kStageVec = NBLK * 16 * kStageRow / 16;     // uint4 per wave
    // Per wave: its K staging area while streaming, its partial (O~) at segment end.
    union alignas(16) WaveArea {
        float o[kTmMax][D + 4];
        u32x4 k[kStageVec];
    };
    struct alignas(16) Smem {
        WaveArea area[kStreams];
        float m[kStreams][kTmMax];
        float l[kStreams][kTmMax];
        __device__ const float* o_at(int stream, int row, int col) const { return &area[stream].o[row][col]; }
    };

    __device__ static void run(const DecodeArgs& a, const Segment& sg, Smem& sm, int cta) {
        const int lane = threadIdx.x & 63;
        const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const int r = lane & 15;   // A row / B column index of the lane
        const int g = lane >> 4;   // k-group of the lane
        const int n_ctx = sg.n_ctx;
        const TileRows tr = tile_rows(a, sg.b, sg.h);

        const int64_t row0 = a.sched.packed
                                 ? (int64_t)tr.hk * a.total_rows + a.table.cu_tok[sg.b]
                                 : ((int64_t)sg.b * a.Hkv + tr.hk) * a.kv_seq_stride;
        const uint32_t slab_bytes = (uint32_t)n_ctx * kRowBytes;
        const buffer_rsrc k_slab = make_slab(a.k + row0 * D, slab_bytes);
        const buffer_rsrc v_slab = make_slab(a.v + row0 * D, slab_bytes);
        const int k_tok = 4 * (r & 3) + (r >> 2);  // token (within a block) this lane feeds as A row r
        // K and V: lane (r, g) loads its kPieces pieces of row 4*j + g, j = 0..3
        const uint32_t v_lane_off = (uint32_t)(w * kCH + g) * kRowBytes + (uint32_t)r * (kPW * 4u);
        char* stage = reinterpret_cast<char*>(sm.area[w].k);
        const uint32_t stage_wr = (uint32_t)g * kStageRow + (uint32_t)r * (kPW * 4u);   // + (blk*16 + 4*j) rows
        const uint32_t stage_rd = (uint32_t)k_tok * kStageRow + (uint32_t)g * 16u;      // + blk*16 rows + 64*c2

        GqaWave<DT, D, NBLK, MB> wv;
        wv.load_q(a, tr, n_ctx, r, g);

        vvec kA[NBLK][4], kB[NBLK][4];
        vvec vA[NBLK][4], vB[NBLK][4];

        auto load_row = [&](const buffer_rsrc& slab, uint32_t o) {
            vvec x;
#pragma unroll
            for (int p = 0; p < kPieces; ++p) {
                if constexpr (kPW == 4) x.p[p] = slab_load16(slab, o + 256u * p);
                else x.p[p] = slab_load8(slab, o + 256u * p);
            }
            return x;
        };
        // Per j and piece one fully coalesced wave-wide load over 4 rows; `off` is the lane's byte
        // offset of the step in the slab (an offset past the slab loads zeros without any traffic).
        auto load_tile = [&](const buffer_rsrc& slab, vvec(&x)[NBLK][4], uint32_t off) {
#pragma unroll
            for (int blk = 0; blk < NBLK; ++blk) {
#pragma unroll
                for (int j = 0; j < 4; ++j) x[blk][j] = load_row(slab, off + (uint32_t)(blk * 16 + 4 * j) * kRowBytes);
            }
        };
        auto step_off = [&](int step) { return v_lane_off + (uint32_t)step * (kTn * kRowBytes); };

        // K rows -> wave-private LDS (lane r: token k_tok, lane group g: piece); frees the registers
        auto stage_k = [&](const vvec(&kraw)[NBLK][4]) {
#pragma unroll
            for (int blk = 0; blk < NBLK; ++blk) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
#pragma unroll
                    for (int p = 0; p < kPieces; ++p)
                        *reinterpret_cast<pvec*>(stage + stage_wr + (uint32_t)(blk * 16 + 4 * j) * kStageRow + 256u * p) =
                            kraw[blk][j].p[p];
                }
            }
            __builtin_amdgcn_wave_barrier();
        };

        // The staged K tile against Q, the online softmax, then P against the V tile in registers.
        auto attend = [&](const vvec(&vb)[NBLK][4], int step) {
            const int base = step * kTn + w * kCH;
            u32x4 kb[NBLK][kKC];
#pragma unroll
            for (int blk = 0; blk < NBLK; ++blk) {
#pragma unroll
                for (int c2 = 0; c2 < kKC; ++c2)
                    kb[blk][c2] = *reinterpret_cast<const u32x4*>(stage + stage_rd + (uint32_t)(blk * 16) * kStageRow + c2 * 64u);
            }
            __builtin_amdgcn_wave_barrier();
            wv.step(kb, base, g, a.scale_log2e, [&](int blk, int j, int i) { return vb[blk][j].dword(i); }, [] {});
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
        if constexpr (DB) {
            // Double-buffered walk: the loads of the next step stay in flight across the
            // arithmetic of this one.
            int k = 0;
            load_tile(k_slab, kA, off_at(0));
            load_tile(v_slab, vA, off_at(0));
            while (k < n_it) {
                load_tile(k_slab, kB, off_at(k + 1));
                load_tile(v_slab, vB, off_at(k + 1));
                stage_k(kA);
                attend(vA, it_first + k);
                if (a.cta_clock && k == 0 && threadIdx.x == 0) a.cta_clock[kClockWords * cta + kClkFirstStep] = wall_clock64();
                load_tile(k_slab, kA, off_at(k + 2));
                load_tile(v_slab, vA, off_at(k + 2));
                if (k + 1 < n_it) {
                    stage_k(kB);
                    attend(vB, it_first + k + 1);
                }
                k += 2;
            }
        } else {
            if constexpr (!kPipelined) {
                // One register buffer: a wave issues one step's loads, consumes them, then issues
                // the next; the other waves of the compute unit cover its memory latency.
                for (int k = 0; k < n_it; ++k) {
                    load_tile(k_slab, kA, off_at(k));
                    load_tile(v_slab, vA, off_at(k));
                    stage_k(kA);
                    attend(vA, it_first + k);
                    if (a.cta_clock && k == 0 && threadIdx.x == 0) a.cta_clock[kClockWords * cta + kClkFirstStep] = wall_clock64();
                }
            } else {
                // One register buffer, software-pipelined: the K registers are free as soon as the
                // tile is staged in LDS, the V registers after the last PV contraction, so the next
                // step's K loads are in flight across this step's arithmetic and its V loads across
                // the next step's scores and softmax.
                load_tile(k_slab, kA, off_at(0));
                load_tile(v_slab, vA, off_at(0));
                for (int k = 0; k < n_it; ++k) {
                    stage_k(kA);
                    load_tile(k_slab, kA, off_at(k + 1));
                    attend(vA, it_first + k);
                    load_tile(v_slab, vA, off_at(k + 1));
                    if (a.cta_clock && k == 0 && threadIdx.x == 0) a.cta_clock[kClockWords * cta + kClkFirstStep] = wall_clock64();
                }
            }
        }

        wv.park(sm, w, r, g, [](int m, int e) { return col_of(m, e); });
        __syncthreads();
    }
};

}  // namespace lean
