// LeanTile inner loop (Algorithm 1) for T_m <= 16 * MB query rows that share one KV head, with the
// K and V tiles staged in LDS: the variant of GqaCore (same contractions, same online softmax,
// same operand layouts) for the shapes whose register tiles leave no room for a second buffer --
// 256 output columns per token (D = 256, or two blocks of 16 query rows at D = 128).
//
// Each wave owns STAGES buffers of one K tile and one V tile (16 * NBLK tokens) in LDS and fills
// them with direct-to-LDS buffer loads (buffer_load_dwordx4 ... lds: no destination registers, so
// the loads of the next STAGES - 1 steps stay in flight across the arithmetic of this one).  A
// wave-wide load writes its 64 pieces of 16 bytes to 1 KiB of consecutive LDS in lane order; what
// a lane fetches is free, so the placement is chosen by the global address each lane asks for:
//
//   K: the KiB holds whole rows; the 16-byte chunk c of row t is stored at chunk position
//      c ^ (t % 16) of its row.  The A operand of S^T = K Q^T (lane r: token 4*(r%4) + r/4,
//      lane group g: chunk 4*c2 + g) is then read with ds_read_b128 from 16 rows at 16 different
//      chunk positions, and there is no staging store (measured: the read costs what the read
//      from GqaCore's padded rows costs, twice a linear one).  Every row is still fetched as
//      one contiguous run of 256 (D = 128) or 512 bytes.
//   V: lane (m, g) fetches what GqaCore loads into registers (row 4*j + g, 16 bytes at m * 16 of
//      each 256-byte piece of the row) and reads back its own slot: LDS is a queue per lane.
//
// The compiler does not order LDS reads against these loads, so the waits are written out: before
// a stage is read, vmcnt leaves only the loads of the later stages outstanding (loads retire in
// issue order); before a stage is refilled, its LDS reads have returned.
#pragma once
#include <type_traits>

#include "lean_device.h"
#include "lean_gqa_core.h"

namespace lean {

#define LEAN_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

template <int N>
__device__ __forceinline__ void wait_loads_outstanding() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void wait_lds_reads() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

template <int DT, int D, int NBLK, int NW, int STAGES, int MB = 1>
struct GqaLdsCore {
    static constexpr int kD = D;
    static constexpr int kDT = DT;
    static constexpr int kTn = NW * NBLK * 16;  // LeanTile
    static constexpr int kCH = NBLK * 16;       // tokens per wave per step
    static constexpr int kThreads = NW * 64;
    static constexpr int kTmMax = 16 * MB;
    static constexpr int kStreams = NW;
    static constexpr int kMinWavesPerSimd = NW <= 4 ? 1 : 2;
    static constexpr int kKC = D / 32;          // 16-byte K pieces per lane per block
    static constexpr int kEV = D / 16;          // head-dim elements per lane per token (V side)
    static constexpr int kPieces = D / 128;     // 16-byte pieces per lane per V row
    static constexpr int kPE = 8;               // head-dim elements per piece
    static_assert(D == 128 || D == 256, "head dim");
    static_assert(STAGES >= 2 && STAGES <= 4, "stages");
    // head-dim index of element e (0..kEV) of the lane with row index m
    __device__ static constexpr int col_of(int m, int e) { return (e / kPE) * (D / kPieces) + m * kPE + e % kPE; }

    static constexpr int kRowBytes = D * 2;
    static constexpr int kChunksPerRow = kRowBytes / 16;
    static constexpr int kTileBytes = kCH * kRowBytes;    // the K or the V tile of one wave and step
    static constexpr int kLoads = kTileBytes / 1024;      // wave-wide loads per tile
    static constexpr int kStageLoads = 2 * kLoads;
    static_assert((STAGES - 1) * kStageLoads < 64, "the load counter has 6 bits");
    struct alignas(16) Stage {
        u32x4 k[kTileBytes / 16];
        u32x4 v[kTileBytes / 16];
    };
    // Per wave: its stage buffers while streaming, its partial (O~) at segment end.
    union alignas(16) WaveArea {
        float o[kTmMax][D + 4];
        Stage st[STAGES];
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

        // What the lane fetches in wave-wide load i of a tile, as a byte offset within the tile.
        uint32_t k_src[kLoads];
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
            const uint32_t pos = (uint32_t)i * 1024u + (uint32_t)lane * 16u;   // where it lands
            const uint32_t row = pos / kRowBytes, chunk = (pos % kRowBytes) / 16u;
            k_src[i] = row * kRowBytes + ((chunk ^ (row & 15u)) & (kChunksPerRow - 1)) * 16u;
        }
        const uint32_t v_src = (uint32_t)g * kRowBytes + (uint32_t)r * 16u;   // + row 16*blk + 4*j, piece p
        // Where the lane reads its K operand chunk 4*c2 + g of token k_tok (+ block and stage offsets)
        uint32_t k_rd[kKC];
#pragma unroll
        for (int c2 = 0; c2 < kKC; ++c2)
            k_rd[c2] = (uint32_t)k_tok * kRowBytes + (((uint32_t)(4 * c2 + g) ^ (uint32_t)k_tok) * 16u);
        Stage* const stages = sm.area[w].st;

        GqaWave<DT, D, NBLK, MB> wv;
        wv.load_q(a, tr, n_ctx, r, g);

        // Fill one stage: `off` is the byte offset of the wave's tile in the slab (an offset past
        // the slab writes zeros to LDS without any memory traffic).
        auto issue = [&](auto stage_index, uint32_t off) {
            constexpr int s = decltype(stage_index)::value;
#pragma unroll
            for (int i = 0; i < kLoads; ++i)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(k_slab, LEAN_LDS_PTR(&stages[s].k[i * 64]), 16, (int)(off + k_src[i]), 0,
                                                         0, kStreamOnce);
#pragma unroll
            for (int blk = 0; blk < NBLK; ++blk) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
#pragma unroll
                    for (int p = 0; p < kPieces; ++p)
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(
                            v_slab, LEAN_LDS_PTR(&stages[s].v[((blk * 4 + j) * kPieces + p) * 64]), 16,
                            (int)(off + v_src + (uint32_t)(blk * 16 + 4 * j) * kRowBytes + 256u * p), 0, 0, kStreamOnce);
                }
            }
        };

        // One staged K tile against Q, the online softmax, then P against the staged V tile.
        auto attend = [&](auto stage_index, int step) {
            constexpr int s = decltype(stage_index)::value;
            const char* kbuf = reinterpret_cast<const char*>(stages[s].k);
            u32x4 kb[NBLK][kKC];
#pragma unroll
            for (int blk = 0; blk < NBLK; ++blk) {
#pragma unroll
                for (int c2 = 0; c2 < kKC; ++c2)
                    kb[blk][c2] = *reinterpret_cast<const u32x4*>(kbuf + (uint32_t)(blk * 16) * kRowBytes + k_rd[c2]);
            }
            u32x4 vb[NBLK][4][kPieces];
#pragma unroll
            for (int blk = 0; blk < NBLK; ++blk) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
#pragma unroll
                    for (int p = 0; p < kPieces; ++p) vb[blk][j][p] = stages[s].v[((blk * 4 + j) * kPieces + p) * 64 + lane];
                }
            }
            wv.step(kb, step * kTn + w * kCH, g, a.scale_log2e, [&](int blk, int j, int i) { return vb[blk][j][i / 4][i % 4]; },
                    [] { wait_lds_reads(); });   // the stage may be refilled once its reads have returned
        };

        const int it_first = sg.local_iter;
        const int n_it = sg.local_iter_end - sg.local_iter;
        // Every stage is refilled unconditionally, past the segment from beyond the slab, so that
        // the number of loads issued after those of a stage is the same constant at every wait.
        constexpr uint32_t kPastSlab = 0xF0000000u;
        const uint32_t wave_off = (uint32_t)(w * kCH) * kRowBytes;
        auto off_at = [&](int k) {
            return k < n_it ? wave_off + (uint32_t)(it_first + k) * (uint32_t)(kTn * kRowBytes) : kPastSlab;
        };
        using S0 = std::integral_constant<int, 0>;
        using S1 = std::integral_constant<int, 1>;
        using S2 = std::integral_constant<int, 2>;
        using S3 = std::integral_constant<int, 3>;
        auto turn = [&](auto stage_index, int k) {
            constexpr int s = decltype(stage_index)::value;
            if (k + s < n_it) {
                wait_loads_outstanding<(STAGES - 1) * kStageLoads>();
                attend(stage_index, it_first + k + s);
                if (a.cta_clock && k + s == 0 && threadIdx.x == 0) a.cta_clock[kClockWords * cta + kClkFirstStep] = wall_clock64();
            }
            issue(stage_index, off_at(k + s + STAGES));
        };
        issue(S0{}, off_at(0));
        issue(S1{}, off_at(1));
        if constexpr (STAGES > 2) issue(S2{}, off_at(2));
        if constexpr (STAGES > 3) issue(S3{}, off_at(3));
        for (int k = 0; k < n_it; k += STAGES) {
            turn(S0{}, k);
            turn(S1{}, k);
            if constexpr (STAGES > 2) turn(S2{}, k);
            if constexpr (STAGES > 3) turn(S3{}, k);
        }
        // the loads still outstanding write (zeros) into the area the partial is parked in next
        wait_loads_outstanding<0>();

        wv.park(sm, w, r, g, [](int m, int e) { return col_of(m, e); });
        __syncthreads();
    }
};

}  // namespace lean
