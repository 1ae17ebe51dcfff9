// Kernel variants: core family x dtype x head dim x tile shape.  The decode kernels are compiled in
// one translation unit per (family, dtype) (lean_kernels.hip, six times); the host side asks them
// for a variant's entry points and shape through the functions declared here.
//   VALU core:  U loads of 16 bytes per lane for K and again for V per step, NW waves;
//               LeanTile T_n = NW * U * 64/(D/8) tokens.
//   MFMA core:  NBLK blocks of 16 tokens per wave per step, NW waves; T_n = NW * NBLK * 16.
//               One (T_m <= 16) or two (T_m <= 32, D <= 128) blocks of 16 query rows per pass.
#pragma once
#include "../../include/lean_attn.h"

namespace lean {

constexpr int kNumShapes = LEAN_ATTN_NUM_TILE_SHAPES;  // tile shapes per (family, dtype, head dim), numbered 1..9 (not every one is built for every family)

struct Variant {
    const void* fn;           // arguments by value (null: no such variant)
    const void* fn_indirect;  // arguments read from a device block (built for the candidate default shapes only)
    int T_n;
    int threads;
};

// shape 1..kNumShapes; D in {64, 128, 256} (two row blocks: {64, 128}); fn == nullptr otherwise
Variant variant_mha_f16(int D, int shape);
Variant variant_mha_bf16(int D, int shape);
Variant variant_gqa_f16(int D, int shape);
Variant variant_gqa_bf16(int D, int shape);
Variant variant_gqa2_f16(int D, int shape);
Variant variant_gqa2_bf16(int D, int shape);

}  // namespace lean
