// The decode kernels of one (core family, dtype): compiled six times, with
//   -DLEAN_TU_FAMILY=0 (VALU single-row core) | 1 (MFMA core, one block of 16 query rows) |
//                    2 (MFMA core, two row blocks)   and   -DLEAN_TU_DT=0 (f16) | 1 (bf16),
// so that the variants build in parallel.  Each unit exports one look-up function
// (lean_variants.h) that hands the host side the kernel entry points of a (head dim, shape).
#include <hip/hip_runtime.h>

#include "lean_device.h"
#include "lean_gqa_core.h"
#include "lean_gqa_lds_core.h"
#include "lean_kernel.h"
#include "lean_mha_core.h"
#include "lean_variants.h"

#if !defined(LEAN_TU_FAMILY) || !defined(LEAN_TU_DT)
#error "compile with -DLEAN_TU_FAMILY=0|1|2 -DLEAN_TU_DT=0|1"
#endif

namespace lean {

template <class Core, bool INDIRECT = false>
static Variant variant_of() {
    const void* indirect = nullptr;
    if constexpr (INDIRECT) indirect = reinterpret_cast<const void*>(&lean_decode_kernel_indirect<Core>);
    return Variant{reinterpret_cast<const void*>(&lean_decode_kernel<Core>), indirect, Core::kTn, Core::kThreads};
}

constexpr int DT = LEAN_TU_DT;
constexpr Variant kNone = {nullptr, nullptr, 0, 0};

#if LEAN_TU_FAMILY == 0
// <loads of 16 bytes per lane per stream, waves, double-buffered>
template <int D>
static Variant shape_of(int shape) {
    switch (shape) {
        case 1: return variant_of<MhaCore<DT, D, 8, 4, true>>();
        case 2: return variant_of<MhaCore<DT, D, 4, 4, true>>();
        case 3: return variant_of<MhaCore<DT, D, 8, 4, false>>();
        case 4: return variant_of<MhaCore<DT, D, 8, 8, false>>();
        case 5: return variant_of<MhaCore<DT, D, 4, 8, false>>();
        case 6: return variant_of<MhaCore<DT, D, 4, 4, false>, true>();
        default: return kNone;
    }
}
#elif LEAN_TU_FAMILY == 1
// <16-token blocks per wave per step, waves, double-buffered>.  At D = 256 the double-buffered shapes
// 1 and 3 do not fit the register file (50-70 spilled registers per lane) and are not built.
template <int D>
static Variant shape_of(int shape) {
    if (D == 256 && (shape == 1 || shape == 3)) return kNone;
    switch (shape) {
        case 1: return variant_of<GqaCore<DT, D == 256 ? 128 : D, 2, 4, true>>();
        case 2: return variant_of<GqaCore<DT, D, 1, 4, true>>();
        case 3: return variant_of<GqaCore<DT, D == 256 ? 128 : D, 1, 8, true>>();
        case 4: return variant_of<GqaCore<DT, D, 1, 8, false>, true>();
        case 5: return variant_of<GqaCore<DT, D, 2, 4, false>, true>();
        case 6: return variant_of<GqaCore<DT, D, 1, 4, false>, true>();
        default: break;
    }
    // K/V staged in LDS by direct loads: <blocks per wave per step, waves, stages>.  Measured on the
    // 256-unit part they stream 0-4 % slower than the register shapes above (the loads that stay in
    // flight across the arithmetic are more than the memory system needs), so no default uses them.
    if constexpr (D >= 128) {
        switch (shape) {
            case 7: return variant_of<GqaLdsCore<DT, D, 256 / D, 4, 2>>();
            case 8: if constexpr (D == 128) return variant_of<GqaLdsCore<DT, D, 1, 8, 2>>(); else return variant_of<GqaLdsCore<DT, D, 1, 2, 2>>();
            case 9: if constexpr (D == 128) return variant_of<GqaLdsCore<DT, D, 1, 4, 2>>(); else break;
            default: break;
        }
    }
    return kNone;
}
#else
// two blocks of 16 query rows per pass over K/V (17..32 rows per output tile, D <= 128)
template <int D>
static Variant shape_of(int shape) {
    switch (shape) {
        case 1: return variant_of<GqaCore<DT, D, 2, 4, true, 2>, true>();
        case 2: return variant_of<GqaCore<DT, D, 1, 4, true, 2>>();
        case 3: case 4: return variant_of<GqaCore<DT, D, 1, 8, false, 2>, true>();
        case 5: return variant_of<GqaCore<DT, D, 2, 4, false, 2>>();
        case 6: return variant_of<GqaCore<DT, D, 1, 4, false, 2>>();
        default: break;
    }
    if constexpr (D == 128) {
        switch (shape) {
            case 7: return variant_of<GqaLdsCore<DT, D, 2, 4, 2, 2>>();
            case 8: return variant_of<GqaLdsCore<DT, D, 1, 8, 2, 2>>();
            case 9: return variant_of<GqaLdsCore<DT, D, 1, 4, 2, 2>>();
            default: break;
        }
    }
    return kNone;
}
#endif

#define LEAN_CAT3(a, b, c) a##b##c
#define LEAN_TU_NAME(fam, dt) LEAN_CAT3(variant_, fam, dt)
#if LEAN_TU_FAMILY == 0
#define LEAN_FAM mha_
#elif LEAN_TU_FAMILY == 1
#define LEAN_FAM gqa_
#else
#define LEAN_FAM gqa2_
#endif
#if LEAN_TU_DT == 0
#define LEAN_DTN f16
#else
#define LEAN_DTN bf16
#endif
#define LEAN_TU_NAME2(fam, dt) LEAN_TU_NAME(fam, dt)

Variant LEAN_TU_NAME2(LEAN_FAM, LEAN_DTN)(int D, int shape) {
    if (D == 64) return shape_of<64>(shape);
    if (D == 128) return shape_of<128>(shape);
#if LEAN_TU_FAMILY != 2
    if (D == 256) return shape_of<256>(shape);
#endif
    return kNone;
}

}  // namespace lean
