// Reciprocal used for the per-reference-element factor 1/|r| of the relative error.
//
// evo.h defines that factor as the correctly rounded binary32 quotient 1.0f / |r|.  On
// gfx950, v_rcp_f32 followed by one Newton step in fused multiply-adds gives exactly
// that quotient for EVERY binary32 input in [2^-126, 2^126): rcp_check.hip compares the
// two over all 2^31 - 2^24 such inputs on the device (no mismatch), and the GPU tests
// run it.  From 2^126 upwards the quotient is subnormal and the shortcut does not hold
// (it differs for every input there), so callers must use the division for those.
#pragma once

#include <hip/hip_runtime.h>

namespace evo {

constexpr float kRecipShortcutBelow = 0x1p126f;

__device__ __forceinline__ float recip_shortcut(float a) {
    const float y = __builtin_amdgcn_rcpf(a);
    const float e = __builtin_fmaf(-a, y, 1.0f);
    return __builtin_fmaf(y, e, y);
}

}  // namespace evo
