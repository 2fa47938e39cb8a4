// Matrix-core helpers shared by the product kernels (gfx950 only).
#pragma once

#include "dab_internal.h"

namespace dab {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

// One 32 x 32 x 64 product of 4-bit floats (E2M1), fp32 accumulate.  Lane l of the A operand holds
// row l % 32 and the 32 k of half l / 32 (sixteen bytes), lane l of the B operand column l % 32 and
// the same k; register v of the result is row (v / 4) * 8 + (l / 32) * 4 + v % 4, column l % 32.
__device__ __forceinline__ v16f mfma_fp4(v4i a, v4i b, v16f c) {
    const v8i a8 = {a.x, a.y, a.z, a.w, 0, 0, 0, 0};
    const v8i b8 = {b.x, b.y, b.z, b.w, 0, 0, 0, 0};
    // cbsz = blgp = 4 selects fp4 for both operands; scale bytes 0x7f = 2^0
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, c, 4, 4, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
}

// Output forms of a product kernel.
enum { kOutY = 0, kOutYDebug = 1, kOutSplit = 2, kOutBits = 3 };

}  // namespace dab
