// Device helpers shared by the float16 matrix-core kernels: the split float16 operand form and the
// loading of fp32 rows in the lane layout of v_mfma_f32_32x32x16_f16.
//
// Split form: 1024 v = hi + lo with hi = fp16(1024 v), lo = fp16(1024 v - hi).  A product of two
// split numbers accumulated as hi*hi + hi*lo + lo*hi in float32 equals 2^20 * (v * w) to about
// 2^-22 relative (the lo*lo term is below 2^-24).  Values below 2.4e-4 in magnitude have a lo part
// under the float16 normal range, where it weighs at most 6e-8 of the unit scale.
//
// Operand layout of v_mfma_f32_32x32x16_f16: A is 32x16 (lane = i + 32*(k/8), element k%8), B is
// 16x32 likewise; D[i][j] sits in lane j + 32*((i/4)%2), register (i%4) + 4*(i/8).  A lane
// (j, half) therefore takes the coordinates 16*kb + 8*half + [0, 8) of row j in block kb.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "kernels.h"

namespace ivftq {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));

// v must be a finished float32 value, not an expression: the only multiplication in here is by a power
// of two and therefore exact.  With an inexact product in its place (v * factor * 1024 folded into one
// multiplication) the compiler contracts that product once into the float16 conversion and once into
// the subtraction; where the float32 product lands on a float16 tie the two round apart, the leading
// part used as operand and the one the trailing part was taken against differ by a unit in the last
// place, and hi + lo is off by 2^-11 (seen as one wrong coordinate in about 0.2 % of the rows).
__device__ __forceinline__ void split_scaled(float v, _Float16& hi, _Float16& lo) {
    const float V = v * kSplitScale;
    hi = (_Float16)V;
    lo = (_Float16)(V - (float)hi);
}

// v[kb][e] = p[16*kb + 8*half + e] for a row of `len` floats at p (zero beyond len, or when the
// row is not valid).  Every load is unconditional on a clamped index, so p must be readable even
// for an invalid row.  vec4: len % 4 == 0 and p 16-byte aligned.  The padded width 16*KB is the
// smallest supported size that holds len, which is within 32 of it: only the last two blocks can
// reach past len, the others are read without a test.
template <int KB>
__device__ __forceinline__ void load_row_blocks(const float* __restrict__ p, bool valid, int len, int vec4,
                                                int half, float (&v)[KB][8]) {
    if (vec4) {
        const float4* q = reinterpret_cast<const float4*>(p);
        const int last4 = len / 4 - 1;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int c = 16 * kb + 8 * half + 4 * e;
                const int i4 = c / 4;
                const bool inside = 16 * kb + 16 <= 16 * KB - 32;      // known when the kernel is compiled
                const float4 t = q[(inside || i4 < last4) ? i4 : last4];
                const bool in = valid && (inside || c < len);
                v[kb][4 * e] = in ? t.x : 0.f; v[kb][4 * e + 1] = in ? t.y : 0.f;
                v[kb][4 * e + 2] = in ? t.z : 0.f; v[kb][4 * e + 3] = in ? t.w : 0.f;
            }
    } else {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int c = 16 * kb + 8 * half + e;
                const bool inside = 16 * kb + 16 <= 16 * KB - 32;
                const float t = p[(inside || c < len) ? c : len - 1];
                v[kb][e] = (valid && (inside || c < len)) ? t : 0.f;
            }
    }
}

// Sum of squares of the whole row (both lane halves together).
template <int KB>
__device__ __forceinline__ float row_norm2(const float (&v)[KB][8]) {
    float n2 = 0.f;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int e = 0; e < 8; ++e) n2 += v[kb][e] * v[kb][e];
    return n2 + __shfl_xor(n2, 32);
}

}  // namespace ivftq
