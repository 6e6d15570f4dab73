// Residual rotation, normalisation, Lloyd-Max quantisation and bit-packing in one kernel
// (Section "Architecture", Indexing: r = x~ - c~_l, rotate by Pi, normalise Pi r, quantise each
// coordinate; Bit accounting: b*d code bits and a float16 norm per vector), plus the query-side
// rotation z = Pi q~ (Section "Architecture", Search).
//
// The rotation is a d x d contraction on the matrix cores (v_mfma_f32_32x32x16_f16 on split float16
// operands with float32 accumulation, see split_f16.h).  A wavefront owns 32 rows; the unit residuals
// are the right-hand operand held in registers, 32-row tiles of Pi stream through LDS as the
// left-hand operand.  In tile t a lane holds, for one row, the rotated coordinates
// 32t + 8g + 4*half + {0..3}; all tiles stay in registers until the norm of Pi r is known.
#include <hip/hip_fp16.h>

#include "kernels.h"
#include "split_f16.h"

namespace ivftq {

namespace {

template <int DP>
struct EncCfg {
    static constexpr int KB = DP / 16;
    static constexpr int NT = DP / 32;
    static constexpr int LDH = DP + 8;                     // halves per LDS row of the Pi tile
    static constexpr size_t pi_bytes = (size_t)2 * 32 * LDH * sizeof(uint16_t);
    static constexpr size_t code_bytes = 4 * 32 * DP;      // per wave: 32 rows x DP bytes
    static constexpr size_t lds_bytes = pi_bytes + 256 * 4 + code_bytes;
    static constexpr int occupancy = DP <= 160 ? 2 : 1;    // wavefronts per SIMD the register budget allows
};

template <int DP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(EncCfg<DP>::occupancy)))
void k_encode(int mode, EncodeArgs a, int vec4) {
    using Cfg = EncCfg<DP>;
    constexpr int KB = Cfg::KB;
    extern __shared__ unsigned char lds_raw[];
    uint16_t* ph = reinterpret_cast<uint16_t*>(lds_raw);           // [32][LDH] hi parts of 32 rows of Pi
    uint16_t* pl = ph + 32 * Cfg::LDH;                               // [32][LDH] lo parts
    float* tau_s = reinterpret_cast<float*>(pl + 32 * Cfg::LDH);     // [256]
    uint8_t* code_s = reinterpret_cast<uint8_t*>(tau_s + 256);

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, half = lane >> 5, j = lane & 31;
    const int64_t row0 = (int64_t)blockIdx.x * kRowsPerWG + wave * 32;
    const int64_t row = row0 + j;
    const bool valid = row < a.n;
    const int d = a.d;
    const int K = 1 << a.b;

    if (mode != 2 && tid < K - 1) tau_s[tid] = a.tau[tid];

    // x~, then the residual against the assigned centroid and its norm gamma.  The rotation acts on
    // the unit residual r/gamma: Pi r / |Pi r| does not depend on the scale of r, and a unit vector
    // keeps the split float16 form accurate however small the residual is.
    float v[KB][8];
    load_row_blocks<KB>(a.x + (valid ? row : 0) * (int64_t)d, valid, d, vec4, half, v);
    const float n2 = row_norm2<KB>(v);
    const bool good = (n2 > 0.f) && (n2 < __builtin_inff());
    const float inv_n = good ? 1.f / sqrtf(n2) : 0.f;   // one division per row, then multiplies
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int e = 0; e < 8; ++e) v[kb][e] *= inv_n;

    int cell = -1;
    float gamma = 0.f;
    if (mode != 2) {
        cell = valid ? a.assign[row] : -1;
        float c[KB][8];
        load_row_blocks<KB>(a.cent + (int64_t)(cell < 0 ? 0 : cell) * a.cent_pitch, cell >= 0, DP, 1, half, c);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int e = 0; e < 8; ++e) v[kb][e] -= c[kb][e];
        gamma = sqrtf(row_norm2<KB>(v));
        const float inv_g = (gamma > 1e-30f) ? 1.f / gamma : 0.f;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int e = 0; e < 8; ++e) v[kb][e] *= inv_g;
    }
    half8 bh[KB], bl[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            _Float16 h, l;
            split_scaled(v[kb][e], h, l);
            bh[kb][e] = h;
            bl[kb][e] = l;
        }

    // u = Pi r^: 32 output coordinates per tile, every tile's accumulator kept until the norm is known
    floatx16 acc[Cfg::NT];
    const uint16_t* ah_base = ph + j * Cfg::LDH + 8 * half;
    const uint16_t* al_base = pl + j * Cfg::LDH + 8 * half;
#pragma unroll
    for (int t = 0; t < Cfg::NT; ++t) {
        __syncthreads();
        for (int e = tid; e < 32 * (DP / 8); e += 256) {
            const int rr = e / (DP / 8), c8 = e % (DP / 8);
            const int64_t src = (int64_t)(t * 32 + rr) * DP + c8 * 8;
            *reinterpret_cast<uint4*>(ph + rr * Cfg::LDH + c8 * 8) = *reinterpret_cast<const uint4*>(a.pi_h + src);
            *reinterpret_cast<uint4*>(pl + rr * Cfg::LDH + c8 * 8) = *reinterpret_cast<const uint4*>(a.pi_l + src);
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[t][q] = 0.f;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const half8 ah = *reinterpret_cast<const half8*>(ah_base + 16 * kb);
            const half8 al = *reinterpret_cast<const half8*>(al_base + 16 * kb);
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh[kb], acc[t], 0, 0, 0);
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bl[kb], acc[t], 0, 0, 0);
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, bh[kb], acc[t], 0, 0, 0);
        }
    }
    constexpr float kUnscale = 1.f / (kSplitScale * kSplitScale);

    if (mode == 2) {
        if (valid) {
#pragma unroll
            for (int t = 0; t < Cfg::NT; ++t)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 o = make_float4(acc[t][4 * g] * kUnscale, acc[t][4 * g + 1] * kUnscale,
                                                 acc[t][4 * g + 2] * kUnscale, acc[t][4 * g + 3] * kUnscale);
                    const int64_t at = row * (int64_t)DP + t * 32 + 8 * g + 4 * half;
                    *reinterpret_cast<float4*>(a.zout + at) = o;
                    if (a.zh_out) {
                        const float z[4] = {o.x, o.y, o.z, o.w};
                        uint16_t h[4], l[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            _Float16 hi, lo;
                            split_scaled(z[e], hi, lo);
                            h[e] = __builtin_bit_cast(uint16_t, hi);
                            l[e] = __builtin_bit_cast(uint16_t, lo);
                        }
                        *reinterpret_cast<uint2*>(a.zh_out + at) = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
                        *reinterpret_cast<uint2*>(a.zl_out + at) = make_uint2(l[0] | ((uint32_t)l[1] << 16), l[2] | ((uint32_t)l[3] << 16));
                    }
                }
        }
        return;
    }

    // |Pi r^| in the accumulators' scale (rows of Pi beyond d are zero, so padded coordinates add nothing)
    float u2 = 0.f;
#pragma unroll
    for (int t = 0; t < Cfg::NT; ++t)
#pragma unroll
        for (int q = 0; q < 16; ++q) u2 += acc[t][q] * acc[t][q];
    u2 += __shfl_xor(u2, 32);
    const float un = sqrtf(u2);
    const float inv_u = (un > 1e-30f) ? 1.f / un : 0.f;   // a zero residual quantises as rho = 0

    // quantise: code = #{i : rho >= tau_i}, by bisection over the ascending boundaries
    uint8_t* my_codes = code_s + wave * (32 * DP) + j * DP;
#pragma unroll
    for (int t = 0; t < Cfg::NT; ++t) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint32_t packed = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float rho = acc[t][4 * g + e] * inv_u;
                int code = 0;
#pragma unroll
                for (int lvl = 7; lvl >= 0; --lvl) {       // straight-line bisection, levels above b skipped
                    const int step = 1 << lvl;
                    if (step < K && rho >= tau_s[code + step - 1]) code += step;
                }
                packed |= (uint32_t)code << (8 * e);
            }
            *reinterpret_cast<uint32_t*>(my_codes + t * 32 + 8 * g + 4 * half) = packed;
        }
    }
    __syncthreads();

    const uint8_t* wave_codes = code_s + wave * (32 * DP);
    if (mode == 1) {
        if (a.codes_flat) {
            const int64_t rows_here = (a.n - row0) < 32 ? (a.n - row0) : 32;
            for (int64_t e = lane; e < rows_here * d; e += 64) {
                const int rl = (int)(e / d), c = (int)(e % d);
                a.codes_flat[row0 * d + e] = wave_codes[rl * DP + c];
            }
        }
        if (valid && half == 0 && a.gamma_flat)
            a.gamma_flat[row] = __half_as_ushort(__float2half_rn(cell >= 0 ? gamma : 0.f));
        return;
    }

    // mode 0: pack b-bit codes into 32-bit words (coordinate j occupies bits [j*b, j*b+b) of the
    // vector's little-endian bit string) and scatter them to the vector's storage slot.
    const int words = a.store.words;
    const int b = a.b;
    for (int item = lane; item < 32 * words; item += 64) {
        const int rl = item & 31, w = item >> 5;
        const int64_t rrow = row0 + rl;
        if (rrow >= a.n) continue;
        const int64_t slot = a.slot[rrow];
        if (slot < 0) continue;
        const int first = (32 * w) / b;
        uint32_t word = 0;
        for (int c = first; c < d; ++c) {
            const int sh = c * b - 32 * w;
            if (sh >= 32) break;
            const uint32_t code = wave_codes[rl * DP + c];
            word |= sh >= 0 ? (code << sh) : (code >> (-sh));
        }
        a.store.codes[((slot >> 6) * words + w) * 64 + (slot & 63)] = word;
    }
    if (valid && half == 0) {
        const int64_t slot = a.slot[row];
        if (slot >= 0) {
            a.store.gamma[slot] = __half_as_ushort(__float2half_rn(gamma));
            a.store.ids[slot] = a.labels ? a.labels[row] : a.label_base + row;
        }
    }
}

template <int DP>
hipError_t run(int mode, const EncodeArgs& a, hipStream_t st) {
    static bool attr_set = false;
    const size_t lds = EncCfg<DP>::lds_bytes;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_encode<DP>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int64_t blocks = (a.n + kRowsPerWG - 1) / kRowsPerWG;
    const int vec4 = (a.d % 4 == 0) && (reinterpret_cast<uintptr_t>(a.x) % 16 == 0);
    hipLaunchKernelGGL(k_encode<DP>, dim3((unsigned)blocks), dim3(256), lds, st, mode, a, vec4);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_encode(int mode, const EncodeArgs& a, hipStream_t st) {
    if (a.n <= 0) return hipSuccess;
    switch (rot_dp(a.d)) {
        case 32: return run<32>(mode, a, st);
        case 64: return run<64>(mode, a, st);
        case 96: return run<96>(mode, a, st);
        case 128: return run<128>(mode, a, st);
        case 160: return run<160>(mode, a, st);
        case 192: return run<192>(mode, a, st);
        case 224: return run<224>(mode, a, st);
        case 256: return run<256>(mode, a, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ivftq
