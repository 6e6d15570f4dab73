// Residual rotation, normalisation, Lloyd-Max quantisation and bit-packing in one kernel
// (Section "Architecture", Indexing: r = x~ - c~_l, rotate by Pi, normalise Pi r, quantise each
// coordinate; Bit accounting: b*d code bits and a float16 norm per vector), plus the query-side
// rotation z = Pi q~ (Section "Architecture", Search).
//
// The rotation is a d x d contraction on the matrix cores (v_mfma_f32_32x32x2_f32, see
// coarse_kernels.hip for the operand layout).  A wavefront owns 32 rows; the residuals are the
// right-hand operand held in registers, 32-row tiles of Pi stream through LDS as the left-hand
// operand.  In tile t a lane holds, for one row, the rotated coordinates 32t + 8g + 4*half + {0..3}.
#include <hip/hip_fp16.h>

#include "kernels.h"

namespace ivftq {

typedef float floatx16 __attribute__((ext_vector_type(16)));

namespace {

template <int DP>
struct EncCfg {
    static constexpr int NT = DP / 32;
    static constexpr int LDP = DP + 1;
    static constexpr size_t pi_floats = 32 * LDP;
    static constexpr size_t code_bytes = 4 * 32 * DP;      // per wave: 32 rows x DP bytes
    static constexpr size_t lds_bytes = pi_floats * 4 + 256 * 4 + code_bytes;
};

// Coordinates k0 + [0, DP/2) of the row at p (len valid floats) into v, zero beyond len.  Every
// load is unconditional on a clamped index, so the compiler emits straight-line code; p must point
// at a readable row even when `valid` is false.
template <int DP>
__device__ __forceinline__ void load_half(const float* __restrict__ p, bool valid, int len, int vec4,
                                          int k0, float (&v)[DP / 2]) {
    if (vec4) {
        const float4* q = reinterpret_cast<const float4*>(p);
        const int last4 = len / 4 - 1;
#pragma unroll
        for (int s = 0; s < DP / 2; s += 4) {
            const int i4 = (k0 + s) / 4;
            const float4 t = q[i4 < last4 ? i4 : last4];
            const bool in = valid && (k0 + s < len);
            v[s] = in ? t.x : 0.f; v[s + 1] = in ? t.y : 0.f; v[s + 2] = in ? t.z : 0.f; v[s + 3] = in ? t.w : 0.f;
        }
    } else {
#pragma unroll
        for (int s = 0; s < DP / 2; ++s) {
            const int i = k0 + s;
            const float t = p[i < len ? i : len - 1];
            v[s] = (valid && i < len) ? t : 0.f;
        }
    }
}

template <int DP>
__global__ __launch_bounds__(256, 2) void k_encode(int mode, EncodeArgs a, int vec4) {
    using Cfg = EncCfg<DP>;
    extern __shared__ float lds[];
    float* pi_tile = lds;                                   // [32][LDP]
    float* tau_s = lds + Cfg::pi_floats;                    // [256]
    uint8_t* code_s = reinterpret_cast<uint8_t*>(tau_s + 256);

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, half = lane >> 5, j = lane & 31;
    const int64_t row0 = (int64_t)blockIdx.x * kRowsPerWG + wave * 32;
    const int64_t row = row0 + j;
    const bool valid = row < a.n;
    const int d = a.d;
    const int K = 1 << a.b;

    if (mode != 2 && tid < K - 1) tau_s[tid] = a.tau[tid];

    // x~ (and the residual against the assigned centroid)
    float r[DP / 2];
    load_half<DP>(a.x + (valid ? row : 0) * (int64_t)d, valid, d, vec4, half * (DP / 2), r);
    float n2 = 0.f;
#pragma unroll
    for (int s = 0; s < DP / 2; ++s) n2 += r[s] * r[s];
    n2 += __shfl_xor(n2, 32);
    const bool good = (n2 > 0.f) && (n2 < __builtin_inff());
    const float nrm = sqrtf(n2);
#pragma unroll
    for (int s = 0; s < DP / 2; ++s) r[s] = good ? r[s] / nrm : 0.f;

    int cell = -1;
    float gamma = 0.f;
    if (mode != 2) {
        cell = valid ? a.assign[row] : -1;
        float c[DP / 2];
        load_half<DP>(a.cent + (int64_t)(cell < 0 ? 0 : cell) * a.cent_pitch, cell >= 0, DP, 1,
                      half * (DP / 2), c);
        float g2 = 0.f;
#pragma unroll
        for (int s = 0; s < DP / 2; ++s) {
            r[s] = r[s] - c[s];
            g2 += r[s] * r[s];
        }
        g2 += __shfl_xor(g2, 32);
        gamma = sqrtf(g2);
    }

    // u = Pi r, 32 output coordinates per tile.  The norm of the whole rotated vector is needed
    // before any coordinate can be quantised, so the tiles are swept twice: once for |Pi r|^2 and
    // once, bit-identically, to quantise.  That keeps one 32x32 accumulator live instead of d/32.
    const float* a_base = pi_tile + j * Cfg::LDP + half * (DP / 2);
    auto rotate_tile = [&](int t) -> floatx16 {
        __syncthreads();
        for (int e = tid; e < 32 * (DP / 4); e += 256) {
            const int rr = e / (DP / 4), q4 = e % (DP / 4);
            const float4 v = *reinterpret_cast<const float4*>(a.pi + (int64_t)(t * 32 + rr) * DP + q4 * 4);
            float* dst = pi_tile + rr * Cfg::LDP + q4 * 4;
            dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
        }
        __syncthreads();
        floatx16 acc;
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[q] = 0.f;
#pragma unroll
        for (int s = 0; s < DP / 2; ++s)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a_base[s], r[s], acc, 0, 0, 0);
        return acc;
    };

    if (mode == 2) {
#pragma unroll 1
        for (int t = 0; t < Cfg::NT; ++t) {
            const floatx16 acc = rotate_tile(t);
            if (valid) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float4 o = make_float4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
                    const int64_t at = row * (int64_t)DP + t * 32 + 8 * g + 4 * half;
                    *reinterpret_cast<float4*>(a.zout + at) = o;
                    if (a.zh_out) {
                        const float v[4] = {o.x, o.y, o.z, o.w};
                        uint16_t h[4], l[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float V = v[e] * kSplitScale;
                            const _Float16 hi = (_Float16)V;
                            const _Float16 lo = (_Float16)(V - (float)hi);
                            h[e] = __builtin_bit_cast(uint16_t, hi);
                            l[e] = __builtin_bit_cast(uint16_t, lo);
                        }
                        *reinterpret_cast<uint2*>(a.zh_out + at) = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
                        *reinterpret_cast<uint2*>(a.zl_out + at) = make_uint2(l[0] | ((uint32_t)l[1] << 16), l[2] | ((uint32_t)l[3] << 16));
                    }
                }
            }
        }
        return;
    }

    // |Pi r| (rows of Pi beyond d are zero, so padded coordinates add nothing)
    float u2 = 0.f;
#pragma unroll 1
    for (int t = 0; t < Cfg::NT; ++t) {
        const floatx16 acc = rotate_tile(t);
#pragma unroll
        for (int q = 0; q < 16; ++q) u2 += acc[q] * acc[q];
    }
    u2 += __shfl_xor(u2, 32);
    const float un = sqrtf(u2);
    const bool degenerate = !(un > 1e-30f);

    // quantise: code = #{i : rho >= tau_i}, by bisection over the ascending boundaries
    uint8_t* my_codes = code_s + wave * (32 * DP) + j * DP;
#pragma unroll 1
    for (int t = 0; t < Cfg::NT; ++t) {
        const floatx16 acc = rotate_tile(t);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint32_t packed = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float rho = degenerate ? 0.f : acc[4 * g + e] / un;
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
