// Coarse scoring on the matrix cores: <x~_i, c~_l> for every data row i and every cell l, with
// either a running argmax (encode step "assign to the nearest centroid by maximum inner product",
// Section "Architecture", Indexing) or the full score matrix (search step "coarse term computed
// exactly", Section "Architecture", Search).
//
// Shape of the work: n x d times d x L with small d (96..200) and a result that is never kept
// (argmax) or kept once (scores).  One wavefront owns 32*R data rows for the whole kernel and holds
// them in registers as the right-hand MFMA operand; centroid tiles stream through LDS and are the
// left-hand operand, so that in each 32x32 result a lane holds one data row's scores against 16
// centroids and the argmax over centroids never crosses lanes until the very end.
//
// Arithmetic: both operands are used in split float16 form (split_f16.h) on
// v_mfma_f32_32x32x16_f16 with float32 accumulation, so a score differs from the float32 dot
// product by about 2e-7, well inside the 1e-5 near-tie allowance, at the float16 matrix rate.
#include "kernels.h"
#include "split_f16.h"

namespace ivftq {

namespace {

constexpr int kNT = 2;                       // 32-centroid tiles per LDS stage
constexpr int kTN = kNT * 32;

template <int DP>
struct CoarseCfg {
    static constexpr int KB = DP / 16;
    static constexpr int LDH = DP + 8;       // halves per LDS row: the 16-byte pad keeps b128 reads conflict free
    static constexpr size_t lds_bytes = (size_t)2 * kTN * LDH * sizeof(uint16_t) + kTN * sizeof(float);
};

// hi[r][c], lo[r][c] = split float16 form of src[r][c]
__global__ void k_split_rows(const float* __restrict__ src, int64_t count, uint16_t* __restrict__ hi,
                             uint16_t* __restrict__ lo) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    _Float16 h, l;
    split_scaled(src[i], h, l);
    hi[i] = __builtin_bit_cast(uint16_t, h);
    lo[i] = __builtin_bit_cast(uint16_t, l);
}

// One 32-row tile of normalised data rows as the B operand (split form).  Returns whether the
// row's norm is usable.
template <int DP>
__device__ __forceinline__ bool load_rows(const float* __restrict__ x, int64_t row, bool valid, int d, int vec4,
                                          int half, half8 (&bh)[DP / 16], half8 (&bl)[DP / 16]) {
    constexpr int KB = DP / 16;
    float v[KB][8];
    load_row_blocks<KB>(x + (valid ? row : 0) * (int64_t)d, valid, d, vec4, half, v);
    const float n2 = row_norm2<KB>(v);
    const bool good = (n2 > 0.f) && (n2 < __builtin_inff());
    const float inv = good ? 1.f / sqrtf(n2) : 0.f;     // one division per row, then multiplies
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            _Float16 h, l;
            split_scaled(v[kb][e] * inv, h, l);
            bh[kb][e] = h;
            bl[kb][e] = l;
        }
    return good;
}

// R = 32-row tiles per wavefront.
template <int DP, int R>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void k_coarse(
    int mode, const float* __restrict__ x, int64_t n, int d, int vec4, const uint16_t* __restrict__ cent_h,
    const uint16_t* __restrict__ cent_l, int cent_pitch, const float* __restrict__ bias, int L, int Lpad,
    int32_t* __restrict__ assign, float* __restrict__ best_out, float* __restrict__ scores,
    int64_t ld_scores, int* __restrict__ flag) {
    using Cfg = CoarseCfg<DP>;
    constexpr int KB = Cfg::KB;
    extern __shared__ unsigned char lds_raw[];
    uint16_t* th = reinterpret_cast<uint16_t*>(lds_raw);            // [TN][LDH] hi parts of the centroid tile
    uint16_t* tl = th + kTN * Cfg::LDH;                               // [TN][LDH] lo parts
    float* tile_bias = reinterpret_cast<float*>(tl + kTN * Cfg::LDH); // [TN]

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, half = lane >> 5, j = lane & 31;
    const int64_t row0 = ((int64_t)blockIdx.x * 4 + wave) * (32 * R);

    half8 bh[R][KB], bl[R][KB];
    bool good[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int64_t row = row0 + 32 * r + j;
        good[r] = load_rows<DP>(x, row, row < n, d, vec4, half, bh[r], bl[r]);
        if (row < n && !good[r] && half == 0) atomicOr(flag, 1);
    }

    float best[R];
    int best_idx[R];
#pragma unroll
    for (int r = 0; r < R; ++r) { best[r] = -__builtin_inff(); best_idx[r] = 0; }
    const uint16_t* ah_base = th + j * Cfg::LDH + 8 * half;
    const uint16_t* al_base = tl + j * Cfg::LDH + 8 * half;
    constexpr float kUnscale = 1.f / (kSplitScale * kSplitScale);

    // gridDim.y workgroups share the centroid stages of one row block (score mode with few rows)
    const int stages = Lpad / kTN, per_y = (stages + (int)gridDim.y - 1) / (int)gridDim.y;
    const int c_lo = (int)blockIdx.y * per_y * kTN;
    const int c_hi = c_lo + per_y * kTN < Lpad ? c_lo + per_y * kTN : Lpad;
    for (int c0 = c_lo; c0 < c_hi; c0 += kTN) {
        __syncthreads();
        // stage TN centroid rows (hi and lo) into LDS, 16 bytes at a time
        for (int e = tid; e < kTN * (DP / 8); e += 256) {
            const int r = e / (DP / 8), c8 = e % (DP / 8);
            const int64_t src = (int64_t)(c0 + r) * cent_pitch + c8 * 8;
            *reinterpret_cast<uint4*>(th + r * Cfg::LDH + c8 * 8) = *reinterpret_cast<const uint4*>(cent_h + src);
            *reinterpret_cast<uint4*>(tl + r * Cfg::LDH + c8 * 8) = *reinterpret_cast<const uint4*>(cent_l + src);
        }
        if (tid < kTN) tile_bias[tid] = bias ? bias[c0 + tid] : 0.f;
        __syncthreads();

        floatx16 acc[R][kNT];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int t = 0; t < kNT; ++t)
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[r][t][q] = 0.f;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
            for (int t = 0; t < kNT; ++t) {
                const half8 ah = *reinterpret_cast<const half8*>(ah_base + t * 32 * Cfg::LDH + 16 * kb);
                const half8 al = *reinterpret_cast<const half8*>(al_base + t * 32 * Cfg::LDH + 16 * kb);
#pragma unroll
                for (int r = 0; r < R; ++r) acc[r][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh[r][kb], acc[r][t], 0, 0, 0);
#pragma unroll
                for (int r = 0; r < R; ++r) acc[r][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bl[r][kb], acc[r][t], 0, 0, 0);
#pragma unroll
                for (int r = 0; r < R; ++r) acc[r][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, bh[r][kb], acc[r][t], 0, 0, 0);
            }
        }

        if (mode == 0 && !bias && c0 + kTN <= L) {
            // plain inner products, whole stage inside the table: compare the raw accumulators
            // (the argmax does not depend on the common 2^20 scale); ascending c, first maximum wins
#pragma unroll
            for (int t = 0; t < kNT; ++t)
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int c = c0 + t * 32 + 8 * (q / 4) + 4 * half + (q % 4);
#pragma unroll
                    for (int r = 0; r < R; ++r)
                        if (acc[r][t][q] > best[r]) { best[r] = acc[r][t][q]; best_idx[r] = c; }
                }
        } else if (mode == 0) {
#pragma unroll
            for (int t = 0; t < kNT; ++t)
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int i = 8 * (q / 4) + 4 * half + (q % 4);
                    const int c = c0 + t * 32 + i;
                    // with a bias the comparison is in true units; without, in accumulator units
                    const float bi = tile_bias[t * 32 + i];
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        const float v = bias ? fmaf(acc[r][t][q], kUnscale, bi) : acc[r][t][q];
                        if (c < L && v > best[r]) { best[r] = v; best_idx[r] = c; }
                    }
                }
        } else {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int64_t row = row0 + 32 * r + j;
                if (row >= n) continue;
#pragma unroll
                for (int t = 0; t < kNT; ++t)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int c = c0 + t * 32 + 8 * g + 4 * half;
                        if (c < ld_scores) {
                            float4 o = make_float4(acc[r][t][4 * g] * kUnscale, acc[r][t][4 * g + 1] * kUnscale,
                                                   acc[r][t][4 * g + 2] * kUnscale, acc[r][t][4 * g + 3] * kUnscale);
                            *reinterpret_cast<float4*>(scores + row * ld_scores + c) = o;
                        }
                    }
            }
        }
    }

    if (mode == 0) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float ob = __shfl_xor(best[r], 32);
            const int oi = __shfl_xor(best_idx[r], 32);
            if (ob > best[r] || (ob == best[r] && oi < best_idx[r])) { best[r] = ob; best_idx[r] = oi; }
            const int64_t row = row0 + 32 * r + j;
            if (row < n && half == 0) {
                if (assign) assign[row] = good[r] ? best_idx[r] : -1;
                if (best_out) best_out[row] = bias ? best[r] : best[r] * kUnscale;
            }
        }
    }
}

template <int DP, int R>
hipError_t run(int mode, const float* x, int64_t n, int d, const uint16_t* cent_h, const uint16_t* cent_l,
               int cent_pitch, const float* bias, int L, int Lpad, int32_t* assign, float* best, float* scores,
               int64_t ld_scores, int* flag, hipStream_t st) {
    static bool attr_set = false;
    const size_t lds = CoarseCfg<DP>::lds_bytes;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_coarse<DP, R>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int64_t rows_per_wg = 4 * 32 * R;
    const int64_t blocks = (n + rows_per_wg - 1) / rows_per_wg;
    const int vec4 = (d % 4 == 0) && (reinterpret_cast<uintptr_t>(x) % 16 == 0);
    // score mode: every (row, centroid) result is independent, so when the rows alone do not fill
    // the chip the centroid stages are split over gridDim.y as well
    int ysplit = 1;
    if (mode == 1)
        while (blocks * ysplit < 512 && ysplit * 2 <= Lpad / kTN) ysplit *= 2;
    hipLaunchKernelGGL((k_coarse<DP, R>), dim3((unsigned)blocks, (unsigned)ysplit), dim3(256), lds, st, mode, x, n, d, vec4, cent_h,
                       cent_l, cent_pitch, bias, L, Lpad, assign, best, scores, ld_scores, flag);
    return hipGetLastError();
}

// Calibration of the float16 matrix pipe: nothing but v_mfma_f32_32x32x16_f16 on operands held in
// registers, four independent accumulators per wavefront, two wavefronts per SIMD.  What this
// reaches with random operand bits is the rate the contraction kernels can be compared with: the
// chip lowers its clock under the switching activity of real data, so it is below the nominal peak.
__global__ __launch_bounds__(256) void k_mfma_peak(const half8* __restrict__ src, float* __restrict__ out, int iters) {
    half8 a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = src[(threadIdx.x * 16 + i) & 4095];
        b[i] = src[(threadIdx.x * 16 + 8 + i) & 4095];
    }
    floatx16 acc[4];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[c][q] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[(i + c) & 7], b[i], acc[c], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int q = 0; q < 16; ++q) s += acc[c][q];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace

hipError_t launch_mfma_peak(const uint16_t* operands, float* out, int blocks, int iters, hipStream_t st) {
    hipLaunchKernelGGL(k_mfma_peak, dim3(blocks), dim3(256), 0, st, reinterpret_cast<const half8*>(operands), out, iters);
    return hipGetLastError();
}

int coarse_dp(int d) {
    static const int sizes[] = {32, 64, 96, 128, 160, 192, 208, 224, 256};
    for (int s : sizes)
        if (d <= s) return s;
    return -1;
}

hipError_t launch_split_rows(const float* src, int64_t count, uint16_t* hi, uint16_t* lo, hipStream_t st) {
    if (count <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_split_rows, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, src, count, hi, lo);
    return hipGetLastError();
}

hipError_t launch_coarse(int mode, const float* x, int64_t n, int d, const uint16_t* cent_h, const uint16_t* cent_l,
                         int cent_pitch, const float* bias, int L, int Lpad, int32_t* assign, float* best,
                         float* scores, int64_t ld_scores, int* flag, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    switch (coarse_dp(d)) {
#define IVFTQ_CASE(DPV, RV) \
    case DPV: return run<DPV, RV>(mode, x, n, d, cent_h, cent_l, cent_pitch, bias, L, Lpad, assign, best, scores, ld_scores, flag, st);
        IVFTQ_CASE(32, 2) IVFTQ_CASE(64, 2) IVFTQ_CASE(96, 2) IVFTQ_CASE(128, 2) IVFTQ_CASE(160, 1)
        IVFTQ_CASE(192, 1) IVFTQ_CASE(208, 1) IVFTQ_CASE(224, 1) IVFTQ_CASE(256, 1)
#undef IVFTQ_CASE
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ivftq
