// Coarse scoring on the matrix cores: <x~_i, c~_l> for every data row i and every cell l, with
// either a running argmax (encode step "assign to the nearest centroid by maximum inner product",
// Section "Architecture", Indexing) or the full score matrix (search step "coarse term computed
// exactly", Section "Architecture", Search).
//
// Shape of the work: n x d times d x L with small d (96..200) and a result that is never kept
// (argmax) or kept once (scores).  One wavefront owns 32 data rows for the whole kernel and holds
// them in registers as the right-hand MFMA operand; centroid tiles stream through LDS and are the
// left-hand operand, so that in the 32x32 result each lane holds one data row's scores against 16
// centroids and the argmax over centroids never crosses lanes until the very end.
//
// v_mfma_f32_32x32x2_f32: A is 32x2 (lane = i + 32k), B is 2x32 (lane = j + 32k), D is 32x32 with
// D[i][j] in lane j + 32*((i/4)%2), register (i%4) + 4*(i/8).  The two k-slots of step s are
// mapped to coordinates s and DP/2 + s, so each lane reads one contiguous half of its row.
#include "kernels.h"

namespace ivftq {

typedef float floatx16 __attribute__((ext_vector_type(16)));

namespace {

template <int DP>
struct CoarseCfg {
    static constexpr int NT = 2;                 // 32-centroid tiles per LDS stage
    static constexpr int TN = NT * 32;
    static constexpr int LDP = DP + 1;           // odd pitch: conflict-free column reads
    static constexpr size_t lds_bytes = (size_t)TN * LDP * sizeof(float) + TN * sizeof(float);
};

// Coordinates half*DP/2 + [0, DP/2) of `row` into v, zero beyond d.  Loads are unconditional on
// clamped indices (straight-line code); an invalid row reads row 0 and is zeroed.
template <int DP>
__device__ __forceinline__ void load_half_row(const float* __restrict__ x, int64_t row, bool valid,
                                              int d, int vec4, int half, float (&v)[DP / 2]) {
    const int k0 = half * (DP / 2);
    const float* p = x + (valid ? row : 0) * (int64_t)d;
    if (vec4) {   // d % 4 == 0 and x 16-byte aligned: whole float4s are in or out of range
        const float4* q = reinterpret_cast<const float4*>(p);
        const int last4 = d / 4 - 1;
#pragma unroll
        for (int s = 0; s < DP / 2; s += 4) {
            const int i4 = (k0 + s) / 4;
            const float4 t = q[i4 < last4 ? i4 : last4];
            const bool in = valid && (k0 + s < d);
            v[s] = in ? t.x : 0.f; v[s + 1] = in ? t.y : 0.f; v[s + 2] = in ? t.z : 0.f; v[s + 3] = in ? t.w : 0.f;
        }
    } else {
#pragma unroll
        for (int s = 0; s < DP / 2; ++s) {
            const int i = k0 + s;
            const float t = p[i < d ? i : d - 1];
            v[s] = (valid && i < d) ? t : 0.f;
        }
    }
}

template <int DP>
__global__ __launch_bounds__(256, 2) void k_coarse(
    int mode, const float* __restrict__ x, int64_t n, int d, int vec4, const float* __restrict__ cent,
    int cent_pitch, const float* __restrict__ bias, int L, int Lpad, int32_t* __restrict__ assign,
    float* __restrict__ best_out, float* __restrict__ scores, int64_t ld_scores, int* __restrict__ flag) {
    using Cfg = CoarseCfg<DP>;
    extern __shared__ float lds[];
    float* tile = lds;
    float* tile_bias = lds + Cfg::TN * Cfg::LDP;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, half = lane >> 5, j = lane & 31;
    const int64_t row = (int64_t)blockIdx.x * kRowsPerWG + wave * 32 + j;
    const bool valid = row < n;

    float bx[DP / 2];
    load_half_row<DP>(x, row, valid, d, vec4, half, bx);
    float n2 = 0.f;
#pragma unroll
    for (int s = 0; s < DP / 2; ++s) n2 += bx[s] * bx[s];
    n2 += __shfl_xor(n2, 32);
    const bool good = (n2 > 0.f) && (n2 < __builtin_inff());
    if (valid && !good && half == 0) atomicOr(flag, 1);
    const float nrm = sqrtf(n2);
#pragma unroll
    for (int s = 0; s < DP / 2; ++s) bx[s] = good ? bx[s] / nrm : 0.f;

    float best = -__builtin_inff();
    int best_idx = 0;
    const float* a_base = tile + j * Cfg::LDP + half * (DP / 2);

    for (int c0 = 0; c0 < Lpad; c0 += Cfg::TN) {
        __syncthreads();
        // stage TN centroid rows (DP columns of the padded table) into LDS
        for (int e = tid; e < Cfg::TN * (DP / 4); e += 256) {
            const int r = e / (DP / 4), q4 = e % (DP / 4);
            const float4 t = *reinterpret_cast<const float4*>(cent + (int64_t)(c0 + r) * cent_pitch + q4 * 4);
            float* dst = tile + r * Cfg::LDP + q4 * 4;
            dst[0] = t.x; dst[1] = t.y; dst[2] = t.z; dst[3] = t.w;
        }
        if (tid < Cfg::TN) tile_bias[tid] = bias ? bias[c0 + tid] : 0.f;
        __syncthreads();

        floatx16 acc[Cfg::NT];
#pragma unroll
        for (int t = 0; t < Cfg::NT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
#pragma unroll
        for (int s = 0; s < DP / 2; ++s) {
#pragma unroll
            for (int t = 0; t < Cfg::NT; ++t) {
                const float a = a_base[t * 32 * Cfg::LDP + s];
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bx[s], acc[t], 0, 0, 0);
            }
        }

        if (mode == 0) {
#pragma unroll
            for (int t = 0; t < Cfg::NT; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int i = 8 * (r / 4) + 4 * half + (r % 4);
                    const int c = c0 + t * 32 + i;
                    const float v = acc[t][r] + tile_bias[t * 32 + i];
                    if (c < L && v > best) { best = v; best_idx = c; }   // ascending c: first maximum wins
                }
        } else if (valid) {
#pragma unroll
            for (int t = 0; t < Cfg::NT; ++t)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int c = c0 + t * 32 + 8 * g + 4 * half;
                    if (c < ld_scores) {
                        float4 o = make_float4(acc[t][4 * g], acc[t][4 * g + 1], acc[t][4 * g + 2], acc[t][4 * g + 3]);
                        *reinterpret_cast<float4*>(scores + row * ld_scores + c) = o;
                    }
                }
        }
    }

    if (mode == 0) {
        const float ob = __shfl_xor(best, 32);
        const int oi = __shfl_xor(best_idx, 32);
        if (ob > best || (ob == best && oi < best_idx)) { best = ob; best_idx = oi; }
        if (valid && half == 0) {
            if (assign) assign[row] = good ? best_idx : -1;
            if (best_out) best_out[row] = best;
        }
    }
}

template <int DP>
hipError_t run(int mode, const float* x, int64_t n, int d, const float* cent, int cent_pitch,
               const float* bias, int L, int Lpad, int32_t* assign, float* best, float* scores,
               int64_t ld_scores, int* flag, hipStream_t st) {
    static bool attr_set = false;
    const size_t lds = CoarseCfg<DP>::lds_bytes;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_coarse<DP>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int64_t blocks = (n + kRowsPerWG - 1) / kRowsPerWG;
    const int vec4 = (d % 4 == 0) && (reinterpret_cast<uintptr_t>(x) % 16 == 0);
    hipLaunchKernelGGL(k_coarse<DP>, dim3((unsigned)blocks), dim3(256), lds, st, mode, x, n, d, vec4, cent,
                       cent_pitch, bias, L, Lpad, assign, best, scores, ld_scores, flag);
    return hipGetLastError();
}

}  // namespace

int coarse_dp(int d) {
    static const int sizes[] = {32, 64, 96, 128, 160, 192, 200, 224, 256};
    for (int s : sizes)
        if (d <= s) return s;
    return -1;
}

hipError_t launch_coarse(int mode, const float* x, int64_t n, int d, const float* cent, int cent_pitch,
                         const float* bias, int L, int Lpad, int32_t* assign, float* best,
                         float* scores, int64_t ld_scores, int* flag, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    switch (coarse_dp(d)) {
#define IVFTQ_CASE(DPV) \
    case DPV: return run<DPV>(mode, x, n, d, cent, cent_pitch, bias, L, Lpad, assign, best, scores, ld_scores, flag, st);
        IVFTQ_CASE(32) IVFTQ_CASE(64) IVFTQ_CASE(96) IVFTQ_CASE(128) IVFTQ_CASE(160)
        IVFTQ_CASE(192) IVFTQ_CASE(200) IVFTQ_CASE(224) IVFTQ_CASE(256)
#undef IVFTQ_CASE
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ivftq
