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

// R = 32-row tiles per wavefront.  VEC4: rows are read 16 bytes at a time (d % 4 == 0, x 16-byte aligned).
template <int DP, int R, bool VEC4>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void k_coarse(
    int mode, const float* __restrict__ x, int64_t n, int d, const uint16_t* __restrict__ cent_h,
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
        good[r] = load_rows<DP>(x, row, row < n, d, VEC4 ? 1 : 0, half, bh[r], bl[r]);
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

// Screening pass of the argmax: only the hi*hi products (one MFMA per block instead of three).  With
// unit vectors the result is off by at most (2^-10 + 2^-22) * sum|a_j b_j| <= 9.8e-4 plus float32
// summation error, so when the best screened score beats the second best by more than twice that, the
// best is the exact argmax as well.  Rows where it does not (and rows without a usable norm) are
// appended to row_list and redone by k_coarse_resolve with all three products; both write assign.
// Per score: best' = max(best, v), second' = med3(best, second, v).
constexpr float kScreenMargin = 2.2e-3f;
constexpr float kScreenNone = -3.0e38f;     // below every score, finite so that tagging its low bits keeps it a number

// 32-centroid tiles per LDS stage of the screening pass (two stages are resident)
template <int DP>
constexpr int screen_nt() { return 2; }

template <int DP>
constexpr size_t screen_lds_bytes() { return (size_t)2 * screen_nt<DP>() * 32 * CoarseCfg<DP>::LDH * sizeof(uint16_t); }

// max(a, b, c) and the middle of (a, b, c) as single instructions.  Written as instructions because the
// scores carry a tag in their low bits (below) and are never NaN, so the quieting that the compiler puts
// in front of a float maximum of an unknown bit pattern would be one wasted operation per score.
__device__ __forceinline__ float max3_raw(float a, float b, float c) {
    float o;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(o) : "v"(a), "v"(b), "v"(c));
    return o;
}

// The 16 scores of tile position t that a lane holds, four at a time.  The position (t, q) replaces
// the low 6 bits of the float32 pattern (a change below 2^-17 of the score's size), so that maxima and
// medians alone carry the index.  With b the running best and s the running second best, two new
// scores u, w give  s' = max(s, med3(b, u, w)),  b' = max(b, u, w).
#define IVFTQ_SCREEN_TAKE(MASKED)                                                                          \
    _Pragma("unroll") for (int q = 0; q < 16; q += 4) {                                                     \
        _Pragma("unroll") for (int r = 0; r < R; ++r) {                                                     \
            float v[4];                                                                                     \
            _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                 \
                v[i] = __uint_as_float((__float_as_uint(acc[r][q + i]) & ~63u) | (unsigned)(t * 16 + q + i)); \
                /* columns q..q+3 of a lane are neighbouring centroids 8*(q/4) + 4*half + i */              \
                if (MASKED) v[i] = (c0 + t * 32 + 2 * q + 4 * half + i < L) ? v[i] : kScreenNone;           \
            }                                                                                               \
            const float m0 = __builtin_amdgcn_fmed3f(best[r], v[0], v[1]);                                  \
            const float b1 = max3_raw(best[r], v[0], v[1]);                                                 \
            const float m1 = __builtin_amdgcn_fmed3f(b1, v[2], v[3]);                                       \
            best[r] = max3_raw(b1, v[2], v[3]);                                                             \
            second[r] = max3_raw(second[r], m0, m1);                                                        \
        }                                                                                                   \
    }

// VEC4: rows are read 16 bytes at a time (d % 4 == 0 and x 16-byte aligned); a template parameter so that
// each instantiation carries one loading path only (with both, the loads of the prologue spill).
template <int DP, int R, bool VEC4>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu((DP <= 128 || R == 1) ? 3 : 2))) void k_coarse_screen(
    const float* __restrict__ x, int64_t n, int d, const uint16_t* __restrict__ cent_h, int cent_pitch,
    int L, int Lpad, int32_t* __restrict__ assign, int32_t* __restrict__ row_list,
    unsigned long long* __restrict__ row_key, int* __restrict__ row_count, float* __restrict__ part) {
    using Cfg = CoarseCfg<DP>;
    constexpr int KB = Cfg::KB;
    extern __shared__ unsigned char lds_raw[];
    constexpr int NT = screen_nt<DP>(), TN = NT * 32;
    // gridDim.y > 1 (short batches): workgroup (x, y) takes the y-th share of the centroid stages and leaves
    // (best, second best, index) of every row in `part`; k_coarse_screen_join puts the shares together
    const int n_stages = Lpad / TN, per_y = (n_stages + (int)gridDim.y - 1) / (int)gridDim.y;
    const int c_lo = (int)blockIdx.y * per_y * TN < Lpad ? (int)blockIdx.y * per_y * TN : Lpad;
    const int c_hi = c_lo + per_y * TN < Lpad ? c_lo + per_y * TN : Lpad;
    uint16_t* th = reinterpret_cast<uint16_t*>(lds_raw);            // [2][TN][LDH] hi parts of the centroids
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, half = lane >> 5, j = lane & 31;
    const int64_t row0 = ((int64_t)blockIdx.x * 4 + wave) * (32 * R);

    half8 bh[R][KB];
    bool good[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int64_t row = row0 + 32 * r + j;
        half8 unused[KB];
        good[r] = load_rows<DP>(x, row, row < n, d, VEC4 ? 1 : 0, half, bh[r], unused);
        __builtin_amdgcn_sched_barrier(0);          // one tile's float32 values at a time in registers
    }
    float best[R], second[R];
    int best_c0[R];
#pragma unroll
    for (int r = 0; r < R; ++r) { best[r] = kScreenNone; second[r] = kScreenNone; best_c0[r] = 0; }
    // Stage s+1 travels global memory -> registers while stage s is multiplied, then registers -> the
    // other LDS buffer; one barrier per stage.
    constexpr int kChunks = TN * (DP / 8);                          // 16-byte pieces of one stage
    constexpr int kPer = (kChunks + 255) / 256;
    uint4 pre[kPer];
#define IVFTQ_SCREEN_FETCH(C0)                                                                     \
    _Pragma("unroll") for (int i = 0; i < kPer; ++i) {                                              \
        int e = tid + 256 * i;                                                                      \
        e = e < kChunks ? e : kChunks - 1;                                                          \
        const int r = e / (DP / 8), c8 = e % (DP / 8);                                              \
        const int c = (C0) + r < Lpad ? (C0) + r : Lpad - 1; /* a stage may reach past the padded rows */ \
        pre[i] = *reinterpret_cast<const uint4*>(cent_h + (int64_t)c * cent_pitch + c8 * 8);        \
    }
#define IVFTQ_SCREEN_STORE(BUF)                                                                    \
    _Pragma("unroll") for (int i = 0; i < kPer; ++i) {                                              \
        const int e = tid + 256 * i;                                                                \
        if (kChunks % 256 == 0 || e < kChunks)                                                      \
            *reinterpret_cast<uint4*>((BUF) + (e / (DP / 8)) * Cfg::LDH + (e % (DP / 8)) * 8) = pre[i]; \
    }
    IVFTQ_SCREEN_FETCH(c_lo)
    IVFTQ_SCREEN_STORE(th)
    __syncthreads();
    int stage = 0;
    for (int c0 = c_lo; c0 < c_hi; c0 += TN, stage ^= 1) {
        IVFTQ_SCREEN_FETCH(c0 + TN)          // unconditional (indices are clamped): after the last stage it is unused
        const uint16_t* ah_base = th + stage * (TN * Cfg::LDH) + j * Cfg::LDH + 8 * half;
        float prev[R];
#pragma unroll
        for (int r = 0; r < R; ++r) prev[r] = best[r];
        // The row operand of a tile is read from LDS a tile ahead: the reads of tile t+1 are issued
        // after the products of tile t and complete while its scores are taken.
        // (up to 128 coordinates; beyond that the registers do not reach and each block is read as it is used)
        constexpr bool kAhead = KB <= 8;
        half8 ah[kAhead ? KB : 1];
        if (kAhead) {
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) ah[kAhead ? kb : 0] = *reinterpret_cast<const half8*>(ah_base + 16 * kb);
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            floatx16 acc[R];
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[r][q] = 0.f;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                const half8 a = kAhead ? ah[kAhead ? kb : 0]
                                       : *reinterpret_cast<const half8*>(ah_base + t * 32 * Cfg::LDH + 16 * kb);
#pragma unroll
                for (int r = 0; r < R; ++r) acc[r] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, bh[r][kb], acc[r], 0, 0, 0);
            }
            if (kAhead && t + 1 < NT) {
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
                    ah[kAhead ? kb : 0] = *reinterpret_cast<const half8*>(ah_base + (t + 1) * 32 * Cfg::LDH + 16 * kb);
            }
            if (c0 + (t + 1) * 32 <= L) {
                IVFTQ_SCREEN_TAKE(false)
            } else {
                IVFTQ_SCREEN_TAKE(true)
            }
        }
        // which stage the best came from is seen from whether the stage changed it
#pragma unroll
        for (int r = 0; r < R; ++r) best_c0[r] = best[r] != prev[r] ? c0 : best_c0[r];
        IVFTQ_SCREEN_STORE(th + (stage ^ 1) * (TN * Cfg::LDH))
        __syncthreads();
    }
#undef IVFTQ_SCREEN_FETCH
#undef IVFTQ_SCREEN_STORE
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const unsigned code = __float_as_uint(best[r]) & 63u;
        int idx = best_c0[r] + (int)(code >> 4) * 32 + 8 * (int)((code & 15u) >> 2) + 4 * half + (int)(code & 3u);
        // the other half of the lane pair saw the other centroids of the same row
        const float ob = __shfl_xor(best[r], 32), os = __shfl_xor(second[r], 32);
        const int oi = __shfl_xor(idx, 32);
        const float s2 = fmaxf(fmaxf(second[r], os), fminf(best[r], ob));
        const float b2 = fmaxf(best[r], ob);
        if (ob > best[r]) idx = oi;
        const int64_t row = row0 + 32 * r + j;
        if (gridDim.y > 1) {
            if (row < n && half == 0) {
                float* pp = part + (row * (int64_t)gridDim.y + blockIdx.y) * 3;
                pp[0] = b2;
                pp[1] = s2;
                pp[2] = __int_as_float(good[r] ? idx : -1 - idx);
            }
            continue;
        }
        if (row < n && half == 0) {
            const bool sure = good[r] && (b2 - s2 > kScreenMargin * kSplitScale * kSplitScale);
            assign[row] = idx;
            if (!sure) {
                const int pos = atomicAdd(row_count, 1);
                row_list[pos] = (int32_t)row;
                row_key[pos] = 0ull;
            }
        }
    }
}
#undef IVFTQ_SCREEN_TAKE

// Shares of a row's screening pass put together: the best of the bests, and as second best the largest of
// every share's second best and of the bests that lost; then the same decision as in the kernel itself.
__global__ void k_coarse_screen_join(const float* __restrict__ part, int64_t n, int shares, int32_t* __restrict__ assign,
                                     int32_t* __restrict__ row_list, unsigned long long* __restrict__ row_key,
                                     int* __restrict__ row_count) {
    const int64_t row = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= n) return;
    float best = kScreenNone, second = kScreenNone;
    int idx = 0;
    bool good = true;
    for (int y = 0; y < shares; ++y) {
        const float* pp = part + (row * shares + y) * 3;
        const float b = pp[0], s2 = pp[1];
        int i = __float_as_int(pp[2]);
        if (i < 0) { good = false; i = -1 - i; }
        if (b > best) { second = fmaxf(second, best); best = b; idx = i; }
        else second = fmaxf(second, b);
        second = fmaxf(second, s2);
    }
    const bool sure = good && (best - second > kScreenMargin * kSplitScale * kSplitScale);
    assign[row] = idx;
    if (!sure) {
        const int pos = atomicAdd(row_count, 1);
        row_list[pos] = (int32_t)row;
        row_key[pos] = 0ull;
    }
}

// The undecided rows of the screening pass, with all three products.  Workgroup (x, y) walks the row
// blocks x, x + gridDim.x, ... of the list (128 rows each, one tile per wavefront) against the y-th share of
// the centroid stages, so that a short list still spreads over the chip; the shares of a row meet in
// row_key[position] through a 64-bit atomic maximum of (order-preserving score bits, ~index), which keeps
// the smallest index among equal scores like the single-kernel argmax does.  A row without a usable norm
// leaves its key at 0.
template <int DP, bool VEC4>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void k_coarse_resolve(
    const float* __restrict__ x, int d, const uint16_t* __restrict__ cent_h,
    const uint16_t* __restrict__ cent_l, int cent_pitch, int L, int Lpad, const int32_t* __restrict__ row_list,
    const int* __restrict__ row_count, unsigned long long* __restrict__ row_key) {
    using Cfg = CoarseCfg<DP>;
    constexpr int KB = Cfg::KB;
    extern __shared__ unsigned char lds_raw[];
    uint16_t* th = reinterpret_cast<uint16_t*>(lds_raw);            // [TN][LDH] hi parts of the centroid tile
    uint16_t* tl = th + kTN * Cfg::LDH;                               // [TN][LDH] lo parts
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, half = lane >> 5, j = lane & 31;
    const int n = *row_count;
    const int stages = Lpad / kTN, per_y = (stages + (int)gridDim.y - 1) / (int)gridDim.y;
    const int c_lo = (int)blockIdx.y * per_y * kTN;
    const int c_hi = c_lo + per_y * kTN < Lpad ? c_lo + per_y * kTN : Lpad;
    if (c_lo >= c_hi) return;
    const uint16_t* ah_base = th + j * Cfg::LDH + 8 * half;
    const uint16_t* al_base = tl + j * Cfg::LDH + 8 * half;

    for (int64_t rb = blockIdx.x; rb * 128 < n; rb += gridDim.x) {
        const int pos = (int)(rb * 128) + wave * 32 + j;
        half8 bh[KB], bl[KB];
        const bool good = load_rows<DP>(x, pos < n ? (int64_t)row_list[pos] : 0, pos < n, d, VEC4 ? 1 : 0, half, bh, bl);
        float best = -__builtin_inff();
        int best_idx = 0;
        for (int c0 = c_lo; c0 < c_hi; c0 += kTN) {
            __syncthreads();                 // the previous stage (or row block) is no longer read
            for (int e = tid; e < kTN * (DP / 8); e += 256) {
                const int r = e / (DP / 8), c8 = e % (DP / 8);
                const int64_t src = (int64_t)(c0 + r) * cent_pitch + c8 * 8;
                *reinterpret_cast<uint4*>(th + r * Cfg::LDH + c8 * 8) = *reinterpret_cast<const uint4*>(cent_h + src);
                *reinterpret_cast<uint4*>(tl + r * Cfg::LDH + c8 * 8) = *reinterpret_cast<const uint4*>(cent_l + src);
            }
            __syncthreads();
            floatx16 acc[kNT];
#pragma unroll
            for (int t = 0; t < kNT; ++t)
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[t][q] = 0.f;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int t = 0; t < kNT; ++t) {
                    const half8 ah = *reinterpret_cast<const half8*>(ah_base + t * 32 * Cfg::LDH + 16 * kb);
                    const half8 al = *reinterpret_cast<const half8*>(al_base + t * 32 * Cfg::LDH + 16 * kb);
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh[kb], acc[t], 0, 0, 0);
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bl[kb], acc[t], 0, 0, 0);
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, bh[kb], acc[t], 0, 0, 0);
                }
            // raw accumulators (the argmax does not depend on the common 2^20 scale); ascending c, first maximum wins
#pragma unroll
            for (int t = 0; t < kNT; ++t)
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int c = c0 + t * 32 + 8 * (q / 4) + 4 * half + (q % 4);
                    if (c < L && acc[t][q] > best) { best = acc[t][q]; best_idx = c; }
                }
        }
        const float ob = __shfl_xor(best, 32);
        const int oi = __shfl_xor(best_idx, 32);
        if (ob > best || (ob == best && oi < best_idx)) { best = ob; best_idx = oi; }
        if (pos < n && half == 0 && good) {
            const unsigned u = __float_as_uint(best);
            const unsigned mono = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
            atomicMax(row_key + pos, ((unsigned long long)mono << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)best_idx));
        }
    }
}

__global__ void k_coarse_resolve_write(const int32_t* __restrict__ row_list, const int* __restrict__ row_count,
                                       const unsigned long long* __restrict__ row_key, int32_t* __restrict__ assign,
                                       int* __restrict__ flag) {
    const int n = *row_count;
    for (int pos = blockIdx.x * blockDim.x + threadIdx.x; pos < n; pos += gridDim.x * blockDim.x) {
        const unsigned long long key = row_key[pos];
        assign[row_list[pos]] = key ? (int32_t)(0xFFFFFFFFu - (unsigned)(key & 0xFFFFFFFFull)) : -1;
        if (!key) atomicOr(flag, 1);
    }
}

// RS = 32-row tiles per wavefront of the screening kernel
template <int DP, int RS>
hipError_t run_screened(const float* x, int64_t n, int d, const uint16_t* cent_h, const uint16_t* cent_l, int cent_pitch,
                        int L, int Lpad, int32_t* assign, int* flag, int32_t* row_list, unsigned long long* row_key,
                        int* row_count, float* part, hipStream_t st) {
    static LdsLimit lim_screen[2], lim_resolve[2];
    const size_t lds_screen = screen_lds_bytes<DP>();
    const size_t lds = (size_t)2 * kTN * CoarseCfg<DP>::LDH * sizeof(uint16_t);
    const int vec4 = (d % 4 == 0) && (reinterpret_cast<uintptr_t>(x) % 16 == 0);
    hipError_t e = vec4 ? lim_screen[1].ensure(reinterpret_cast<const void*>(k_coarse_screen<DP, RS, true>), lds_screen)
                        : lim_screen[0].ensure(reinterpret_cast<const void*>(k_coarse_screen<DP, RS, false>), lds_screen);
    if (e == hipSuccess)
        e = vec4 ? lim_resolve[1].ensure(reinterpret_cast<const void*>(k_coarse_resolve<DP, true>), lds)
                 : lim_resolve[0].ensure(reinterpret_cast<const void*>(k_coarse_resolve<DP, false>), lds);
    if (e != hipSuccess) return e;
    const int64_t blocks_s = (n + 4 * 32 * RS - 1) / (4 * 32 * RS);
    // A short batch gives few workgroups, each walking every centroid stage on its own (90 us at 4096
    // centroids however few rows there are): with room for the partial results the stages are shared out
    // over gridDim.y until about 1024 workgroups are in the launch, at least two stages each.
    int shares = 1;
    if (part)
        while (shares < kScreenMaxShares && blocks_s * shares < 1024 && (Lpad / (screen_nt<DP>() * 32)) >= 4 * shares) shares *= 2;
    const dim3 grid_s((unsigned)blocks_s, (unsigned)shares);
    if (vec4)
        hipLaunchKernelGGL((k_coarse_screen<DP, RS, true>), grid_s, dim3(256), lds_screen, st, x, n, d,
                           cent_h, cent_pitch, L, Lpad, assign, row_list, row_key, row_count, part);
    else
        hipLaunchKernelGGL((k_coarse_screen<DP, RS, false>), grid_s, dim3(256), lds_screen, st, x, n, d,
                           cent_h, cent_pitch, L, Lpad, assign, row_list, row_key, row_count, part);
    if (shares > 1)
        hipLaunchKernelGGL(k_coarse_screen_join, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const float*)part, n, shares,
                           assign, row_list, row_key, row_count);
    // the undecided rows: about four centroid stages per workgroup, at most 512 x 16 workgroups
    const int stages = Lpad / kTN;
    const int ysplit = std::min(16, (stages + 3) / 4);
    const int64_t row_blocks = (n + 127) / 128;
    const dim3 grid_r((unsigned)std::min<int64_t>(row_blocks, 512), (unsigned)ysplit);
    if (vec4)
        hipLaunchKernelGGL((k_coarse_resolve<DP, true>), grid_r, dim3(256), lds, st, x, d, cent_h, cent_l, cent_pitch, L, Lpad,
                           (const int32_t*)row_list, (const int*)row_count, row_key);
    else
        hipLaunchKernelGGL((k_coarse_resolve<DP, false>), grid_r, dim3(256), lds, st, x, d, cent_h, cent_l, cent_pitch, L, Lpad,
                           (const int32_t*)row_list, (const int*)row_count, row_key);
    hipLaunchKernelGGL(k_coarse_resolve_write, dim3((unsigned)std::min<int64_t>((n + 255) / 256, 256)), dim3(256), 0, st,
                       (const int32_t*)row_list, (const int*)row_count, (const unsigned long long*)row_key, assign, flag);
    return hipGetLastError();
}

template <int DP, int R>
hipError_t run(int mode, const float* x, int64_t n, int d, const uint16_t* cent_h, const uint16_t* cent_l,
               int cent_pitch, const float* bias, int L, int Lpad, int32_t* assign, float* best, float* scores,
               int64_t ld_scores, int* flag, hipStream_t st) {
    static LdsLimit lim[2];
    const size_t lds = CoarseCfg<DP>::lds_bytes;
    const int64_t rows_per_wg = 4 * 32 * R;
    const int64_t blocks = (n + rows_per_wg - 1) / rows_per_wg;
    const int vec4 = (d % 4 == 0) && (reinterpret_cast<uintptr_t>(x) % 16 == 0);
    const hipError_t e = vec4 ? lim[1].ensure(reinterpret_cast<const void*>(k_coarse<DP, R, true>), lds)
                              : lim[0].ensure(reinterpret_cast<const void*>(k_coarse<DP, R, false>), lds);
    if (e != hipSuccess) return e;
    // score mode: every (row, centroid) result is independent, so when the rows alone do not fill
    // the chip the centroid stages are split over gridDim.y as well
    int ysplit = 1;
    if (mode == 1)
        while (blocks * ysplit < 512 && ysplit * 2 <= Lpad / kTN) ysplit *= 2;
    if (vec4)
        hipLaunchKernelGGL((k_coarse<DP, R, true>), dim3((unsigned)blocks, (unsigned)ysplit), dim3(256), lds, st, mode, x, n, d,
                           cent_h, cent_l, cent_pitch, bias, L, Lpad, assign, best, scores, ld_scores, flag);
    else
        hipLaunchKernelGGL((k_coarse<DP, R, false>), dim3((unsigned)blocks, (unsigned)ysplit), dim3(256), lds, st, mode, x, n, d,
                           cent_h, cent_l, cent_pitch, bias, L, Lpad, assign, best, scores, ld_scores, flag);
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

hipError_t launch_coarse_screened(const float* x, int64_t n, int d, const uint16_t* cent_h, const uint16_t* cent_l,
                                  int cent_pitch, int L, int Lpad, int32_t* assign, int* flag, int32_t* row_list,
                                  unsigned long long* row_key, int* row_count, float* part, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    switch (coarse_dp(d)) {
#define IVFTQ_CASE(DPV, RS) \
    case DPV: return run_screened<DPV, RS>(x, n, d, cent_h, cent_l, cent_pitch, L, Lpad, assign, flag, row_list, row_key, row_count, part, st);
        IVFTQ_CASE(32, 2) IVFTQ_CASE(64, 2) IVFTQ_CASE(96, 2) IVFTQ_CASE(128, 2) IVFTQ_CASE(160, 2)
        IVFTQ_CASE(192, 2) IVFTQ_CASE(208, 2) IVFTQ_CASE(224, 2) IVFTQ_CASE(256, 2)
#undef IVFTQ_CASE
        default: return hipErrorInvalidValue;
    }
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
