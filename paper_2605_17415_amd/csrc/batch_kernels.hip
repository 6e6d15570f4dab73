// Query-batched list scan on the matrix cores (Section "Architecture", Search: the residual
// estimate gamma * <Pi q~, C[code]> for every vector of every probed list).
//
// In a large query batch each inverted list is probed by many queries (Q * nprobe / nlist of them
// on average), so the scan of one list against all of its queries is a dense contraction:
// [vectors of the list] x [d] times [d] x [queries probing the list].  The (query, probe) pairs are
// regrouped by list, and one workgroup takes one list and up to 32*NQ of its queries: the de-quantised
// codes of 32 vectors are the left MFMA operand (held in registers and reused for every query tile),
// the rotated queries are the right operand (a panel in LDS), fp32 in, fp32 accumulate, so the
// estimate keeps float32 accuracy.  In the 32x32 result a lane holds one query's scores against 16
// vectors; it adds the coarse term, scales by the stored norm and keeps only scores that reach the
// query's threshold (the k-th best score of its nearest lists, found beforehand by the exact
// streaming scan), appending them to a short per-query candidate list.
#include <hip/hip_fp16.h>

#include "kernels.h"

namespace ivftq {

typedef float floatx16 __attribute__((ext_vector_type(16)));

namespace {

// ---- regrouping (query, probe) pairs by list ---------------------------------------------------

// key[q*np + p] = list probed, or -1 for the probes the streaming scan already covered
__global__ void k_pair_keys(const int32_t* __restrict__ probe, const int32_t* __restrict__ first, int64_t nq,
                            int np, int32_t* __restrict__ key) {
    const int64_t it = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (it >= nq * np) return;
    const int64_t q = it / np;
    const int p = (int)(it % np);
    key[it] = (p >= first[q]) ? probe[it] : -1;
}

// pair_off[l] = first pair of list l (as int64, the form the ranking kernel takes);
// tile_off[l] = first workgroup tile of list l, tile_off[L] = number of tiles.  One workgroup.
__global__ __launch_bounds__(1024) void k_pair_prefix(const uint32_t* __restrict__ count, int L, int tq,
                                                      int64_t* __restrict__ pair_off,
                                                      int32_t* __restrict__ tile_off) {
    __shared__ uint32_t part_c[1024], part_t[1024];
    const int tid = threadIdx.x;
    const int per = (L + 1023) / 1024;
    uint32_t c = 0, t = 0;
    for (int e = 0; e < per; ++e) {
        const int l = tid * per + e;
        if (l < L) { c += count[l]; t += (count[l] + tq - 1) / tq; }
    }
    part_c[tid] = c;
    part_t[tid] = t;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {            // inclusive scan
        const uint32_t ac = tid >= o ? part_c[tid - o] : 0, at = tid >= o ? part_t[tid - o] : 0;
        __syncthreads();
        part_c[tid] += ac;
        part_t[tid] += at;
        __syncthreads();
    }
    uint32_t rc = part_c[tid] - c, rt = part_t[tid] - t;
    for (int e = 0; e < per; ++e) {
        const int l = tid * per + e;
        if (l < L) {
            pair_off[l] = rc;
            tile_off[l] = (int32_t)rt;
            rc += count[l];
            rt += (count[l] + tq - 1) / tq;
        }
    }
    if (tid == 1023) { pair_off[L] = part_c[1023]; tile_off[L] = (int32_t)part_t[1023]; }
}

__global__ void k_scatter_pairs(const int64_t* __restrict__ slot, int64_t n, int32_t* __restrict__ pairs) {
    const int64_t it = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (it >= n) return;
    const int64_t s = slot[it];
    if (s >= 0) pairs[s] = (int32_t)it;
}

// ---- the batched scan ----------------------------------------------------------------------------

template <int DP, int NQ>
struct BatchCfg {
    static constexpr int TQ = NQ * 32;
    static constexpr int LDP = DP + 1;
    static constexpr size_t lds_bytes = ((size_t)TQ * LDP + 3 * TQ + 256) * sizeof(float);
};

// Code of coordinate j from the packed words of one vector (coordinate j occupies bits [j*B, j*B+B)).
template <int B, int W>
__device__ __forceinline__ uint32_t code_at(const uint32_t (&w)[W], int j) {
    const int bit = j * B, wi = bit >> 5, sh = bit & 31;
    uint32_t v = w[wi] >> sh;
    if (sh + B > 32 && wi + 1 < W) v |= w[wi + 1] << (32 - sh);
    return v & ((1u << B) - 1u);
}

template <int DP, int B, int NQ>
__global__ __launch_bounds__(256, 2) void k_batch_scan(BatchScanArgs a) {
    using Cfg = BatchCfg<DP, NQ>;
    constexpr int W = (B * DP + 31) / 32;        // words that can hold DP coordinates
    extern __shared__ float lds[];
    float* zp = lds;                              // [TQ][LDP] rotated queries of this tile
    float* s_coarse = zp + Cfg::TQ * Cfg::LDP;    // [TQ] coarse term of each (query, this list)
    float* s_thr = s_coarse + Cfg::TQ;            // [TQ] threshold of each query
    int32_t* s_q = reinterpret_cast<int32_t*>(s_thr + Cfg::TQ);   // [TQ] query number
    float* s_cb = reinterpret_cast<float*>(s_q + Cfg::TQ);        // [256] codebook

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, half = lane >> 5, jl = lane & 31;

    // which (list, query tile) this workgroup owns
    const int total_tiles = a.tile_off[a.L];
    if ((int)blockIdx.x >= total_tiles) return;
    int lo = 0, hi = a.L;                         // largest l with tile_off[l] <= blockIdx.x
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (a.tile_off[mid] <= (int)blockIdx.x) lo = mid; else hi = mid;
    }
    const int l = lo;
    const int tile = blockIdx.x - a.tile_off[l];
    const int64_t pair0 = a.pair_off[l] + (int64_t)tile * Cfg::TQ;
    const int64_t pair_end = a.pair_off[l + 1];
    const int nq_tile = (int)((pair_end - pair0) < Cfg::TQ ? (pair_end - pair0) : Cfg::TQ);
    const int n_l = a.store.list_size[l];
    if (n_l == 0 || nq_tile <= 0) return;

    // stage the query panel
    for (int e = tid; e < Cfg::TQ; e += 256) {
        int32_t q = -1;
        float sc = 0.f, th = __builtin_inff();
        if (e < nq_tile) {
            const int32_t it = a.pairs[pair0 + e];
            q = it / a.np;
            sc = a.coarse[it];
            th = a.thresh[(int64_t)q * a.thresh_stride];
        }
        s_q[e] = q;
        s_coarse[e] = sc;
        s_thr[e] = th;
    }
    if (tid < (1 << B)) s_cb[tid] = a.cb[tid];
    __syncthreads();
    for (int e = tid; e < Cfg::TQ * (DP / 4); e += 256) {
        const int r = e / (DP / 4), c4 = e % (DP / 4);
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        const int32_t q = s_q[r];
        if (q >= 0) v = *reinterpret_cast<const float4*>(a.z + (int64_t)q * a.z_pitch + c4 * 4);
        float* dst = zp + r * Cfg::LDP + c4 * 4;
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    }
    __syncthreads();

    const int words = a.store.words;
    const int64_t base_slot = a.store.list_off[l];
    const int nslab = (n_l + 31) / 32;
    const int n_qt = (nq_tile + 31) / 32;
    const float* b_base = zp + jl * Cfg::LDP + half;

    for (int slab = wave; slab < nslab; slab += 4) {
        // de-quantise 32 vectors: this lane takes vector jl, coordinates of parity `half`
        const int v_mine = slab * 32 + jl;
        const int64_t slot = base_slot + (v_mine < n_l ? v_mine : n_l - 1);
        const uint32_t* wp = a.store.codes + (slot >> 6) * words * 64 + (slot & 63);
        uint32_t wv[W];
#pragma unroll
        for (int w = 0; w < W; ++w) wv[w] = (w < words) ? wp[(int64_t)w * 64] : 0u;
        float av[DP / 2];
#pragma unroll
        for (int s = 0; s < DP / 2; ++s) {
            const uint32_t c0 = code_at<B, W>(wv, 2 * s), c1 = code_at<B, W>(wv, 2 * s + 1);
            av[s] = s_cb[half ? c1 : c0];
        }
        // norms of the 16 rows this lane sees in the result
        float g[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int v = slab * 32 + 8 * (r / 4) + 4 * half + (r % 4);
            g[r] = (v < n_l) ? __half2float(__ushort_as_half(a.store.gamma[base_slot + v])) : __builtin_nanf("");
        }
        for (int qt = 0; qt < n_qt; ++qt) {
            floatx16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
            const float* bq = b_base + qt * 32 * Cfg::LDP;
#pragma unroll
            for (int s = 0; s < DP / 2; ++s)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[s], bq[2 * s], acc, 0, 0, 0);
            const int e = qt * 32 + jl;
            const float sq = s_coarse[e], th = s_thr[e];
            const int32_t q = s_q[e];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float sc = fmaf(g[r], acc[r], sq);        // NaN (row beyond the list) fails the test
                if (sc >= th && q >= 0) {
                    const int v = slab * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                    const int pos = atomicAdd(&a.cand_cnt[q], 1);
                    if (pos < a.cap) {
                        a.cand_score[(int64_t)q * a.cap + pos] = sc;
                        a.cand_slot[(int64_t)q * a.cap + pos] = base_slot + v;
                    }
                }
            }
        }
    }
}

// ---- merging the streaming top-k of the nearest lists with the batched candidates ----------------

__device__ __forceinline__ uint32_t okey(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(256) void k_merge(MergeArgs a) {
    extern __shared__ unsigned char smem[];
    const int64_t q = blockIdx.x;
    const int tid = threadIdx.x;
    const int cnt = a.cand_cnt[q];
    const bool overflow = cnt > a.cap;
    if (tid == 0) a.gate[q] = overflow ? 1 : 0;
    if (overflow) return;                        // the exact streaming pass redoes this query
    const int total = a.k + cnt;
    int size = 1;
    while (size < total) size <<= 1;
    uint32_t* s_key = reinterpret_cast<uint32_t*>(smem);
    float* s_val = reinterpret_cast<float*>(s_key + size);
    int64_t* s_lab = reinterpret_cast<int64_t*>(s_val + size);
    for (int i = tid; i < size; i += 256) {
        float v = -__builtin_inff();
        int64_t lab = INT64_MAX;
        uint32_t key = 0;
        if (i < a.k) {
            lab = a.first_ids[q * a.k + i];
            v = a.first_scores[q * a.k + i];
            if (lab >= 0) key = okey(v); else lab = INT64_MAX;
        } else if (i < total) {
            v = a.cand_score[q * a.cap + (i - a.k)];
            lab = a.ids[a.cand_slot[q * a.cap + (i - a.k)]];
            key = okey(v);
        }
        s_key[i] = key; s_val[i] = v; s_lab[i] = lab;
    }
    __syncthreads();
    for (int sz = 2; sz <= size; sz <<= 1) {
        for (int stride = sz >> 1; stride > 0; stride >>= 1) {
            for (int i = tid; i < size / 2; i += 256) {
                const int lo_i = 2 * i - (i & (stride - 1));
                const int hi_i = lo_i + stride;
                const bool up = ((lo_i & sz) == 0);
                const uint32_t k0 = s_key[lo_i], k1 = s_key[hi_i];
                const int64_t l0 = s_lab[lo_i], l1 = s_lab[hi_i];
                const bool first_before = (k0 > k1) || (k0 == k1 && l0 <= l1);
                if (first_before != up) {
                    s_key[lo_i] = k1; s_key[hi_i] = k0;
                    s_lab[lo_i] = l1; s_lab[hi_i] = l0;
                    const float t = s_val[lo_i]; s_val[lo_i] = s_val[hi_i]; s_val[hi_i] = t;
                }
            }
            __syncthreads();
        }
    }
    for (int i = tid; i < a.k; i += 256) {
        const bool real = s_key[i] != 0;
        a.out_scores[q * a.k + i] = real ? s_val[i] : -__builtin_inff();
        a.out_ids[q * a.k + i] = real ? s_lab[i] : -1;
    }
}

template <int DP, int B, int NQ>
hipError_t run_batch(const BatchScanArgs& a, int max_tiles, hipStream_t st) {
    static bool attr_set = false;
    const size_t lds = BatchCfg<DP, NQ>::lds_bytes;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_batch_scan<DP, B, NQ>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((k_batch_scan<DP, B, NQ>), dim3((unsigned)max_tiles), dim3(256), lds, st, a);
    return hipGetLastError();
}

}  // namespace

int batch_tile_queries(int d, int b) {
    const int dp = rot_dp(d);
    if (b < 2 || b > 4) return 0;
    if (dp == 64 || dp == 96 || dp == 128) return 128;
    if (dp == 224) return 64;
    return 0;
}

hipError_t launch_pair_keys(const int32_t* probe, const int32_t* first, int64_t nq, int np, int32_t* key,
                            hipStream_t st) {
    const int64_t n = nq * np;
    hipLaunchKernelGGL(k_pair_keys, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, probe, first, nq, np, key);
    return hipGetLastError();
}

hipError_t launch_pair_prefix(const uint32_t* count, int L, int tq, int64_t* pair_off, int32_t* tile_off,
                              hipStream_t st) {
    hipLaunchKernelGGL(k_pair_prefix, dim3(1), dim3(1024), 0, st, count, L, tq, pair_off, tile_off);
    return hipGetLastError();
}

hipError_t launch_scatter_pairs(const int64_t* slot, int64_t n, int32_t* pairs, hipStream_t st) {
    hipLaunchKernelGGL(k_scatter_pairs, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, slot, n, pairs);
    return hipGetLastError();
}

hipError_t launch_batch_scan(const BatchScanArgs& a, int d, int b, int max_tiles, hipStream_t st) {
    if (max_tiles <= 0) return hipSuccess;
    const int dp = rot_dp(d);
#define IVFTQ_BATCH(DPV, NQV)                                              \
    if (dp == DPV) {                                                       \
        if (b == 2) return run_batch<DPV, 2, NQV>(a, max_tiles, st);       \
        if (b == 3) return run_batch<DPV, 3, NQV>(a, max_tiles, st);       \
        if (b == 4) return run_batch<DPV, 4, NQV>(a, max_tiles, st);       \
    }
    IVFTQ_BATCH(64, 4) IVFTQ_BATCH(96, 4) IVFTQ_BATCH(128, 4) IVFTQ_BATCH(224, 2)
#undef IVFTQ_BATCH
    return hipErrorInvalidValue;
}

hipError_t launch_merge(const MergeArgs& a, int64_t nq, hipStream_t st) {
    if (nq <= 0) return hipSuccess;
    int size = 1;
    while (size < a.k + a.cap) size <<= 1;
    const size_t lds = (size_t)size * 16;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_merge),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(k_merge, dim3((unsigned)nq), dim3(256), lds, st, a);
    return hipGetLastError();
}

}  // namespace ivftq
