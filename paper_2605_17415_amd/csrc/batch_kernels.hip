// Query-batched list scan on the matrix cores (Section "Architecture", Search: the residual
// estimate gamma * <Pi q~, C[code]> for every vector of every probed list).
//
// In a large query batch each inverted list is probed by many queries (Q * nprobe / nlist of them
// on average), so the scan of one list against all of its queries is a dense contraction:
// [vectors of the list] x [d] times [d] x [queries probing the list].  The (query, probe) pairs are
// regrouped by list, and one workgroup takes one list and up to 32*NQ of its queries: the de-quantised
// codes of 32 vectors are the left MFMA operand (held in registers and reused for every query tile),
// the rotated queries are the right operand (a panel in LDS); operands are split float16 pairs and
// accumulation is float32, so the estimate keeps float32 accuracy (see below).  In the 32x32 result a lane holds one query's scores against 16
// vectors; it adds the coarse term, scales by the stored norm and keeps only scores that reach the
// query's threshold (the k-th best score of its nearest lists, found beforehand by the exact
// streaming scan), appending them to a short per-query candidate list.
#include <hip/hip_fp16.h>

#include <type_traits>

#include "kernels.h"

namespace ivftq {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));

namespace {

// ---- regrouping (query, probe) pairs by list ---------------------------------------------------
//
// Pairs are bucketed with atomic counters: bucket l holds the pairs (q, p < first[q]) of list l
// (each query's nearest lists, scanned first to find its threshold), bucket L + l the others.  The order of the pairs inside a bucket (and so
// which tile a query lands in) may change from run to run; results do not, because a score depends
// only on its own (query, vector) pair and the final merge orders candidates by (score, label).

__global__ void k_pair_count(const int32_t* __restrict__ probe, const int32_t* __restrict__ first, int64_t nq,
                             int np, int L, uint32_t* __restrict__ count) {
    const int64_t it = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (it >= nq * np) return;
    const int late = (int)(it % np) >= first[it / np];
    atomicAdd(&count[probe[it] + (late ? L : 0)], 1u);
}

// Over the 2L buckets: pair_off[b] = first pair of bucket b; tile_off[b] = first workgroup tile of
// bucket b (entry 2L = totals); cursor[b] = 0.  One workgroup; L here is the number of buckets.
__global__ __launch_bounds__(1024) void k_pair_prefix(const uint32_t* __restrict__ count, int L, int tq,
                                                      int64_t* __restrict__ pair_off,
                                                      int32_t* __restrict__ tile_off,
                                                      uint32_t* __restrict__ cursor) {
    __shared__ uint32_t part_c[1024], part_t[1024];
    const int tid = threadIdx.x;
    const int per = (L + 1023) / 1024;
    uint32_t c = 0, t = 0;
    for (int e = 0; e < per; ++e) {
        const int l = tid * per + e;
        if (l < L) { c += count[l]; t += (count[l] + tq - 1) / tq; cursor[l] = 0; }
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

__global__ void k_pair_scatter(const int32_t* __restrict__ probe, const int32_t* __restrict__ first, int64_t nq,
                               int np, int L, const int64_t* __restrict__ pair_off,
                               uint32_t* __restrict__ cursor, int32_t* __restrict__ pairs) {
    const int64_t it = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (it >= nq * np) return;
    const int late = (int)(it % np) >= first[it / np];
    const int bkt = probe[it] + (late ? L : 0);
    pairs[pair_off[bkt] + atomicAdd(&cursor[bkt], 1u)] = (int32_t)it;
}

// The same two steps with the counters privatised in LDS: a workgroup takes kPairChunk consecutive
// pairs, counts them per bucket in LDS, and touches each global counter once per bucket it met
// (thousands of pairs hit the same few thousand counters, so per-pair global atomics serialise).
// In the scatter step that one global atomic reserves the workgroup's range inside the bucket.
constexpr int kPairChunk = 4096;
constexpr int kPairLdsBuckets = 16384;      // 2L must not exceed this (64 KB of LDS)

__global__ __launch_bounds__(1024) void k_pair_count_lds(const int32_t* __restrict__ probe,
                                                         const int32_t* __restrict__ first, int64_t nq, int np,
                                                         int L, uint32_t* __restrict__ count) {
    extern __shared__ uint32_t bins[];                   // [2L]
    for (int i = threadIdx.x; i < 2 * L; i += 1024) bins[i] = 0u;
    __syncthreads();
    const int64_t begin = (int64_t)blockIdx.x * kPairChunk, total = nq * np;
    const int64_t end = begin + kPairChunk < total ? begin + kPairChunk : total;
    for (int64_t it = begin + threadIdx.x; it < end; it += 1024) {
        const int late = (int)(it % np) >= first[it / np];
        atomicAdd(&bins[probe[it] + (late ? L : 0)], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 2 * L; i += 1024)
        if (bins[i]) atomicAdd(&count[i], bins[i]);
}

__global__ __launch_bounds__(1024) void k_pair_scatter_lds(const int32_t* __restrict__ probe,
                                                           const int32_t* __restrict__ first, int64_t nq, int np,
                                                           int L, const int64_t* __restrict__ pair_off,
                                                           uint32_t* __restrict__ cursor, int32_t* __restrict__ pairs) {
    extern __shared__ uint32_t bins[];                   // [2L] count, then first position of this workgroup's range
    for (int i = threadIdx.x; i < 2 * L; i += 1024) bins[i] = 0u;
    __syncthreads();
    const int64_t begin = (int64_t)blockIdx.x * kPairChunk, total = nq * np;
    const int64_t end = begin + kPairChunk < total ? begin + kPairChunk : total;
    for (int64_t it = begin + threadIdx.x; it < end; it += 1024) {
        const int late = (int)(it % np) >= first[it / np];
        atomicAdd(&bins[probe[it] + (late ? L : 0)], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 2 * L; i += 1024) {
        const uint32_t c = bins[i];
        bins[i] = c ? atomicAdd(&cursor[i], c) : 0u;      // this workgroup's pairs of bucket i start here
    }
    __syncthreads();
    for (int64_t it = begin + threadIdx.x; it < end; it += 1024) {
        const int late = (int)(it % np) >= first[it / np];
        const int bkt = probe[it] + (late ? L : 0);
        pairs[pair_off[bkt] + atomicAdd(&bins[bkt], 1u)] = (int32_t)it;
    }
}

// ---- the batched scan ----------------------------------------------------------------------------
//
// Arithmetic: both operands are used in split float16 form, 1024*v = hi + lo with hi = fp16(1024 v)
// and lo = fp16(1024 v - hi), and the product is accumulated as hi*hi + hi*lo + lo*hi on
// v_mfma_f32_32x32x16_f16 with float32 accumulation (the lo*lo term, below 2^-24 relative, is
// dropped).  Each part carries 11 significant bits, so the result matches a float32 contraction to
// about 2e-7 relative while running on the float16 matrix pipe; the 2^-20 of the two scale factors
// is folded into the stored norm.
//
// v_mfma_f32_32x32x16_f16: A is 32x16 (lane = i + 32*(k/8), element k%8), B is 16x32 likewise,
// D as for the 32x32 float32 form: D[i][j] in lane j + 32*((i/4)%2), register (i%4) + 4*(i/8).

template <int DP, int B, int NQ>
struct BatchCfg {
    static constexpr int TQ = NQ * 32;
    static constexpr int LDH = DP + 8;            // halves per panel row: 16-byte pad keeps b128 reads conflict free
    static constexpr int PT = 1 << (2 * B);       // entries of the code-pair tables
    static constexpr size_t lds_bytes = (size_t)TQ * LDH * 2 * sizeof(uint16_t) + 4 * TQ * sizeof(float) + 2 * PT * 4;   // panels + per-query words + pair tables
    static constexpr size_t lds_bytes_threshold = lds_bytes - (size_t)TQ * LDH * sizeof(uint16_t);                      // without the lo panel
};

// WAVES = wavefronts per workgroup, OCC = wavefronts per SIMD the register budget is set for.
// DENSE (the nearest lists, every score stored): the queries are the row operand and the vectors the
// column operand, so a lane holds one vector's scores against 16 queries and the stores of a
// query's scores coalesce.  Otherwise (threshold pass) the roles are swapped: a lane holds one
// query's scores against 16 vectors and needs that query's coarse term and threshold only once.
// The threshold pass multiplies the leading float16 parts only (one product instead of three): the
// accumulator starts at acc0 = 2^20 * kappa, kappa bounding the error of such a sum for a unit query, so
// what is compared with the threshold and appended is an upper bound of the true score (true score in
// [u - 2*kappa*gamma, u]); k_merge re-scores from the packed codes the few that can still matter.
template <int DP, int B, int NQ, int WAVES, int OCC, bool DENSE>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(OCC)))
void k_batch_scan(BatchScanArgs a) {
    using Cfg = BatchCfg<DP, B, NQ>;
    constexpr int KB = DP / 16;                   // 16-coordinate blocks
    constexpr int NT = WAVES * 64;
    extern __shared__ unsigned char lds_raw[];
    uint16_t* zh = reinterpret_cast<uint16_t*>(lds_raw);          // [TQ][LDH] hi parts of the rotated queries
    uint16_t* zl = zh + Cfg::TQ * Cfg::LDH;                         // [TQ][LDH] lo parts
    float* s_coarse = reinterpret_cast<float*>(DENSE ? zl + Cfg::TQ * Cfg::LDH : zl);   // [TQ] (the threshold pass keeps no lo panel)
    float* s_thr = s_coarse + Cfg::TQ;                              // [TQ] threshold, or (dense) offset of the pair's scores
    int32_t* s_q = reinterpret_cast<int32_t*>(s_thr + Cfg::TQ);     // [TQ]
    int32_t* s_p = s_q + Cfg::TQ;                                   // [TQ] probe rank of the pair
    uint32_t* tab_h = reinterpret_cast<uint32_t*>(s_p + Cfg::TQ);   // [PT] hi parts of a code pair, packed
    uint32_t* tab_l = tab_h + Cfg::PT;                              // [PT] lo parts

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, half = lane >> 5, jl = lane & 31;

    // which (bucket, query tile) this workgroup owns, among the buckets [bucket_lo, bucket_hi)
    const int my_tile = (int)blockIdx.x + a.tile_off[a.bucket_lo];
    if (my_tile >= a.tile_off[a.bucket_hi]) return;
    int lo_l = a.bucket_lo, hi_l = a.bucket_hi;   // largest bucket with tile_off[bucket] <= my_tile
    while (hi_l - lo_l > 1) {
        const int mid = (lo_l + hi_l) >> 1;
        if (a.tile_off[mid] <= my_tile) lo_l = mid; else hi_l = mid;
    }
    const int bkt = lo_l;
    const int l = bkt >= a.L ? bkt - a.L : bkt;
    const int tile = my_tile - a.tile_off[bkt];
    const int64_t pair0 = a.pair_off[bkt] + (int64_t)tile * Cfg::TQ;
    const int64_t pair_end = a.pair_off[bkt + 1];
    const int nq_tile = (int)((pair_end - pair0) < Cfg::TQ ? (pair_end - pair0) : Cfg::TQ);
    const int n_l = a.store.list_size[l];
    if (n_l == 0 || nq_tile <= 0) return;

    const int words = a.store.words;
    const int64_t base_slot = a.store.list_off[l];
    const int nslab = (n_l + 31) / 32;
    const int n_qt = (nq_tile + 31) / 32;
    const uint16_t* bh_base = zh + jl * Cfg::LDH + 8 * half;
    const uint16_t* bl_base = zl + jl * Cfg::LDH + 8 * half;
    constexpr float kUnscale = 1.f / (kSplitScale * kSplitScale);

    // Raw words and norms of a slab are fetched one slab ahead so that their latency hides behind
    // the matrix work of the current slab; the first slab's behind the staging below.
    constexpr int NW = (B == 3 || B == 5) ? 2 : 1; // 24- and 40-bit chunks straddle two words
    auto fetch = [&](int slab, uint32_t (&w)[KB][NW], uint32_t (&gp)[8]) {
        const int v_mine = slab * 32 + jl;         // this lane de-quantises vector jl of the slab
        const int64_t slot = base_slot + (v_mine < n_l ? v_mine : n_l - 1);
        const uint32_t* wp = a.store.codes + (slot >> 6) * words * 64 + (slot & 63);
        // Blocks whose words exist for both halves of the wavefront (the same for every lane) are loaded at constant
        // offsets with no tests in between: all of them when the rows are as long as the panel, all but the last
        // for a row that ends inside the last block (d = 200 in a 208-wide panel); else block by block.
        const int last_whole = ((16 * (KB - 1) + 8) * B) >> 5;      // first word of the last block's upper half
        if (NW == 1 && last_whole < words) {
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) w[kb][0] = wp[(int64_t)(((16 * kb + 8 * half) * B) >> 5) * 64];
        } else if (NW == 1 && KB > 1 && (((16 * (KB - 2) + 8) * B) >> 5) < words) {
#pragma unroll
            for (int kb = 0; kb < KB - 1; ++kb) w[kb][0] = wp[(int64_t)(((16 * kb + 8 * half) * B) >> 5) * 64];
            const int wi = ((16 * (KB - 1) + 8 * half) * B) >> 5;
            w[KB - 1][0] = wi < words ? wp[(int64_t)wi * 64] : 0u;
        } else {
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                const int wi = ((16 * kb + 8 * half) * B) >> 5;
                // the words of both halves of the wavefront exist (again the same for every lane): plain loads;
                // else (the padding beyond a row shorter than the panel) lane by lane
                if ((((16 * kb + 8) * B) >> 5) + NW - 1 < words) {
#pragma unroll
                    for (int e = 0; e < NW; ++e) w[kb][e] = wp[(int64_t)(wi + e) * 64];
                } else {
#pragma unroll
                    for (int e = 0; e < NW; ++e) w[kb][e] = (wi + e < words) ? wp[(int64_t)(wi + e) * 64] : 0u;
                }
            }
        }
        if (DENSE) {                               // float16 norm of the lane's own vector (NaN beyond the list)
            gp[0] = v_mine < n_l ? (uint32_t)a.store.gamma[slot] : 0x7E00u;
        } else {
            // float16 norms of the lane's 16 result rows: four runs of four consecutive vectors, 8 bytes each
            // (8-byte aligned: lists start at multiples of 64 slots).  A list's slots reach to a multiple of 64,
            // so the reads stay inside the array also in the last slab, whose rows beyond the list are then
            // replaced by NaN.
            const uint16_t* gb = a.store.gamma + base_slot + slab * 32 + 4 * half;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const uint2 pr2 = *reinterpret_cast<const uint2*>(gb + 8 * g);
                gp[2 * g] = pr2.x;
                gp[2 * g + 1] = pr2.y;
            }
            if (slab * 32 + 32 > n_l) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int v = slab * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                    if (v >= n_l) gp[r / 2] = (r & 1) ? ((gp[r / 2] & 0xFFFFu) | 0x7E000000u) : ((gp[r / 2] & 0xFFFF0000u) | 0x7E00u);
                }
            }
        }
    };

    uint32_t cw[KB][NW], cg[8], nw[KB][NW], ng[8];
    int slab = wave;
    if (slab < nslab) fetch(slab, cw, cg);

    // stage the query panel and the code-pair tables
    for (int e = tid; e < Cfg::TQ; e += NT) {
        int32_t q = -1, pr = 0;
        float sc = 0.f, th = __builtin_inff();
        if (e < nq_tile) {
            const int32_t it = a.pairs[pair0 + e];
            q = it / a.np;
            pr = it - q * a.np;
            sc = a.coarse[it];
            if (DENSE) th = __int_as_float(a.cand_off[(int64_t)q * (a.np + 1) + (it - q * a.np)]);
            else th = a.thresh[(int64_t)q * a.thresh_stride];
        }
        s_q[e] = q;
        s_p[e] = pr;
        s_coarse[e] = sc;
        s_thr[e] = th;
    }
    for (int e = tid; e < Cfg::PT; e += NT) {
        uint32_t hp = 0, lp = 0;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const float V = a.cb[(e >> (t * B)) & ((1 << B) - 1)] * kSplitScale;
            const _Float16 hi = (_Float16)V;
            const _Float16 lo = (_Float16)(V - (float)hi);
            hp |= (uint32_t)__builtin_bit_cast(uint16_t, hi) << (16 * t);
            lp |= (uint32_t)__builtin_bit_cast(uint16_t, lo) << (16 * t);
        }
        tab_h[e] = hp;
        if (DENSE) tab_l[e] = lp;
    }
    __syncthreads();
    for (int e = tid; e < Cfg::TQ * (DP / 8); e += NT) {           // 16-byte pieces
        const int r = e / (DP / 8), c8 = e % (DP / 8);
        uint4 vh = make_uint4(0, 0, 0, 0), vl = make_uint4(0, 0, 0, 0);
        const int32_t q = s_q[r];
        if (q >= 0) {
            vh = *reinterpret_cast<const uint4*>(a.zh + (int64_t)q * a.z_pitch + c8 * 8);
            if (DENSE) vl = *reinterpret_cast<const uint4*>(a.zl + (int64_t)q * a.z_pitch + c8 * 8);
        }
        *reinterpret_cast<uint4*>(zh + r * Cfg::LDH + c8 * 8) = vh;
        if (DENSE) *reinterpret_cast<uint4*>(zl + r * Cfg::LDH + c8 * 8) = vl;
    }
    __syncthreads();

    // acc0 in every element, kept in registers for the whole kernel (hidden from the compiler, which would
    // otherwise write the 16 registers anew from scalars for every tile)
    // (not for 3 and 5 stored bits, whose chunks straddle words and take the registers this would need)
    floatx16 acc_init;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_init[r] = DENSE ? 0.f : a.acc0;
    if (!DENSE && NW == 1) asm volatile("" : "+v"(acc_init));

    while (slab < nslab) {
        const int next = slab + WAVES;
        if (next < nslab) fetch(next, nw, ng);

        // de-quantise: coordinates 16*kb + 8*half + [0, 8) of vector jl, two codes per table look-up
        half8 ah[KB], al[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const int sh = ((16 * kb + 8 * half) * B) & 31;
            // the 8 codes of this lane's block: 8*B bits starting at bit sh of the first word
            typename std::conditional<(8 * B > 32), uint64_t, uint32_t>::type chunk = cw[kb][0] >> sh;
            if (NW == 2) chunk = (decltype(chunk))((((uint64_t)cw[kb][NW - 1] << 32) | cw[kb][0]) >> sh);
            uint32_t hv[4], lv[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const uint32_t idx = (uint32_t)(chunk >> (2 * B * t)) & (uint32_t)(Cfg::PT - 1);
                hv[t] = tab_h[idx];
                lv[t] = DENSE ? tab_l[idx] : 0u;
            }
            ah[kb] = __builtin_bit_cast(half8, make_uint4(hv[0], hv[1], hv[2], hv[3]));
            al[kb] = __builtin_bit_cast(half8, make_uint4(lv[0], lv[1], lv[2], lv[3]));
        }
        if constexpr (!DENSE) {
            // ---- threshold pass.  A lane holds one query's 16 accumulators per tile; row r is the vector
            // 8*(r/4) + 4*half + r%4 of the slab, its norm the half r%2 of cg[r/2] (NaN beyond the list).
            // (the register is hidden from the compiler at the point of use: it would otherwise convert all 16
            // norms once per slab, ahead of the tiles, although only the rare tile with a candidate reads them)
            auto norm_of = [&](int r) -> float {
                uint32_t pr = cg[r / 2];
                if constexpr (DP <= 128) asm volatile("" : "+v"(pr));     // (beyond: measured slower, it spills)
                return kUnscale * __half2float(__ushort_as_half((uint16_t)((r & 1) ? (pr >> 16) : (pr & 0xFFFFu))));
            };
            // the largest norm among this lane's rows (packed float16 maxima, which skip the NaNs)
            typedef _Float16 half2v __attribute__((ext_vector_type(2)));
            half2v gm = __builtin_bit_cast(half2v, cg[0]);
#pragma unroll
            for (int r = 1; r < 8; ++r) gm = __builtin_elementwise_max(gm, __builtin_bit_cast(half2v, cg[r]));
            const float g_max = kUnscale * fmaxf((float)gm[0], (float)gm[1]);
            // No row of a tile can reach the threshold unless the largest accumulator times the largest norm
            // does: g_max >= g_r >= 0 and a_max >= max(acc_r, 0), and a correctly rounded fused multiply-add
            // never decreases when its exact value grows, so fmaf(g_max, a_max, sq) >= fmaf(g_r, acc_r, sq).
            auto take = [&](const floatx16& acc, int qt) {
                const int e = qt * 32 + jl;
                const float sq = s_coarse[e], th = s_thr[e];
                const int32_t q = s_q[e];
                float a_max = 0.f;
#pragma unroll
                for (int r = 0; r < 16; r += 2) a_max = fmaxf(fmaxf(a_max, acc[r]), acc[r + 1]);
                if (fmaf(g_max, a_max, sq) >= th && q >= 0) {        // rare: some row of this lane may reach the threshold
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float sc_r = fmaf(norm_of(r), acc[r], sq);   // upper bound of the score; NaN never passes
                        if (sc_r >= th) {
                            const int v = slab * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                            const int pos = atomicAdd(&a.cand_cnt[q], 1);
                            if (pos < a.cap) {
                                a.cand_score[(int64_t)q * a.cap + pos] = sc_r;
                                a.cand_slot[(int64_t)q * a.cap + pos] = (base_slot + v) | ((int64_t)s_p[e] << kCandProbeShift);
                            }
                        }
                    }
                }
            };
            // two query tiles at a time: their products are independent, so one tile's matrix instructions
            // and LDS reads fill the waits of the other's; the first product of a tile starts from the block
            // that holds the error bound in every element
            // (only where the register budget of the launch shape has room for a second accumulator block:
            // at three wavefronts per SIMD it spilled and the pass took half as long again)
            constexpr bool kPairs = OCC <= 2 && NW == 1;
            int qt = 0;
            for (; kPairs && qt + 1 < n_qt; qt += 2) {
                const uint16_t* b0 = bh_base + qt * 32 * Cfg::LDH;
                const uint16_t* b1 = b0 + 32 * Cfg::LDH;
                floatx16 acc0, acc1;
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) {
                    const half8 h0 = *reinterpret_cast<const half8*>(b0 + 16 * kb);
                    const half8 h1 = *reinterpret_cast<const half8*>(b1 + 16 * kb);
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[kb], h0, kb ? acc0 : acc_init, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[kb], h1, kb ? acc1 : acc_init, 0, 0, 0);
                }
                take(acc0, qt);
                take(acc1, qt + 1);
            }
            for (; qt < n_qt; ++qt) {
                const uint16_t* b0 = bh_base + qt * 32 * Cfg::LDH;
                floatx16 acc0;
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) {
                    const half8 h0 = *reinterpret_cast<const half8*>(b0 + 16 * kb);
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[kb], h0, kb ? acc0 : acc_init, 0, 0, 0);
                }
                take(acc0, qt);
            }
        } else {
        float g[16];                               // 2^-20 * norm of this lane's vector (NaN beyond the list)
#pragma unroll
        for (int r = 0; r < 16; ++r) g[r] = kUnscale * __half2float(__ushort_as_half((uint16_t)(cg[0] & 0xFFFFu)));
        for (int qt = 0; qt < n_qt; ++qt) {
            floatx16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
            const uint16_t* bhq = bh_base + qt * 32 * Cfg::LDH;
            const uint16_t* blq = bl_base + qt * 32 * Cfg::LDH;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                const half8 bh = *reinterpret_cast<const half8*>(bhq + 16 * kb);
                const half8 bl = *reinterpret_cast<const half8*>(blq + 16 * kb);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(bh, ah[kb], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(bl, ah[kb], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(bh, al[kb], acc, 0, 0, 0);
            }
            // result row r of this lane: query 8*(r/4) + 4*half + r%4 of the tile, vector jl of the slab
            const int v = slab * 32 + jl;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                // rows 4g .. 4g+3 belong to the queries 8g .. 8g+7 of this tile: a sparse tile (a list that
                // is among the nearest of few queries) skips the groups it has no query for
                if (qt * 32 + 8 * (r / 4) >= nq_tile) break;
                const int e = qt * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                const int32_t q = s_q[e];
                if (q >= 0 && v < n_l)
                    a.scores[(int64_t)q * a.m_stride + __float_as_int(s_thr[e]) + v] = fmaf(g[r], acc[r], s_coarse[e]);
            }
        }
        }
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int e = 0; e < NW; ++e) cw[kb][e] = nw[kb][e];
#pragma unroll
        for (int r = 0; r < 8; ++r) cg[r] = ng[r];
        slab = next;
    }
}

// ---- merging the streaming top-k of the nearest lists with the batched candidates ----------------

__device__ __forceinline__ uint32_t okey(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// ---- merge: first-pass top-k and threshold-pass candidates -> the k best --------------------------
//
// One workgroup per query.  First-pass entries carry exact scores; a candidate carries an upper bound u
// of its score, the score itself lying in [u - 2*kappa*gamma, u].  All entries are sorted by upper bound;
// R = the smallest lower bound among the k entries with the largest upper bounds is a lower bound of the
// k-th largest score, so only the entries with u >= R (a prefix of the sorted order, a few more than k)
// can be among the k best.  Those are re-scored from the packed codes in float32 (each
// wavefront takes entries in turn, lane j sums coordinates j, j+64, ...), sorted again by (score desc,
// label asc) and the k best written.  A query whose candidate list overflowed is appended to the gate list.
__device__ __forceinline__ void merge_sort_desc(uint32_t* s_key, float* s_val, int64_t* s_lab, uint8_t* s_flag,
                                                int size, int tid, bool by_label) {
    for (int sz = 2; sz <= size; sz <<= 1) {
        for (int stride = sz >> 1; stride > 0; stride >>= 1) {
            for (int i = tid; i < size / 2; i += 256) {
                const int lo_i = 2 * i - (i & (stride - 1));
                const int hi_i = lo_i + stride;
                const bool up = ((lo_i & sz) == 0);
                const uint32_t k0 = s_key[lo_i], k1 = s_key[hi_i];
                const int64_t l0 = s_lab[lo_i], l1 = s_lab[hi_i];
                const bool first_before = (k0 > k1) || (k0 == k1 && (!by_label || l0 <= l1));
                if (first_before != up) {
                    s_key[lo_i] = k1; s_key[hi_i] = k0;
                    s_lab[lo_i] = l1; s_lab[hi_i] = l0;
                    const float t = s_val[lo_i]; s_val[lo_i] = s_val[hi_i]; s_val[hi_i] = t;
                    const uint8_t f = s_flag[lo_i]; s_flag[lo_i] = s_flag[hi_i]; s_flag[hi_i] = f;
                }
            }
            __syncthreads();
        }
    }
}

__global__ __launch_bounds__(256) void k_merge(MergeArgs a) {
    extern __shared__ unsigned char smem[];
    __shared__ int s_bound;      // order-preserving key (sign bit flipped for a signed minimum) of the lower bound R
    __shared__ int s_prefix;
    const int64_t q = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int cnt = a.cand_cnt[q];
    const bool overflow = cnt > a.cap;
    if (tid == 0 && overflow) a.gate[1 + atomicAdd(&a.gate[0], 1)] = (int32_t)q;   // listed for the exact pass
    if (overflow) return;                        // the exact streaming pass redoes this query
    if (cnt == 0) {                              // nothing beat the threshold: the first pass's k best stand as they are
        for (int i = tid; i < a.k; i += 256) {
            a.out_scores[q * a.k + i] = a.first_scores[q * a.k + i];
            a.out_ids[q * a.k + i] = a.first_ids[q * a.k + i];
        }
        return;
    }
    const int total = a.k + cnt;
    int size = 1;
    while (size < total) size <<= 1;
    uint32_t* s_key = reinterpret_cast<uint32_t*>(smem);
    float* s_val = reinterpret_cast<float*>(s_key + size);
    int64_t* s_lab = reinterpret_cast<int64_t*>(s_val + size);     // label, or (flag 1) the packed slot of a candidate
    uint8_t* s_flag = reinterpret_cast<uint8_t*>(s_lab + size);    // 1: candidate whose score is still an upper bound
    float* s_z = reinterpret_cast<float*>(smem + (((size_t)size * 17 + 3) & ~(size_t)3));   // [d] the query's rotated coordinates
    for (int j = tid; j < a.d; j += 256) s_z[j] = a.z[q * a.z_pitch + j];
    if (tid == 0) { s_bound = INT32_MAX; s_prefix = 0; }
    __syncthreads();
    for (int i = tid; i < size; i += 256) {
        float v = -__builtin_inff();
        int64_t lab = INT64_MAX;
        uint32_t key = 0;
        uint8_t flag = 0;
        if (i < a.k) {
            lab = a.first_ids[q * a.k + i];
            v = a.first_scores[q * a.k + i];
            if (lab >= 0) key = okey(v); else lab = INT64_MAX;
        } else if (i < total) {
            v = a.cand_score[q * a.cap + (i - a.k)];
            lab = a.cand_slot[q * a.cap + (i - a.k)];
            key = okey(v);
            flag = 1;
        }
        s_key[i] = key; s_val[i] = v; s_lab[i] = lab; s_flag[i] = flag;
    }
    __syncthreads();
    merge_sort_desc(s_key, s_val, s_lab, s_flag, size, tid, false);
    // The k entries with the largest upper bounds have scores of at least their lower bounds, so the
    // smallest of those lower bounds is a lower bound of the k-th largest score.
    const bool have_k = s_key[a.k - 1] != 0u;
    if (have_k) {
        float lo_min = __builtin_inff();
        for (int i = tid; i < a.k; i += 256) {
            float lo = s_val[i];
            if (s_flag[i]) {
                const int64_t slot = s_lab[i] & (((int64_t)1 << kCandProbeShift) - 1);
                lo -= 2.f * a.kappa * __half2float(__ushort_as_half(a.store.gamma[slot]));
            }
            lo_min = fminf(lo_min, lo);
        }
        for (int o = 32; o > 0; o >>= 1) lo_min = fminf(lo_min, __shfl_xor(lo_min, o));
        if (lane == 0) atomicMin(reinterpret_cast<int*>(&s_bound), (int)okey(lo_min) ^ (int)0x80000000);   // signed order of the keys
    }
    __syncthreads();
    // the prefix that can still hold one of the k best
    const uint32_t bound_key = have_k ? ((uint32_t)s_bound ^ 0x80000000u) : 0u;
    for (int i = tid; i < size; i += 256) {
        const bool in = s_key[i] != 0u && s_key[i] >= bound_key;
        const bool next_in = i + 1 < size && s_key[i + 1] != 0u && s_key[i + 1] >= bound_key;
        if (in && !next_in) s_prefix = i + 1;
    }
    __syncthreads();
    const int prefix = s_prefix;
    // exact scores and labels for the candidates in the prefix: 16 lanes per candidate, lane t sums the
    // coordinates t, t+16, ... (the query's rotated coordinates were staged in LDS above)
    const uint32_t mask = (1u << a.b) - 1u;
    const int grp = tid >> 4, gl = tid & 15;
    for (int i = grp; i < prefix; i += 16) {
        if (!s_flag[i]) continue;                 // uniform over the 16 lanes
        const int64_t packed = s_lab[i];
        const int64_t slot = packed & (((int64_t)1 << kCandProbeShift) - 1);
        const int pr = (int)(packed >> kCandProbeShift);
        const uint32_t* wp = a.store.codes + (slot >> 6) * a.store.words * 64 + (slot & 63);
        float acc = 0.f;
        for (int j = gl; j < a.d; j += 16) {
            const int bit = j * a.b, w = bit >> 5, o = bit & 31;
            uint32_t v = wp[(int64_t)w * 64] >> o;
            if (o + a.b > 32) v |= wp[(int64_t)(w + 1) * 64] << (32 - o);
            acc += s_z[j] * a.cb[v & mask];
        }
        for (int o = 8; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 16);
        if (gl == 0) {
            const float sc = a.coarse[q * a.np + pr] + __half2float(__ushort_as_half(a.store.gamma[slot])) * acc;
            s_val[i] = sc;
            s_key[i] = okey(sc);
            s_lab[i] = a.ids ? a.ids[slot] : slot;
        }
    }
    __syncthreads();
    for (int i = tid; i < prefix; i += 256) s_flag[i] = 0;
    __syncthreads();
    // entries beyond the prefix are out; sort the prefix (padded to a power of two) by exact score, then label
    int psize = 1;
    while (psize < prefix) psize <<= 1;
    for (int i = prefix + tid; i < psize; i += 256) { s_key[i] = 0u; s_val[i] = -__builtin_inff(); s_lab[i] = INT64_MAX; s_flag[i] = 0; }
    __syncthreads();
    merge_sort_desc(s_key, s_val, s_lab, s_flag, psize, tid, true);
    for (int i = tid; i < a.k; i += 256) {
        const bool real = i < prefix && s_key[i] != 0u;
        a.out_scores[q * a.k + i] = real ? s_val[i] : -__builtin_inff();
        a.out_ids[q * a.k + i] = real ? s_lab[i] : -1;
    }
}

// WD, OD: wavefronts per workgroup and per SIMD of the dense pass; WT, OT: of the threshold pass (which is
// lighter in registers and LDS, so smaller workgroups let several share a compute unit and overlap their set-up).
template <int DP, int B, int NQ, int WD, int OD, int WT, int OT>
hipError_t run_batch(const BatchScanArgs& a, int max_tiles, hipStream_t st) {
    static LdsLimit lim_threshold, lim_dense;
    const size_t lds = BatchCfg<DP, B, NQ>::lds_bytes;
    const size_t lds_threshold = BatchCfg<DP, B, NQ>::lds_bytes_threshold;
    hipError_t e = a.dense ? lim_dense.ensure(reinterpret_cast<const void*>(k_batch_scan<DP, B, NQ, WD, OD, true>), lds)
                           : lim_threshold.ensure(reinterpret_cast<const void*>(k_batch_scan<DP, B, NQ, WT, OT, false>), lds_threshold);
    if (e != hipSuccess) return e;
    if (a.dense)
        hipLaunchKernelGGL((k_batch_scan<DP, B, NQ, WD, OD, true>), dim3((unsigned)max_tiles), dim3(WD * 64), lds, st, a);
    else
        hipLaunchKernelGGL((k_batch_scan<DP, B, NQ, WT, OT, false>), dim3((unsigned)max_tiles), dim3(WT * 64), lds_threshold, st, a);
    return hipGetLastError();
}

}  // namespace

// Panel width of the batched scan for rows of d coordinates: the padded width of the rotated queries (a multiple
// of 32), except that 193 ... 208 coordinates take 13 blocks of 16 rather than 14 (d = 200: a fourteenth less to
// de-quantise and multiply).
static int batch_dp(int d) { return (d > 192 && d <= 208) ? 208 : rot_dp(d); }

int batch_tile_queries(int d, int b) {
    const int dp = batch_dp(d);
    if (b < 2 || b > 5) return 0;
    if (dp == 64 || dp == 96 || dp == 128) return 128;
    if (dp == 208 || dp == 224) return 128;
    return 0;
}

hipError_t launch_pair_grouping(const int32_t* probe, const int32_t* first, int64_t nq, int np, int L, int tq,
                               uint32_t* count, uint32_t* cursor, int64_t* pair_off, int32_t* tile_off,
                               int32_t* pairs, hipStream_t st) {
    const int64_t n = nq * np;
    if (n <= 0) return hipSuccess;
    hipError_t e = launch_fill_u32(count, 2 * L, 0u, st);
    if (e != hipSuccess) return e;
    if (2 * L <= kPairLdsBuckets) {
        static LdsLimit lim_count, lim_scatter;
        const size_t most = (size_t)kPairLdsBuckets * sizeof(uint32_t);
        e = lim_count.ensure(reinterpret_cast<const void*>(k_pair_count_lds), most);
        if (e == hipSuccess) e = lim_scatter.ensure(reinterpret_cast<const void*>(k_pair_scatter_lds), most);
        if (e != hipSuccess) return e;
        const unsigned blocks = (unsigned)((n + kPairChunk - 1) / kPairChunk);
        const size_t lds = (size_t)2 * L * sizeof(uint32_t);
        hipLaunchKernelGGL(k_pair_count_lds, dim3(blocks), dim3(1024), lds, st, probe, first, nq, np, L, count);
        hipLaunchKernelGGL(k_pair_prefix, dim3(1), dim3(1024), 0, st, count, 2 * L, tq, pair_off, tile_off, cursor);
        hipLaunchKernelGGL(k_pair_scatter_lds, dim3(blocks), dim3(1024), lds, st, probe, first, nq, np, L, pair_off, cursor, pairs);
        return hipGetLastError();
    }
    const unsigned blocks = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(k_pair_count, dim3(blocks), dim3(256), 0, st, probe, first, nq, np, L, count);
    hipLaunchKernelGGL(k_pair_prefix, dim3(1), dim3(1024), 0, st, count, 2 * L, tq, pair_off, tile_off, cursor);
    hipLaunchKernelGGL(k_pair_scatter, dim3(blocks), dim3(256), 0, st, probe, first, nq, np, L, pair_off, cursor, pairs);
    return hipGetLastError();
}

hipError_t launch_batch_scan(const BatchScanArgs& a, int d, int b, int max_tiles, hipStream_t st) {
    if (max_tiles <= 0) return hipSuccess;
    const int dp = batch_dp(d);
    // <coordinates, queries per tile / 32, wavefronts per SIMD of the dense pass, wavefronts per workgroup and per
    // SIMD of the threshold pass>; the dense pass runs eight wavefronts per workgroup
#define IVFTQ_BATCH(DPV, NQV, OCCV, WT, OT)                                                                       \
    if (dp == DPV) {                                                                                              \
        if (b == 2) return run_batch<DPV, 2, NQV, 8, OCCV, WT, OT>(a, max_tiles, st);             \
        if (b == 3) return run_batch<DPV, 3, NQV, 8, OCCV, WT, OT>(a, max_tiles, st);             \
        if (b == 4) return run_batch<DPV, 4, NQV, 8, OCCV, WT, OT>(a, max_tiles, st);             \
        if (b == 5) return run_batch<DPV, 5, NQV, 8, OCCV, WT, OT>(a, max_tiles, st);             \
    }
    IVFTQ_BATCH(64, 4, 2, 4, 3)
    IVFTQ_BATCH(96, 4, 2, 4, 3)
    IVFTQ_BATCH(128, 4, 2, 4, 3)
    IVFTQ_BATCH(208, 4, 2, 4, 2)
    IVFTQ_BATCH(224, 4, 2, 4, 2)
#undef IVFTQ_BATCH
    return hipErrorInvalidValue;
}

hipError_t launch_merge(const MergeArgs& a, int64_t nq, hipStream_t st) {
    if (nq <= 0) return hipSuccess;
    int size = 1;
    while (size < a.k + a.cap) size <<= 1;
    const size_t lds = (size_t)size * 17 + 4 + (size_t)a.d * sizeof(float);
    static LdsLimit lim;
    const hipError_t e = lim.ensure(reinterpret_cast<const void*>(k_merge), 128 * 1024);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_merge, dim3((unsigned)nq), dim3(256), lds, st, a);
    return hipGetLastError();
}

}  // namespace ivftq
