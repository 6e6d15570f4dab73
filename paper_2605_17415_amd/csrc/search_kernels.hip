// Search-side kernels (Section "Architecture", Search): the scan of the probed lists, which adds
// the residual estimate gamma * <Pi q~, C[code]> to the exact coarse term, and the per-query
// selection of the best k (also used to pick the nprobe best cells).
#include <hip/hip_fp16.h>

#include <algorithm>

#include "kernels.h"

namespace ivftq {

namespace {

// ---- candidate offsets -----------------------------------------------------------------------

// Also, when asked: first[q] = the number of leading probes whose lists are scored densely to find
// the query's threshold (see the kernel), or np when all probed cells together hold too few vectors.
__global__ __launch_bounds__(256) void k_cand_offsets(const int32_t* __restrict__ probe, int64_t nq, int np,
                                                      const int32_t* __restrict__ list_size, int32_t* __restrict__ cand_off,
                                                      int k, int cap, int32_t* __restrict__ first,
                                                      int32_t* __restrict__ cand_cnt, int32_t* __restrict__ gate) {
    // one wavefront per query: 64 probes at a time, running sum over the lanes
    const int lane = threadIdx.x & 63;
    const int64_t q = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (q >= nq) return;
    int32_t run = 0;
    for (int p0 = 0; p0 < np; p0 += 64) {
        const int p = p0 + lane;
        const int32_t size = p < np ? list_size[probe[q * np + p]] : 0;
        int32_t incl = size;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int32_t t = __shfl_up(incl, o);
            if (lane >= o) incl += t;
        }
        if (p < np) cand_off[q * (np + 1) + p] = run + incl - size;
        run += __shfl(incl, 63);
    }
    if (lane == 0) cand_off[q * (np + 1) + np] = run;
    if (!first) return;
    // Were the prefix a random sample of P of the query's T candidates, its k-th score would be beaten by
    // about k*(T-P)/P of the others; P = f*k*T/cap (f = kPrefixFactorX2/2) keeps that near cap/f even then.
    // The nearest lists hold the best candidates, so in practice far fewer pass (and a list that does
    // overflow sends its query to the exact pass).  At least k vectors, so that a threshold exists.
    int64_t need = (kPrefixFactorX2 * (int64_t)k * run + 2 * cap - 1) / (2 * cap);
    if (need < k) need = k;
    // the first p >= 1 whose lists 0 .. p-1 together reach `need` (np when none does)
    int p1 = np;
    int32_t run2 = 0;
    for (int p0 = 0; p0 < np && p1 == np; p0 += 64) {
        const int p = p0 + lane;
        const int32_t size = p < np ? list_size[probe[q * np + p]] : 0;
        int32_t incl = size;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int32_t t = __shfl_up(incl, o);
            if (lane >= o) incl += t;
        }
        const uint64_t reached = __ballot(p < np && (int64_t)(run2 + incl) >= need);
        if (reached) p1 = p0 + (int)__builtin_ctzll(reached) + 1;
        run2 += __shfl(incl, 63);
    }
    if (lane == 0) {
        first[q] = p1;
        // the counters of the batched scan start at zero (cleared here rather than by launches of their own)
        if (cand_cnt) cand_cnt[q] = 0;
        if (gate && q == 0) gate[0] = 0;
    }
}

// ---- list scan: a row of workgroups per query walks its probed lists ---------------------------
//
// The query's rotated coordinates and the 2^b centroid values are combined once per workgroup
// into a table lut[j][e] = z_j * C[e] in LDS (the per-query ADC table the paper's own scan uses,
// Appendix "Why cascade does not yield a speedup"); a lane then owns one stored vector at a time,
// reads its packed words with 256-byte-per-wavefront coalesced loads and sums d table entries.
// When the table would not fit LDS (large b and d) DIRECT keeps z and C separately and multiplies
// per coordinate instead.
template <int B, bool DIRECT>
__global__ __launch_bounds__(256) void k_list_scan(const float* __restrict__ z, int z_pitch, int d,
                                                   const float* __restrict__ cb,
                                                   const int32_t* __restrict__ probe,
                                                   const float* __restrict__ coarse,
                                                   const int32_t* __restrict__ cand_off, int np,
                                                   ListStore store, int64_t q_begin,
                                                   float* __restrict__ scores, int64_t m_stride,
                                                   const int32_t* __restrict__ p_limit,
                                                   const int32_t* __restrict__ gate, int gate_begin, int gate_rows,
                                                   int metric, const float* __restrict__ qnorm) {
    constexpr int K = 1 << B;
    extern __shared__ float lut[];     // [d][K], or z[d] followed by C[K] when DIRECT
    // gate (may be null): of the gate[0] queries listed in gate[1..], entries [gate_begin, gate_begin +
    // gate_rows) are processed instead of all queries, entry g writing score row g - gate_begin; the grid's
    // y extent is then fixed and each workgroup row walks the list
    int64_t n_rows = gridDim.y;
    if (gate) n_rows = gate[0] < gate_begin + gate_rows ? gate[0] : gate_begin + gate_rows;
    for (int64_t row_i = (gate ? gate_begin : 0) + blockIdx.y; row_i < n_rows; row_i += gridDim.y) {
    const int64_t qi = gate ? gate[1 + row_i] : row_i;     // index inside this pass
    const int64_t score_row = gate ? row_i - gate_begin : qi;
    const int64_t q = q_begin + qi;
    const int p_end = p_limit ? p_limit[q] : np;
    if ((int)blockIdx.x >= p_end) continue;
    const float qn = metric ? qnorm[q] : 1.f;
    __syncthreads();                   // the table of the previous query is no longer read

    if constexpr (DIRECT) {
        for (int e = threadIdx.x; e < d; e += 256) lut[e] = z[q * z_pitch + e];
        for (int e = threadIdx.x; e < K; e += 256) lut[d + e] = cb[e];
    } else {
        for (int e = threadIdx.x; e < d * K; e += 256) lut[e] = z[q * z_pitch + (e >> B)] * cb[e & (K - 1)];
    }
    __syncthreads();
    auto term = [&](int j, uint32_t code) -> float {
        if constexpr (DIRECT) return lut[j] * lut[d + code];
        else return lut[j * K + code];
    };

    const int words = store.words;
    for (int p = blockIdx.x; p < p_end; p += gridDim.x) {
    const int l = probe[q * np + p];
    const int n_l = store.list_size[l];
    const float s_l = coarse[q * np + p];
    const int64_t base_slot = store.list_off[l];
    float* out = scores + score_row * m_stride + cand_off[q * (np + 1) + p];

    // a list is dealt out in rounds of 256 vectors to the gridDim.z workgroups that share it
    for (int v = threadIdx.x + 256 * (int)blockIdx.z; v < n_l; v += 256 * (int)gridDim.z) {
        const int64_t slot = base_slot + v;
        const uint32_t* wp = store.codes + (slot >> 6) * words * 64 + (slot & 63);
        float acc = 0.f;
        // A row is walked in chunks of 32 coordinates = B packed words, whose codes sit at bit positions known at
        // compile time.
        int chunks = 0;                // whole chunks summed by the table lookups below
        if constexpr (!DIRECT && B >= 2) {   // (one-bit codes: the two bits below a code are not a single neighbour's)
            // Table lookups without address arithmetic.  The codes of a word are split by the parity of their
            // position into two masked copies, so that the bits below a code are zero; a bit-field extract that
            // starts two bits below the code then yields the code times four, the byte offset of its table entry.
            // The chunk loop is unrolled against the longest row the table fits, which makes the coordinate's part
            // of the address an immediate of the LDS read: per code one extract, one read and one add, per word
            // two masks.  (A code in the lowest two bits of a word is shifted up and masked instead, one that
            // straddles two words is taken from the aligned pair.)  The next chunk's words are fetched before the
            // current one is summed.  Coordinates beyond the last whole chunk take the loop further down.
            // longest row: the table fits 64 KB (4K bytes per coordinate) and the library takes d <= 256
            constexpr int kMaxCoords = (64 * 1024 / (K * 4)) < 256 ? (64 * 1024 / (K * 4)) : 256;
            constexpr int kMaxChunks = kMaxCoords / 32;
            // The table's LDS address: the lookups address LDS by number (offset of the entry plus an
            // immediate), which holds when the table starts at LDS address 0 -- it is this kernel's only
            // shared array; were it ever placed elsewhere, every chunk takes the loop further down instead.
            typedef __attribute__((address_space(3))) const float lds_float;
            uint32_t lut_at = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) float*)lut;
            asm volatile("" : "+s"(lut_at));
            // opaque, so that the tests below stay scalar compares inside the loop instead of a set of flags
            // computed ahead of it
            chunks = lut_at == 0 ? ((d >> 5) < kMaxChunks ? (d >> 5) : kMaxChunks) : 0;
            asm volatile("" : "+s"(chunks));
            uint32_t cur[B];
            if (chunks > 0) {
#pragma unroll
                for (int u = 0; u < B; ++u) cur[u] = wp[u * 64];
            }
#pragma unroll
            for (int c = 0; c < kMaxChunks; ++c) {
                if (c >= chunks) break;
                uint32_t nxt[B];
                if (c + 1 < chunks) {
#pragma unroll
                    for (int u = 0; u < B; ++u) nxt[u] = wp[((c + 1) * B + u) * 64];
                }
                uint32_t par[B][2];    // word u with only its whole codes of even / odd position kept
#pragma unroll
                for (int u = 0; u < B; ++u) {
                    uint32_t m[2] = {0u, 0u};
#pragma unroll
                    for (int t = 0; t < 32; ++t)
                        if (((t * B) >> 5) == u && ((t * B) & 31) + B <= 32) m[t & 1] |= (uint32_t)(K - 1) << ((t * B) & 31);
                    par[u][0] = cur[u] & m[0];
                    par[u][1] = cur[u] & m[1];
                    asm("" : "+v"(par[u][0]));   // keeps each lookup one bit-field extract: with the cleared
                    asm("" : "+v"(par[u][1]));   // bits known, the compiler rewrites it as a shift and a mask
                }
#pragma unroll
                for (int t = 0; t < 32; ++t) {
                    const int wi = (t * B) >> 5, sh = (t * B) & 31;
                    uint32_t off4;
                    if (sh + B > 32)   // straddles: sh > 24
                        off4 = __builtin_amdgcn_alignbit(cur[wi + 1 < B ? wi + 1 : wi], cur[wi], sh - 2) & ((uint32_t)(K - 1) << 2);
                    else if (sh < 2)
                        off4 = (cur[wi] << (2 - sh)) & ((uint32_t)(K - 1) << 2);
                    else
                        off4 = __builtin_amdgcn_ubfe(par[wi][t & 1], sh - 2, B + 2);
                    acc += *(lds_float*)(off4 + (uint32_t)((c * 32 + t) * K * 4));
                }
#pragma unroll
                for (int u = 0; u < B; ++u) cur[u] = nxt[u];
            }
        }
        // the rest (a last chunk of fewer than 32 coordinates; every chunk when the table is not in LDS): every
        // code is one bit-field extract (two shifts where it straddles a word) plus the address arithmetic
        for (int w0 = chunks * B; w0 < words; w0 += B) {
            uint32_t wd[B + 1];
#pragma unroll
            for (int u = 0; u < B; ++u) wd[u] = (w0 + u < words) ? wp[(w0 + u) * 64] : 0u;
            wd[B] = 0u;
            const int j0 = (w0 / B) * 32;
            const bool whole = j0 + 32 <= d;
#pragma unroll
            for (int t = 0; t < 32; ++t) {
                constexpr int kBits = B;
                const int wi = (t * kBits) >> 5, sh = (t * kBits) & 31;
                const uint32_t code = (sh + kBits <= 32)
                    ? __builtin_amdgcn_ubfe(wd[wi], sh, kBits)
                    : (((wd[wi] >> sh) | (wd[wi + 1] << (32 - sh))) & (uint32_t)(K - 1));
                if (whole || j0 + t < d) acc += term(j0 + t, code);
            }
        }
        const float g = __half2float(__ushort_as_half(store.gamma[slot]));
        float sc = s_l + g * acc;
        if (metric) {                  // ranking key of a raw metric (see launch_metric_finish)
            const float xn = store.xnorm[slot];
            sc = metric == 1 ? xn * sc : fmaf(2.f * xn * qn, sc, -xn * xn);
        }
        out[v] = sc;
    }
    }
    }
}

// Selected ranking keys of a raw metric -> metric values (keys of missing results are -inf).
__global__ void k_metric_finish(float* __restrict__ scores, int64_t nq, int k, int metric, const float* __restrict__ qnorm) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nq * k) return;
    const float qn = qnorm[i / k], key = scores[i];
    scores[i] = metric == 1 ? qn * key : qn * qn - key;       // -inf stays -inf (inner product) or becomes +inf (distance)
}

// ---- selection: k largest of a row ------------------------------------------------------------
//
// Exact radix selection on an order-preserving 32-bit key (four 8-bit digits, most significant
// first), then the survivors are labelled and sorted by (value desc, label asc) with a bitonic
// network in LDS.  Among values equal to the k-th one, those with the smallest column are kept.

__device__ __forceinline__ uint32_t order_key(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int kSelU = 8;        // groups of 64 columns loaded together by k_select
constexpr int kSelSmallU = 8;   // and by k_select_small beyond its registers
constexpr int kSelCand = 512;   // most keys the short cut of k_select sorts directly

// COPIES: counters per digit in the histogram (a power of two; 8 pays for long rows, 1 for short ones, where
// clearing and summing the copies costs more than the collisions they avoid).
template <int MODE, int COPIES>
__global__ __launch_bounds__(256) void k_select(SelectArgs a) {
    constexpr int kHistCopies = COPIES;
    extern __shared__ unsigned char smem[];
    int kpad = 1;
    while (kpad < a.k) kpad <<= 1;
    // kHistCopies counters per digit, chosen by lane: keys of one row often share their leading byte, and
    // 64 lanes adding to one LDS word are served one after the other
    uint32_t* hist = reinterpret_cast<uint32_t*>(smem);               // [256][kHistCopies]
    uint32_t* ctrl = hist + 256 * kHistCopies;                        // [8]
    uint32_t* wave_cnt = ctrl + 8;                                    // [4]
    uint32_t* s_key = wave_cnt + 4;                                   // [kpad]
    uint32_t* s_col = s_key + kpad;                                   // [kpad]
    int64_t* s_lab = reinterpret_cast<int64_t*>(s_col + kpad);   // [kpad], 8-byte aligned: 268 + 2*kpad words
    uint32_t* c_key = reinterpret_cast<uint32_t*>(s_lab + kpad);      // [kSelCand] keys of the short cut ...
    uint32_t* c_col = c_key + kSelCand;                               // [kSelCand] ... and their columns

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // gate (may be null): a.gate[0] rows, listed in a.gate[1..], are processed instead of all
    int64_t n_rows = a.rows;
    if (a.gate) n_rows = a.gate[0] < a.gate_begin + a.gate_rows ? a.gate[0] : a.gate_begin + a.gate_rows;
    for (int64_t row_i = (a.gate ? a.gate_begin : 0) + blockIdx.x; row_i < n_rows; row_i += gridDim.x) {
    const int64_t row = a.gate ? a.gate[1 + row_i] : row_i;
    const float* vals = a.vals + (a.gate ? row_i - a.gate_begin : row) * a.stride;
    const int64_t q = a.q_begin + row;
    __syncthreads();                   // LDS of the previous row is no longer read
    const int m = (MODE == 0) ? a.m_fixed
                              : a.cand_off[q * (a.np + 1) + (a.p_limit ? a.p_limit[q] : a.np)];
    const int k = a.k;
    const int take = m < k ? m : k;

    for (int i = tid; i < kpad; i += 256) { s_key[i] = 0u; s_col[i] = 0xFFFFFFFFu; s_lab[i] = INT64_MAX; }

    // each wavefront owns a contiguous quarter [w_begin, w_end) of the row
    const int chunk = ((m + 3) / 4 + 63) & ~63;
    const int w_begin = wave * chunk < m ? wave * chunk : m;
    const int w_end = (w_begin + chunk < m) ? w_begin + chunk : m;
    uint32_t prefix = 0, mask = 0;
    uint32_t need = (uint32_t)take;
    // Short cut.  Every thread takes the largest key of the columns tid, tid + 256, ...; at least `take`
    // values reach the take-th largest of these 256 maxima, so it is a lower bound of the take-th largest
    // value, and with the columns dealt out round-robin about -256 ln(1 - take/256) values reach it
    // whatever the row looks like (127 for take = 100, 355 for 192; beyond that too many).  Those are gathered and sorted by (key desc, column asc): the first
    // `take` of them are the winners the radix search below would pick (same rule for keys equal to the
    // last one).  Two reads of the row instead of six; if more than kSelCand values reach the bound the
    // radix search runs after all.
    bool picked = false;
    if (take > 0 && m > k && take <= 192 && m >= 2048) {
        uint32_t best = 0;            // below every key of a number
        for (int i0 = 0; i0 < m; i0 += 256 * kSelU) {
            float v[kSelU];
#pragma unroll
            for (int u = 0; u < kSelU; ++u) {
                const int i = i0 + 256 * u + tid;
                v[u] = vals[i < m ? i : m - 1];
            }
#pragma unroll
            for (int u = 0; u < kSelU; ++u) {
                const uint32_t key = order_key(v[u]);
                if (i0 + 256 * u + tid < m && key > best) best = key;
            }
        }
        c_key[tid] = best;
        if (tid == 0) { ctrl[4] = 0; ctrl[5] = 0; }
        __syncthreads();
        // rank of this thread's maximum among the 256 (larger first, thread number breaks ties)
        uint32_t rank = 0;
        for (int j = 0; j < 256; j += 4) {
            const uint4 o = *reinterpret_cast<const uint4*>(c_key + j);
            rank += (o.x > best || (o.x == best && j < tid)) ? 1u : 0u;
            rank += (o.y > best || (o.y == best && j + 1 < tid)) ? 1u : 0u;
            rank += (o.z > best || (o.z == best && j + 2 < tid)) ? 1u : 0u;
            rank += (o.w > best || (o.w == best && j + 3 < tid)) ? 1u : 0u;
        }
        if (rank == (uint32_t)take - 1u) ctrl[4] = best;
        __syncthreads();
        const uint32_t bound = ctrl[4];
        __syncthreads();               // the maxima are no longer read: c_key is filled anew
        for (int i0 = 0; i0 < m; i0 += 256 * kSelU) {
            float v[kSelU];
#pragma unroll
            for (int u = 0; u < kSelU; ++u) {
                const int i = i0 + 256 * u + tid;
                v[u] = vals[i < m ? i : m - 1];
            }
#pragma unroll
            for (int u = 0; u < kSelU; ++u) {
                const int i = i0 + 256 * u + tid;
                const uint32_t key = order_key(v[u]);
                if (i < m && key >= bound) {
                    const uint32_t pos = atomicAdd(&ctrl[5], 1u);
                    if (pos < (uint32_t)kSelCand) { c_key[pos] = key; c_col[pos] = (uint32_t)i; }
                }
            }
        }
        __syncthreads();
        const uint32_t found = ctrl[5];
        if (found <= (uint32_t)kSelCand) {          // uniform over the workgroup
            int cpad = 1;
            while (cpad < (int)found) cpad <<= 1;
            for (int i = (int)found + tid; i < cpad; i += 256) { c_key[i] = 0u; c_col[i] = 0xFFFFFFFFu; }
            __syncthreads();
            for (int size = 2; size <= cpad; size <<= 1) {
                for (int stride = size >> 1; stride > 0; stride >>= 1) {
                    for (int i = tid; i < cpad / 2; i += 256) {
                        const int lo_i = 2 * i - (i & (stride - 1));
                        const int hi_i = lo_i + stride;
                        const bool up = ((lo_i & size) == 0);
                        const uint32_t k0 = c_key[lo_i], k1 = c_key[hi_i];
                        const uint32_t c0 = c_col[lo_i], c1 = c_col[hi_i];
                        const bool first_before = (k0 > k1) || (k0 == k1 && c0 <= c1);
                        if (first_before != up) {
                            c_key[lo_i] = k1; c_key[hi_i] = k0;
                            c_col[lo_i] = c1; c_col[hi_i] = c0;
                        }
                    }
                    __syncthreads();
                }
            }
            for (int i = tid; i < take; i += 256) { s_key[i] = c_key[i]; s_col[i] = c_col[i]; }
            picked = true;
        }
        __syncthreads();
    }
    if (picked) {
        // winners are in place
    } else if (take > 0 && m > k) {
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
#pragma unroll
            for (int e = 0; e < kHistCopies; ++e) hist[tid + 256 * e] = 0;
            __syncthreads();
            // kSelU groups of 64 columns per step, their loads in flight together (the pass is bound by the
            // latency of reading the row, not by its arithmetic)
            for (int i0 = w_begin; i0 < w_end; i0 += 64 * kSelU) {
                float v[kSelU];
#pragma unroll
                for (int u = 0; u < kSelU; ++u) {
                    const int i = i0 + 64 * u + lane;
                    v[u] = vals[i < w_end ? i : w_end - 1];
                }
#pragma unroll
                for (int u = 0; u < kSelU; ++u) {
                    const uint32_t key = order_key(v[u]);
                    if (i0 + 64 * u + lane < w_end && (key & mask) == prefix)
                        atomicAdd(&hist[((key >> shift) & 255u) * kHistCopies + (lane & (kHistCopies - 1))], 1u);
                }
            }
            __syncthreads();
            if (wave == 0) {
                // the digit where the count of keys with larger digits first reaches `need`: lane l owns the
                // digits 4l .. 4l+3, a suffix sum over the lanes gives what lies above each lane
                uint32_t h[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    h[e] = 0;
#pragma unroll
                    for (int c = 0; c < kHistCopies; ++c) h[e] += hist[(lane * 4 + e) * kHistCopies + c];
                }
                const uint32_t own = h[0] + h[1] + h[2] + h[3];
                uint32_t incl = own;
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) {
                    const uint32_t t = __shfl_down(incl, o);
                    if (lane + o < 64) incl += t;
                }
                uint32_t above = incl - own;
                int found = -1;
                uint32_t before = 0;
#pragma unroll
                for (int e = 3; e >= 0; --e) {
                    if (found < 0 && above < need && above + h[e] >= need) { found = lane * 4 + e; before = above; }
                    above += h[e];
                }
                if (found >= 0) { ctrl[0] = (uint32_t)found; ctrl[1] = need - before; }   // exactly one lane (need >= 1)
            }
            __syncthreads();
            prefix |= ctrl[0] << shift;
            mask |= 255u << shift;
            need = ctrl[1];
            __syncthreads();
        }
    } else {
        need = 0;   // everything is taken (m <= k): threshold below every key
    }
    // now: keys > prefix are all kept (take - need of them); `need` of the keys == prefix are kept
    const bool all = !(take > 0 && m > k);
    if (tid == 0) { ctrl[2] = 0; ctrl[3] = 0; }
    __syncthreads();
    const uint32_t n_above = (uint32_t)take - need;
    if (take > 0 && !picked) {
        // Keys above the threshold go anywhere in the first n_above places (atomic counter).  Keys equal to it
        // are taken in column order: each wavefront owns a contiguous quarter of the row, counts its ties in a
        // first sweep and, once the counts of the wavefronts before it are known, places them in a second.
        uint32_t my_ties = 0;
        for (int i0 = w_begin; i0 < w_end; i0 += 64 * kSelU) {
            float v[kSelU];
#pragma unroll
            for (int u = 0; u < kSelU; ++u) {
                const int i = i0 + 64 * u + lane;
                v[u] = vals[i < w_end ? i : w_end - 1];
            }
#pragma unroll
            for (int u = 0; u < kSelU; ++u) {
                const int i = i0 + 64 * u + lane;
                const uint32_t key = order_key(v[u]);
                const bool above = i < w_end && (all || key > prefix);
                const bool tie = i < w_end && !all && key == prefix;
                if (above) {
                    const uint32_t pos = atomicAdd(&ctrl[2], 1u);
                    s_key[pos] = key;
                    s_col[pos] = (uint32_t)i;
                }
                my_ties += (uint32_t)__popcll(__ballot(tie));
            }
        }
        if (lane == 0) wave_cnt[wave] = my_ties;
        __syncthreads();
        uint32_t before = 0;
        for (int w = 0; w < wave; ++w) before += wave_cnt[w];
        for (int i0 = w_begin; i0 < w_end && before < need && my_ties > 0; i0 += 64) {
            const int i = i0 + lane;
            uint32_t key = 0;
            bool tie = false;
            if (i < w_end) {
                key = order_key(vals[i]);
                tie = !all && key == prefix;
            }
            const uint64_t bal = __ballot(tie);
            const uint32_t rank = before + (uint32_t)__popcll(bal & ((1ull << lane) - 1ull));
            if (tie && rank < need) {
                s_key[n_above + rank] = key;
                s_col[n_above + rank] = (uint32_t)i;
            }
            before += (uint32_t)__popcll(bal);
        }
    }
    __syncthreads();

    // labels
    for (int i = tid; i < take; i += 256) {
        const uint32_t col = s_col[i];
        if (MODE == 0) {
            s_lab[i] = (int64_t)col;
        } else {
            const int32_t* off = a.cand_off + q * (a.np + 1);
            int lo = 0, hi = a.np;          // largest p with off[p] <= col
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (off[mid] <= (int32_t)col) lo = mid; else hi = mid;
            }
            const int l = a.probe[q * a.np + lo];
            const int64_t slot = a.list_off[l] + ((int32_t)col - off[lo]);
            s_lab[i] = a.ids ? a.ids[slot] : slot;       // without a label table the slot itself is the result
        }
    }
    __syncthreads();

    // bitonic sort, descending key then ascending label; empty entries (key 0, label max) sink
    for (int size = 2; size <= kpad; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int i = tid; i < kpad / 2; i += 256) {
                const int lo_i = 2 * i - (i & (stride - 1));
                const int hi_i = lo_i + stride;
                const bool up = ((lo_i & size) == 0);
                const uint32_t k0 = s_key[lo_i], k1 = s_key[hi_i];
                const int64_t l0 = s_lab[lo_i], l1 = s_lab[hi_i];
                const bool first_before = (k0 > k1) || (k0 == k1 && l0 <= l1);   // lo already precedes hi
                if (first_before != up) {
                    s_key[lo_i] = k1; s_key[hi_i] = k0;
                    s_lab[lo_i] = l1; s_lab[hi_i] = l0;
                    const uint32_t c0 = s_col[lo_i]; s_col[lo_i] = s_col[hi_i]; s_col[hi_i] = c0;
                }
            }
            __syncthreads();
        }
    }

    for (int i = tid; i < k; i += 256) {
        const bool real = i < take;
        const float v = real ? vals[s_col[i]] : -__builtin_inff();
        if (a.out_vals) a.out_vals[row * k + i] = v;
        if (MODE == 0) { if (a.out_i32) a.out_i32[row * k + i] = real ? (int32_t)s_lab[i] : -1; }
        else { if (a.out_i64) a.out_i64[row * k + i] = real ? s_lab[i] : -1; }
    }
    }
}

// ---- selection for short rows: one wavefront per row ------------------------------------------
//
// For rows of at most kSmallM values (bound known to the host) and k <= 64 a wavefront does the whole selection on its own,
// without workgroup barriers: the k-th largest key is found by a four-pass radix search (8 bits per
// pass, a 256-bin histogram private to the wavefront, a suffix sum over the lanes), then the values
// above it and, in column order, as many equal to it as are still needed are compacted with
// ballots.  The first 64*NV columns of the row are loaded once, all loads in flight together, and
// every pass takes them from registers; columns beyond that (long rows are rare) are re-read from
// memory in each pass.  A wavefront needs little LDS, so many rows are in flight per compute unit.  A final bitonic pass over the lanes orders the winners by (value desc, label asc).

// MODE 2 and 3 are the two halves of a selection in two steps, for calls with so few rows that one wavefront
// per row would leave the chip idle: MODE 2 takes the k best of every (query, probed list) stretch of a score
// row, with labels, MODE 3 the k best of a query's np * k survivors (labels looked up, not computed).
constexpr int kSmallM = 16384;
constexpr int kShortcutTake = 32;     // the lane-maxima short cut pays up to this many winners (beyond, too many keys reach the bound)

// WIDE: the instantiation for more than kShortcutTake winners (its second short cut costs the common case of
// fewer winners a fifth of its speed when both sit in one kernel).
template <int MODE, int NV, bool WIDE = false>
// (probe selection, MODE 0, is held to the registers of four wavefronts per SIMD: 10,000 rows over 4096 cells
// take 0.072 ms so, 0.100 ms at the two wavefronts its unconstrained register count allows; the result rows of
// MODE 1 lose from the same limit)
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(MODE == 0 ? 4 : 1, 8))) void k_select_small(SelectArgs a) {
    __shared__ uint32_t s_work[4][256 + 64];             // per wavefront: 256 bins, 64 winning columns
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t n_rows = a.rows;
    if (a.gate) n_rows = a.gate[0] < a.gate_begin + a.gate_rows ? a.gate[0] : a.gate_begin + a.gate_rows;
    for (int64_t row_i = (a.gate ? a.gate_begin : 0) + (int64_t)blockIdx.x * 4 + wave; row_i < n_rows; row_i += (int64_t)gridDim.x * 4) {
    const int64_t row = a.gate ? a.gate[1 + row_i] : row_i;
    // MODE 2: row = (query, probe rank); the stretch of that list in the query's score row
    const int64_t q = a.q_begin + (MODE == 2 ? row / a.np : row);
    const int sub_p = MODE == 2 ? (int)(row % a.np) : 0;
    int m, sub_off = 0;
    if (MODE == 0 || MODE == 3) {
        m = a.m_fixed;
    } else if (MODE == 1) {
        m = a.cand_off[q * (a.np + 1) + (a.p_limit ? a.p_limit[q] : a.np)];
    } else {
        const int32_t* off = a.cand_off + q * (a.np + 1);
        sub_off = off[sub_p];
        m = (a.p_limit && sub_p >= a.p_limit[q]) ? 0 : off[sub_p + 1] - sub_off;
    }
    const int k = a.k;
    const int take = m < k ? m : k;
    const float* vals = MODE == 2 ? a.vals + (row / a.np) * a.stride + sub_off
                                  : a.vals + (a.gate ? row_i - a.gate_begin : row) * a.stride;
    uint32_t* hist = s_work[wave];                                      // [256]
    int* win_col = reinterpret_cast<int*>(hist + 256);                  // [64]
    const float ninf = -__builtin_inff();
    auto key_of = [](float v) -> uint32_t { return v != v ? 0u : order_key(v); };   // NaN sorts last

    win_col[lane] = -1;
    uint32_t keys[NV];                                   // key of column e*64 + lane (unused beyond m)
#pragma unroll
    for (int e = 0; e < NV; ++e) {
        const int i = e * 64 + lane;
        keys[e] = key_of(vals[i < m ? i : 0]);
    }

    // Short cut.  The take-th largest of the 64 lane maxima is reached by at least `take` keys (one per lane
    // that holds such a maximum), so every winner is among the keys that reach it; there are seldom many more
    // than `take` of them.  When at most 64 do, they are compacted into the lanes, sorted by (key desc, column
    // asc) and the first `take` are the winners: the same set as the radix search below would pick.
    bool done = false;
    if (take > 0 && take <= kShortcutTake) {
        uint32_t lane_max = 0u;
#pragma unroll
        for (int e = 0; e < NV; ++e) lane_max = (e * 64 + lane < m && keys[e] > lane_max) ? keys[e] : lane_max;
        for (int i0 = NV * 64; i0 < m; i0 += 64 * kSelSmallU) {
            float v[kSelSmallU];
#pragma unroll
            for (int u = 0; u < kSelSmallU; ++u) { const int i = i0 + 64 * u + lane; v[u] = vals[i < m ? i : m - 1]; }
#pragma unroll
            for (int u = 0; u < kSelSmallU; ++u) {
                const uint32_t key = key_of(v[u]);
                lane_max = (i0 + 64 * u + lane < m && key > lane_max) ? key : lane_max;
            }
        }
        uint32_t sorted = lane_max;                      // the lane maxima in descending order over the lanes
#pragma unroll
        for (int size = 2; size <= 64; size <<= 1) {
#pragma unroll
            for (int stride = size >> 1; stride > 0; stride >>= 1) {
                const uint32_t other = __shfl_xor(sorted, stride);
                const bool lower = (lane & stride) == 0, up = (lane & size) == 0;
                const bool keep = (lower == up) ? (sorted >= other) : (sorted <= other);
                sorted = keep ? sorted : other;
            }
        }
        const uint32_t reach = __shfl(sorted, take - 1);
        if (reach != 0u) {
            uint32_t* c_key = hist;                      // [64] keys that reach it, [64] their columns
            int* c_col = reinterpret_cast<int*>(hist + 64);
            uint32_t count = 0;
            auto collect = [&](int i, uint32_t key) {
                const bool in = i < m && key >= reach;
                const uint64_t b = __ballot(in);
                const uint32_t pos = count + (uint32_t)__popcll(b & (((uint64_t)1 << lane) - 1));
                if (in && pos < 64u) { c_key[pos] = key; c_col[pos] = i; }
                count += (uint32_t)__popcll(b);
            };
#pragma unroll
            for (int e = 0; e < NV; ++e)
                if (e * 64 < m) collect(e * 64 + lane, keys[e]);
            for (int i0 = NV * 64; i0 < m && count <= 64u; i0 += 64 * kSelSmallU) {
                float v[kSelSmallU];
#pragma unroll
                for (int u = 0; u < kSelSmallU; ++u) { const int i = i0 + 64 * u + lane; v[u] = vals[i < m ? i : m - 1]; }
#pragma unroll
                for (int u = 0; u < kSelSmallU; ++u)
                    if (i0 + 64 * u < m) collect(i0 + 64 * u + lane, key_of(v[u]));
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if (count <= 64u) {
                uint32_t ck = lane < (int)count ? c_key[lane] : 0u;
                int cc = lane < (int)count ? c_col[lane] : INT32_MAX;
#pragma unroll
                for (int size = 2; size <= 64; size <<= 1) {
#pragma unroll
                    for (int stride = size >> 1; stride > 0; stride >>= 1) {
                        const uint32_t ok = __shfl_xor(ck, stride);
                        const int oc = __shfl_xor(cc, stride);
                        const bool lower = (lane & stride) == 0, up = (lane & size) == 0;
                        const bool mine_first = (ck > ok) || (ck == ok && cc <= oc);
                        const bool keep = (lower == up) ? mine_first : !mine_first;
                        if (!keep) { ck = ok; cc = oc; }
                    }
                }
                if (lane < take) win_col[lane] = cc;
                done = true;
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();         // the words of `hist` are free again
        }
    }
    // The same idea for up to 64 winners, with two maxima per lane (over the even and over the odd 64-column
    // blocks of the row): the take-th largest of these 128 is again reached by at least `take` keys, and by few
    // more.  It is found by bisection on the key's bits (two ballots a bit); up to 128 keys that reach it are
    // compacted into LDS and every one counts the keys that precede it in (key desc, column asc) order, which is
    // its place among the winners.
    if (WIDE && !done && take > kShortcutTake && take <= 64) {
        uint32_t gm0 = 0u, gm1 = 0u;
#pragma unroll
        for (int e = 0; e < NV; ++e) {
            const bool in = e * 64 + lane < m;
            if (e & 1) gm1 = (in && keys[e] > gm1) ? keys[e] : gm1;
            else gm0 = (in && keys[e] > gm0) ? keys[e] : gm0;
        }
        static_assert(NV % 2 == 0 && kSelSmallU % 2 == 0, "block parity below");
        for (int i0 = NV * 64; i0 < m; i0 += 64 * kSelSmallU) {
            float v[kSelSmallU];
#pragma unroll
            for (int u = 0; u < kSelSmallU; ++u) { const int i = i0 + 64 * u + lane; v[u] = vals[i < m ? i : m - 1]; }
#pragma unroll
            for (int u = 0; u < kSelSmallU; ++u) {
                const uint32_t key = key_of(v[u]);
                const bool in = i0 + 64 * u + lane < m;
                if (u & 1) gm1 = (in && key > gm1) ? key : gm1;
                else gm0 = (in && key > gm0) ? key : gm0;
            }
        }
        uint32_t reach = 0u;
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t test = reach | (1u << bit);
            const int cnt = __popcll(__ballot(gm0 >= test)) + __popcll(__ballot(gm1 >= test));
            if (cnt >= take) reach = test;
        }
        if (reach != 0u) {
            uint32_t* c_key = hist;                      // [128] keys that reach it, [128] their columns
            int* c_col = reinterpret_cast<int*>(hist + 128);
            uint32_t count = 0;
            auto collect = [&](int i, uint32_t key) {
                const bool in = i < m && key >= reach;
                const uint64_t b = __ballot(in);
                const uint32_t pos = count + (uint32_t)__popcll(b & (((uint64_t)1 << lane) - 1));
                if (in && pos < 128u) { c_key[pos] = key; c_col[pos] = i; }
                count += (uint32_t)__popcll(b);
            };
#pragma unroll
            for (int e = 0; e < NV; ++e)
                if (e * 64 < m) collect(e * 64 + lane, keys[e]);
            for (int i0 = NV * 64; i0 < m && count <= 128u; i0 += 64 * kSelSmallU) {
                float v[kSelSmallU];
#pragma unroll
                for (int u = 0; u < kSelSmallU; ++u) { const int i = i0 + 64 * u + lane; v[u] = vals[i < m ? i : m - 1]; }
#pragma unroll
                for (int u = 0; u < kSelSmallU; ++u)
                    if (i0 + 64 * u < m) collect(i0 + 64 * u + lane, key_of(v[u]));
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if (count <= 128u) {
                const int n_c = (int)count;
                const bool has0 = lane < n_c, has1 = lane + 64 < n_c;
                const uint32_t k0 = has0 ? c_key[lane] : 0u, k1 = has1 ? c_key[lane + 64] : 0u;
                const int c0 = has0 ? c_col[lane] : 0, c1 = has1 ? c_col[lane + 64] : 0;
                int r0 = 0, r1 = 0;
                for (int jj = 0; jj < n_c; ++jj) {
                    const uint32_t kj = c_key[jj];
                    const int cj = c_col[jj];
                    r0 += (kj > k0 || (kj == k0 && cj < c0)) ? 1 : 0;
                    r1 += (kj > k1 || (kj == k1 && cj < c1)) ? 1 : 0;
                }
                if (has0 && r0 < take) win_col[r0] = c0;
                if (has1 && r1 < take) win_col[r1] = c1;
                done = true;
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();         // the words of `hist` are free again
        }
    }
    if (!done) {
    // radix search for the take-th largest key
    uint32_t prefix = 0, mask = 0, need = (uint32_t)take;
    // Leading bytes that every key of the row shares (scores of one query usually share sign and exponent)
    // need no pass: their histogram would be one bin that all lanes hit at once.
    int top_shift = 24;
    if (take > 0) {
        const uint32_t first = __builtin_amdgcn_readfirstlane(keys[0]);
        uint32_t diff = 0u;
#pragma unroll
        for (int e = 0; e < NV; ++e) diff |= (e * 64 + lane < m) ? (keys[e] ^ first) : 0u;
        for (int i0 = NV * 64; i0 < m; i0 += 64 * kSelSmallU) {                               // columns beyond the registers,
            float v[kSelSmallU];                                                               // kSelSmallU loads in flight together
#pragma unroll
            for (int u = 0; u < kSelSmallU; ++u) { const int i = i0 + 64 * u + lane; v[u] = vals[i < m ? i : m - 1]; }
#pragma unroll
            for (int u = 0; u < kSelSmallU; ++u) diff |= key_of(v[u]) ^ first;                  // a clamped column repeats the last one
        }
        if (__ballot((diff >> 24) != 0u) == 0ull) {
            prefix = first & 0xFF000000u; mask = 0xFF000000u; top_shift = 16;
            if (__ballot((diff >> 16) != 0u) == 0ull) { prefix = first & 0xFFFF0000u; mask = 0xFFFF0000u; top_shift = 8; }
        }
    }
    if (take > 0) {
        for (int shift = top_shift; shift >= 0; shift -= 8) {
#pragma unroll
            for (int e = 0; e < 4; ++e) hist[lane * 4 + e] = 0u;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int e = 0; e < NV; ++e)
                if (e * 64 + lane < m && (keys[e] & mask) == prefix) atomicAdd(&hist[(keys[e] >> shift) & 255u], 1u);
            for (int i0 = NV * 64; i0 < m; i0 += 64 * kSelSmallU) {
                float v[kSelSmallU];
#pragma unroll
                for (int u = 0; u < kSelSmallU; ++u) { const int i = i0 + 64 * u + lane; v[u] = vals[i < m ? i : m - 1]; }
#pragma unroll
                for (int u = 0; u < kSelSmallU; ++u) {
                    const uint32_t key = key_of(v[u]);
                    if (i0 + 64 * u + lane < m && (key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            // lane l owns digits 4l .. 4l+3; above = how many keys have a digit beyond this lane's
            uint32_t h[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) h[e] = hist[lane * 4 + e];
            const uint32_t own = h[0] + h[1] + h[2] + h[3];
            uint32_t incl = own;                                     // inclusive suffix sum over lanes
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t t = __shfl_down(incl, o);
                if (lane + o < 64) incl += t;
            }
            uint32_t above = incl - own;
            // the digit where the running count first reaches `need`, scanning digits downwards
            int found = -1;
            uint32_t before = 0;
#pragma unroll
            for (int e = 3; e >= 0; --e) {
                if (found < 0 && above < need && above + h[e] >= need) { found = lane * 4 + e; before = above; }
                above += h[e];
            }
            const uint64_t who = __ballot(found >= 0);               // exactly one lane while need >= 1
            const int src = who ? (int)__builtin_ctzll(who) : 0;
            const int dgt = __shfl(found, src);
            before = __shfl(before, src);
            need -= before;
            prefix |= (uint32_t)dgt << shift;
            mask |= 255u << shift;
        }
    }
    // keys above the threshold, then `need` keys equal to it in column order
    const uint32_t n_above = (uint32_t)take - need;
    uint32_t base_gt = 0, base_eq = 0;
    auto place = [&](int i, uint32_t key) {
        const bool gt = i < m && key > prefix;
        const bool eq = i < m && key == prefix;
        const uint64_t bg = __ballot(gt), be = __ballot(eq);
        const uint64_t below = ((uint64_t)1 << lane) - 1;
        if (gt) win_col[base_gt + (uint32_t)__popcll(bg & below)] = i;
        const uint32_t rank_eq = base_eq + (uint32_t)__popcll(be & below);
        if (eq && rank_eq < need) win_col[n_above + rank_eq] = i;
        base_gt += (uint32_t)__popcll(bg);
        base_eq += (uint32_t)__popcll(be);
    };
    if (take > 0) {
#pragma unroll
        for (int e = 0; e < NV; ++e)
            if (e * 64 < m) place(e * 64 + lane, keys[e]);
        for (int i0 = NV * 64; i0 < m; i0 += 64 * kSelSmallU) {
            float v[kSelSmallU];
#pragma unroll
            for (int u = 0; u < kSelSmallU; ++u) { const int i = i0 + 64 * u + lane; v[u] = vals[i < m ? i : m - 1]; }
#pragma unroll
            for (int u = 0; u < kSelSmallU; ++u)
                if (i0 + 64 * u < m) place(i0 + 64 * u + lane, key_of(v[u]));
        }
    }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const int out_c = lane < take ? win_col[lane] : -1;
    float out_v = out_c >= 0 ? vals[out_c] : ninf;

    // labels, then order equal values by label
    int64_t lab = INT64_MAX;
    if (out_c >= 0) {
        if (MODE == 0) {
            lab = out_c;
        } else if (MODE == 2) {
            const int64_t slot = a.list_off[a.probe[q * a.np + sub_p]] + out_c;
            lab = a.ids ? a.ids[slot] : slot;
        } else if (MODE == 3) {
            lab = a.lab_in[row * a.m_fixed + out_c];
        } else {
            lab = 0;      // placeholder, resolved below by the whole wavefront
        }
    }
    if (MODE == 1) {
        // probe rank of each winner: the last p with cand_off[p] <= column.  Up to 256 probes the row of
        // offsets is staged in the wavefront's LDS words (the histogram is no longer needed) and every
        // winner bisects there; beyond that the offsets are handed round with shuffles, 64 at a time.
        const int32_t* off = a.cand_off + q * (a.np + 1);
        int rank = 0, rank_off = 0;
        if (a.np <= 256) {
            int32_t* s_off = reinterpret_cast<int32_t*>(hist);
            for (int p = lane; p < a.np; p += 64) s_off[p] = off[p];
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            int lo = 0, hi = a.np;               // off[0] = 0 <= column
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (s_off[mid] <= out_c) lo = mid; else hi = mid;
            }
            rank = lo;
            rank_off = s_off[lo];
        } else {
            for (int base = 0; base < a.np; base += 64) {
                const int p = base + lane;
                const int32_t mine_off = p < a.np ? off[p] : INT32_MAX;
                const int span = a.np - base < 64 ? a.np - base : 64;
                for (int t = 0; t < span; ++t) {
                    const int32_t o = __shfl(mine_off, t);
                    if (o <= out_c) { rank = base + t; rank_off = o; }
                }
            }
        }
        if (out_c >= 0) {
            const int64_t slot = a.list_off[a.probe[q * a.np + rank]] + (out_c - rank_off);
            lab = a.ids ? a.ids[slot] : slot;
        }
    }
    // order the winners by (value desc, label asc): a bitonic network over the first nsort >= take lanes
    // (the others hold nothing); the value travels as its key and is decoded at the end
    uint32_t key = out_c >= 0 ? key_of(out_v) : 0u;
    if (MODE == 3 && lab < 0) key = 0u;              // a survivor slot that the first step left empty
    const int nsort = take <= 8 ? 8 : take <= 16 ? 16 : take <= 32 ? 32 : 64;
#pragma unroll
    for (int size = 2; size <= 64; size <<= 1) {
        if (size > nsort) break;
#pragma unroll
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            const uint32_t ok = __shfl_xor(key, stride);
            const int64_t ol = __shfl_xor(lab, stride);
            const bool lower = (lane & stride) == 0;     // this lane holds the earlier position of the pair
            const bool up = (lane & size) == 0;          // block sorted into final order (best first)
            const bool mine_first = (key > ok) || (key == ok && lab <= ol);
            const bool keep = (lower == up) ? mine_first : !mine_first;
            if (!keep) { key = ok; lab = ol; }
        }
    }
    out_v = __uint_as_float((key & 0x80000000u) ? (key ^ 0x80000000u) : ~key);     // inverse of order_key
    if (lane < k) {
        const bool real = key != 0u;
        if (a.out_vals) a.out_vals[row * k + lane] = real ? out_v : ninf;
        if (MODE == 0) { if (a.out_i32) a.out_i32[row * k + lane] = real ? (int32_t)lab : -1; }
        else { if (a.out_i64) a.out_i64[row * k + lane] = real ? lab : -1; }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();   // the wavefront's LDS words are free for its next row
    }
}

// ---- re-ranking on raw vectors (Section "Architecture", Search: optional) -----------------------
//
// One workgroup per query: each wavefront takes candidates in turn and computes <q, x> / (|q| |x|)
// from the raw rows, then the workgroup sorts (score desc, label asc) in LDS and emits the k best,
// dropping repeated labels.
__global__ __launch_bounds__(256) void k_rerank(RerankArgs a) {
    extern __shared__ unsigned char smem[];
    int size = 1;
    while (size < a.r) size <<= 1;
    uint32_t* s_key = reinterpret_cast<uint32_t*>(smem);
    float* s_val = reinterpret_cast<float*>(s_key + size);
    int64_t* s_lab = reinterpret_cast<int64_t*>(s_val + size);
    const int64_t q = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* qv = a.q + q * a.d;
    float qr[4];
    float qq = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int j = lane + 64 * e;
        qr[e] = j < a.d ? qv[j] : 0.f;
        qq += qr[e] * qr[e];
    }
    for (int o = 32; o > 0; o >>= 1) qq += __shfl_xor(qq, o);
    for (int c = wave; c < size; c += 4) {
        const int64_t id = c < a.r ? a.cand[q * a.r + c] : -1;
        float xy = 0.f, xx = 0.f;
        if (id >= 0 && id < a.n_rows) {
            const float* xv = a.x + id * a.d;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = lane + 64 * e;
                const float v = j < a.d ? xv[j] : 0.f;
                xy += v * qr[e];
                xx += v * v;
            }
        }
        for (int o = 32; o > 0; o >>= 1) { xy += __shfl_xor(xy, o); xx += __shfl_xor(xx, o); }
        if (lane == 0) {
            const bool ok = id >= 0 && id < a.n_rows && xx > 0.f && qq > 0.f;
            const float sc = ok ? xy / sqrtf(xx * qq) : -__builtin_inff();
            s_key[c] = (ok && sc == sc) ? order_key(sc) : 0u;
            s_val[c] = sc;
            s_lab[c] = ok ? id : INT64_MAX;
        }
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
                    const float v0 = s_val[lo_i]; s_val[lo_i] = s_val[hi_i]; s_val[hi_i] = v0;
                }
            }
            __syncthreads();
        }
    }
    if (tid == 0) {
        int out = 0;
        int64_t prev = INT64_MAX;
        for (int i = 0; i < size && out < a.k; ++i) {
            if (s_key[i] == 0u) break;
            if (s_lab[i] == prev) continue;                  // the same label again: equal score, adjacent
            prev = s_lab[i];
            a.out_scores[q * a.k + out] = s_val[i];
            a.out_ids[q * a.k + out] = s_lab[i];
            ++out;
        }
        for (; out < a.k; ++out) { a.out_scores[q * a.k + out] = -__builtin_inff(); a.out_ids[q * a.k + out] = -1; }
    }
}

// ---- cascade search, pass 2 (Appendix "Cascade search via Lloyd-Max bin ordinality") ------------
//
// One workgroup per query.  Each wavefront takes kept candidates in turn: finds the probed list that
// holds the slot (lanes over the query's probes), then lane j sums the coordinates j, j+64, ... from
// the packed words; the workgroup sorts (score desc, label asc) in LDS and emits the k best.
__global__ __launch_bounds__(256) void k_cascade_rescore(CascadeArgs a) {
    extern __shared__ unsigned char smem[];
    int size = 1;
    while (size < a.n_keep) size <<= 1;
    uint32_t* s_key = reinterpret_cast<uint32_t*>(smem);
    float* s_val = reinterpret_cast<float*>(s_key + size);
    int64_t* s_lab = reinterpret_cast<int64_t*>(s_val + size);
    const int64_t q = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t mask = (1u << a.b) - 1u;
    float zr[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int j = lane + 64 * e;
        zr[e] = j < a.d ? a.z[q * a.z_pitch + j] : 0.f;
    }
    for (int c = wave; c < size; c += 4) {
        const int64_t slot = c < a.n_keep ? a.cand[q * a.n_keep + c] : -1;
        int p_found = -1;
        if (slot >= 0) {
            for (int base = 0; base < a.np && p_found < 0; base += 64) {
                const int p = base + lane;
                bool hit = false;
                if (p < a.np) {
                    const int l = a.probe[q * a.np + p];
                    const int64_t off = a.store.list_off[l];
                    hit = slot >= off && slot < off + a.store.list_size[l];
                }
                const unsigned long long m = __ballot(hit);
                if (m) p_found = base + __ffsll((long long)m) - 1;
            }
        }
        float acc = 0.f;
        if (p_found >= 0) {
            const uint32_t* wp = a.store.codes + (slot >> 6) * a.store.words * 64 + (slot & 63);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = lane + 64 * e;
                if (j < a.d) {
                    const int bit = j * a.b, w = bit >> 5, o = bit & 31;
                    uint32_t v = wp[(int64_t)w * 64] >> o;
                    if (o + a.b > 32) v |= wp[(int64_t)(w + 1) * 64] << (32 - o);
                    acc += zr[e] * a.cb[v & mask];
                }
            }
        }
        for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
        if (lane == 0) {
            const bool ok = p_found >= 0;
            float sc = -__builtin_inff();
            if (ok) sc = a.coarse[q * a.np + p_found] + __half2float(__ushort_as_half(a.store.gamma[slot])) * acc;
            s_key[c] = (ok && sc == sc) ? order_key(sc) : 0u;
            s_val[c] = sc;
            s_lab[c] = ok ? a.ids[slot] : INT64_MAX;
        }
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
                    const float v0 = s_val[lo_i]; s_val[lo_i] = s_val[hi_i]; s_val[hi_i] = v0;
                }
            }
            __syncthreads();
        }
    }
    for (int i = tid; i < a.k; i += 256) {
        const bool real = i < size && s_key[i] != 0u;
        a.out_scores[q * a.k + i] = real ? s_val[i] : -__builtin_inff();
        a.out_ids[q * a.k + i] = real ? s_lab[i] : -1;
    }
}

}  // namespace

hipError_t launch_cascade_rescore(const CascadeArgs& a, int64_t nq, hipStream_t st) {
    if (nq <= 0) return hipSuccess;
    int size = 1;
    while (size < a.n_keep) size <<= 1;
    const size_t lds = (size_t)size * 16;
    hipLaunchKernelGGL(k_cascade_rescore, dim3((unsigned)nq), dim3(256), lds, st, a);
    return hipGetLastError();
}

hipError_t launch_rerank(const RerankArgs& a, int64_t nq, hipStream_t st) {
    if (nq <= 0) return hipSuccess;
    int size = 1;
    while (size < a.r) size <<= 1;
    const size_t lds = (size_t)size * 16;
    hipLaunchKernelGGL(k_rerank, dim3((unsigned)nq), dim3(256), lds, st, a);
    return hipGetLastError();
}

hipError_t launch_cand_offsets(const int32_t* probe, int64_t nq, int np, const int32_t* list_size,
                               int32_t* cand_off, int k, int cap, int32_t* first, int32_t* cand_cnt, int32_t* gate,
                               hipStream_t st) {
    if (nq <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_cand_offsets, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, st, probe, nq, np,
                       list_size, cand_off, k, cap, first, cand_cnt, gate);
    return hipGetLastError();
}

hipError_t launch_list_scan(const float* z, int z_pitch, int d, int b, const float* cb,
                            const int32_t* probe, const float* coarse, const int32_t* cand_off,
                            int np, const ListStore& store, int64_t q_begin, int64_t q_count,
                            float* scores, int64_t m_stride, const int32_t* p_limit, const int32_t* gate,
                            int gate_begin, int gate_rows, int blocks_per_query, int slices, int metric, const float* qnorm,
                            hipStream_t st) {
    if (q_count <= 0) return hipSuccess;
    if (metric && (!qnorm || !store.xnorm)) return hipErrorInvalidValue;
    const size_t lut_bytes = (size_t)d * (1u << b) * sizeof(float);
    const bool direct = lut_bytes > 64 * 1024;
    const size_t lds = direct ? (size_t)(d + (1 << b)) * sizeof(float) : lut_bytes;
    // gated: a fixed number of workgroup rows walks the list of marked queries
    dim3 grid((unsigned)(blocks_per_query > 0 ? blocks_per_query : np), (unsigned)(gate ? std::min<int64_t>(std::min<int64_t>(q_count, gate_rows), 256) : q_count));
    // slices: every list is dealt out in rounds of 256 vectors to that many workgroups (grid z, the slowest
    // dimension of the dispatch order: the launch works through the index one slice at a time)
    if (!gate) grid.z = (unsigned)std::max(1, std::min(slices, 64));
#define IVFTQ_SCAN(BV)                                                                              \
    case BV:                                                                                        \
        if (direct)                                                                                 \
            hipLaunchKernelGGL((k_list_scan<BV, true>), grid, dim3(256), lds, st, z, z_pitch, d, cb, probe, \
                               coarse, cand_off, np, store, q_begin, scores, m_stride, p_limit, gate, gate_begin, gate_rows, metric, qnorm); \
        else                                                                                        \
            hipLaunchKernelGGL((k_list_scan<BV, false>), grid, dim3(256), lds, st, z, z_pitch, d, cb, probe, \
                               coarse, cand_off, np, store, q_begin, scores, m_stride, p_limit, gate, gate_begin, gate_rows, metric, qnorm); \
        break;
    switch (b) {
        IVFTQ_SCAN(1) IVFTQ_SCAN(2) IVFTQ_SCAN(3) IVFTQ_SCAN(4)
        IVFTQ_SCAN(5) IVFTQ_SCAN(6) IVFTQ_SCAN(7) IVFTQ_SCAN(8)
        default: return hipErrorInvalidValue;
    }
#undef IVFTQ_SCAN
    return hipGetLastError();
}

hipError_t launch_metric_finish(float* scores, int64_t nq, int k, int metric, const float* qnorm, hipStream_t st) {
    if (nq <= 0 || metric == 0) return hipSuccess;
    hipLaunchKernelGGL(k_metric_finish, dim3((unsigned)((nq * k + 255) / 256)), dim3(256), 0, st, scores, nq, k, metric, qnorm);
    return hipGetLastError();
}

// Longest row the one-wavefront-per-row kernel takes.  Probe selection (mode 0, every row has m_fixed values):
// its short cuts (up to 64 winners) beat the workgroup-per-row kernel well beyond the columns it holds in
// registers (10,000 rows over 4096 cells: 0.069 ms for 32 winners, against 0.145 ms); result rows (mode 1)
// are mostly much shorter than their bound.
constexpr int kSmallMax0Shortcut = 8192, kSmallMax1 = kSmallM;
hipError_t launch_select(int mode, const SelectArgs& a_in, hipStream_t st) {
    if (a_in.rows <= 0) return hipSuccess;
    SelectArgs a = a_in;
    if (mode == 2 || mode == 3) {
        if (a.k > 64 || a.gate || (mode == 3 && !a.lab_in)) return hipErrorInvalidValue;
        const int bound = mode == 2 ? a.m_bound : a.m_fixed;
        const unsigned blocks = (unsigned)((a.rows + 3) / 4);
        if (mode == 2) {
            if (bound <= 1536) hipLaunchKernelGGL((k_select_small<2, 16>), dim3(blocks), dim3(256), 0, st, a);
            else hipLaunchKernelGGL((k_select_small<2, 32>), dim3(blocks), dim3(256), 0, st, a);
        } else {
            if (bound <= 1536) hipLaunchKernelGGL((k_select_small<3, 16>), dim3(blocks), dim3(256), 0, st, a);
            else hipLaunchKernelGGL((k_select_small<3, 32>), dim3(blocks), dim3(256), 0, st, a);
        }
        return hipGetLastError();
    }
    // short rows and small k: the one-wavefront-per-row kernel
    const int m_bound = mode == 0 ? a.m_fixed : a.m_bound;
    if (a.k <= 64 && m_bound > 0 && m_bound <= (mode == 0 ? kSmallMax0Shortcut : kSmallMax1)) {
        const size_t lds = 0;
        const unsigned blocks = (unsigned)((a.gate ? std::min<int64_t>(std::min<int64_t>(a.rows, a.gate_rows), 1024) : a.rows) + 3) / 4;
#define IVFTQ_SMALL(NVV)                                                                            \
        if (mode == 0 && a.k > kShortcutTake) hipLaunchKernelGGL((k_select_small<0, NVV, true>), dim3(blocks), dim3(256), lds, st, a);  \
        else if (mode == 0) hipLaunchKernelGGL((k_select_small<0, NVV>), dim3(blocks), dim3(256), lds, st, a);  \
        else if (a.k > kShortcutTake) hipLaunchKernelGGL((k_select_small<1, NVV, true>), dim3(blocks), dim3(256), lds, st, a);  \
        else hipLaunchKernelGGL((k_select_small<1, NVV>), dim3(blocks), dim3(256), lds, st, a);
        if (m_bound <= 1536 || mode == 1) { IVFTQ_SMALL(16) } else { IVFTQ_SMALL(32) }
#undef IVFTQ_SMALL
        return hipGetLastError();
    }
    int kpad = 1;
    while (kpad < a.k) kpad <<= 1;
    const int copies = (m_bound == 0 || m_bound > 8192) ? 8 : 1;
    const size_t lds = (256 * copies + 8 + 4) * 4 + (size_t)kpad * 8 + 8 + (size_t)kpad * 8 + (size_t)kSelCand * 8;
    const unsigned wgs = (unsigned)(a.gate ? std::min<int64_t>(std::min<int64_t>(a.rows, a.gate_rows), 256) : a.rows);
    if (copies == 8) {
        if (mode == 0) hipLaunchKernelGGL((k_select<0, 8>), dim3(wgs), dim3(256), lds, st, a);
        else hipLaunchKernelGGL((k_select<1, 8>), dim3(wgs), dim3(256), lds, st, a);
    } else {
        if (mode == 0) hipLaunchKernelGGL((k_select<0, 1>), dim3(wgs), dim3(256), lds, st, a);
        else hipLaunchKernelGGL((k_select<1, 1>), dim3(wgs), dim3(256), lds, st, a);
    }
    return hipGetLastError();
}

}  // namespace ivftq
