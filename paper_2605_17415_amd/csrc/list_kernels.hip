// Inverted-list bookkeeping for appends (Section "Architecture": "new vectors enter at any
// time"; Section "Streaming Experiments": append-only ingest with constant coarse parameters) and
// the centroid-update half of coarse k-means (Section "Architecture", Indexing).
//
// An append must place row i of the batch at position (old size of its list) + (number of earlier
// batch rows of the same list), so that list order equals arrival order and results never depend
// on scheduling.  That is a stable counting sort by cell number, done in three small kernels:
// per-segment histograms, a column-wise running sum over segments, and an in-order rank inside
// each segment by one wavefront.
#include <hip/hip_fp16.h>

#include "kernels.h"

namespace ivftq {

namespace {

__global__ __launch_bounds__(256) void k_segment_hist(const int32_t* __restrict__ assign, int64_t n,
                                                      int64_t seg_len, int L, uint32_t* __restrict__ seg_hist) {
    extern __shared__ uint32_t hist[];
    for (int l = threadIdx.x; l < L; l += 256) hist[l] = 0;
    __syncthreads();
    const int64_t begin = (int64_t)blockIdx.x * seg_len;
    const int64_t end = begin + seg_len < n ? begin + seg_len : n;
    for (int64_t i = begin + threadIdx.x; i < end; i += 256) {
        const int a = assign[i];
        if (a >= 0 && a < L) atomicAdd(&hist[a], 1u);
    }
    __syncthreads();
    for (int l = threadIdx.x; l < L; l += 256) seg_hist[(int64_t)blockIdx.x * L + l] = hist[l];
}

// Column-wise exclusive running sum over segments.  A workgroup takes 16 lists; its 1024 threads split the
// segments into 64 parts (a sixteen-lane group per part), so each of the two passes over a column is 64 wide
// and a launch has L/16 workgroups.
__global__ __launch_bounds__(1024) void k_segment_scan(uint32_t* __restrict__ seg_hist, int nseg, int L,
                                                       uint32_t* __restrict__ batch_count) {
    __shared__ uint32_t part_sum[64][16];
    const int li = threadIdx.x & 15, part = threadIdx.x >> 4;
    const int l = blockIdx.x * 16 + li;
    const int chunk = (nseg + 63) / 64;
    const int s0 = part * chunk < nseg ? part * chunk : nseg;
    const int s1 = (s0 + chunk < nseg) ? s0 + chunk : nseg;
    uint32_t sum = 0;
    if (l < L)
        for (int s = s0; s < s1; ++s) sum += seg_hist[(int64_t)s * L + l];
    part_sum[part][li] = sum;
    __syncthreads();
    uint32_t run = 0;
    for (int p = 0; p < part; ++p) run += part_sum[p][li];
    if (l < L) {
        for (int s = s0; s < s1; ++s) {
            const uint32_t t = seg_hist[(int64_t)s * L + l];
            seg_hist[(int64_t)s * L + l] = run;
            run += t;
        }
        if (part == 63) batch_count[l] = run;
    }
}

// One wavefront walks its segment 64 rows at a time, in order.
__global__ __launch_bounds__(64) void k_stable_rank(const int32_t* __restrict__ assign, int64_t n,
                                                    int64_t seg_len, int L,
                                                    const uint32_t* __restrict__ seg_hist,
                                                    const int64_t* __restrict__ list_base,
                                                    int64_t* __restrict__ slot,
                                                    const int64_t* __restrict__ batch_base,
                                                    int32_t* __restrict__ order, int2* __restrict__ order_cell) {
    extern __shared__ uint32_t cnt[];
    const int lane = threadIdx.x;
    for (int l = lane; l < L; l += 64) cnt[l] = seg_hist[(int64_t)blockIdx.x * L + l];
    __syncthreads();
    const int64_t begin = (int64_t)blockIdx.x * seg_len;
    const int64_t end = begin + seg_len < n ? begin + seg_len : n;
    const int nbits = 32 - __builtin_clz((unsigned)L);                      // bits of the numbers 0 .. L
    for (int64_t g = begin; g < end; g += 64) {
        const int64_t i = g + lane;
        int key = (i < end) ? assign[i] : -1;
        if (key >= L) key = -1;
        // lanes holding the same cell number: one ballot per bit of the number narrows the set (rows without a
        // cell carry the number L, which no other row has)
        const uint32_t kbits = (uint32_t)(key >= 0 ? key : L);
        uint64_t same = ~0ull;
        for (int bit = 0; bit < nbits; ++bit) {
            const bool set = (kbits >> bit) & 1u;
            const uint64_t bal = __ballot(set);
            same &= set ? bal : ~bal;
        }
        const int lower = __popcll(same & ((1ull << lane) - 1ull));        // earlier rows of this group in the same cell
        const bool later = (same >> lane) > 1ull;                          // a later row of the group is in it too
        uint32_t base = 0;
        if (key >= 0) {
            base = cnt[key];
            if (slot) slot[i] = list_base[key] + (int64_t)(base + lower);
            if (order) order[batch_base[key] + (int64_t)(base + lower)] = (int32_t)i;
            if (order_cell) order_cell[batch_base[key] + (int64_t)(base + lower)] = make_int2((int)i, key);
        } else if (i < end && slot) {
            slot[i] = -1;
        }
        __syncthreads();
        if (key >= 0 && !later) cnt[key] = base + lower + 1;
        __syncthreads();
    }
}

__global__ __launch_bounds__(256) void k_copy_lists(ListStore from, ListStore to) {
    const int l = blockIdx.x;
    const int64_t size = from.list_size[l];
    if (size == 0) return;
    const int64_t src = from.list_off[l], dst = to.list_off[l];
    const int words = from.words;
    const int64_t nblk = (size + 63) / 64;
    const int64_t total_words = nblk * words * 64;
    const uint32_t* s = from.codes + (src >> 6) * words * 64;
    uint32_t* t = to.codes + (dst >> 6) * words * 64;
    for (int64_t e = (int64_t)blockIdx.y * 256 + threadIdx.x; e < total_words; e += (int64_t)gridDim.y * 256)
        t[e] = s[e];
    if (to.head && from.head) {
        const int64_t head_total = nblk * from.head_words * 64;
        const uint32_t* hs = from.head + (src >> 6) * from.head_words * 64;
        uint32_t* ht = to.head + (dst >> 6) * from.head_words * 64;
        for (int64_t e = (int64_t)blockIdx.y * 256 + threadIdx.x; e < head_total; e += (int64_t)gridDim.y * 256)
            ht[e] = hs[e];
    }
    for (int64_t e = (int64_t)blockIdx.y * 256 + threadIdx.x; e < size; e += (int64_t)gridDim.y * 256) {
        to.gamma[dst + e] = from.gamma[src + e];
        to.ids[dst + e] = from.ids[src + e];
        if (to.xnorm) to.xnorm[dst + e] = from.xnorm ? from.xnorm[src + e] : 0.f;
    }
}

__global__ __launch_bounds__(256) void k_pack_scatter(const uint8_t* __restrict__ codes,
                                                      const uint16_t* __restrict__ gamma,
                                                      const float* __restrict__ xnorm,
                                                      const int64_t* __restrict__ labels, int64_t label_base,
                                                      const int64_t* __restrict__ slot, int64_t n, int d,
                                                      int b, ListStore store) {
    const int words = store.words;
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= n * words) return;
    const int64_t row = item / words;
    const int w = (int)(item % words);
    const int64_t s = slot[row];
    if (s < 0) return;
    const uint8_t* c = codes + row * d;
    uint32_t word = 0;
    for (int j = (32 * w) / b; j < d; ++j) {        // coordinate j occupies bits [j*b, j*b + b)
        const int sh = j * b - 32 * w;
        if (sh >= 32) break;
        const uint32_t code = c[j];
        word |= sh >= 0 ? (code << sh) : (code >> (-sh));
    }
    store.codes[((s >> 6) * words + w) * 64 + (s & 63)] = word;
    if (store.head && w < store.head_words) {      // word w of the top-bit plane: coordinate j at bits [j*beta, j*beta + beta)
        const int beta = b - store.head_shift;
        uint32_t hword = 0;
        for (int j = (32 * w) / beta; j < d; ++j) {
            const int sh = j * beta - 32 * w;
            if (sh >= 32) break;
            const uint32_t code = (uint32_t)c[j] >> store.head_shift;
            hword |= sh >= 0 ? (code << sh) : (code >> (-sh));
        }
        store.head[((s >> 6) * store.head_words + w) * 64 + (s & 63)] = hword;
    }
    if (w == 0) {
        store.gamma[s] = gamma[row];
        store.ids[s] = labels ? labels[row] : label_base + row;
        if (store.xnorm) store.xnorm[s] = xnorm ? xnorm[row] : 0.f;
    }
}

__global__ void k_fill_u32(uint32_t* p, int64_t n, uint32_t v) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = v;
}

// ---- k-means ------------------------------------------------------------------------------------

// out[l] = sum of count[l'] over l' < l, for up to 16384 entries, by one workgroup.
__global__ __launch_bounds__(1024) void k_exclusive_scan(const uint32_t* __restrict__ count, int L,
                                                         int64_t* __restrict__ out) {
    __shared__ int64_t part[1024];
    const int per = (L + 1023) / 1024;
    const int lo = threadIdx.x * per < L ? threadIdx.x * per : L;
    const int hi = lo + per < L ? lo + per : L;
    int64_t sum = 0;
    for (int l = lo; l < hi; ++l) sum += count[l];
    part[threadIdx.x] = sum;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {            // inclusive running sum over the 1024 parts
        const int64_t add = threadIdx.x >= o ? part[threadIdx.x - o] : 0;
        __syncthreads();
        part[threadIdx.x] += add;
        __syncthreads();
    }
    int64_t run = part[threadIdx.x] - sum;
    for (int l = lo; l < hi; ++l) { out[l] = run; run += count[l]; }
}

// Sum of the normalised rows of each cell, in a fixed order: workgroup l walks the rows
// order[base[l] .. base[l] + count[l]) of its cell, wavefront w taking every fourth row from the w-th on,
// a lane the coordinates lane, lane + 64, ...; the four partial sums are then added in the order 0, 1, 2, 3.
// Nothing depends on scheduling, so the same input gives the same bits on every run.
__global__ __launch_bounds__(256) void k_kmeans_cell_sums(const float* __restrict__ x, int d,
                                                          const int32_t* __restrict__ order,
                                                          const int64_t* __restrict__ base,
                                                          const uint32_t* __restrict__ count,
                                                          float* __restrict__ sums, int pitch) {
    __shared__ float part[4][kMaxD];
    const int l = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t first = base[l];
    const int cnt = (int)count[l];
    float acc[kMaxD / 64];
#pragma unroll
    for (int t = 0; t < kMaxD / 64; ++t) acc[t] = 0.f;
    for (int p = wave; p < cnt; p += 4) {
        const float* row = x + (int64_t)order[first + p] * d;
        float v[kMaxD / 64];
        float n2 = 0.f;
#pragma unroll
        for (int t = 0; t < kMaxD / 64; ++t) {
            const int j = lane + 64 * t;
            v[t] = j < d ? row[j] : 0.f;
            n2 += v[t] * v[t];
        }
        for (int o = 32; o > 0; o >>= 1) n2 += __shfl_xor(n2, o);
        const float nrm = sqrtf(n2);
#pragma unroll
        for (int t = 0; t < kMaxD / 64; ++t) acc[t] += v[t] / nrm;
    }
#pragma unroll
    for (int t = 0; t < kMaxD / 64; ++t) part[wave][lane + 64 * t] = acc[t];
    __syncthreads();
    for (int j = threadIdx.x; j < d; j += 256)
        sums[(int64_t)l * pitch + j] = ((part[0][j] + part[1][j]) + part[2][j]) + part[3][j];
}

__global__ __launch_bounds__(64) void k_kmeans_update(float* __restrict__ cent, int pitch,
                                                      const float* __restrict__ sums,
                                                      const uint32_t* __restrict__ counts,
                                                      float* __restrict__ bias, int L, int d) {
    const int l = blockIdx.x, lane = threadIdx.x;
    if (l >= L) { if (lane == 0) bias[l] = -__builtin_inff(); return; }
    const uint32_t c = counts[l];
    float n2 = 0.f;
    for (int j = lane; j < d; j += 64) {
        float v = cent[(int64_t)l * pitch + j];
        if (c > 0) { v = sums[(int64_t)l * pitch + j] / (float)c; cent[(int64_t)l * pitch + j] = v; }
        n2 += v * v;
    }
    for (int o = 32; o > 0; o >>= 1) n2 += __shfl_xor(n2, o);
    if (lane == 0) bias[l] = -0.5f * n2;
}

__global__ __launch_bounds__(64) void k_copy_rows_normalised(const float* __restrict__ x, int d,
                                                             const int64_t* __restrict__ src_row,
                                                             const int32_t* __restrict__ dst,
                                                             float* __restrict__ cent, int pitch) {
    const int lane = threadIdx.x;
    const int64_t row = src_row[blockIdx.x];
    const int l = dst[blockIdx.x];
    float n2 = 0.f;
    for (int j = lane; j < d; j += 64) { const float v = x[row * d + j]; n2 += v * v; }
    for (int o = 32; o > 0; o >>= 1) n2 += __shfl_xor(n2, o);
    const float nrm = sqrtf(n2);
    for (int j = lane; j < d; j += 64) cent[(int64_t)l * pitch + j] = nrm > 0.f ? x[row * d + j] / nrm : 0.f;
}

// Reconstruction of stored vectors (Section "Adaptive coarse refresh", Refresh self-containedness):
// x^ = c~_l + gamma * Pi^T C[code].  A workgroup takes 32 consecutive vectors of one list: their
// de-quantised coordinates go to LDS as rho[k][v], then thread j accumulates output coordinate j of
// all 32 vectors, x^_j = sum_k Pi[k][j] rho_k (row k of Pi is read coalesced across the threads, the
// 32 values of rho[k][.] are LDS broadcasts), and rows are written whole.  Rows come out in list
// order: list l starts at row out_off[l]; labels_out gets the stored labels in the same order.
__global__ __launch_bounds__(256) void k_reconstruct(ListStore store, const float* __restrict__ cent, int cent_pitch,
                                                     const float* __restrict__ pi, int pi_pitch,
                                                     const float* __restrict__ cb, int d, int b,
                                                     const int64_t* __restrict__ out_off,
                                                     float* __restrict__ x_out, int64_t* __restrict__ labels_out) {
    extern __shared__ float rho[];                     // [d][32], then 32 norms
    float* gam = rho + (size_t)d * 32;
    const int l = blockIdx.y;
    const int n_l = store.list_size[l];
    const int v0 = blockIdx.x * 32;
    if (v0 >= n_l) return;
    const int tid = threadIdx.x;
    const int64_t base_slot = store.list_off[l];
    const int words = store.words;
    const uint32_t mask = (1u << b) - 1u;
    for (int e = tid; e < 32 * d; e += 256) {
        const int v = e & 31, k = e >> 5;
        float val = 0.f;
        if (v0 + v < n_l) {
            const int64_t slot = base_slot + v0 + v;
            const uint32_t* wp = store.codes + (slot >> 6) * (int64_t)words * 64 + (slot & 63);
            const int bit = k * b, w = bit >> 5, sh = bit & 31;
            uint32_t code = wp[(int64_t)w * 64] >> sh;
            if (sh + b > 32) code |= wp[(int64_t)(w + 1) * 64] << (32 - sh);
            val = cb[code & mask];
        }
        rho[k * 32 + v] = val;
    }
    if (tid < 32) {
        const bool in = v0 + tid < n_l;
        gam[tid] = in ? __half2float(__ushort_as_half(store.gamma[base_slot + v0 + tid])) : 0.f;
        if (in && labels_out) labels_out[out_off[l] + v0 + tid] = store.ids[base_slot + v0 + tid];
    }
    __syncthreads();
    const int j = tid;
    if (j >= d) return;
    float acc[32];
#pragma unroll
    for (int v = 0; v < 32; ++v) acc[v] = 0.f;
    for (int k = 0; k < d; ++k) {
        const float p = pi[(int64_t)k * pi_pitch + j];
        const float4* r4 = reinterpret_cast<const float4*>(rho + k * 32);
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            const float4 r = r4[g];
            acc[4 * g] = fmaf(p, r.x, acc[4 * g]); acc[4 * g + 1] = fmaf(p, r.y, acc[4 * g + 1]);
            acc[4 * g + 2] = fmaf(p, r.z, acc[4 * g + 2]); acc[4 * g + 3] = fmaf(p, r.w, acc[4 * g + 3]);
        }
    }
    const float c = cent[(int64_t)l * cent_pitch + j];
#pragma unroll
    for (int v = 0; v < 32; ++v)
        if (v0 + v < n_l) x_out[(out_off[l] + v0 + v) * (int64_t)d + j] = fmaf(gam[v], acc[v], c);
}

// dst[t] = src[idx[t]] for rows of d floats
__global__ __launch_bounds__(64) void k_gather_rows(const float* __restrict__ src, int d,
                                                    const int64_t* __restrict__ idx, float* __restrict__ dst) {
    const int64_t row = idx[blockIdx.x];
    for (int j = threadIdx.x; j < d; j += 64) dst[(int64_t)blockIdx.x * d + j] = src[row * d + j];
}

__global__ __launch_bounds__(64) void k_normalise_centroids(float* __restrict__ cent, int pitch,
                                                            float* __restrict__ bias, int d) {
    const int l = blockIdx.x, lane = threadIdx.x;
    float n2 = 0.f;
    for (int j = lane; j < d; j += 64) { const float v = cent[(int64_t)l * pitch + j]; n2 += v * v; }
    for (int o = 32; o > 0; o >>= 1) n2 += __shfl_xor(n2, o);
    const float nrm = sqrtf(n2);
    for (int j = lane; j < d; j += 64)
        if (nrm > 0.f) cent[(int64_t)l * pitch + j] /= nrm;
    if (lane == 0) bias[l] = 0.f;
}

// Deterministic: one workgroup, fixed summation order.
__global__ __launch_bounds__(256) void k_inertia(const float* __restrict__ best, int64_t n, double* out) {
    __shared__ double part[256];
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += 256) s += 1.0 - 2.0 * (double)best[i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if (threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = part[0];
}

}  // namespace

hipError_t launch_segment_hist(const int32_t* assign, int64_t n, int64_t seg_len, int nseg, int L,
                               uint32_t* seg_hist, hipStream_t st) {
    hipLaunchKernelGGL(k_segment_hist, dim3(nseg), dim3(256), (size_t)L * 4, st, assign, n, seg_len, L, seg_hist);
    return hipGetLastError();
}

hipError_t launch_segment_scan(uint32_t* seg_hist, int nseg, int L, uint32_t* batch_count, hipStream_t st) {
    hipLaunchKernelGGL(k_segment_scan, dim3((L + 15) / 16), dim3(1024), 0, st, seg_hist, nseg, L, batch_count);
    return hipGetLastError();
}

hipError_t launch_stable_rank(const int32_t* assign, int64_t n, int64_t seg_len, int nseg, int L,
                              const uint32_t* seg_hist, const int64_t* list_base, int64_t* slot,
                              const int64_t* batch_base, int32_t* order, int2* order_cell, hipStream_t st) {
    hipLaunchKernelGGL(k_stable_rank, dim3(nseg), dim3(64), (size_t)L * 4, st, assign, n, seg_len, L,
                       seg_hist, list_base, slot, batch_base, order, order_cell);
    return hipGetLastError();
}

hipError_t launch_copy_lists(const ListStore& from, const ListStore& to, int L, hipStream_t st) {
    hipLaunchKernelGGL(k_copy_lists, dim3(L, 8), dim3(256), 0, st, from, to);
    return hipGetLastError();
}

hipError_t launch_pack_scatter(const uint8_t* codes, const uint16_t* gamma, const float* xnorm, const int64_t* labels,
                               int64_t label_base, const int64_t* slot, int64_t n, int d, int b,
                               const ListStore& store, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    const int64_t items = n * store.words;
    hipLaunchKernelGGL(k_pack_scatter, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, codes, gamma, xnorm,
                       labels, label_base, slot, n, d, b, store);
    return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)blocks), dim3(256), 0, st, p, n, v);
    return hipGetLastError();
}

hipError_t launch_exclusive_scan(const uint32_t* count, int L, int64_t* out, hipStream_t st) {
    if (L < 1 || L > kMaxList) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_exclusive_scan, dim3(1), dim3(1024), 0, st, count, L, out);
    return hipGetLastError();
}

hipError_t launch_kmeans_cell_sums(const float* x, int d, const int32_t* order, const int64_t* base,
                                   const uint32_t* count, int L, float* sums, int pitch, hipStream_t st) {
    if (d > kMaxD) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_kmeans_cell_sums, dim3(L), dim3(256), 0, st, x, d, order, base, count, sums, pitch);
    return hipGetLastError();
}

hipError_t launch_kmeans_update(float* cent, int pitch, const float* sums, const uint32_t* counts,
                                float* bias, int L, int Lpad, int d, hipStream_t st) {
    hipLaunchKernelGGL(k_kmeans_update, dim3(Lpad), dim3(64), 0, st, cent, pitch, sums, counts, bias, L, d);
    return hipGetLastError();
}

hipError_t launch_copy_rows_normalised(const float* x, int d, const int64_t* src_row, const int32_t* dst,
                                       int count, float* cent, int pitch, hipStream_t st) {
    if (count <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_copy_rows_normalised, dim3(count), dim3(64), 0, st, x, d, src_row, dst, cent, pitch);
    return hipGetLastError();
}

hipError_t launch_reconstruct(const ListStore& store, int L, int max_list, const float* cent, int cent_pitch,
                              const float* pi, int pi_pitch, const float* cb, int d, int b, const int64_t* out_off,
                              float* x_out, int64_t* labels_out, hipStream_t st) {
    if (max_list <= 0) return hipSuccess;
    const size_t lds = ((size_t)d * 32 + 32) * sizeof(float);
    hipLaunchKernelGGL(k_reconstruct, dim3((unsigned)((max_list + 31) / 32), (unsigned)L), dim3(256), lds, st, store, cent,
                       cent_pitch, pi, pi_pitch, cb, d, b, out_off, x_out, labels_out);
    return hipGetLastError();
}

hipError_t launch_gather_rows(const float* src, int d, const int64_t* idx, int64_t count, float* dst, hipStream_t st) {
    if (count <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_gather_rows, dim3((unsigned)count), dim3(64), 0, st, src, d, idx, dst);
    return hipGetLastError();
}

hipError_t launch_normalise_centroids(float* cent, int pitch, float* bias, int L, int d, hipStream_t st) {
    hipLaunchKernelGGL(k_normalise_centroids, dim3(L), dim3(64), 0, st, cent, pitch, bias, d);
    return hipGetLastError();
}

hipError_t launch_inertia(const float* best, int64_t n, double* out, hipStream_t st) {
    hipLaunchKernelGGL(k_inertia, dim3(1), dim3(256), 0, st, best, n, out);
    return hipGetLastError();
}

}  // namespace ivftq
