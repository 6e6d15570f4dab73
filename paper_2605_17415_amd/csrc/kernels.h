// Internal launcher declarations shared by the HIP translation units of libivftq.
// Nothing here is part of the public ABI (see include/ivftq.h for that).
#pragma once
#include <cmath>
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>

namespace ivftq {

constexpr int kSlotsPerBlock = 64;   // vectors interleaved in one storage block (= one wavefront)
constexpr int kRowsPerWG = 128;      // data rows one workgroup of the contraction kernels owns
constexpr int kMaxD = 256;
constexpr int kMaxList = 16384;
constexpr int kMaxK = 2048;
constexpr int kPrefixFactorX2 = 2;   // twice the factor f in: dense prefix >= f * k * T / cap vectors
constexpr int kStreamWorkgroups = 8192;             // workgroups the streaming scan aims to launch at least
constexpr int64_t kStreamSliceBytes = 150ll << 20;  // part of the packed index one slice of a large streaming scan covers
constexpr int kMaxGridCells = 4096;  // entries of the quantiser's uniform-grid index (32 KB of LDS)

// Split float16 form used by the float16 matrix-core kernels: V = 1024*v, hi = fp16(V),
// lo = fp16(V - hi).  hi + lo equals V to about 2^-22 relative; the factor keeps lo in the normal
// float16 range for every |v| > 2.4e-4 (below that lo is at most 6e-8 of v's scale).
constexpr float kSplitScale = 1024.f;

// Raises a kernel's dynamic-LDS limit where a launch needs more than the default.  The attribute belongs
// to a (kernel, device) pair, so what has been set is remembered per device (one object per kernel);
// two threads that race here both set it, which is harmless.
class LdsLimit {
  public:
    hipError_t ensure(const void* kernel, size_t bytes) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= kDevices) return hipErrorInvalidDevice;
        if (bytes <= set_[dev].load(std::memory_order_acquire)) return hipSuccess;
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e == hipSuccess) set_[dev].store(bytes, std::memory_order_release);
        return e;
    }

  private:
    static constexpr int kDevices = 64;
    std::atomic<size_t> set_[kDevices] = {};
};

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }
inline int64_t round_up64(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

// Padded dimension used by the coarse-scoring kernel (smallest instantiated size >= d).
int coarse_dp(int d);
// Padded dimension used by the rotation kernel (multiple of 32).
inline int rot_dp(int d) { return round_up(d, 32); }
// 32-bit words of packed codes per vector.
inline int code_words(int b, int d) { return (b * d + 31) / 32; }

// Inverted-list storage as the kernels see it.  Slot s of the pool lives in storage block s/64,
// lane s%64; word w of its code sits at codes[(s/64 * words + w) * 64 + s%64], so a wavefront
// reading word w of 64 neighbouring vectors touches 256 contiguous bytes.
struct ListStore {
    uint32_t* codes;
    uint16_t* gamma;          // float16 bit patterns, one per slot
    int64_t* ids;             // labels, one per slot
    float* xnorm;             // |x| of the raw input row, one per slot; null unless the index keeps a raw metric
    const int64_t* list_off;  // [nlist] first slot of each list (multiple of 64)
    const int32_t* list_size; // [nlist] vectors stored in each list
    int words;
    // Optional second copy of the top (b - head_shift) bits of every code, packed the same way in head_words
    // words per vector (pass 1 of the cascade search reads these instead of the full codes); null = not kept.
    uint32_t* head; int head_words; int head_shift;
};

// ---- contraction kernels (split float16 MFMA) --------------------------------------------------------

// mode 0: assign[i] = argmax_c (<x~_i, cent_c> + bias_c), best[i] that value (either may be null)
// mode 1: scores[i*ld_scores + c] = <x~_i, cent_c> for c < L
// x: n x d raw rows (normalised inside).  cent_h / cent_l: split float16 form of the centroid table
// [Lpad][cent_pitch], zero padded, Lpad % 64 == 0 (made by launch_split_rows).
// flag: set to 1 when a row has zero or non-finite norm (that row gets assign -1).
hipError_t launch_coarse(int mode, const float* x, int64_t n, int d, const uint16_t* cent_h, const uint16_t* cent_l,
                         int cent_pitch, const float* bias, int L, int Lpad, int32_t* assign, float* best,
                         float* scores, int64_t ld_scores, int* flag, hipStream_t st);
// The argmax of mode 0 (no bias) in two steps: a screening pass with the hi*hi products alone decides
// every row whose best score is clearly ahead, the rest (listed in row_list, counted in *row_count,
// which the caller clears) is redone with all three products.  assign as for launch_coarse.  row_list
// and row_key are scratch arrays of n entries.  part (may be null): 3 * kScreenMaxShares floats of scratch
// per row; with it a short batch shares the centroid stages out over several workgroups per row tile.
constexpr int kScreenMaxShares = 16;
hipError_t launch_coarse_screened(const float* x, int64_t n, int d, const uint16_t* cent_h, const uint16_t* cent_l,
                                  int cent_pitch, int L, int Lpad, int32_t* assign, int* flag, int32_t* row_list,
                                  unsigned long long* row_key, int* row_count, float* part, hipStream_t st);
// hi[i], lo[i] = split float16 form of src[i]
hipError_t launch_split_rows(const float* src, int64_t count, uint16_t* hi, uint16_t* lo, hipStream_t st);

// Pure-MFMA calibration loop: `blocks` workgroups of 4 wavefronts, each wavefront issues 32*iters
// v_mfma_f32_32x32x16_f16.  operands: 4096*8 float16 values (any finite bits); out: blocks*256 floats.
hipError_t launch_mfma_peak(const uint16_t* operands, float* out, int blocks, int iters, hipStream_t st);

// Rotation family.  pi_h/pi_l: split form of Pi, [DP][DP] zero padded, DP = rot_dp(d).
// mode 0: residual -> rotate -> quantise -> pack into the list store at slot[row]
// mode 1: same, but write unpacked codes / fp16 norms to flat arrays (any may be null)
// mode 2: z_i = Pi x~_i written to zout[i*DP + j] (no centroid, no quantiser)
// q_grid: the quantiser's uniform-grid index (host_math.h), q_cells entries of (boundary, index bits).
// order_cell (mode 0): position p of the batch in list order holds row order_cell[p].x, which belongs to list
// order_cell[p].y and goes to slot list_base[l] + p - batch_base[l] (neighbouring lanes store to neighbouring
// slots, and neither the cell nor the slot of a row has to be fetched by row number).  Modes 1 and 2 take the
// rows in input order and read assign[row].
struct EncodeArgs {
    const float* x; int64_t n; int d; int b;
    const float* cent; int cent_pitch;
    const uint16_t* pi_h; const uint16_t* pi_l;   // split float16 form of Pi, [DP][DP]
    const float2* q_grid; int q_cells; float q_scale, q_offset;
    const int32_t* assign;
    // mode 0
    const int2* order_cell; const int64_t* list_base; const int64_t* batch_base;
    ListStore store; const int64_t* labels; int64_t label_base;
    // mode 1
    uint8_t* codes_flat; uint16_t* gamma_flat;
    // mode 2
    float* zout;
    uint16_t* zh_out; uint16_t* zl_out;   // optional: split float16 form of 1024*z (see split_scaled)
    float* norm_out;                      // optional (mode 2): |x_i| of every input row
};


hipError_t launch_encode(int mode, const EncodeArgs& a, hipStream_t st);

// ---- list bookkeeping -------------------------------------------------------------------------

// seg_hist[s*L + l] = number of rows of segment s assigned to list l (rows with assign < 0 skipped)
hipError_t launch_segment_hist(const int32_t* assign, int64_t n, int64_t seg_len, int nseg, int L,
                               uint32_t* seg_hist, hipStream_t st);
// in place: seg_hist[s][l] <- sum_{s'<s} seg_hist[s'][l];  batch_count[l] <- column total
hipError_t launch_segment_scan(uint32_t* seg_hist, int nseg, int L, uint32_t* batch_count, hipStream_t st);
// slot[i] = list_base[l] + (rank of row i among the batch rows of list l, in input order); slot and
// list_base may be null when only the order is wanted.
// order (may be null): the batch's rows grouped by list, lists ascending, input order inside a list:
// order[batch_base[l] + rank] = i, with batch_base the exclusive running sum of the batch's rows per list.
// order_cell (may be null): the same order with the list beside the row, order_cell[...] = (i, l).
hipError_t launch_stable_rank(const int32_t* assign, int64_t n, int64_t seg_len, int nseg, int L,
                              const uint32_t* seg_hist, const int64_t* list_base, int64_t* slot,
                              const int64_t* batch_base, int32_t* order, int2* order_cell, hipStream_t st);
// pack already-quantised rows (codes: n x d bytes, one bin number each) into their storage slots
// xnorm (may be null): raw norms of the rows, stored when the store keeps them
hipError_t launch_pack_scatter(const uint8_t* codes, const uint16_t* gamma, const float* xnorm, const int64_t* labels,
                               int64_t label_base, const int64_t* slot, int64_t n, int d, int b,
                               const ListStore& store, hipStream_t st);
// copy every list from one pool layout to another (same words per vector)
hipError_t launch_copy_lists(const ListStore& from, const ListStore& to, int L, hipStream_t st);
hipError_t launch_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t st);

// x_out[out_off[l] + v] = cent_l + gamma * Pi^T C[code] for vector v of list l (rows of d floats, list
// order), labels_out (may be null) the stored labels in the same order.  pi: fp32 [.][pi_pitch].
hipError_t launch_reconstruct(const ListStore& store, int L, int max_list, const float* cent, int cent_pitch,
                              const float* pi, int pi_pitch, const float* cb, int d, int b, const int64_t* out_off,
                              float* x_out, int64_t* labels_out, hipStream_t st);
// dst[t] = src[idx[t]], rows of d floats
hipError_t launch_gather_rows(const float* src, int d, const int64_t* idx, int64_t count, float* dst, hipStream_t st);

// ---- k-means pieces ---------------------------------------------------------------------------

// out[l] = sum of count[l'] over l' < l (L <= kMaxList)
hipError_t launch_exclusive_scan(const uint32_t* count, int L, int64_t* out, hipStream_t st);
// sums[l][j] = sum of x~_ij over the rows order[base[l] .. base[l] + count[l]) of cell l, added in a fixed
// order (bit-reproducible); rows are normalised on the fly
hipError_t launch_kmeans_cell_sums(const float* x, int d, const int32_t* order, const int64_t* base,
                                   const uint32_t* count, int L, float* sums, int pitch, hipStream_t st);
// cent[l] = sums[l]/counts[l] for non-empty cells; bias[l] = -|cent_l|^2/2 (padding rows: bias -inf)
hipError_t launch_kmeans_update(float* cent, int pitch, const float* sums, const uint32_t* counts,
                                float* bias, int L, int Lpad, int d, hipStream_t st);
// cent[dst[t]] = normalised row src_row[t] of x
hipError_t launch_copy_rows_normalised(const float* x, int d, const int64_t* src_row, const int32_t* dst,
                                       int count, float* cent, int pitch, hipStream_t st);
// normalise centroid rows in place; bias <- 0 for real rows
hipError_t launch_normalise_centroids(float* cent, int pitch, float* bias, int L, int d, hipStream_t st);
// sum over rows of (1 - 2*best_i) in double
hipError_t launch_inertia(const float* best, int64_t n, double* out, hipStream_t st);

// ---- search -----------------------------------------------------------------------------------

// cand_off[q*(np+1) + p] = sum_{p'<p} list_size[probe[q][p']]
// first (may be null): first[q] = shortest probe prefix (>= 1 cell) holding at least
// max(k, 2*k*T/cap) vectors, T the query's candidate total; np if there is none.  With `first`, cand_cnt[q]
// and gate[0] (each may be null) are set to zero: the counters the batched scan and its merge add to.
hipError_t launch_cand_offsets(const int32_t* probe, int64_t nq, int np, const int32_t* list_size,
                               int32_t* cand_off, int k, int cap, int32_t* first, int32_t* cand_cnt, int32_t* gate,
                               hipStream_t st);
// scores[row*m_stride + cand_off[q][p] + i] = coarse[q][p] + gamma_i * sum_j z_qj * C[code_ij]
hipError_t launch_list_scan(const float* z, int z_pitch, int d, int b, const float* cb,
                            const int32_t* probe, const float* coarse, const int32_t* cand_off,
                            int np, const ListStore& store, int64_t q_begin, int64_t q_count,
                            float* scores, int64_t m_stride, const int32_t* p_limit, const int32_t* gate,
                            int gate_begin, int gate_rows, int blocks_per_query, int slices, int metric, const float* qnorm,
                            hipStream_t st);
// metric 0: the score is the estimate s^ of <q~, x~> itself.  Raw metrics (the store keeps |x|, qnorm[q] = |q|):
// the scan writes a key that ranks like the metric and launch_metric_finish turns the selected keys into values:
//   metric 1 (inner product): key = |x| s^,                 value = |q| key            (descending)
//   metric 2 (squared L2):    key = 2 |x| |q| s^ - |x|^2,   value = |q|^2 - key        (ascending; missing: +inf)
hipError_t launch_metric_finish(float* scores, int64_t nq, int k, int metric, const float* qnorm, hipStream_t st);
// p_limit (may be null): only probes p < p_limit[q] are scanned.  gate (may be null; row = the query's index
// without it): of the gate[0] queries listed in gate[1..] only entries [gate_begin, gate_begin + gate_rows) are
// processed, entry g into score row g - gate_begin, so a buffer of gate_rows rows serves any number of listed
// queries in several launches.  blocks_per_query: workgroups per query (0 = one per probe), each
// walking its share of the probes; slices (not with a gate): workgroups that share every list.

// Per row: the k largest of m values, sorted by (value desc, label asc).
// mode 0 (probe selection): m = m_fixed for every row, label = column; writes int32 labels.
// mode 1 (results): row q has m = cand_off[q][np] values; column -> (probe p, position) -> label
//                   ids[list_off[probe[q][p]] + position]; writes int64 labels.
struct SelectArgs {
    const float* vals; int64_t stride; int64_t rows; int k;
    int m_fixed;
    const int32_t* cand_off; const int32_t* probe; int np; int64_t q_begin;
    const int32_t* p_limit;   // mode 1: row q only has the candidates of probes p < p_limit[q] (null = all)
    const int32_t* gate;      // null = all rows; else of the gate[0] rows listed in gate[1..] the entries
    int gate_begin, gate_rows;   // [gate_begin, gate_begin + gate_rows) are processed, entry g reading vals row g - gate_begin
    const int64_t* list_off; const int64_t* ids;
    float* out_vals; int32_t* out_i32; int64_t* out_i64;
    int m_bound;      // mode 1: host-side upper bound of any row's length (0 = unknown); picks the kernel
    // Selection in two steps (k <= 64, no gate): mode 2 treats `rows` = queries x np rows, row (q, p) being the
    // stretch of probe p in score row q, and writes k (value, label) pairs per row (m_bound = longest list);
    // mode 3 selects among the m_fixed = np * k survivors of a query, whose labels it reads from lab_in.
    const int64_t* lab_in;
};
hipError_t launch_select(int mode, const SelectArgs& a, hipStream_t st);

// Exact re-ranking: out = the k candidates of each query with the largest <q~, x~> computed from raw
// rows (x: n_rows x d, addressed by label), ordered by (score desc, label asc), repeats dropped.
struct RerankArgs {
    const float* q; const float* x; int64_t n_rows; int d;
    const int64_t* cand; int r; int k;
    float* out_scores; int64_t* out_ids;
};
hipError_t launch_rerank(const RerankArgs& a, int64_t nq, hipStream_t st);

// Pass 2 of the cascade search: the candidates of each query (slot numbers, -1 = none) are scored
// with the full codes, score = coarse term of the candidate's list + gamma * sum_j z_j cb[code_j],
// and the k best by (score desc, label asc) are written out.
struct CascadeArgs {
    const float* z; int z_pitch; int d; int b;
    const float* cb;                       // 2^b levels
    const int32_t* probe; const float* coarse; int np;     // [nq][np]
    ListStore store;
    const int64_t* ids;                    // label of a slot
    const int64_t* cand; int n_keep; int k;
    float* out_scores; int64_t* out_ids;
};
hipError_t launch_cascade_rescore(const CascadeArgs& a, int64_t nq, hipStream_t st);

// ---- query-batched scan ------------------------------------------------------------------------

// Queries one workgroup of the batched scan takes per tile for this (d, b); 0 = shape not covered
// (the streaming scan is used instead).
int batch_tile_queries(int d, int b);

// Buckets the (query, probe) pairs: bucket l holds the pairs (q, p < first[q]) of list l, bucket
// L + l the pairs (q, p >= first[q]).  pairs[pair_off[b] ...] holds the flat pair numbers q*np + p
// of bucket b; tile_off[b] counts workgroup tiles of tq queries (both arrays have 2L+1 entries).
// count and cursor are scratch arrays of 2L entries.
hipError_t launch_pair_grouping(const int32_t* probe, const int32_t* first, int64_t nq, int np, int L, int tq,
                                uint32_t* count, uint32_t* cursor, int64_t* pair_off, int32_t* tile_off,
                                int32_t* pairs, hipStream_t st);

struct BatchScanArgs {
    const uint16_t* zh; const uint16_t* zl; int z_pitch;   // split rotated queries, [nq][z_pitch] halves
    const float* cb;
    const int32_t* pairs; const int64_t* pair_off; const int32_t* tile_off;
    const float* coarse;                 // [nq*np] coarse term of each (query, probe)
    const float* thresh; int thresh_stride;   // threshold of query q at thresh[q*thresh_stride]
    ListStore store; int np; int L;
    int bucket_lo, bucket_hi;            // buckets this launch covers
    // threshold mode: cand_score = upper bound of the score (see acc0), cand_slot = slot | probe rank << kCandProbeShift
    float* cand_score; int64_t* cand_slot; int32_t* cand_cnt; int cap;
    float acc0;                          // 2^20 * kappa: start value of the threshold pass's accumulators
    // dense mode (the nearest lists): every score goes to scores[q*m_stride + cand_off[q][p] + v]
    int dense; float* scores; int64_t m_stride; const int32_t* cand_off;
};
hipError_t launch_batch_scan(const BatchScanArgs& a, int d, int b, int max_tiles, hipStream_t st);

constexpr int kCandProbeShift = 48;      // a candidate's probe rank sits above its slot number (slots < 2^48, ranks < 2^12)

// kappa with |sum_j z_j c_j - 2^-20 sum_j fp16(1024 z_j) fp16(1024 c_j)| <= kappa for |z| <= 1 and
// codebook values of magnitude <= cmax in d coordinates (each leading part is within 2^-11 relative
// of its value, Cauchy-Schwarz, |c| <= sqrt(d) cmax), with room for float32 accumulation.
inline float screen_kappa(int d, float cmax) { return (0x1p-10f + 0x1p-16f) * 1.002f * sqrtf((float)d) * cmax; }

struct MergeArgs {
    const float* first_scores; const int64_t* first_ids;     // [nq][k] from the streaming pass (exact scores)
    // candidates of the threshold pass: upper bounds u of the score (true score in [u - 2*kappa*gamma, u])
    const float* cand_score; const int64_t* cand_slot; const int32_t* cand_cnt; int cap;
    float kappa;
    const float* z; int z_pitch; int d; int b; const float* cb;   // rotated queries (float32) and levels, for re-scoring
    const float* coarse; int np;                                  // [nq][np] coarse terms
    ListStore store;
    const int64_t* ids;                                       // labels by slot (null: the slot is the label)
    int k; float* out_scores; int64_t* out_ids;
    int32_t* gate;                                            // [1 + nq]: count (cleared by the caller), then the queries whose candidate list overflowed
};
hipError_t launch_merge(const MergeArgs& a, int64_t nq, hipStream_t st);

}  // namespace ivftq
