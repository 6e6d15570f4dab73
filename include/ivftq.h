/*
 * ivftq.h -- C ABI of the IVF-TQ hot path for AMD MI355X (gfx950).
 *
 * IVF-TQ (arxiv 2605.17415, Section "IVF-TQ / Architecture") is an inverted-file index whose
 * residual layer needs no training: a fixed Haar rotation Pi followed by a Lloyd-Max scalar
 * quantiser that depends only on (b, d).  This library holds the two data-parallel halves of
 * that method as hand-written HIP kernels:
 *
 *   encode : x~ = x/|x| ; l = argmax_l <x~, c~_l> ; r = x~ - c~_l ; gamma = |r| ;
 *            rho = Pi r / |Pi r| ; code_j = bin of rho_j ; append (id, codes, fp16 gamma) to list l
 *   search : q~ = q/|q| ; s_l = <q~, c~_l> for all l ; probe the nprobe best cells ; z = Pi q~ ;
 *            score_i = s_l + gamma_i * sum_j z_j * C[code_ij] ; k best scores per query
 *
 * Conventions
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device memory on the
 *     current device.  The caller owns every buffer it passes; the library owns the index.
 *   - All matrices are dense row-major float32 unless stated.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Device work is
 *     queued on it.  Calls that hand data back to the host, and ivftq_encode_add /
 *     ivftq_train_coarse (which size storage from device results), synchronise that stream
 *     before returning; ivftq_search and ivftq_encode_only return with work still queued.
 *     Calls without a stream argument (ivftq_reset, ivftq_set_coarse, ivftq_set_rotation,
 *     ivftq_export_list) first wait for the stream of the most recent call on the index that
 *     took one; a caller who spreads one index over several streams orders them itself.
 *   - Every call returns an ivftq_status; nothing throws or aborts across this boundary.
 *     Arguments are validated before any kernel is launched.  ivftq_last_error() gives a
 *     thread-local message for the most recent failure.
 *   - An index is not thread-safe: one call at a time per index.
 *   - Limits: 1 <= b <= 8, 8 <= d <= 256, 1 <= nlist <= 16384, 1 <= nprobe <= min(nlist, 2048),
 *     1 <= k <= 2048.
 */
#ifndef IVFTQ_H
#define IVFTQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ivftq_index ivftq_index; /* opaque, library-owned */

/* Where an index gets its device memory (spec boundary: the caller's framework, e.g. PyTorch's
 * caching allocator, provides device memory; the library provides the kernels).  alloc returns `bytes`
 * bytes of device memory on the current device, aligned to at least 256 bytes, or NULL when it has
 * none; release takes back a pointer that alloc returned.  Both get the ctx pointer given at creation.
 * They are called from the thread that makes the library call, never from a kernel or another thread,
 * and a NULL from alloc makes that call return IVFTQ_OOM with the stored vectors unchanged. */
typedef void* (*ivftq_alloc_fn)(size_t bytes, void* ctx);
typedef void (*ivftq_free_fn)(void* ptr, void* ctx);

typedef int ivftq_status;
enum {
    IVFTQ_OK = 0,
    IVFTQ_INVALID_ARG = 1,   /* NULL pointer, size or parameter out of range */
    IVFTQ_BAD_STATE = 2,     /* e.g. encode or search before the coarse centroids exist */
    IVFTQ_OOM = 3,           /* device or host allocation failed */
    IVFTQ_HIP_ERROR = 4,     /* a HIP runtime call failed */
    IVFTQ_ZERO_NORM = 5,     /* an input row has zero or non-finite norm; nothing was appended */
    IVFTQ_UNSUPPORTED = 6    /* a size beyond the limits listed above */
};

/* What ivftq_search ranks by and returns (ivftq_set_metric). */
enum {
    IVFTQ_METRIC_COSINE = 0, /* the paper's setting: estimated <q~, x~> of the normalised vectors, descending */
    IVFTQ_METRIC_IP = 1,     /* estimated <q, x> of the raw vectors, descending */
    IVFTQ_METRIC_L2 = 2      /* estimated |q - x|^2 of the raw vectors, ascending */
};

/* ---- constants fixed by (b, d, seed): no device needed -------------------------------- */

/* Lloyd-Max codebook for the coordinate density of a uniform point on the unit sphere in R^d,
 * f_d(t) ~ (1 - t^2)^((d-3)/2)  (Appendix "Proofs of the rate-distortion bounds", Lemma 1).
 * centroids_out: host, 2^b floats, ascending.  boundaries_out: host, 2^b - 1 floats, the
 * midpoints of neighbouring centroids; coordinate value v gets code #{i : v >= boundary_i},
 * i.e. bins are [tau_i, tau_{i+1}) (Appendix "Sign-bit refinement").  Computed in double and
 * rounded to float. */
ivftq_status ivftq_build_codebook(int b, int d, float* centroids_out, float* boundaries_out);

/* Stage 1 at b bits plus the sign-bit refinement (Appendix "Sign-bit refinement": one more bit per
 * coordinate, s = 1[v >= c_i] for the value's bin i, reconstruction by the mean of the half-bin) as
 * one quantiser with 2^(b+1) levels, which is how the library stores and scans it:
 * boundaries_out (2^(b+1) - 1 floats) = the Stage-1 centroids and boundaries interleaved,
 * levels_out (2^(b+1) floats): entry 2i + s = E[T | T in half-bin (i, s)] under the density the
 * codebook is designed for.  #{j : v >= boundaries_out[j]} = 2*code + s.  1 <= b <= 7.  Host. */
ivftq_status ivftq_build_refined_codebook(int b, int d, float* levels_out, float* boundaries_out);

/* The table through which the encode kernel evaluates  code = #{i : v >= boundary_i}  (same
 * passage as above) with one lookup: the real line is cut into *cells_out equal cells (the two
 * outermost open-ended), cell(v) = clamp((int)(v * *scale_out + *offset_out), 0, cells - 1) in float
 * arithmetic, and  code = index_out[cell] + (v >= boundary_out[cell]).  For inspection and host-side
 * tests; all pointers host.  boundary_out / index_out (either may be NULL) need `capacity` >= cells
 * entries, else IVFTQ_INVALID_ARG; call with both NULL to learn the size.  IVFTQ_UNSUPPORTED if
 * (b, d) would need more than 4096 cells (then ivftq_create fails the same way).  sign_bit = 1:
 * the table of the merged quantiser of ivftq_build_refined_codebook. */
ivftq_status ivftq_quantiser_grid(int b, int sign_bit, int d, int capacity, int* cells_out,
                                  float* scale_out, float* offset_out, float* boundary_out,
                                  int32_t* index_out);

/* Haar-distributed orthogonal matrix (same appendix, Setup): QR of a d x d Gaussian matrix with
 * the sign of each column fixed so that diag(R) > 0.  pi_out: host, d*d floats, row-major, acting
 * as u = Pi r.  The first form draws the Gaussian matrix from `seed`; the second takes it from
 * the caller (g: host, d*d doubles, row-major) so that two implementations can be compared. */
ivftq_status ivftq_haar_rotation(int d, uint64_t seed, float* pi_out);
ivftq_status ivftq_haar_from_gaussian(int d, const double* g, float* pi_out);

/* ---- index life cycle ------------------------------------------------------------------ */

/* New empty index on the current HIP device: builds the (b, d) codebook and a Haar rotation from
 * rotation_seed.  Coarse centroids must be trained or set before encoding or searching.
 * alloc_fn / free_fn / alloc_ctx: all device memory of the index (constants, inverted lists, work
 * space) is obtained and returned through them; both NULL = hipMalloc / hipFree.  List storage
 * grows by allocating the larger pool before the old one is released, work buffers by releasing
 * first; everything is released by ivftq_destroy.  If alloc_fn returns NULL here the result is
 * IVFTQ_OOM and *out stays NULL. */
ivftq_status ivftq_create(int d, int b, int nlist, uint64_t rotation_seed, ivftq_alloc_fn alloc_fn,
                          ivftq_free_fn free_fn, void* alloc_ctx, ivftq_index** out);
/* The same with the sign-bit refinement switched on (sign_bit = 1): b Stage-1 bits + 1 refinement
 * bit are stored per coordinate, b + 1 <= 8.  Codes reported and accepted by the other calls are
 * then the merged ones, 2*code + s in [0, 2^(b+1)), and ivftq_get_codebook returns the tables of
 * ivftq_build_refined_codebook.  sign_bit = 0 is ivftq_create. */
ivftq_status ivftq_create_refined(int d, int b, int sign_bit, int nlist, uint64_t rotation_seed,
                                  ivftq_alloc_fn alloc_fn, ivftq_free_fn free_fn, void* alloc_ctx,
                                  ivftq_index** out);
/* Waits for the whole device (work of any stream may still use the index's memory), then returns
 * every buffer through free_fn. */
ivftq_status ivftq_destroy(ivftq_index* index);
/* Remove every stored vector.  Constants, the capacity already reserved for the lists and the
 * search workspace are kept, so the index can be filled again without allocating.  Waits for the
 * stream of the most recent call. */
ivftq_status ivftq_reset(ivftq_index* index);

/* Coarse partition (Section "Architecture", Indexing): Lloyd k-means on the L2-normalised rows of
 * x_dev (device, n x d), `niter` iterations, nearest mean in Euclidean distance; the final
 * centroids are L2-normalised.  init_rows_host: host, nlist distinct row numbers used as initial
 * centres, or NULL to draw them from `seed`.  An empty cell is re-seeded from a member of the
 * largest cell.  Needs n >= nlist.  inertia_out (host, may be NULL) receives the k-means
 * objective of the last assignment step.  The sums of an iteration are taken in a fixed order, so the
 * same rows, initial rows and seed give the same centroids bit for bit on every run.  The index's
 * centroids change only when the call succeeds.  Synchronises. */
ivftq_status ivftq_train_coarse(ivftq_index* index, const float* x_dev, int64_t n, int niter,
                                const int64_t* init_rows_host, uint64_t seed, double* inertia_out,
                                void* stream);

/* Inject / read back constants (host pointers).  centroids: nlist x d, rows are used as given
 * (they should be unit vectors).  pi: d x d, must be orthogonal to float32 rounding
 * (|Pi Pi^T - I|_F <= 2e-6, else IVFTQ_INVALID_ARG and the index keeps its rotation): the encode uses
 * |Pi r| = |r| (Section "Architecture", Indexing).  Setting either on a non-empty index is BAD_STATE. */
ivftq_status ivftq_set_coarse(ivftq_index* index, const float* centroids_host);
ivftq_status ivftq_get_coarse(const ivftq_index* index, float* centroids_host);
ivftq_status ivftq_set_rotation(ivftq_index* index, const float* pi_host);
ivftq_status ivftq_get_rotation(const ivftq_index* index, float* pi_host);
/* centroids_out: 2^b floats, boundaries_out: 2^b - 1 floats (either may be NULL). */
ivftq_status ivftq_get_codebook(const ivftq_index* index, float* centroids_out, float* boundaries_out);

/* ---- encode (Section "Architecture", Indexing and Bit accounting) ---------------------- */

/* Encode the n rows of x_dev (device, n x d) and append each to the inverted list of its coarse
 * cell, in input order.  ids_dev: device, n int64 labels, or NULL for consecutive labels
 * continuing from ivftq_ntotal().  Stored per vector: b*d code bits, a float16 residual norm and
 * the label.  On IVFTQ_ZERO_NORM nothing is appended.  Waits for the stream once (after the coarse
 * assignment, to size the lists on the host); the encode kernel itself and the update of the list
 * sizes are left running on the stream, so x_dev and ids_dev must stay valid until the stream has
 * passed them.  Later calls on the same stream see the appended vectors. */
ivftq_status ivftq_encode_add(ivftq_index* index, const float* x_dev, int64_t n,
                              const int64_t* ids_dev, void* stream);

/* Append vectors that are already encoded (the storage half of encode on its own, e.g. to import
 * an index built elsewhere).  assign_dev: n int32 cell numbers in [0, nlist); codes_dev: n x d
 * uint8 bin numbers in [0, 2^b); gamma_dev: n float16 bit patterns; ids_dev: n int64 labels or NULL
 * for consecutive labels.  All device pointers.  Rows are appended in input order.  A cell number
 * out of range gives IVFTQ_INVALID_ARG and nothing is appended.  Stream behaviour as for
 * ivftq_encode_add: one wait, then the packing runs on the stream. */
ivftq_status ivftq_add_encoded(ivftq_index* index, int64_t n, const int32_t* assign_dev,
                               const uint8_t* codes_dev, const uint16_t* gamma_dev,
                               const int64_t* ids_dev, void* stream);

/* Encode without storing.  Any output may be NULL.  assign_dev: n int32 cell numbers;
 * codes_dev: n x d uint8 bin numbers (one per byte); gamma_dev: n float16 bit patterns of |r|.
 * Rows with zero norm get cell -1.  Asynchronous. */
ivftq_status ivftq_encode_only(ivftq_index* index, const float* x_dev, int64_t n,
                               int32_t* assign_dev, uint8_t* codes_dev, uint16_t* gamma_dev,
                               void* stream);

/* ivftq_encode_only for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical
 * outputs, but the work arrays of the coarse assignment (and the cell numbers when assign_dev is NULL)
 * live in a static device array inside the library, 1 MiB + 256 bytes on every GPU the library has run
 * on, instead of the index's grow-only buffers: the call allocates and frees nothing (no hipMalloc, no
 * allocator callback) and issues kernel launches only.  n <= 65536, else IVFTQ_UNSUPPORTED and nothing
 * is launched.  All calls on one GPU share that array (whatever index they are for), so two calls that
 * overlap in time on one GPU race: keep them on one stream or order them.  ivftq_assign_undecided does
 * not cover this call.  Asynchronous. */
ivftq_status ivftq_encode_only_noalloc(ivftq_index* index, const float* x_dev, int64_t n,
                                       int32_t* assign_dev, uint8_t* codes_dev, uint16_t* gamma_dev,
                                       void* stream);

/* Re-ranking on raw vectors (same section: optional).  For each of the nq queries the r candidate
 * labels cand_ids_dev[q*r ..] (e.g. the ids ivftq_search returned for k = r; -1 and labels outside
 * [0, n_rows) are skipped, repeats count once) are scored exactly, <q~, x~> from the raw rows
 * x_dev[label*d ..] normalised on the fly, and the k best are written in descending order, ties by
 * smaller label, missing results as (-inf, -1).  The library keeps no raw vectors: x_dev is the
 * caller's n_rows x d matrix addressed by label.  All pointers device; 1 <= k <= r <= 2048;
 * asynchronous on the stream. */
ivftq_status ivftq_rerank(int d, const float* q_dev, int64_t nq, const float* x_dev, int64_t n_rows,
                          const int64_t* cand_ids_dev, int r, int k, float* scores_dev,
                          int64_t* ids_dev, void* stream);

/* ---- adaptive coarse refresh (Section "Adaptive coarse refresh") ------------------------ */

/* Reconstructions of every stored vector, x^ = c~_l + |r| * Pi^T C[code] (Refresh
 * self-containedness), in list order (list 0 first, storage order inside a list).  x_out_dev: device,
 * ivftq_ntotal() x d floats; ids_out_dev: device, ivftq_ntotal() int64 labels in the same order, or
 * NULL.  Synchronises. */
ivftq_status ivftq_reconstruct(ivftq_index* index, float* x_out_dev, int64_t* ids_out_dev, void* stream);

/* Replace the coarse centroids (host, nlist x d, unit rows) and re-assign and re-encode every stored
 * vector from its reconstruction against them; rotation and codebook stay as they are.  Labels are
 * kept; list order afterwards is the old list order filtered by new cell.  Allocates ntotal x d floats
 * of device memory for the duration of the call.  If the re-append fails (out of memory) the index
 * is left empty.  Synchronises. */
ivftq_status ivftq_reencode(ivftq_index* index, const float* centroids_host, void* stream);

/* The whole refresh (Algorithm of that section): reconstruct everything, take a sample stratified
 * across the lists (list l gives round(sample_n * n_l / ntotal) of its vectors, at least one, evenly
 * spaced in storage order), run ivftq_train_coarse on the sample (niter, init_rows_host -- rows of the
 * sample -- or seed, inertia_out as there), then re-encode as ivftq_reencode does.  If the training
 * fails the index is unchanged. */
ivftq_status ivftq_refresh_coarse(ivftq_index* index, int64_t sample_n, int niter,
                                  const int64_t* init_rows_host, uint64_t seed, double* inertia_out,
                                  void* stream);

/* ---- search (Section "Architecture", Search) ------------------------------------------- */

/* For each of the nq rows of q_dev (device, nq x d): scores_dev[nq x k] (float32, descending)
 * and ids_dev[nq x k] (int64 labels) of the k largest estimated inner products <q~, x~> among the
 * vectors of the nprobe cells with the largest <q~, c~_l>.  Equal scores are ordered by label.
 * Queries with fewer than k candidates are padded with label -1 and score -infinity.
 * Asynchronous on `stream`; uses workspace owned by the index, which only grows: once a call of the
 * same (nq, nprobe, k) has run on the index as it stands, further calls allocate nothing, do not
 * synchronise with the host and issue kernel launches only, so they may be recorded into a HIP graph.
 * A later call that needs more workspace (more queries, probes or results, or a larger index)
 * replaces the buffers, and graphs recorded before it must not be replayed any more: run the
 * largest shape once before recording. */
ivftq_status ivftq_search(ivftq_index* index, const float* q_dev, int64_t nq, int nprobe, int k,
                          float* scores_dev, int64_t* ids_dev, void* stream);

/* The first two steps of search on their own: probe_dev[nq x nprobe] int32 cell numbers ordered
 * by decreasing <q~, c~_l> (ties: smaller cell first) and coarse_dev[nq x nprobe] those inner
 * products.  Either output may be NULL.  Asynchronous. */
ivftq_status ivftq_coarse_probe(ivftq_index* index, const float* q_dev, int64_t nq, int nprobe,
                                int32_t* probe_dev, float* coarse_dev, void* stream);

/* ---- inspection ------------------------------------------------------------------------ */

int64_t ivftq_ntotal(const ivftq_index* index);
ivftq_status ivftq_list_size(const ivftq_index* index, int list, int64_t* n_out);
/* Copy one inverted list to the host in stored order.  ids_host: n int64; codes_host: n x d uint8
 * (unpacked bin numbers); gamma_host: n float16 bit patterns.  Any may be NULL.  Waits for the
 * stream of the most recent call. */
ivftq_status ivftq_export_list(const ivftq_index* index, int list, int64_t* ids_host,
                               uint8_t* codes_host, uint16_t* gamma_host);
/* Bytes of device memory the stored vectors occupy (codes + norms + labels, without slack; with a raw
 * metric 4 more per vector). */
int64_t ivftq_index_bytes(const ivftq_index* index);
/* Scan strategy of ivftq_search: 0 = default (the query-batched matrix-core scan when (d, b) is one
 * of its instantiated shapes, nprobe > 1 and the call is large enough for it to pay: the bytes a
 * per-query stream of the probed lists would read exceed 2.3 times the part of the index the call
 * touches plus 0.25 GB, a few hundred queries on a 10M-vector index; else the streaming scan, whose
 * shorter chain of kernels is faster for smaller calls), 1 = streaming scan only (a row of workgroups
 * per query walks its probed lists), 2 = the batched scan wherever the shape allows, whatever the
 * size of the call.  Results obey the same contract in every mode. */
ivftq_status ivftq_set_search_mode(ivftq_index* index, int mode);
/* Raw metrics.  The paper puts every vector on the unit sphere (Section "Architecture", Indexing), where
 * inner product, cosine and L2 rank alike; this switch serves inputs whose lengths matter, with nothing
 * but one stored float32 per vector, |x|, beside the paper's record: from the estimate s^ of <q~, x~>,
 *     <q, x> = |q| |x| s^          and          |q - x|^2 = |q|^2 + |x|^2 - 2 |q| |x| s^.
 * Cells are still probed by <q~, c~_l> and the codes are those of the normalised vector.  Switching
 * between cosine and a raw metric needs an empty index (BAD_STATE otherwise); between IP and L2 it
 * is free.  With a raw metric: ivftq_encode_add stores |x| too, encoded vectors are appended with
 * ivftq_add_encoded_raw, ivftq_search returns metric values (L2: smallest first, missing results
 * +infinity) from the streaming scan, and ivftq_search_cascade, ivftq_reencode and
 * ivftq_refresh_coarse return IVFTQ_UNSUPPORTED. */
ivftq_status ivftq_set_metric(ivftq_index* index, int metric);
/* ivftq_add_encoded for an index with a raw metric: xnorm_dev holds n float32 norms |x| (device). */
ivftq_status ivftq_add_encoded_raw(ivftq_index* index, int64_t n, const int32_t* assign_dev,
                                   const uint8_t* codes_dev, const uint16_t* gamma_dev,
                                   const float* xnorm_dev, const int64_t* ids_dev, void* stream);
/* The stored norms of one list in stored order (host, n float32); BAD_STATE for a cosine index.
 * Waits for the stream of the most recent call. */
ivftq_status ivftq_export_norms(const ivftq_index* index, int list, float* norms_host);

/* Upper limit, in bytes, of the per-search score workspace (default 4 GiB, at least 1 MiB or
 * IVFTQ_INVALID_ARG); queries are processed in as many passes as that allows.  A pass walks every
 * probed list again, so fewer passes are faster; the results do not depend on the limit. */
ivftq_status ivftq_set_workspace_limit(ivftq_index* index, int64_t bytes);

/* ---- per-kernel timing (measurement aid) ------------------------------------------------ */

/* While enabled, every kernel launch made for this index is bracketed by two HIP events recorded
 * on the launch stream.  ivftq_profile_read waits for the recorded events, adds up the elapsed time and
 * the number of launches per kernel class since the last read (ms_out, launches_out: host arrays
 * of ivftq_profile_kernel_count() entries) and clears the records.  Enabling or disabling clears
 * them too.  Kernel classes are named by ivftq_profile_kernel_name(id). */
ivftq_status ivftq_profile_enable(ivftq_index* index, int on);
ivftq_status ivftq_profile_read(ivftq_index* index, double* ms_out, int64_t* launches_out);
int ivftq_profile_kernel_count(void);
const char* ivftq_profile_kernel_name(int id);

/* Cascade search (Appendix "Cascade search via Lloyd-Max bin ordinality"): pass 1 ranks every
 * candidate of the probed lists from the top `beta` bits of each stored Stage-1 code, reconstructed
 * with the coarsened codebook below, and keeps the n_keep best per query; pass 2 scores those with
 * the full stored codes (Stage 1 and, if the index has it, the sign bit) and returns the k best,
 * outputs as ivftq_search.  1 <= beta <= Stage-1 bits, k <= n_keep <= 2048.  If the index keeps a
 * plane of exactly the top beta bits (ivftq_set_cascade_plane) pass 1 reads that plane, beta/b of the
 * bytes of the full codes; otherwise it reads the full codes through a table that ignores the low
 * bits.  The two give the same scores.  With n_keep at least the number of candidates, or beta equal
 * to the Stage-1 bits, the result is that of ivftq_search.  Candidates that tie in pass 1 at the
 * n_keep-th place are kept in slot order. */
ivftq_status ivftq_search_cascade(ivftq_index* index, const float* q_dev, int64_t nq, int nprobe, int k,
                                  int beta, int n_keep, float* scores_dev, int64_t* ids_dev, void* stream);

/* MSB-first storage for the cascade search (same appendix, "Cascade algorithm"): beside the packed
 * codes the index keeps the top beta bits of every coordinate once more, packed the same way in
 * ceil(beta*d/32) words per vector, so that pass 1 streams only those.  beta = 0 switches the plane
 * off (the default).  1 <= beta <= Stage-1 bits and beta < stored bits, else IVFTQ_INVALID_ARG; the
 * index must be empty (IVFTQ_BAD_STATE otherwise).  Costs beta*d more bits per vector (see
 * ivftq_index_bytes); every append path fills the plane, every other call ignores it. */
ivftq_status ivftq_set_cascade_plane(ivftq_index* index, int beta);
/* The plane's content for one list in stored order: head_codes_host gets n x d uint8, each the top
 * beta bits of the coordinate's code.  BAD_STATE without a plane.  Waits for the stream of the most
 * recent call. */
ivftq_status ivftq_export_cascade_plane(const ivftq_index* index, int list, uint8_t* head_codes_host);

/* The coarsened codebook of pass 1 (host only): values_out[g], g < 2^beta, is the mean of the
 * sphere-coordinate density over the union of the 2^(b-beta) Stage-1 bins whose codes start with g
 * (with sign_bit != 0: computed from the merged 2^(b+1)-level table, the same numbers). */
ivftq_status ivftq_build_coarsened_codebook(int b, int sign_bit, int d, int beta, float* values_out);

/* Measurement aid: how many rows of the most recent ivftq_encode_add / ivftq_encode_only call on this
 * index the screening pass of the coarse assignment (float16 leading parts only) left undecided and
 * handed to the full-precision pass (Algorithm "Encode", coarse assignment step; the assignment is
 * the full-precision one either way).  Waits for `stream`. */
ivftq_status ivftq_assign_undecided(ivftq_index* index, int64_t* count_out, void* stream);

/* Measurement aid: what the query-batched scan of the most recent ivftq_search / ivftq_search_cascade on this
 * index did in its last pass over the queries (Section "Architecture", Search; beyond each query's nearest lists the scan keeps only the
 * candidates whose upper bound reaches the k-th best score of those lists): queries_out = queries of that pass
 * (0 when the streaming scan ran), redone_out = those whose candidate list overflowed and that were redone by
 * the exact streaming scan, max_candidates_out / mean_candidates_out = candidates collected per query.  Any
 * output may be NULL.  Waits for `stream`. */
ivftq_status ivftq_scan_stats(ivftq_index* index, int64_t* queries_out, int64_t* redone_out,
                              int64_t* max_candidates_out, double* mean_candidates_out, void* stream);

/* Measurement aid: the rate (TFLOP/s, 2*32*32*16 flop per instruction) that a loop of nothing but
 * v_mfma_f32_32x32x16_f16, the instruction every contraction of this library uses, reaches on the
 * current device, two wavefronts per SIMD, operands in registers.  random_operands != 0: operands
 * with random sign and mantissa bits (the switching activity of real data, under which the chip
 * lowers its clock); 0: all operands 1.0.  Allocates and frees its own small buffers; synchronises. */
ivftq_status ivftq_measure_mfma_rate(int random_operands, double* tflops_out);

const char* ivftq_last_error(void);
const char* ivftq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* IVFTQ_H */
