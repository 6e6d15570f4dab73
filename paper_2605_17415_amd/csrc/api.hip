// C ABI of libivftq: argument checking, index life cycle, storage growth and the launch
// sequences of encode (Section "Architecture", Indexing) and search (same section, Search).
// All arithmetic of the hot path happens in the kernels; the host only sizes buffers and orders
// launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <numeric>
#include <string>
#include <unordered_set>
#include <vector>

#include "../../include/ivftq.h"
#include "host_math.h"
#include "kernels.h"

using namespace ivftq;

namespace {

thread_local std::string g_error;

ivftq_status fail(ivftq_status code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_error = buf;
    return code;
}

#define HIP_TRY(expr)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return fail(e_ == hipErrorOutOfMemory ? IVFTQ_OOM : IVFTQ_HIP_ERROR, "%s: %s",    \
                        #expr, hipGetErrorString(e_));                                        \
    } while (0)

// Where device memory comes from: the caller's callbacks (ivftq_create), or hipMalloc / hipFree
// when none were given.
struct Allocator {
    ivftq_alloc_fn alloc = nullptr;
    ivftq_free_fn free = nullptr;
    void* ctx = nullptr;
    void* get(size_t bytes) const {
        if (alloc) return alloc(bytes, ctx);
        void* p = nullptr;
        if (hipMalloc(&p, bytes) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
        return p;
    }
    void put(void* p) const {
        if (!p) return;
        if (alloc) free(p, ctx); else (void)hipFree(p);
    }
};
const Allocator kHipAllocator{};

// Grow-only device buffer.  Contents are not kept across a growth.
struct DevBuf {
    void* p = nullptr;
    size_t bytes = 0;
    const Allocator* al = &kHipAllocator;
    DevBuf() = default;
    explicit DevBuf(const Allocator* a) : al(a) {}
    hipError_t ensure(size_t need) {
        if (need <= bytes) return hipSuccess;
        release();
        p = al->get(need);
        if (!p) return hipErrorOutOfMemory;
        bytes = need;
        return hipSuccess;
    }
    void release() { al->put(p); p = nullptr; bytes = 0; }
    template <class T> T* as() const { return static_cast<T*>(p); }
};

// Grow-only pinned host buffer (staging for small asynchronous copies in both directions).
struct PinnedBuf {
    void* p = nullptr;
    size_t bytes = 0;
    hipError_t ensure(size_t need) {
        if (need <= bytes) return hipSuccess;
        if (p) { (void)hipHostFree(p); p = nullptr; bytes = 0; }
        hipError_t e = hipHostMalloc(&p, need, hipHostMallocDefault);
        if (e == hipSuccess) bytes = need; else p = nullptr;
        return e;
    }
    void release() { if (p) (void)hipHostFree(p); p = nullptr; bytes = 0; }
};

// kernel classes for the optional per-launch timing
enum ProfId { P_ASSIGN, P_COARSE_SCORES, P_ENCODE, P_ROTATE_Q, P_SEG_HIST, P_SEG_SCAN, P_RANK, P_PACK,
              P_COPY_LISTS, P_SELECT_PROBE, P_CAND_OFF, P_LIST_SCAN, P_SELECT_TOPK, P_KMEANS_UPDATE, P_KMEANS_SUMS,
              P_PAIR_GROUP, P_BATCH_FIRST, P_BATCH_SCAN, P_MERGE, P_CASCADE, P_COUNT };
const char* const kProfNames[P_COUNT] = {"coarse_assign", "coarse_scores", "encode_rotate_quantise_pack",
                                         "rotate_queries", "segment_hist", "segment_scan", "stable_rank",
                                         "pack_scatter", "copy_lists", "select_probes", "cand_offsets",
                                         "list_scan", "select_topk", "kmeans_update", "kmeans_cell_sums", "pair_grouping",
                                         "batch_scan_nearest", "batch_scan", "merge_topk", "cascade_rescore"};
struct ProfRec { int id; hipEvent_t a, b; };
// Timing events are recycled process-wide: creating one per launch costs more than the launch.
std::mutex g_event_mutex;
std::vector<hipEvent_t> g_event_pool;

uint64_t splitmix(uint64_t& s) {
    uint64_t z = (s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Scratch of the allocation-free entry point (ivftq_encode_only_noalloc): the work arrays of the coarse
// assignment for up to kNoAllocRows rows.  Layout: 256 bytes of flags and counters | 8-byte keys | int32 row
// numbers | int32 cell numbers.  Every GPU the library runs on holds its own copy until the process ends.
constexpr int64_t kNoAllocRows = 65536;
constexpr size_t kNoAllocBytes = 256 + (size_t)kNoAllocRows * (8 + 4 + 4);
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

}  // namespace

static __device__ __align__(256) unsigned char scratch[kNoAllocBytes];

namespace {

// Device address of `scratch` on the current device (looked up once per device; in host code the array's
// name is only a handle for this look-up, never an address).
hipError_t scratch_on_current_device(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

struct ivftq_index {
    int d = 0, b = 0, nlist = 0, K = 0, dp = 0, lpad = 0, words = 0;   // b: bits stored per coordinate (Stage 1 + sign bit)
    int sign_bit = 0;
    bool refreshing = false;   // set while ivftq_refresh_coarse re-trains the centroids of a non-empty index
    int q_cells = 0; float q_scale = 0.f, q_offset = 0.f;   // quantiser grid (host_math.h)
    bool has_coarse = false;
    std::vector<float> h_cent, h_pi, h_cb, h_tau;
    // device constants
    DevBuf cent, cent_h, cent_l, bias, pi, pi_h, pi_l, cb, q_grid;   // cent_h/cent_l: split float16 form of cent
    // list storage
    DevBuf codes, gamma, ids, d_off, d_size;
    DevBuf xnorm;          // |x| per slot, kept only for a raw metric (ivftq_set_metric)
    DevBuf head;           // top plane_beta bits of every code once more, packed alike (ivftq_set_cascade_plane); unused when plane_beta == 0
    int plane_beta = 0, head_words = 0;
    int metric = IVFTQ_METRIC_COSINE;
    DevBuf w_qnorm;        // |q| per query of the current search pass
    std::vector<int64_t> h_off, h_cap;
    std::vector<int32_t> h_size;
    int64_t pool_slots = 0;
    PinnedBuf pin;   // [L u32 batch counts | 16 B flag | 2L i64 bases | L i32 sizes], see place_rows / commit_rows
    int64_t ntotal = 0;
    // workspace
    DevBuf w_assign, w_slot, w_order, w_hist, w_count, w_base, w_flag, w_best, w_undecided;
    DevBuf cb_cascade, w_keep, w_keep_scores;   // cascade search: pass-1 table (for cascade_beta), kept slots and their pass-1 scores
    int cascade_beta = 0;
    DevBuf w_S, w_probe, w_coarse, w_z, w_candoff, w_scores;
    DevBuf w_sums, w_counts, w_zero, w_rows, w_dst, w_obj;
    DevBuf t_cent, t_cent_h, t_cent_l, t_bias;   // k-means works on its own tables; the index's change only on success
    DevBuf w_zh, w_zl;
    DevBuf w_first, w_fscores, w_fids, w_pairs, w_pairoff, w_tileoff, w_cscore, w_cslot, w_ccnt, w_gate;
    DevBuf w_stage_s, w_stage_i;      // survivors of the first step of a selection in two steps
    DevBuf w_part;                    // partial results of a coarse assignment whose centroid stages are shared out
    int64_t last_batched_queries = 0;   // queries of the last pass of the most recent batched search (ivftq_scan_stats)
    int search_mode = 0;   // 0 auto, 1 streaming scan only, 2 batched scan whenever the shape allows
    int64_t ws_limit = (int64_t)4 << 30;
    bool prof_on = false;
    std::vector<ProfRec> prof;
    Allocator alloc;                  // every DevBuf of the index draws from it
    hipStream_t last_stream = nullptr;   // stream of the most recent call that took one (ivftq_reset and the host read-backs wait for it)

    std::vector<DevBuf*> buffers() {
        return {&cent, &cent_h, &cent_l, &pi_h, &pi_l, &bias, &pi, &cb, &q_grid, &codes, &gamma, &ids, &xnorm, &head, &w_qnorm, &d_off, &d_size, &w_assign,
                &w_slot, &w_order, &w_hist, &w_count, &w_base, &w_flag, &w_best, &w_undecided, &cb_cascade, &w_keep, &w_keep_scores,
                &w_S, &w_probe, &w_coarse, &w_z, &w_candoff, &w_scores, &w_sums, &w_counts, &w_zero, &w_rows, &w_dst, &w_obj,
                &t_cent, &t_cent_h, &t_cent_l, &t_bias, &w_first, &w_fscores, &w_fids, &w_pairs, &w_pairoff, &w_tileoff, &w_cscore,
                &w_cslot, &w_ccnt, &w_gate, &w_zh, &w_zl, &w_stage_s, &w_stage_i, &w_part};
    }
    explicit ivftq_index(const Allocator& a) : alloc(a) {
        for (DevBuf* bfr : buffers()) bfr->al = &alloc;
    }
    ivftq_index(const ivftq_index&) = delete;
    ivftq_index& operator=(const ivftq_index&) = delete;

    ListStore store() const {
        ListStore s;
        s.codes = codes.as<uint32_t>();
        s.gamma = gamma.as<uint16_t>();
        s.ids = ids.as<int64_t>();
        s.xnorm = metric != IVFTQ_METRIC_COSINE ? xnorm.as<float>() : nullptr;
        s.list_off = d_off.as<int64_t>();
        s.list_size = d_size.as<int32_t>();
        s.words = words;
        s.head = plane_beta ? head.as<uint32_t>() : nullptr;
        s.head_words = head_words;
        s.head_shift = plane_beta ? b - plane_beta : 0;
        return s;
    }
    // The top-bit plane seen as a store of plane_beta-bit codes (same slots, norms and labels).
    ListStore head_store() const {
        ListStore s = store();
        s.codes = head.as<uint32_t>();
        s.words = head_words;
        s.head = nullptr; s.head_words = 0; s.head_shift = 0;
        return s;
    }
    ~ivftq_index() {
        for (ProfRec& r : prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
        for (DevBuf* bfr : buffers()) bfr->release();
        pin.release();
    }
};

namespace {

// Runs one launch; when profiling is on, brackets it with events on the launch stream.
template <class F>
hipError_t timed(ivftq_index* ix, hipStream_t st, int id, F&& launch) {
    if (!ix->prof_on) return launch();
    ProfRec r{id, nullptr, nullptr};
    hipError_t e = hipSuccess;
    {
        std::lock_guard<std::mutex> lock(g_event_mutex);
        for (hipEvent_t* ev : {&r.a, &r.b}) {
            if (!g_event_pool.empty()) { *ev = g_event_pool.back(); g_event_pool.pop_back(); }
            else if ((e = hipEventCreate(ev)) != hipSuccess) return e;
        }
    }
    e = hipEventRecord(r.a, st);
    if (e != hipSuccess) return e;
    e = launch();
    hipError_t e2 = hipEventRecord(r.b, st);
    ix->prof.push_back(r);
    return e != hipSuccess ? e : e2;
}

void drop_profile(ivftq_index* ix) {
    std::lock_guard<std::mutex> lock(g_event_mutex);
    for (ProfRec& r : ix->prof) { g_event_pool.push_back(r.a); g_event_pool.push_back(r.b); }
    ix->prof.clear();
}

// The coarse kernel reads the centroid table in split float16 form; call after every change of it.
hipError_t refresh_split(ivftq_index* ix, hipStream_t st) {
    return launch_split_rows(ix->cent.as<float>(), (int64_t)ix->lpad * ix->dp, ix->cent_h.as<uint16_t>(),
                             ix->cent_l.as<uint16_t>(), st);
}

ivftq_status upload_coarse(ivftq_index* ix) {
    std::vector<float> padded((size_t)ix->lpad * ix->dp, 0.f);
    for (int l = 0; l < ix->nlist; ++l)
        std::memcpy(&padded[(size_t)l * ix->dp], &ix->h_cent[(size_t)l * ix->d], sizeof(float) * ix->d);
    HIP_TRY(hipStreamSynchronize(ix->last_stream));      // nothing queued earlier may still read the old table
    HIP_TRY(hipMemcpy(ix->cent.p, padded.data(), padded.size() * sizeof(float), hipMemcpyHostToDevice));
    std::vector<float> zero(ix->lpad, 0.f);
    HIP_TRY(hipMemcpy(ix->bias.p, zero.data(), zero.size() * sizeof(float), hipMemcpyHostToDevice));
    HIP_TRY(refresh_split(ix, nullptr));
    HIP_TRY(hipStreamSynchronize(nullptr));
    return IVFTQ_OK;
}

ivftq_status upload_rotation(ivftq_index* ix) {
    // The encode kernel quantises Pi r^ without dividing by |Pi r^| (= 1 for an orthogonal Pi), so
    // the rotation has to be orthogonal to float32 rounding: the defect bounds | |Pi r^|^2 - 1 |.
    const double defect = orthogonality_defect(ix->d, ix->h_pi.data());
    if (!(defect <= 2e-6))
        return fail(IVFTQ_INVALID_ARG, "rotation is not orthogonal: |Pi Pi^T - I|_F = %.3g (limit 2e-6)", defect);
    std::vector<float> padded((size_t)ix->dp * ix->dp, 0.f);
    for (int i = 0; i < ix->d; ++i)
        std::memcpy(&padded[(size_t)i * ix->dp], &ix->h_pi[(size_t)i * ix->d], sizeof(float) * ix->d);
    HIP_TRY(hipStreamSynchronize(ix->last_stream));
    HIP_TRY(hipMemcpy(ix->pi.p, padded.data(), padded.size() * sizeof(float), hipMemcpyHostToDevice));
    HIP_TRY(launch_split_rows(ix->pi.as<float>(), (int64_t)ix->dp * ix->dp, ix->pi_h.as<uint16_t>(),
                              ix->pi_l.as<uint16_t>(), nullptr));
    HIP_TRY(hipStreamSynchronize(nullptr));
    return IVFTQ_OK;
}

// Make every list able to hold need[l] vectors.  Lists keep their contents; the pool is rebuilt
// with a quarter of slack per list whenever one list would overflow.
ivftq_status ensure_capacity(ivftq_index* ix, const std::vector<int64_t>& need, hipStream_t st) {
    bool ok = ix->pool_slots > 0;
    for (int l = 0; ok && l < ix->nlist; ++l) ok = need[l] <= ix->h_cap[l];
    if (ok) return IVFTQ_OK;

    std::vector<int64_t> cap(ix->nlist), off(ix->nlist);
    int64_t total = 0;
    for (int l = 0; l < ix->nlist; ++l) {
        int64_t want = need[l] + need[l] / 4 + kSlotsPerBlock;
        cap[l] = round_up64(std::max(ix->h_cap.empty() ? 0 : ix->h_cap[l], want), kSlotsPerBlock);
        off[l] = total;
        total += cap[l];
    }
    const bool raw = ix->metric != IVFTQ_METRIC_COSINE;
    DevBuf ncodes(&ix->alloc), ngamma(&ix->alloc), nids(&ix->alloc), noff(&ix->alloc), nxnorm(&ix->alloc), nhead(&ix->alloc);
    hipError_t e = ncodes.ensure((size_t)total * ix->words * sizeof(uint32_t));
    if (e == hipSuccess) e = ngamma.ensure((size_t)total * sizeof(uint16_t));
    if (e == hipSuccess) e = nids.ensure((size_t)total * sizeof(int64_t));
    if (e == hipSuccess) e = noff.ensure((size_t)ix->nlist * sizeof(int64_t));
    if (e == hipSuccess && raw) e = nxnorm.ensure((size_t)total * sizeof(float));
    if (e == hipSuccess && ix->plane_beta) e = nhead.ensure((size_t)total * ix->head_words * sizeof(uint32_t));
    if (e != hipSuccess) {
        ncodes.release(); ngamma.release(); nids.release(); noff.release(); nxnorm.release(); nhead.release();
        return fail(IVFTQ_OOM, "growing list storage to %lld slots: %s", (long long)total, hipGetErrorString(e));
    }
    HIP_TRY(hipMemcpyAsync(noff.p, off.data(), off.size() * sizeof(int64_t), hipMemcpyHostToDevice, st));
    if (ix->ntotal > 0) {
        ListStore from = ix->store(), to = from;
        to.codes = ncodes.as<uint32_t>();
        to.gamma = ngamma.as<uint16_t>();
        to.ids = nids.as<int64_t>();
        to.xnorm = raw ? nxnorm.as<float>() : nullptr;
        to.head = ix->plane_beta ? nhead.as<uint32_t>() : nullptr;
        to.list_off = noff.as<int64_t>();
        HIP_TRY(timed(ix, st, P_COPY_LISTS, [&] { return launch_copy_lists(from, to, ix->nlist, st); }));
    }
    HIP_TRY(hipStreamSynchronize(st));   // `off` is pageable host memory; old pool is about to be freed
    ix->codes.release(); ix->gamma.release(); ix->ids.release(); ix->d_off.release(); ix->xnorm.release(); ix->head.release();
    ix->codes = ncodes; ix->gamma = ngamma; ix->ids = nids; ix->d_off = noff; ix->xnorm = nxnorm; ix->head = nhead;
    ix->h_cap = cap;
    ix->h_off = off;
    ix->pool_slots = total;
    return IVFTQ_OK;
}

ivftq_status check_index(const ivftq_index* ix) {
    if (!ix) return fail(IVFTQ_INVALID_ARG, "index is NULL");
    return IVFTQ_OK;
}

// Rows per segment of the stable counting sort (one wavefront ranks a segment, one histogram row of L counters
// per segment): as many segments as keep the chip busy (up to 4096), at least 128 rows each, and at most
// 16M counters in all.
int64_t segment_length(int64_t n, int L) {
    const int64_t max_segments = std::max<int64_t>(64, std::min<int64_t>(4096, ((int64_t)16 << 20) / L));
    return round_up64(std::max<int64_t>((n + max_segments - 1) / max_segments, 128), 64);
}

// The stream a call works on; remembered so that calls without a stream argument know what to wait for.
hipStream_t use_stream(ivftq_index* ix, void* stream) {
    ix->last_stream = static_cast<hipStream_t>(stream);
    return ix->last_stream;
}

}  // namespace

extern "C" {

const char* ivftq_last_error(void) { return g_error.c_str(); }
const char* ivftq_version(void) { return "ivftq-gfx950 0.1"; }

ivftq_status ivftq_build_codebook(int b, int d, float* centroids_out, float* boundaries_out) {
    if (b < 1 || b > 8 || d < 3) return fail(IVFTQ_INVALID_ARG, "need 1 <= b <= 8 and d >= 3 (b=%d d=%d)", b, d);
    if (!centroids_out && !boundaries_out) return fail(IVFTQ_INVALID_ARG, "both outputs NULL");
    std::vector<double> c, t;
    if (!build_codebook(b, d, c, t)) return fail(IVFTQ_INVALID_ARG, "codebook construction failed");
    if (centroids_out) for (size_t i = 0; i < c.size(); ++i) centroids_out[i] = (float)c[i];
    if (boundaries_out) for (size_t i = 0; i < t.size(); ++i) boundaries_out[i] = (float)t[i];
    return IVFTQ_OK;
}

ivftq_status ivftq_build_refined_codebook(int b, int d, float* levels_out, float* boundaries_out) {
    if (b < 1 || b > 7 || d < 3) return fail(IVFTQ_INVALID_ARG, "need 1 <= b <= 7 and d >= 3 (b=%d d=%d)", b, d);
    if (!levels_out && !boundaries_out) return fail(IVFTQ_INVALID_ARG, "both outputs NULL");
    std::vector<double> lv, bd, c, t;
    if (!build_refined_codebook(b, d, lv, bd) || !build_codebook(b, d, c, t))
        return fail(IVFTQ_INVALID_ARG, "codebook construction failed");
    if (levels_out) for (size_t i = 0; i < lv.size(); ++i) levels_out[i] = (float)lv[i];
    // the boundaries are the float32 Stage-1 centroids and boundaries themselves, interleaved
    if (boundaries_out) for (size_t i = 0; i < bd.size(); ++i) boundaries_out[i] = (float)bd[i];
    return IVFTQ_OK;
}

ivftq_status ivftq_quantiser_grid(int b, int sign_bit, int d, int capacity, int* cells_out, float* scale_out,
                                  float* offset_out, float* boundary_out, int32_t* index_out) {
    if (!cells_out || !scale_out || !offset_out) return fail(IVFTQ_INVALID_ARG, "output pointer is NULL");
    if (sign_bit != 0 && sign_bit != 1) return fail(IVFTQ_INVALID_ARG, "sign_bit=%d is neither 0 nor 1", sign_bit);
    if (b < 1 || b + sign_bit > 8) return fail(IVFTQ_INVALID_ARG, "b=%d (+%d sign bit) outside [1, 8]", b, sign_bit);
    std::vector<float> c((size_t)1 << (b + sign_bit)), tau(((size_t)1 << (b + sign_bit)) - 1);
    ivftq_status s = sign_bit ? ivftq_build_refined_codebook(b, d, c.data(), tau.data())
                              : ivftq_build_codebook(b, d, c.data(), tau.data());
    if (s != IVFTQ_OK) return s;
    QuantiserGrid grid;
    if (!build_quantiser_grid(tau, kMaxGridCells, grid))
        return fail(IVFTQ_UNSUPPORTED, "quantiser grid for b=%d+%d d=%d needs more than %d cells", b, sign_bit, d, kMaxGridCells);
    *cells_out = grid.cells; *scale_out = grid.scale; *offset_out = grid.offset;
    if (boundary_out || index_out) {
        if (capacity < grid.cells) return fail(IVFTQ_INVALID_ARG, "capacity %d below the %d cells of the grid", capacity, grid.cells);
        if (boundary_out) std::copy(grid.boundary.begin(), grid.boundary.end(), boundary_out);
        if (index_out) std::copy(grid.index.begin(), grid.index.end(), index_out);
    }
    return IVFTQ_OK;
}

ivftq_status ivftq_haar_from_gaussian(int d, const double* g, float* pi_out) {
    if (d < 1 || !g || !pi_out) return fail(IVFTQ_INVALID_ARG, "bad argument to ivftq_haar_from_gaussian");
    std::vector<double> q;
    if (!haar_from_gaussian(d, g, q)) return fail(IVFTQ_INVALID_ARG, "matrix is rank deficient");
    for (size_t i = 0; i < q.size(); ++i) pi_out[i] = (float)q[i];
    return IVFTQ_OK;
}

ivftq_status ivftq_haar_rotation(int d, uint64_t seed, float* pi_out) {
    if (d < 1 || !pi_out) return fail(IVFTQ_INVALID_ARG, "bad argument to ivftq_haar_rotation");
    std::vector<double> g;
    gaussian_matrix(d, seed, g);
    return ivftq_haar_from_gaussian(d, g.data(), pi_out);
}

ivftq_status ivftq_create(int d, int b, int nlist, uint64_t rotation_seed, ivftq_alloc_fn alloc_fn,
                          ivftq_free_fn free_fn, void* alloc_ctx, ivftq_index** out) {
    return ivftq_create_refined(d, b, 0, nlist, rotation_seed, alloc_fn, free_fn, alloc_ctx, out);
}

ivftq_status ivftq_create_refined(int d, int b_stage1, int sign_bit, int nlist, uint64_t rotation_seed,
                                  ivftq_alloc_fn alloc_fn, ivftq_free_fn free_fn, void* alloc_ctx, ivftq_index** out) {
    if (!out) return fail(IVFTQ_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if ((alloc_fn == nullptr) != (free_fn == nullptr))
        return fail(IVFTQ_INVALID_ARG, "alloc_fn and free_fn must both be given or both be NULL");
    if (sign_bit != 0 && sign_bit != 1) return fail(IVFTQ_INVALID_ARG, "sign_bit=%d is neither 0 nor 1", sign_bit);
    if (b_stage1 < 1 || b_stage1 + sign_bit > 8)
        return fail(IVFTQ_INVALID_ARG, "b=%d (+%d sign bit) outside [1, 8] bits per coordinate", b_stage1, sign_bit);
    const int b = b_stage1 + sign_bit;       // bits stored per coordinate: everything below works on the merged quantiser
    if (d < 8) return fail(IVFTQ_INVALID_ARG, "d=%d below 8", d);
    if (nlist < 1) return fail(IVFTQ_INVALID_ARG, "nlist=%d below 1", nlist);
    if (d > kMaxD) return fail(IVFTQ_UNSUPPORTED, "d=%d above %d", d, kMaxD);
    if (nlist > kMaxList) return fail(IVFTQ_UNSUPPORTED, "nlist=%d above %d", nlist, kMaxList);
    Allocator al;
    al.alloc = alloc_fn; al.free = free_fn; al.ctx = alloc_ctx;
    ivftq_index* ix = new (std::nothrow) ivftq_index(al);
    if (!ix) return fail(IVFTQ_OOM, "host allocation failed");
    ix->d = d; ix->b = b; ix->nlist = nlist; ix->K = 1 << b;
    ix->dp = rot_dp(d);
    ix->lpad = round_up(nlist, 64);
    ix->words = code_words(b, d);
    ix->h_cb.resize(ix->K);
    ix->h_tau.resize(ix->K - 1);
    ix->h_pi.resize((size_t)d * d);
    ix->h_cent.assign((size_t)nlist * d, 0.f);
    ix->h_size.assign(nlist, 0);
    ix->h_cap.assign(nlist, 0);
    ix->h_off.assign(nlist, 0);
    ix->sign_bit = sign_bit;
    ivftq_status s = sign_bit ? ivftq_build_refined_codebook(b_stage1, d, ix->h_cb.data(), ix->h_tau.data())
                              : ivftq_build_codebook(b, d, ix->h_cb.data(), ix->h_tau.data());
    if (s == IVFTQ_OK) s = ivftq_haar_rotation(d, rotation_seed, ix->h_pi.data());
    if (s != IVFTQ_OK) { delete ix; return s; }
    auto guard = [&](hipError_t e, const char* what) -> ivftq_status {
        if (e == hipSuccess) return IVFTQ_OK;
        ivftq_status code = fail(e == hipErrorOutOfMemory ? IVFTQ_OOM : IVFTQ_HIP_ERROR, "%s: %s", what,
                                 hipGetErrorString(e));
        return code;
    };
    QuantiserGrid grid;
    if (!build_quantiser_grid(ix->h_tau, kMaxGridCells, grid)) {
        delete ix;
        return fail(IVFTQ_UNSUPPORTED, "quantiser grid for b=%d d=%d needs more than %d cells", b, d, kMaxGridCells);
    }
    ix->q_cells = grid.cells; ix->q_scale = grid.scale; ix->q_offset = grid.offset;
    std::vector<uint32_t> grid_words((size_t)2 * grid.cells);
    for (int i = 0; i < grid.cells; ++i) {
        std::memcpy(&grid_words[2 * i], &grid.boundary[i], 4);
        grid_words[2 * i + 1] = (uint32_t)grid.index[i];
    }
    std::vector<int32_t> zeros(nlist, 0);
    hipError_t e = ix->cent.ensure((size_t)ix->lpad * ix->dp * sizeof(float));
    if (e == hipSuccess) e = ix->cent_h.ensure((size_t)ix->lpad * ix->dp * sizeof(uint16_t));
    if (e == hipSuccess) e = ix->cent_l.ensure((size_t)ix->lpad * ix->dp * sizeof(uint16_t));
    if (e == hipSuccess) e = ix->bias.ensure((size_t)ix->lpad * sizeof(float));
    if (e == hipSuccess) e = ix->pi.ensure((size_t)ix->dp * ix->dp * sizeof(float));
    if (e == hipSuccess) e = ix->pi_h.ensure((size_t)ix->dp * ix->dp * sizeof(uint16_t));
    if (e == hipSuccess) e = ix->pi_l.ensure((size_t)ix->dp * ix->dp * sizeof(uint16_t));
    if (e == hipSuccess) e = ix->cb.ensure(256 * sizeof(float));
    if (e == hipSuccess) e = ix->q_grid.ensure(grid_words.size() * sizeof(uint32_t));
    if (e == hipSuccess) e = hipMemcpy(ix->q_grid.p, grid_words.data(), grid_words.size() * sizeof(uint32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = ix->d_size.ensure((size_t)nlist * sizeof(int32_t));
    if (e == hipSuccess) e = ix->d_off.ensure((size_t)nlist * sizeof(int64_t));
    if (e == hipSuccess) e = ix->w_flag.ensure(64);
    if (e == hipSuccess) e = hipMemcpy(ix->cb.p, ix->h_cb.data(), ix->K * sizeof(float), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(ix->d_size.p, zeros.data(), nlist * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemset(ix->d_off.p, 0, (size_t)nlist * sizeof(int64_t));
    if (e == hipSuccess) { void* unused = nullptr; e = scratch_on_current_device(&unused); }
    if ((s = guard(e, "device set-up")) != IVFTQ_OK) { delete ix; return s; }
    if ((s = upload_rotation(ix)) != IVFTQ_OK) { delete ix; return s; }
    *out = ix;
    return IVFTQ_OK;
}

ivftq_status ivftq_destroy(ivftq_index* index) {
    if (!index) return IVFTQ_OK;
    (void)hipDeviceSynchronize();
    delete index;
    return IVFTQ_OK;
}

ivftq_status ivftq_reset(ivftq_index* ix) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    std::fill(ix->h_size.begin(), ix->h_size.end(), 0);
    HIP_TRY(launch_fill_u32(ix->d_size.as<uint32_t>(), ix->nlist, 0u, ix->last_stream));
    HIP_TRY(hipStreamSynchronize(ix->last_stream));
    ix->ntotal = 0;
    return IVFTQ_OK;
}

ivftq_status ivftq_set_coarse(ivftq_index* ix, const float* centroids_host) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (!centroids_host) return fail(IVFTQ_INVALID_ARG, "centroids_host is NULL");
    if (ix->ntotal > 0) return fail(IVFTQ_BAD_STATE, "centroids cannot change once vectors are stored");
    for (size_t i = 0; i < (size_t)ix->nlist * ix->d; ++i)
        if (!std::isfinite(centroids_host[i])) return fail(IVFTQ_INVALID_ARG, "non-finite centroid value");
    std::copy(centroids_host, centroids_host + (size_t)ix->nlist * ix->d, ix->h_cent.begin());
    ivftq_status s = upload_coarse(ix);
    if (s == IVFTQ_OK) ix->has_coarse = true;
    return s;
}

ivftq_status ivftq_get_coarse(const ivftq_index* ix, float* centroids_host) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (!centroids_host) return fail(IVFTQ_INVALID_ARG, "centroids_host is NULL");
    if (!ix->has_coarse) return fail(IVFTQ_BAD_STATE, "no coarse centroids yet");
    std::copy(ix->h_cent.begin(), ix->h_cent.end(), centroids_host);
    return IVFTQ_OK;
}

ivftq_status ivftq_set_rotation(ivftq_index* ix, const float* pi_host) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (!pi_host) return fail(IVFTQ_INVALID_ARG, "pi_host is NULL");
    if (ix->ntotal > 0) return fail(IVFTQ_BAD_STATE, "rotation cannot change once vectors are stored");
    for (size_t i = 0; i < (size_t)ix->d * ix->d; ++i)
        if (!std::isfinite(pi_host[i])) return fail(IVFTQ_INVALID_ARG, "non-finite rotation entry");
    std::vector<float> previous = ix->h_pi;
    std::copy(pi_host, pi_host + (size_t)ix->d * ix->d, ix->h_pi.begin());
    ivftq_status s = upload_rotation(ix);
    if (s != IVFTQ_OK) ix->h_pi = previous;          // a rejected matrix leaves the index as it was
    return s;
}

ivftq_status ivftq_get_rotation(const ivftq_index* ix, float* pi_host) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (!pi_host) return fail(IVFTQ_INVALID_ARG, "pi_host is NULL");
    std::copy(ix->h_pi.begin(), ix->h_pi.end(), pi_host);
    return IVFTQ_OK;
}

ivftq_status ivftq_get_codebook(const ivftq_index* ix, float* centroids_out, float* boundaries_out) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (centroids_out) std::copy(ix->h_cb.begin(), ix->h_cb.end(), centroids_out);
    if (boundaries_out) std::copy(ix->h_tau.begin(), ix->h_tau.end(), boundaries_out);
    return IVFTQ_OK;
}

ivftq_status ivftq_set_search_mode(ivftq_index* ix, int mode) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (mode < 0 || mode > 2) return fail(IVFTQ_INVALID_ARG, "search mode %d outside [0, 2]", mode);
    ix->search_mode = mode;
    return IVFTQ_OK;
}

ivftq_status ivftq_set_metric(ivftq_index* ix, int metric) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (metric != IVFTQ_METRIC_COSINE && metric != IVFTQ_METRIC_IP && metric != IVFTQ_METRIC_L2)
        return fail(IVFTQ_INVALID_ARG, "metric %d is none of IVFTQ_METRIC_COSINE / _IP / _L2", metric);
    const bool raw_now = ix->metric != IVFTQ_METRIC_COSINE, raw_then = metric != IVFTQ_METRIC_COSINE;
    if (raw_now != raw_then && ix->ntotal > 0)
        return fail(IVFTQ_BAD_STATE, "vectors are stored %s their norms: the metric can only change between inner product and L2",
                    raw_now ? "with" : "without");
    if (raw_now != raw_then) {       // the (empty) lists are laid out again at the next append, with or without norms
        std::fill(ix->h_cap.begin(), ix->h_cap.end(), 0);
        ix->pool_slots = 0;
    }
    ix->metric = metric;
    return IVFTQ_OK;
}

ivftq_status ivftq_set_cascade_plane(ivftq_index* ix, int beta) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    const int b1 = ix->b - (ix->sign_bit ? 1 : 0);
    if (beta < 0 || beta > b1 || (beta != 0 && beta >= ix->b))
        return fail(IVFTQ_INVALID_ARG, "beta=%d: a plane of the top bits needs 1 <= beta <= %d Stage-1 bits and fewer bits than the %d stored (0 = none)",
                    beta, b1, ix->b);
    if (ix->ntotal > 0) return fail(IVFTQ_BAD_STATE, "the layout cannot change once vectors are stored");
    if (beta == ix->plane_beta) return IVFTQ_OK;
    ix->plane_beta = beta;
    ix->head_words = beta ? code_words(beta, ix->d) : 0;
    std::fill(ix->h_cap.begin(), ix->h_cap.end(), 0);      // the (empty) lists are laid out again at the next append
    ix->pool_slots = 0;
    return IVFTQ_OK;
}

ivftq_status ivftq_export_cascade_plane(const ivftq_index* ix, int list, uint8_t* head_codes_host) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (list < 0 || list >= ix->nlist || !head_codes_host) return fail(IVFTQ_INVALID_ARG, "bad list number or NULL output");
    if (!ix->plane_beta) return fail(IVFTQ_BAD_STATE, "the index keeps no plane of top bits");
    const int64_t n = ix->h_size[list];
    if (n == 0) return IVFTQ_OK;
    HIP_TRY(hipStreamSynchronize(ix->last_stream));
    const int64_t off = ix->h_off[list], nblk = (n + 63) / 64;
    const int hw = ix->head_words, beta = ix->plane_beta;
    std::vector<uint32_t> raw((size_t)nblk * hw * 64);
    HIP_TRY(hipMemcpy(raw.data(), ix->head.as<uint32_t>() + (off / 64) * hw * 64, raw.size() * sizeof(uint32_t), hipMemcpyDeviceToHost));
    const uint32_t mask = (1u << beta) - 1u;
    for (int64_t v = 0; v < n; ++v) {
        const uint32_t* blk = &raw[(size_t)(v / 64) * hw * 64 + (v % 64)];
        for (int j = 0; j < ix->d; ++j) {
            const int bit = j * beta, w = bit >> 5, sh = bit & 31;
            uint64_t two = blk[(size_t)w * 64];
            if (w + 1 < hw) two |= (uint64_t)blk[(size_t)(w + 1) * 64] << 32;
            head_codes_host[v * ix->d + j] = (uint8_t)((two >> sh) & mask);
        }
    }
    return IVFTQ_OK;
}

ivftq_status ivftq_export_norms(const ivftq_index* ix, int list, float* norms_host) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (list < 0 || list >= ix->nlist || !norms_host) return fail(IVFTQ_INVALID_ARG, "bad list number or NULL output");
    if (ix->metric == IVFTQ_METRIC_COSINE) return fail(IVFTQ_BAD_STATE, "the index keeps no norms (cosine metric)");
    const int64_t n = ix->h_size[list];
    if (n == 0) return IVFTQ_OK;
    HIP_TRY(hipStreamSynchronize(ix->last_stream));
    HIP_TRY(hipMemcpy(norms_host, ix->xnorm.as<float>() + ix->h_off[list], n * sizeof(float), hipMemcpyDeviceToHost));
    return IVFTQ_OK;
}

ivftq_status ivftq_set_workspace_limit(ivftq_index* ix, int64_t bytes) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (bytes < (1 << 20)) return fail(IVFTQ_INVALID_ARG, "workspace limit below 1 MiB");
    ix->ws_limit = bytes;
    return IVFTQ_OK;
}

ivftq_status ivftq_profile_enable(ivftq_index* ix, int on) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    for (const ProfRec& r : ix->prof) HIP_TRY(hipEventSynchronize(r.b));
    drop_profile(ix);
    ix->prof_on = on != 0;
    return IVFTQ_OK;
}

int ivftq_profile_kernel_count(void) { return P_COUNT; }

const char* ivftq_profile_kernel_name(int id) { return (id >= 0 && id < P_COUNT) ? kProfNames[id] : ""; }

ivftq_status ivftq_measure_mfma_rate(int random_operands, double* tflops_out) {
    if (!tflops_out) return fail(IVFTQ_INVALID_ARG, "tflops_out is NULL");
    int dev = 0, cus = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const int blocks = 2 * cus, iters = 2000;                 // two wavefronts per SIMD
    std::vector<uint16_t> h(4096 * 8);
    uint64_t s = 0x243F6A8885A308D3ull;
    for (auto& v : h) {
        s = s * 6364136223846793005ull + 1442695040888963407ull;
        // random sign and mantissa, exponent of values in [1, 64): finite, no subnormals
        const uint16_t bits = (uint16_t)(s >> 40);
        v = random_operands ? (uint16_t)((bits & 0x83FF) | (uint16_t)((15 + ((bits >> 10) % 6)) << 10)) : (uint16_t)0x3C00;
    }
    struct Scratch { DevBuf operands, out; ~Scratch() { operands.release(); out.release(); } } scratch;
    DevBuf& operands = scratch.operands;
    DevBuf& out = scratch.out;
    HIP_TRY(operands.ensure(h.size() * sizeof(uint16_t)));
    HIP_TRY(out.ensure((size_t)blocks * 256 * sizeof(float)));
    HIP_TRY(hipMemcpy(operands.p, h.data(), h.size() * sizeof(uint16_t), hipMemcpyHostToDevice));
    hipEvent_t e0, e1;
    HIP_TRY(hipEventCreate(&e0));
    HIP_TRY(hipEventCreate(&e1));
    HIP_TRY(launch_mfma_peak(operands.as<uint16_t>(), out.as<float>(), blocks, 20, nullptr));
    HIP_TRY(hipEventRecord(e0, nullptr));
    HIP_TRY(launch_mfma_peak(operands.as<uint16_t>(), out.as<float>(), blocks, iters, nullptr));
    HIP_TRY(hipEventRecord(e1, nullptr));
    HIP_TRY(hipEventSynchronize(e1));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, e0, e1));
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    const double flops = (double)blocks * 4 * iters * 32 * (2.0 * 32 * 32 * 16);
    *tflops_out = flops / (ms * 1e-3) / 1e12;
    return IVFTQ_OK;
}

ivftq_status ivftq_profile_read(ivftq_index* ix, double* ms_out, int64_t* launches_out) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (!ms_out || !launches_out) return fail(IVFTQ_INVALID_ARG, "output pointer is NULL");
    for (int i = 0; i < P_COUNT; ++i) { ms_out[i] = 0.0; launches_out[i] = 0; }
    for (const ProfRec& r : ix->prof) {
        float ms = 0.f;
        HIP_TRY(hipEventSynchronize(r.b));
        HIP_TRY(hipEventElapsedTime(&ms, r.a, r.b));
        ms_out[r.id] += ms;
        launches_out[r.id] += 1;
    }
    drop_profile(ix);
    return IVFTQ_OK;
}

int64_t ivftq_ntotal(const ivftq_index* ix) { return ix ? ix->ntotal : -1; }

int64_t ivftq_index_bytes(const ivftq_index* ix) {
    if (!ix) return -1;
    return ix->ntotal * ((int64_t)(ix->words + (ix->plane_beta ? ix->head_words : 0)) * 4 + 2 + 8 +
                         (ix->metric != IVFTQ_METRIC_COSINE ? 4 : 0));
}

ivftq_status ivftq_list_size(const ivftq_index* ix, int list, int64_t* n_out) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (list < 0 || list >= ix->nlist || !n_out) return fail(IVFTQ_INVALID_ARG, "bad list number or NULL output");
    *n_out = ix->h_size[list];
    return IVFTQ_OK;
}

ivftq_status ivftq_export_list(const ivftq_index* ix, int list, int64_t* ids_host, uint8_t* codes_host,
                               uint16_t* gamma_host) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (list < 0 || list >= ix->nlist) return fail(IVFTQ_INVALID_ARG, "list %d outside [0, %d)", list, ix->nlist);
    const int64_t n = ix->h_size[list];
    if (n == 0) return IVFTQ_OK;
    HIP_TRY(hipStreamSynchronize(ix->last_stream));
    const int64_t off = ix->h_off[list];
    if (ids_host)
        HIP_TRY(hipMemcpy(ids_host, ix->ids.as<int64_t>() + off, n * sizeof(int64_t), hipMemcpyDeviceToHost));
    if (gamma_host)
        HIP_TRY(hipMemcpy(gamma_host, ix->gamma.as<uint16_t>() + off, n * sizeof(uint16_t), hipMemcpyDeviceToHost));
    if (codes_host) {
        const int64_t nblk = (n + 63) / 64;
        std::vector<uint32_t> raw((size_t)nblk * ix->words * 64);
        HIP_TRY(hipMemcpy(raw.data(), ix->codes.as<uint32_t>() + (off / 64) * ix->words * 64,
                          raw.size() * sizeof(uint32_t), hipMemcpyDeviceToHost));
        const uint32_t maskK = (uint32_t)ix->K - 1;
        for (int64_t v = 0; v < n; ++v) {
            const uint32_t* blk = &raw[(size_t)(v / 64) * ix->words * 64 + (v % 64)];
            for (int j = 0; j < ix->d; ++j) {
                const int bit = j * ix->b, w = bit >> 5, sh = bit & 31;
                uint64_t two = blk[(size_t)w * 64];
                if (w + 1 < ix->words) two |= (uint64_t)blk[(size_t)(w + 1) * 64] << 32;
                codes_host[v * ix->d + j] = (uint8_t)((two >> sh) & maskK);
            }
        }
    }
    return IVFTQ_OK;
}

// ---------------------------------------------------------------------------------------------

ivftq_status ivftq_train_coarse(ivftq_index* ix, const float* x_dev, int64_t n, int niter,
                                const int64_t* init_rows_host, uint64_t seed, double* inertia_out,
                                void* stream) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (!x_dev) return fail(IVFTQ_INVALID_ARG, "x_dev is NULL");
    if (n < ix->nlist) return fail(IVFTQ_INVALID_ARG, "need at least nlist=%d training rows, got %lld", ix->nlist, (long long)n);
    if (niter < 0) return fail(IVFTQ_INVALID_ARG, "niter=%d is negative", niter);
    if (ix->ntotal > 0 && !ix->refreshing) return fail(IVFTQ_BAD_STATE, "centroids cannot change once vectors are stored");
    hipStream_t st = use_stream(ix, stream);
    const int L = ix->nlist, d = ix->d, pitch = ix->dp;

    std::vector<int64_t> init(L);
    if (init_rows_host) {
        std::unordered_set<int64_t> seen;
        for (int l = 0; l < L; ++l) {
            init[l] = init_rows_host[l];
            if (init[l] < 0 || init[l] >= n) return fail(IVFTQ_INVALID_ARG, "initial row %lld outside [0, n)", (long long)init[l]);
            if (!seen.insert(init[l]).second) return fail(IVFTQ_INVALID_ARG, "initial rows are not distinct");
        }
    } else {
        std::unordered_set<int64_t> seen;
        uint64_t s = seed ^ 0xA5A5A5A55A5A5A5Aull;
        for (int l = 0; l < L;) {
            const int64_t r = (int64_t)(splitmix(s) % (uint64_t)n);
            if (seen.insert(r).second) init[l++] = r;
        }
    }
    std::vector<int32_t> dst(L);
    std::iota(dst.begin(), dst.end(), 0);

    // The iterations run on tables of their own (t_*): the index keeps its centroids until training has succeeded.
    const size_t table = (size_t)ix->lpad * pitch;
    const int64_t seg_len = segment_length(n, L);
    const int nseg = (int)((n + seg_len - 1) / seg_len);
    HIP_TRY(ix->w_rows.ensure((size_t)L * sizeof(int64_t)));
    HIP_TRY(ix->w_dst.ensure((size_t)L * sizeof(int32_t)));
    HIP_TRY(ix->w_sums.ensure(table * sizeof(float)));
    HIP_TRY(ix->w_counts.ensure((size_t)ix->lpad * sizeof(uint32_t)));
    HIP_TRY(ix->w_zero.ensure((size_t)ix->lpad * sizeof(uint32_t)));
    HIP_TRY(ix->w_assign.ensure((size_t)n * sizeof(int32_t)));
    HIP_TRY(ix->w_best.ensure((size_t)n * sizeof(float)));
    HIP_TRY(ix->w_obj.ensure(sizeof(double)));
    HIP_TRY(ix->w_order.ensure((size_t)n * sizeof(int32_t)));
    HIP_TRY(ix->w_hist.ensure((size_t)nseg * L * sizeof(uint32_t)));
    HIP_TRY(ix->w_base.ensure((size_t)2 * L * sizeof(int64_t)));
    HIP_TRY(ix->t_cent.ensure(table * sizeof(float)));
    HIP_TRY(ix->t_cent_h.ensure(table * sizeof(uint16_t)));
    HIP_TRY(ix->t_cent_l.ensure(table * sizeof(uint16_t)));
    HIP_TRY(ix->t_bias.ensure((size_t)ix->lpad * sizeof(float)));
    float* cent = ix->t_cent.as<float>();
    float* bias = ix->t_bias.as<float>();
    uint32_t* counts_dev = ix->w_counts.as<uint32_t>();
    int64_t* cell_base = ix->w_base.as<int64_t>();

    HIP_TRY(launch_fill_u32(ix->t_cent.as<uint32_t>(), (int64_t)table, 0u, st));
    HIP_TRY(launch_fill_u32(ix->w_zero.as<uint32_t>(), ix->lpad, 0u, st));
    HIP_TRY(launch_fill_u32(ix->w_counts.as<uint32_t>(), ix->lpad, 0u, st));
    HIP_TRY(launch_fill_u32(ix->w_flag.as<uint32_t>(), 1, 0u, st));
    HIP_TRY(hipMemcpyAsync(ix->w_rows.p, init.data(), L * sizeof(int64_t), hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(ix->w_dst.p, dst.data(), L * sizeof(int32_t), hipMemcpyHostToDevice, st));
    HIP_TRY(launch_copy_rows_normalised(x_dev, d, ix->w_rows.as<int64_t>(), ix->w_dst.as<int32_t>(), L, cent, pitch, st));
    HIP_TRY(timed(ix, st, P_KMEANS_UPDATE, [&] { return launch_kmeans_update(cent, pitch, ix->w_sums.as<float>(), ix->w_zero.as<uint32_t>(),
                                 bias, L, ix->lpad, d, st); }));
    HIP_TRY(hipStreamSynchronize(st));

    std::vector<uint32_t> counts(L);
    std::vector<int32_t> h_assign;
    uint64_t rs = seed ^ 0x1234567887654321ull;
    double inertia = std::nan("");
    for (int it = 0; it < niter; ++it) {
        HIP_TRY(launch_split_rows(cent, (int64_t)table, ix->t_cent_h.as<uint16_t>(), ix->t_cent_l.as<uint16_t>(), st));
        HIP_TRY(timed(ix, st, P_ASSIGN, [&] { return launch_coarse(0, x_dev, n, d, ix->t_cent_h.as<uint16_t>(), ix->t_cent_l.as<uint16_t>(), pitch, bias, L, ix->lpad,
                              ix->w_assign.as<int32_t>(), ix->w_best.as<float>(), nullptr, 0,
                              ix->w_flag.as<int>(), st); }));
        // Sums per cell in a fixed order (two runs give the same bits): the rows are grouped by cell with the
        // stable counting sort of the append path, then one workgroup adds up the rows of a cell.
        HIP_TRY(timed(ix, st, P_SEG_HIST, [&] { return launch_segment_hist(ix->w_assign.as<int32_t>(), n, seg_len, nseg, L, ix->w_hist.as<uint32_t>(), st); }));
        HIP_TRY(timed(ix, st, P_SEG_SCAN, [&] { return launch_segment_scan(ix->w_hist.as<uint32_t>(), nseg, L, counts_dev, st); }));
        HIP_TRY(launch_exclusive_scan(counts_dev, L, cell_base, st));
        HIP_TRY(timed(ix, st, P_RANK, [&] { return launch_stable_rank(ix->w_assign.as<int32_t>(), n, seg_len, nseg, L, ix->w_hist.as<uint32_t>(), nullptr,
                                   nullptr, cell_base, ix->w_order.as<int32_t>(), nullptr, st); }));
        HIP_TRY(timed(ix, st, P_KMEANS_SUMS, [&] { return launch_kmeans_cell_sums(x_dev, d, ix->w_order.as<int32_t>(), cell_base, counts_dev, L,
                                        ix->w_sums.as<float>(), pitch, st); }));
        HIP_TRY(timed(ix, st, P_KMEANS_UPDATE, [&] { return launch_kmeans_update(cent, pitch, ix->w_sums.as<float>(), counts_dev, bias, L, ix->lpad, d, st); }));
        if (it == niter - 1) HIP_TRY(launch_inertia(ix->w_best.as<float>(), n, ix->w_obj.as<double>(), st));
        HIP_TRY(hipMemcpyAsync(counts.data(), ix->w_counts.p, L * sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        int flag = 0;
        HIP_TRY(hipMemcpyAsync(&flag, ix->w_flag.p, sizeof(int), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        if (flag) return fail(IVFTQ_ZERO_NORM, "a training row has zero or non-finite norm");
        if (it == niter - 1) HIP_TRY(hipMemcpy(&inertia, ix->w_obj.p, sizeof(double), hipMemcpyDeviceToHost));

        std::vector<int32_t> empty;
        for (int l = 0; l < L; ++l) if (counts[l] == 0) empty.push_back(l);
        if (!empty.empty()) {
            // re-seed each empty cell from a member of the largest cell
            const int big = (int)(std::max_element(counts.begin(), counts.end()) - counts.begin());
            h_assign.resize(n);
            HIP_TRY(hipMemcpy(h_assign.data(), ix->w_assign.p, n * sizeof(int32_t), hipMemcpyDeviceToHost));
            std::vector<int64_t> members;
            for (int64_t i = 0; i < n; ++i) if (h_assign[i] == big) members.push_back(i);
            std::vector<int64_t> rows(empty.size());
            for (size_t t = 0; t < empty.size(); ++t) rows[t] = members[splitmix(rs) % members.size()];
            HIP_TRY(hipMemcpy(ix->w_rows.p, rows.data(), rows.size() * sizeof(int64_t), hipMemcpyHostToDevice));
            HIP_TRY(hipMemcpy(ix->w_dst.p, empty.data(), empty.size() * sizeof(int32_t), hipMemcpyHostToDevice));
            HIP_TRY(launch_copy_rows_normalised(x_dev, d, ix->w_rows.as<int64_t>(), ix->w_dst.as<int32_t>(),
                                                (int)empty.size(), cent, pitch, st));
            HIP_TRY(timed(ix, st, P_KMEANS_UPDATE, [&] { return launch_kmeans_update(cent, pitch, ix->w_sums.as<float>(),
                                         ix->w_zero.as<uint32_t>(), bias, L, ix->lpad, d, st); }));
            HIP_TRY(hipStreamSynchronize(st));
        }
    }
    HIP_TRY(launch_normalise_centroids(cent, pitch, bias, L, d, st));
    std::vector<float> padded((size_t)L * pitch);
    HIP_TRY(hipMemcpyAsync(padded.data(), cent, padded.size() * sizeof(float), hipMemcpyDeviceToHost, st));
    // success: the index takes the new table over (same stream, so later calls on it see the new centroids)
    HIP_TRY(hipMemcpyAsync(ix->cent.p, cent, table * sizeof(float), hipMemcpyDeviceToDevice, st));
    HIP_TRY(launch_fill_u32(ix->bias.as<uint32_t>(), ix->lpad, 0u, st));
    HIP_TRY(refresh_split(ix, st));
    HIP_TRY(hipStreamSynchronize(st));
    for (int l = 0; l < L; ++l)
        std::memcpy(&ix->h_cent[(size_t)l * d], &padded[(size_t)l * pitch], sizeof(float) * d);
    ix->has_coarse = true;
    if (inertia_out) *inertia_out = inertia;
    return IVFTQ_OK;
}

// ---------------------------------------------------------------------------------------------

namespace {

// Steps shared by every append: count the rows of each list, make room, and give each row its
// slot (list order = arrival order).  `assign` holds a cell number per row; with zero_norm_flag
// the flag word written by the coarse kernel is checked too.  Nothing is modified on failure.
ivftq_status place_rows(ivftq_index* ix, const int32_t* assign, int64_t n, bool zero_norm_flag, bool want_order,
                        std::vector<int64_t>& need, hipStream_t st) {
    const int L = ix->nlist;
    const int64_t seg_len = segment_length(n, L);
    const int nseg = (int)((n + seg_len - 1) / seg_len);
    HIP_TRY(ix->w_hist.ensure((size_t)nseg * L * sizeof(uint32_t)));
    HIP_TRY(ix->w_count.ensure((size_t)L * sizeof(uint32_t)));
    HIP_TRY(ix->w_base.ensure((size_t)2 * L * sizeof(int64_t)));
    if (want_order) HIP_TRY(ix->w_order.ensure((size_t)n * sizeof(int2)));
    HIP_TRY(timed(ix, st, P_SEG_HIST, [&] { return launch_segment_hist(assign, n, seg_len, nseg, L, ix->w_hist.as<uint32_t>(), st); }));
    HIP_TRY(timed(ix, st, P_SEG_SCAN, [&] { return launch_segment_scan(ix->w_hist.as<uint32_t>(), nseg, L, ix->w_count.as<uint32_t>(), st); }));
    // pinned staging: [L u32 batch counts | 16 B flag | 2L i64 bases | L i32 list sizes]
    const size_t off_flag = (size_t)round_up(L, 4) * sizeof(uint32_t), off_base = off_flag + 16;
    const size_t off_size = off_base + (size_t)2 * L * sizeof(int64_t);
    HIP_TRY(ix->pin.ensure(off_size + (size_t)L * sizeof(int32_t)));
    char* pin = static_cast<char*>(ix->pin.p);
    const uint32_t* count = reinterpret_cast<const uint32_t*>(pin);
    const int* flag = reinterpret_cast<const int*>(pin + off_flag);
    int64_t* base = reinterpret_cast<int64_t*>(pin + off_base);   // [0, L): first free slot of each list; [L, 2L): first position in the batch order
    HIP_TRY(hipMemcpyAsync(pin, ix->w_count.p, L * sizeof(uint32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(pin + off_flag, ix->w_flag.p, sizeof(int), hipMemcpyDeviceToHost, st));
    // The one host synchronisation of an append: the host decides here whether the lists have room.
    // It also means every earlier use of the staging buffer by this stream has completed.
    HIP_TRY(hipStreamSynchronize(st));
    if (zero_norm_flag && *flag)
        return fail(IVFTQ_ZERO_NORM, "an input row has zero or non-finite norm; nothing was appended");
    int64_t placed = 0;
    for (int l = 0; l < L; ++l) placed += count[l];
    if (placed != n) return fail(IVFTQ_INVALID_ARG, "%lld rows carry a cell number outside [0, nlist)", (long long)(n - placed));

    need.resize(L);
    for (int l = 0; l < L; ++l) need[l] = (int64_t)ix->h_size[l] + count[l];
    for (int l = 0; l < L; ++l)
        if (need[l] > INT32_MAX) return fail(IVFTQ_UNSUPPORTED, "list %d would exceed 2^31-1 vectors", l);
    ivftq_status s = ensure_capacity(ix, need, st);
    if (s != IVFTQ_OK) return s;
    int64_t run = 0;
    for (int l = 0; l < L; ++l) {
        base[l] = ix->h_off[l] + ix->h_size[l];
        base[L + l] = run;
        run += count[l];
    }
    HIP_TRY(hipMemcpyAsync(ix->w_base.p, base, (size_t)2 * L * sizeof(int64_t), hipMemcpyHostToDevice, st));
    // encode_add takes the rows in list order and derives their slots from the position (order_cell); add_encoded
    // packs in input order and needs the slot of every row
    HIP_TRY(timed(ix, st, P_RANK, [&] { return launch_stable_rank(assign, n, seg_len, nseg, L, ix->w_hist.as<uint32_t>(), ix->w_base.as<int64_t>(),
                               want_order ? nullptr : ix->w_slot.as<int64_t>(), ix->w_base.as<int64_t>() + L,
                               nullptr, want_order ? ix->w_order.as<int2>() : nullptr, st); }));
    return IVFTQ_OK;
}

// Records the new list sizes; the device copy is updated in stream order (no host wait).
ivftq_status commit_rows(ivftq_index* ix, const std::vector<int64_t>& need, int64_t n, hipStream_t st) {
    const int L = ix->nlist;
    const size_t off_size = (size_t)round_up(L, 4) * sizeof(uint32_t) + 16 + (size_t)2 * L * sizeof(int64_t);
    int32_t* sizes = reinterpret_cast<int32_t*>(static_cast<char*>(ix->pin.p) + off_size);   // allocated by place_rows
    for (int l = 0; l < L; ++l) sizes[l] = ix->h_size[l] = (int32_t)need[l];
    HIP_TRY(hipMemcpyAsync(ix->d_size.p, sizes, (size_t)L * sizeof(int32_t), hipMemcpyHostToDevice, st));
    ix->ntotal += n;
    return IVFTQ_OK;
}

// Coarse assignment of n rows (Algorithm "Encode", nearest centroid by inner product): screening pass
// plus the exact pass over the rows it left undecided.  w_flag[0] = a row without a usable norm,
// w_flag[1] = number of undecided rows.
constexpr int64_t kScreenShareRows = 1 << 19;     // beyond this the row tiles alone fill the chip
ivftq_status assign_rows(ivftq_index* ix, const float* x_dev, int64_t n, int32_t* assign, hipStream_t st) {
    // keys (8 bytes each) first, then the row numbers
    HIP_TRY(ix->w_undecided.ensure((size_t)n * (sizeof(unsigned long long) + sizeof(int32_t))));
    // short batches share the centroid stages out over several workgroups and need room for the partial results
    float* part = nullptr;
    if (n <= kScreenShareRows) {
        HIP_TRY(ix->w_part.ensure((size_t)n * kScreenMaxShares * 3 * sizeof(float)));
        part = ix->w_part.as<float>();
    }
    HIP_TRY(launch_fill_u32(ix->w_flag.as<uint32_t>(), 2, 0u, st));
    HIP_TRY(timed(ix, st, P_ASSIGN, [&] {
        return launch_coarse_screened(x_dev, n, ix->d, ix->cent_h.as<uint16_t>(), ix->cent_l.as<uint16_t>(), ix->dp,
                                      ix->nlist, ix->lpad, assign, ix->w_flag.as<int>(),
                                      reinterpret_cast<int32_t*>(ix->w_undecided.as<unsigned long long>() + n),
                                      ix->w_undecided.as<unsigned long long>(), ix->w_flag.as<int>() + 1, part, st);
    }));
    return IVFTQ_OK;
}

}  // namespace

ivftq_status ivftq_scan_stats(ivftq_index* ix, int64_t* queries_out, int64_t* redone_out, int64_t* max_candidates_out,
                              double* mean_candidates_out, void* stream) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    hipStream_t st = use_stream(ix, stream);
    const int64_t n = ix->last_batched_queries;
    if (queries_out) *queries_out = n;
    if (redone_out) *redone_out = 0;
    if (max_candidates_out) *max_candidates_out = 0;
    if (mean_candidates_out) *mean_candidates_out = 0.0;
    if (n <= 0) return IVFTQ_OK;
    std::vector<int32_t> cnt(n);
    int32_t gated = 0;
    HIP_TRY(hipMemcpyAsync(cnt.data(), ix->w_ccnt.p, n * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(&gated, ix->w_gate.p, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    int64_t mx = 0;
    double sum = 0.0;
    for (int32_t c : cnt) { mx = std::max<int64_t>(mx, c); sum += c; }
    if (redone_out) *redone_out = gated;
    if (max_candidates_out) *max_candidates_out = mx;
    if (mean_candidates_out) *mean_candidates_out = sum / (double)n;
    return IVFTQ_OK;
}

ivftq_status ivftq_assign_undecided(ivftq_index* ix, int64_t* count_out, void* stream) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (!count_out) return fail(IVFTQ_INVALID_ARG, "count_out is NULL");
    hipStream_t st = use_stream(ix, stream);
    int v = 0;
    HIP_TRY(hipMemcpyAsync(&v, ix->w_flag.as<int>() + 1, sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    *count_out = v;
    return IVFTQ_OK;
}

ivftq_status ivftq_encode_only(ivftq_index* ix, const float* x_dev, int64_t n, int32_t* assign_dev,
                               uint8_t* codes_dev, uint16_t* gamma_dev, void* stream) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (n < 0) return fail(IVFTQ_INVALID_ARG, "n=%lld is negative", (long long)n);
    if (n == 0) return IVFTQ_OK;
    if (!x_dev) return fail(IVFTQ_INVALID_ARG, "x_dev is NULL");
    if (!ix->has_coarse) return fail(IVFTQ_BAD_STATE, "coarse centroids not trained or set");
    if (n > ((int64_t)1 << 31) - 1) return fail(IVFTQ_UNSUPPORTED, "more than 2^31-1 rows in one call");
    hipStream_t st = use_stream(ix, stream);
    HIP_TRY(ix->w_assign.ensure((size_t)n * sizeof(int32_t)));
    int32_t* assign = assign_dev ? assign_dev : ix->w_assign.as<int32_t>();
    { ivftq_status sa = assign_rows(ix, x_dev, n, assign, st); if (sa != IVFTQ_OK) return sa; }
    if (codes_dev || gamma_dev) {
        EncodeArgs a{};
        a.x = x_dev; a.n = n; a.d = ix->d; a.b = ix->b;
        a.cent = ix->cent.as<float>(); a.cent_pitch = ix->dp;
        a.pi_h = ix->pi_h.as<uint16_t>(); a.pi_l = ix->pi_l.as<uint16_t>();
        a.q_grid = ix->q_grid.as<float2>(); a.q_cells = ix->q_cells; a.q_scale = ix->q_scale; a.q_offset = ix->q_offset;
        a.assign = assign;
        a.codes_flat = codes_dev; a.gamma_flat = gamma_dev;
        HIP_TRY(timed(ix, st, P_ENCODE, [&] { return launch_encode(1, a, st); }));
    }
    return IVFTQ_OK;
}

ivftq_status ivftq_encode_only_noalloc(ivftq_index* ix, const float* x_dev, int64_t n, int32_t* assign_dev,
                                       uint8_t* codes_dev, uint16_t* gamma_dev, void* stream) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (n < 0) return fail(IVFTQ_INVALID_ARG, "n=%lld is negative", (long long)n);
    if (n > kNoAllocRows)
        return fail(IVFTQ_UNSUPPORTED, "n=%lld above the %lld rows the static scratch of ivftq_encode_only_noalloc holds",
                    (long long)n, (long long)kNoAllocRows);
    if (n == 0) return IVFTQ_OK;
    if (!x_dev) return fail(IVFTQ_INVALID_ARG, "x_dev is NULL");
    if (!ix->has_coarse) return fail(IVFTQ_BAD_STATE, "coarse centroids not trained or set");
    hipStream_t st = use_stream(ix, stream);
    void* base = nullptr;
    HIP_TRY(scratch_on_current_device(&base));
    unsigned char* sp = static_cast<unsigned char*>(base);
    int* flags = reinterpret_cast<int*>(sp);                                          // [0] bad norm, [1] undecided rows
    unsigned long long* row_key = reinterpret_cast<unsigned long long*>(sp + 256);
    int32_t* row_list = reinterpret_cast<int32_t*>(sp + 256 + (size_t)kNoAllocRows * 8);
    int32_t* own_assign = reinterpret_cast<int32_t*>(sp + 256 + (size_t)kNoAllocRows * 12);
    int32_t* assign = assign_dev ? assign_dev : own_assign;
    // the scratch keeps the previous call's contents: the counters start from zero, the keys and row numbers
    // are written before they are read (one entry per listed row)
    HIP_TRY(launch_fill_u32(reinterpret_cast<uint32_t*>(flags), 2, 0u, st));
    HIP_TRY(launch_coarse_screened(x_dev, n, ix->d, ix->cent_h.as<uint16_t>(), ix->cent_l.as<uint16_t>(), ix->dp,
                                   ix->nlist, ix->lpad, assign, flags, row_list, row_key, flags + 1, nullptr, st));
    if (codes_dev || gamma_dev) {
        EncodeArgs a{};
        a.x = x_dev; a.n = n; a.d = ix->d; a.b = ix->b;
        a.cent = ix->cent.as<float>(); a.cent_pitch = ix->dp;
        a.pi_h = ix->pi_h.as<uint16_t>(); a.pi_l = ix->pi_l.as<uint16_t>();
        a.q_grid = ix->q_grid.as<float2>(); a.q_cells = ix->q_cells; a.q_scale = ix->q_scale; a.q_offset = ix->q_offset;
        a.assign = assign;
        a.codes_flat = codes_dev; a.gamma_flat = gamma_dev;
        HIP_TRY(launch_encode(1, a, st));
    }
    return IVFTQ_OK;
}

ivftq_status ivftq_encode_add(ivftq_index* ix, const float* x_dev, int64_t n, const int64_t* ids_dev,
                              void* stream) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (n < 0) return fail(IVFTQ_INVALID_ARG, "n=%lld is negative", (long long)n);
    if (n == 0) return IVFTQ_OK;
    if (!x_dev) return fail(IVFTQ_INVALID_ARG, "x_dev is NULL");
    if (!ix->has_coarse) return fail(IVFTQ_BAD_STATE, "coarse centroids not trained or set");
    if (n > ((int64_t)1 << 31) - 1) return fail(IVFTQ_UNSUPPORTED, "more than 2^31-1 rows in one call");
    hipStream_t st = use_stream(ix, stream);
    const int L = ix->nlist;

    // 1. coarse assignment
    HIP_TRY(ix->w_assign.ensure((size_t)n * sizeof(int32_t)));
    { ivftq_status sa = assign_rows(ix, x_dev, n, ix->w_assign.as<int32_t>(), st); if (sa != IVFTQ_OK) return sa; }

    // 2.-4. room for the new vectors and the stable position of every row
    std::vector<int64_t> need;
    ivftq_status s = place_rows(ix, ix->w_assign.as<int32_t>(), n, true, true, need, st);
    if (s != IVFTQ_OK) return s;
    // 5. rotate / quantise / pack straight into the lists
    EncodeArgs a{};
    a.x = x_dev; a.n = n; a.d = ix->d; a.b = ix->b;
    a.cent = ix->cent.as<float>(); a.cent_pitch = ix->dp;
    a.pi_h = ix->pi_h.as<uint16_t>(); a.pi_l = ix->pi_l.as<uint16_t>();
        a.q_grid = ix->q_grid.as<float2>(); a.q_cells = ix->q_cells; a.q_scale = ix->q_scale; a.q_offset = ix->q_offset;
    a.store = ix->store();
    a.order_cell = ix->w_order.as<int2>();     // rows in list order: neighbouring lanes store to neighbouring slots
    a.list_base = ix->w_base.as<int64_t>();
    a.batch_base = ix->w_base.as<int64_t>() + L;
    a.labels = ids_dev; a.label_base = ix->ntotal;
    HIP_TRY(timed(ix, st, P_ENCODE, [&] { return launch_encode(0, a, st); }));
    return commit_rows(ix, need, n, st);
}

namespace {

ivftq_status add_encoded_rows(ivftq_index* ix, int64_t n, const int32_t* assign_dev, const uint8_t* codes_dev,
                              const uint16_t* gamma_dev, const float* xnorm_dev, const int64_t* ids_dev, void* stream) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (n < 0) return fail(IVFTQ_INVALID_ARG, "n=%lld is negative", (long long)n);
    if (n == 0) return IVFTQ_OK;
    if (!assign_dev || !codes_dev || !gamma_dev) return fail(IVFTQ_INVALID_ARG, "input pointer is NULL");
    if (!ix->has_coarse) return fail(IVFTQ_BAD_STATE, "coarse centroids not trained or set");
    if (n > ((int64_t)1 << 31) - 1) return fail(IVFTQ_UNSUPPORTED, "more than 2^31-1 rows in one call");
    hipStream_t st = use_stream(ix, stream);
    HIP_TRY(ix->w_slot.ensure((size_t)n * sizeof(int64_t)));
    HIP_TRY(launch_fill_u32(ix->w_flag.as<uint32_t>(), 1, 0u, st));
    std::vector<int64_t> need;
    ivftq_status s = place_rows(ix, assign_dev, n, false, false, need, st);
    if (s != IVFTQ_OK) return s;
    HIP_TRY(timed(ix, st, P_PACK, [&] { return launch_pack_scatter(codes_dev, gamma_dev, xnorm_dev, ids_dev, ix->ntotal, ix->w_slot.as<int64_t>(), n, ix->d,
                                ix->b, ix->store(), st); }));
    return commit_rows(ix, need, n, st);
}

}  // namespace

ivftq_status ivftq_add_encoded(ivftq_index* ix, int64_t n, const int32_t* assign_dev, const uint8_t* codes_dev,
                               const uint16_t* gamma_dev, const int64_t* ids_dev, void* stream) {
    if (ix && ix->metric != IVFTQ_METRIC_COSINE)
        return fail(IVFTQ_BAD_STATE, "the index keeps a raw metric: its vectors need their norms (ivftq_add_encoded_raw)");
    return add_encoded_rows(ix, n, assign_dev, codes_dev, gamma_dev, nullptr, ids_dev, stream);
}

ivftq_status ivftq_add_encoded_raw(ivftq_index* ix, int64_t n, const int32_t* assign_dev, const uint8_t* codes_dev,
                                   const uint16_t* gamma_dev, const float* xnorm_dev, const int64_t* ids_dev, void* stream) {
    if (ix && ix->metric == IVFTQ_METRIC_COSINE)
        return fail(IVFTQ_BAD_STATE, "the index keeps no norms (cosine metric): use ivftq_add_encoded");
    if (ix && n > 0 && !xnorm_dev) return fail(IVFTQ_INVALID_ARG, "xnorm_dev is NULL");
    return add_encoded_rows(ix, n, assign_dev, codes_dev, gamma_dev, xnorm_dev, ids_dev, stream);
}

// ---------------------------------------------------------------------------------------------

// ---- adaptive coarse refresh (Section "Adaptive coarse refresh") ----------------------------------

namespace {

struct ScopedBuf {
    DevBuf b;
    explicit ScopedBuf(const Allocator* a) : b(a) {}
    ~ScopedBuf() { b.release(); }
};

// x_out[row] = reconstruction of the vector at list-order position row, ids_out its label
ivftq_status reconstruct_all(ivftq_index* ix, float* x_out, int64_t* ids_out, hipStream_t st) {
    const int L = ix->nlist;
    std::vector<int64_t> off(L);
    int64_t run = 0;
    int max_list = 0;
    for (int l = 0; l < L; ++l) { off[l] = run; run += ix->h_size[l]; max_list = std::max(max_list, (int)ix->h_size[l]); }
    HIP_TRY(ix->w_base.ensure((size_t)2 * L * sizeof(int64_t)));
    HIP_TRY(hipMemcpyAsync(ix->w_base.p, off.data(), (size_t)L * sizeof(int64_t), hipMemcpyHostToDevice, st));
    HIP_TRY(launch_reconstruct(ix->store(), L, max_list, ix->cent.as<float>(), ix->dp, ix->pi.as<float>(), ix->dp,
                               ix->cb.as<float>(), ix->d, ix->b, ix->w_base.as<int64_t>(), x_out, ids_out, st));
    HIP_TRY(hipStreamSynchronize(st));      // `off` is pageable host memory
    return IVFTQ_OK;
}

// Empties the lists and appends the n rows again (against whatever centroids the index now has).
ivftq_status readd_all(ivftq_index* ix, const float* x, const int64_t* ids, int64_t n, hipStream_t st) {
    std::fill(ix->h_size.begin(), ix->h_size.end(), 0);
    HIP_TRY(launch_fill_u32(ix->d_size.as<uint32_t>(), ix->nlist, 0u, st));
    ix->ntotal = 0;
    ivftq_status s = ivftq_encode_add(ix, x, n, ids, st);
    if (s == IVFTQ_OK) HIP_TRY(hipStreamSynchronize(st));   // x and ids are about to be freed by the caller
    return s;
}

}  // namespace

ivftq_status ivftq_reconstruct(ivftq_index* ix, float* x_out_dev, int64_t* ids_out_dev, void* stream) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (!x_out_dev) return fail(IVFTQ_INVALID_ARG, "x_out_dev is NULL");
    if (ix->ntotal == 0) return IVFTQ_OK;
    return reconstruct_all(ix, x_out_dev, ids_out_dev, use_stream(ix, stream));
}

ivftq_status ivftq_reencode(ivftq_index* ix, const float* centroids_host, void* stream) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (!centroids_host) return fail(IVFTQ_INVALID_ARG, "centroids_host is NULL");
    if (!ix->has_coarse) return fail(IVFTQ_BAD_STATE, "no coarse centroids yet");
    if (ix->metric != IVFTQ_METRIC_COSINE && ix->ntotal > 0)
        return fail(IVFTQ_UNSUPPORTED, "re-encoding does not carry the stored norms of a raw-metric index");
    for (size_t i = 0; i < (size_t)ix->nlist * ix->d; ++i)
        if (!std::isfinite(centroids_host[i])) return fail(IVFTQ_INVALID_ARG, "non-finite centroid value");
    hipStream_t st = use_stream(ix, stream);
    const int64_t n = ix->ntotal;
    ScopedBuf xh(&ix->alloc), lab(&ix->alloc);
    if (n > 0) {
        HIP_TRY(xh.b.ensure((size_t)n * ix->d * sizeof(float)));
        HIP_TRY(lab.b.ensure((size_t)n * sizeof(int64_t)));
        ivftq_status s = reconstruct_all(ix, xh.b.as<float>(), lab.b.as<int64_t>(), st);
        if (s != IVFTQ_OK) return s;
    }
    std::copy(centroids_host, centroids_host + (size_t)ix->nlist * ix->d, ix->h_cent.begin());
    ivftq_status s = upload_coarse(ix);
    if (s != IVFTQ_OK || n == 0) return s;
    return readd_all(ix, xh.b.as<float>(), lab.b.as<int64_t>(), n, st);
}

ivftq_status ivftq_refresh_coarse(ivftq_index* ix, int64_t sample_n, int niter, const int64_t* init_rows_host,
                                  uint64_t seed, double* inertia_out, void* stream) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (!ix->has_coarse || ix->ntotal == 0) return fail(IVFTQ_BAD_STATE, "nothing stored to refresh from");
    if (ix->metric != IVFTQ_METRIC_COSINE)
        return fail(IVFTQ_UNSUPPORTED, "re-encoding does not carry the stored norms of a raw-metric index");
    if (sample_n < ix->nlist) return fail(IVFTQ_INVALID_ARG, "sample of %lld below nlist=%d", (long long)sample_n, ix->nlist);
    if (niter < 0) return fail(IVFTQ_INVALID_ARG, "niter=%d is negative", niter);
    hipStream_t st = use_stream(ix, stream);
    const int L = ix->nlist;
    const int64_t n = ix->ntotal;
    ScopedBuf xh(&ix->alloc), lab(&ix->alloc), sample(&ix->alloc), rows(&ix->alloc);
    HIP_TRY(xh.b.ensure((size_t)n * ix->d * sizeof(float)));
    HIP_TRY(lab.b.ensure((size_t)n * sizeof(int64_t)));
    ivftq_status s = reconstruct_all(ix, xh.b.as<float>(), lab.b.as<int64_t>(), st);
    if (s != IVFTQ_OK) return s;
    // stratified sample: list l gives round(sample_n * n_l / n) of its vectors (at least one, at most
    // all), evenly spaced in storage order
    std::vector<int64_t> pick;
    int64_t first = 0;
    for (int l = 0; l < L; ++l) {
        const int64_t n_l = ix->h_size[l];
        if (n_l > 0) {
            const int64_t s_l = std::min<int64_t>(n_l, std::max<int64_t>(1, (2 * sample_n * n_l + n) / (2 * n)));
            for (int64_t t = 0; t < s_l; ++t) pick.push_back(first + (t * n_l) / s_l);
        }
        first += n_l;
    }
    if ((int64_t)pick.size() < L) return fail(IVFTQ_INVALID_ARG, "the sample holds %lld vectors, fewer than nlist=%d", (long long)pick.size(), L);
    HIP_TRY(rows.b.ensure(pick.size() * sizeof(int64_t)));
    HIP_TRY(sample.b.ensure(pick.size() * ix->d * sizeof(float)));
    HIP_TRY(hipMemcpyAsync(rows.b.p, pick.data(), pick.size() * sizeof(int64_t), hipMemcpyHostToDevice, st));
    HIP_TRY(launch_gather_rows(xh.b.as<float>(), ix->d, rows.b.as<int64_t>(), (int64_t)pick.size(), sample.b.as<float>(), st));
    HIP_TRY(hipStreamSynchronize(st));
    ix->refreshing = true;
    s = ivftq_train_coarse(ix, sample.b.as<float>(), (int64_t)pick.size(), niter, init_rows_host, seed, inertia_out, st);
    ix->refreshing = false;
    if (s != IVFTQ_OK) return s;              // a failed training leaves centroids and lists as they were
    return readd_all(ix, xh.b.as<float>(), lab.b.as<int64_t>(), n, st);
}

namespace {

ivftq_status check_query_args(const ivftq_index* ix, const float* q_dev, int64_t nq, int nprobe) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    if (nq < 0) return fail(IVFTQ_INVALID_ARG, "nq=%lld is negative", (long long)nq);
    if (nq > 0 && !q_dev) return fail(IVFTQ_INVALID_ARG, "q_dev is NULL");
    if (nprobe < 1 || nprobe > ix->nlist) return fail(IVFTQ_INVALID_ARG, "nprobe=%d outside [1, nlist=%d]", nprobe, ix->nlist);
    if (nprobe > kMaxK) return fail(IVFTQ_UNSUPPORTED, "nprobe=%d above %d", nprobe, kMaxK);
    if (!ix->has_coarse) return fail(IVFTQ_BAD_STATE, "coarse centroids not trained or set");
    return IVFTQ_OK;
}

// coarse scores for `count` queries starting at q, then the nprobe best cells of each
ivftq_status coarse_and_probe(ivftq_index* ix, const float* q, int64_t count, int nprobe, int32_t* probe,
                              float* coarse, hipStream_t st) {
    const int64_t ldS = round_up(ix->nlist, 4);
    HIP_TRY(timed(ix, st, P_COARSE_SCORES, [&] { return launch_coarse(1, q, count, ix->d, ix->cent_h.as<uint16_t>(), ix->cent_l.as<uint16_t>(), ix->dp, nullptr, ix->nlist, ix->lpad, nullptr,
                          nullptr, ix->w_S.as<float>(), ldS, ix->w_flag.as<int>(), st); }));
    SelectArgs sa{};
    sa.vals = ix->w_S.as<float>(); sa.stride = ldS; sa.rows = count; sa.k = nprobe; sa.m_fixed = ix->nlist;
    sa.out_vals = coarse; sa.out_i32 = probe;
    HIP_TRY(timed(ix, st, P_SELECT_PROBE, [&] { return launch_select(0, sa, st); }));
    return IVFTQ_OK;
}

}  // namespace

ivftq_status ivftq_rerank(int d, const float* q_dev, int64_t nq, const float* x_dev, int64_t n_rows,
                          const int64_t* cand_ids_dev, int r, int k, float* scores_dev, int64_t* ids_dev, void* stream) {
    if (d < 1 || d > kMaxD) return fail(IVFTQ_INVALID_ARG, "d=%d outside [1, %d]", d, kMaxD);
    if (nq < 0 || n_rows < 0) return fail(IVFTQ_INVALID_ARG, "negative count");
    if (r < 1 || r > kMaxK) return fail(IVFTQ_INVALID_ARG, "r=%d outside [1, %d]", r, kMaxK);
    if (k < 1 || k > r) return fail(IVFTQ_INVALID_ARG, "k=%d outside [1, r=%d]", k, r);
    if (nq == 0) return IVFTQ_OK;
    if (!q_dev || !x_dev || !cand_ids_dev || !scores_dev || !ids_dev) return fail(IVFTQ_INVALID_ARG, "pointer is NULL");
    RerankArgs a{q_dev, x_dev, n_rows, d, cand_ids_dev, r, k, scores_dev, ids_dev};
    HIP_TRY(launch_rerank(a, nq, static_cast<hipStream_t>(stream)));
    return IVFTQ_OK;
}

ivftq_status ivftq_coarse_probe(ivftq_index* ix, const float* q_dev, int64_t nq, int nprobe,
                                int32_t* probe_dev, float* coarse_dev, void* stream) {
    ivftq_status s = check_query_args(ix, q_dev, nq, nprobe);
    if (s != IVFTQ_OK) return s;
    if (nq == 0) return IVFTQ_OK;
    hipStream_t st = use_stream(ix, stream);
    const int64_t ldS = round_up(ix->nlist, 4);
    const int64_t qc = std::max<int64_t>(1, std::min<int64_t>(nq, ix->ws_limit / (ldS * 4)));
    HIP_TRY(ix->w_S.ensure((size_t)qc * ldS * sizeof(float)));
    for (int64_t q0 = 0; q0 < nq; q0 += qc) {
        const int64_t cnt = std::min(qc, nq - q0);
        s = coarse_and_probe(ix, q_dev + q0 * ix->d, cnt, nprobe, probe_dev ? probe_dev + q0 * nprobe : nullptr,
                             coarse_dev ? coarse_dev + q0 * nprobe : nullptr, st);
        if (s != IVFTQ_OK) return s;
    }
    return IVFTQ_OK;
}

}  // extern "C"

namespace {

// The search proper.  cb: the 2^b reconstruction values the scans use; labels: label of every slot, or
// null to return slot numbers instead (pass 1 of the cascade search, which needs to find the codes again).
ivftq_status search_core(ivftq_index* ix, const float* q_dev, int64_t nq, int nprobe, int k, const float* cb,
                         const ListStore& codes_store, int bits, const int64_t* labels, float* scores_dev,
                         int64_t* ids_dev, void* stream) {
    ivftq_status s = check_query_args(ix, q_dev, nq, nprobe);
    if (s != IVFTQ_OK) return s;
    if (k < 1) return fail(IVFTQ_INVALID_ARG, "k=%d below 1", k);
    if (k > kMaxK) return fail(IVFTQ_UNSUPPORTED, "k=%d above %d", k, kMaxK);
    if (nq == 0) return IVFTQ_OK;
    if (!scores_dev || !ids_dev) return fail(IVFTQ_INVALID_ARG, "output pointer is NULL");
    hipStream_t st = use_stream(ix, stream);

    // upper bound of candidates per query: the nprobe largest lists
    std::vector<int32_t> sizes(ix->h_size);
    std::partial_sort(sizes.begin(), sizes.begin() + nprobe, sizes.end(), std::greater<int32_t>());
    int64_t m_bound = 0;
    for (int p = 0; p < nprobe; ++p) m_bound += sizes[p];
    if (m_bound > INT32_MAX - 4) return fail(IVFTQ_UNSUPPORTED, "more than 2^31 candidates per query");
    const int64_t m_stride = std::max<int64_t>(4, round_up64(m_bound, 4));
    const int64_t ldS = round_up(ix->nlist, 4);

    // Scan strategy.  Streaming: a row of workgroups per query walks its probed lists, every score written,
    // exact selection.  Batched: pairs regrouped by list and scanned on the matrix cores against a
    // threshold from each query's nearest lists.  The streaming scan's time follows the bytes it reads, once
    // per query; the batched path reads a list once per 128 queries, so its time follows the part of the
    // index the call touches, but it is a chain of about fourteen kernels with a fixed cost of its own.
    // Batched when the streamed bytes exceed kBatchedGain times the touched bytes plus kBatchedFixedBytes
    // (measured crossovers with nprobe 32 / 32 / 64 at 1M x 128, 10M x 96, 10M x 200: about 200, 380 and
    // 170 queries, i.e. 0.41 / 1.5 / 2.7 GB streamed against an index of 0.066 / 0.58 / 1.04 GB).  Mode 2
    // asks for the batched path whatever the size of the call.
    constexpr double kBatchedGain = 2.3, kBatchedFixedBytes = 0.25e9;
    const int tq = batch_tile_queries(ix->d, bits);
    const int metric = ix->metric;      // a raw metric ranks by a per-vector transform of the estimate: streaming scan only
    const double vec_bytes = (double)codes_store.words * 4 + 2;
    const double index_bytes = (double)ix->ntotal * vec_bytes;
    const double streamed = (double)nq * nprobe * ((double)ix->ntotal / ix->nlist) * vec_bytes;
    const double touched = index_bytes * std::min(1.0, (double)nq * nprobe / ix->nlist);
    const bool batched = tq > 0 && nprobe > 1 && ix->search_mode != 1 && metric == IVFTQ_METRIC_COSINE &&
                         (ix->search_mode == 2 || streamed >= kBatchedGain * touched + kBatchedFixedBytes);
    const int cap = std::min(2048, std::max(512, 16 * k));
    // error bound of a residual sum taken from the leading float16 parts alone (threshold pass)
    float cmax = 0.f;
    for (float v : ix->h_cb) cmax = std::max(cmax, std::fabs(v));
    const float kappa = screen_kappa(ix->d, cmax);
    // Score rows.  The batched path stores scores of the dense prefix only (it stops at the first list that
    // brings it to max(k, k*T/cap) vectors, so it is shorter than that plus the largest list); full-length
    // rows are needed for the queries redone exactly, which take turns in gate_rows rows of the same buffer.
    // The streaming path stores every score.  Queries per pass: as many as the workspace limit allows, since
    // every pass walks every probed list again.
    const int64_t need_max = std::max<int64_t>(k, (kPrefixFactorX2 * (int64_t)k * m_bound + 2 * cap - 1) / (2 * cap));
    const int64_t row_stride = batched ? std::min<int64_t>(m_stride, round_up64(need_max + sizes[0], 4)) : m_stride;
    int64_t qc = ix->ws_limit / (4 * std::max(row_stride, ldS));
    qc = std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(qc, nq), 32768));
    const int64_t gate_rows = std::max<int64_t>(1, std::min<int64_t>(qc, ix->ws_limit / (4 * m_stride)));
    const int64_t score_floats = batched ? std::max(qc * row_stride, gate_rows * m_stride) : qc * m_stride;

    HIP_TRY(ix->w_S.ensure((size_t)qc * ldS * sizeof(float)));
    HIP_TRY(ix->w_scores.ensure((size_t)score_floats * sizeof(float)));
    HIP_TRY(ix->w_probe.ensure((size_t)qc * nprobe * sizeof(int32_t)));
    HIP_TRY(ix->w_coarse.ensure((size_t)qc * nprobe * sizeof(float)));
    HIP_TRY(ix->w_candoff.ensure((size_t)qc * (nprobe + 1) * sizeof(int32_t)));
    HIP_TRY(ix->w_z.ensure((size_t)qc * ix->dp * sizeof(float)));
    if (metric) HIP_TRY(ix->w_qnorm.ensure((size_t)qc * sizeof(float)));
    const int64_t n_pairs = qc * nprobe;
    if (batched) {
        HIP_TRY(ix->w_zh.ensure((size_t)qc * ix->dp * sizeof(uint16_t)));
        HIP_TRY(ix->w_zl.ensure((size_t)qc * ix->dp * sizeof(uint16_t)));
        HIP_TRY(ix->w_first.ensure((size_t)qc * sizeof(int32_t)));
        HIP_TRY(ix->w_fscores.ensure((size_t)qc * k * sizeof(float)));
        HIP_TRY(ix->w_fids.ensure((size_t)qc * k * sizeof(int64_t)));
        HIP_TRY(ix->w_pairs.ensure((size_t)n_pairs * sizeof(int32_t)));
        HIP_TRY(ix->w_count.ensure((size_t)4 * ix->nlist * sizeof(uint32_t)));
        HIP_TRY(ix->w_pairoff.ensure((size_t)(2 * ix->nlist + 1) * sizeof(int64_t)));
        HIP_TRY(ix->w_tileoff.ensure((size_t)(2 * ix->nlist + 1) * sizeof(int32_t)));
        HIP_TRY(ix->w_cscore.ensure((size_t)qc * cap * sizeof(float)));
        HIP_TRY(ix->w_cslot.ensure((size_t)qc * cap * sizeof(int64_t)));
        HIP_TRY(ix->w_ccnt.ensure((size_t)qc * sizeof(int32_t)));
        HIP_TRY(ix->w_gate.ensure((size_t)(qc + 1) * sizeof(int32_t)));
    }
    // Streaming path with so few queries that one wavefront per score row would leave the chip idle (the
    // selection then takes longer than the scan): select per (query, list) first.  Needs what the
    // one-wavefront kernel takes: k <= 64 and lists and survivor rows within its reach.
    const bool two_step = !batched && nq <= 64 && k <= 64 && nprobe > 1 && sizes[0] <= 16384 && (int64_t)nprobe * k <= 16384;
    if (two_step) {
        HIP_TRY(ix->w_stage_s.ensure((size_t)qc * nprobe * k * sizeof(float)));
        HIP_TRY(ix->w_stage_i.ensure((size_t)qc * nprobe * k * sizeof(int64_t)));
    }

    for (int64_t q0 = 0; q0 < nq; q0 += qc) {
        const int64_t cnt = std::min(qc, nq - q0);
        const float* q = q_dev + q0 * ix->d;
        s = coarse_and_probe(ix, q, cnt, nprobe, ix->w_probe.as<int32_t>(), ix->w_coarse.as<float>(), st);
        if (s != IVFTQ_OK) return s;
        EncodeArgs ea{};
        ea.x = q; ea.n = cnt; ea.d = ix->d; ea.b = ix->b;
        ea.pi_h = ix->pi_h.as<uint16_t>(); ea.pi_l = ix->pi_l.as<uint16_t>(); ea.zout = ix->w_z.as<float>();
        if (batched) { ea.zh_out = ix->w_zh.as<uint16_t>(); ea.zl_out = ix->w_zl.as<uint16_t>(); }
        if (metric) ea.norm_out = ix->w_qnorm.as<float>();
        HIP_TRY(timed(ix, st, P_ROTATE_Q, [&] { return launch_encode(2, ea, st); }));
        int32_t* first = batched ? ix->w_first.as<int32_t>() : nullptr;
        HIP_TRY(timed(ix, st, P_CAND_OFF, [&] {
            return launch_cand_offsets(ix->w_probe.as<int32_t>(), cnt, nprobe, ix->d_size.as<int32_t>(),
                                       ix->w_candoff.as<int32_t>(), k, cap, first,
                                       batched ? ix->w_ccnt.as<int32_t>() : nullptr, batched ? ix->w_gate.as<int32_t>() : nullptr, st); }));
        auto stream_scan = [&](const int32_t* gate, int gate_begin, int blocks_per_query, int slices = 1) {
            return launch_list_scan(ix->w_z.as<float>(), ix->dp, ix->d, bits, cb,
                                    ix->w_probe.as<int32_t>(), ix->w_coarse.as<float>(),
                                    ix->w_candoff.as<int32_t>(), nprobe, codes_store, 0, cnt,
                                    ix->w_scores.as<float>(), m_stride, nullptr, gate, gate_begin, (int)gate_rows,
                                    blocks_per_query, slices, metric, ix->w_qnorm.as<float>(), st);
        };
        SelectArgs sa{};
        sa.vals = ix->w_scores.as<float>(); sa.stride = m_stride; sa.rows = cnt; sa.k = k;
        sa.cand_off = ix->w_candoff.as<int32_t>(); sa.probe = ix->w_probe.as<int32_t>(); sa.np = nprobe;
        sa.q_begin = 0;
        sa.list_off = ix->d_off.as<int64_t>(); sa.ids = labels;
        sa.out_vals = scores_dev + q0 * k; sa.out_i64 = ids_dev + q0 * k;
        sa.m_bound = (int)m_stride;

        if (!batched) {
            ix->last_batched_queries = 0;
            // Slices.  A call that reads more bytes than the packed index holds reads lists again and again, but
            // the index (580 MB at 10M x 96) is larger than the 256 MB memory-side cache, so little of it would
            // still be there.  Every list is therefore dealt out in rounds of 256 vectors to `slices` workgroups
            // that the launch runs one slice after the other: each slice covers about kStreamSliceBytes of the
            // index, which stay cached while all queries pass over them (10M x 96, 4096 queries: scan 3.37 ->
            // 2.69 ms with 4 slices; 2 slices, 290 MB each, gain nothing; rounds of 64 vectors lose the gain).
            const int64_t typical = std::max<int64_t>(1, ix->ntotal / ix->nlist * nprobe);     // candidates per query
            const int64_t bytes_per_vec = (int64_t)codes_store.words * 4 + 2 + (metric ? 4 : 0);
            const int64_t index_bytes = ix->ntotal * bytes_per_vec;
            int64_t slices = 1;
            if (cnt * typical * bytes_per_vec > index_bytes)
                slices = std::max<int64_t>(1, std::min<int64_t>(64, (index_bytes + kStreamSliceBytes - 1) / kStreamSliceBytes));
            // workgroups per query and slice: each builds the query's table once and walks its share of the
            // probes; fewer per query as the batch grows, as long as the launch still fills the chip
            const int per_query = (int)std::min<int64_t>(nprobe, std::max<int64_t>(1, kStreamWorkgroups / (cnt * slices)));
            // a handful of queries: one workgroup per (query, list) leaves most of the chip idle and each walks
            // its list in a dozen rounds, so the lists are split until about 2048 workgroups are in the launch
            slices = std::max(slices, std::min<int64_t>(16, 2048 / ((int64_t)per_query * cnt)));
            // and, while a share of a typical list still fills two rounds, until about 8192 are (64 queries at
            // 10M x 96: scan 0.100 -> 0.070 ms)
            slices = std::max(slices, std::min<int64_t>(kStreamWorkgroups / ((int64_t)per_query * cnt), ix->ntotal / ix->nlist / 512));
            HIP_TRY(timed(ix, st, P_LIST_SCAN, [&] { return stream_scan(nullptr, 0, per_query, (int)slices); }));
            if (two_step) {
                // a handful of rows: one wavefront per (query, list) first, then one per query over the survivors
                SelectArgs s_a = sa, s_b = sa;
                s_a.rows = cnt * nprobe; s_a.m_bound = sizes[0];
                s_a.out_vals = ix->w_stage_s.as<float>(); s_a.out_i64 = ix->w_stage_i.as<int64_t>();
                s_b.vals = ix->w_stage_s.as<float>(); s_b.stride = (int64_t)nprobe * k; s_b.m_fixed = nprobe * k;
                s_b.lab_in = ix->w_stage_i.as<int64_t>();
                HIP_TRY(timed(ix, st, P_SELECT_TOPK, [&] { return launch_select(2, s_a, st); }));
                HIP_TRY(timed(ix, st, P_SELECT_TOPK, [&] { return launch_select(3, s_b, st); }));
            } else {
                HIP_TRY(timed(ix, st, P_SELECT_TOPK, [&] { return launch_select(1, sa, st); }));
            }
            HIP_TRY(launch_metric_finish(scores_dev + q0 * k, cnt, k, metric, ix->w_qnorm.as<float>(), st));
            continue;
        }

        // 1. (query, probe) pairs bucketed by list; the nearest lists of each query in their own buckets
        ix->last_batched_queries = cnt;
        const int64_t np_items = cnt * nprobe;
        HIP_TRY(timed(ix, st, P_PAIR_GROUP, [&] {
            hipError_t e = launch_pair_grouping(ix->w_probe.as<int32_t>(), first, cnt, nprobe, ix->nlist, tq,
                                                ix->w_count.as<uint32_t>(), ix->w_count.as<uint32_t>() + 2 * ix->nlist,
                                                ix->w_pairoff.as<int64_t>(), ix->w_tileoff.as<int32_t>(),
                                                ix->w_pairs.as<int32_t>(), st);
            return e; }));
        BatchScanArgs ba{};
        ba.zh = ix->w_zh.as<uint16_t>(); ba.zl = ix->w_zl.as<uint16_t>(); ba.z_pitch = ix->dp;
        ba.cb = cb;
        ba.pairs = ix->w_pairs.as<int32_t>(); ba.pair_off = ix->w_pairoff.as<int64_t>();
        ba.tile_off = ix->w_tileoff.as<int32_t>();
        ba.coarse = ix->w_coarse.as<float>();
        ba.store = codes_store; ba.np = nprobe; ba.L = ix->nlist;
        ba.cand_score = ix->w_cscore.as<float>(); ba.cand_slot = ix->w_cslot.as<int64_t>();
        ba.cand_cnt = ix->w_ccnt.as<int32_t>(); ba.cap = cap;
        ba.acc0 = kappa * kSplitScale * kSplitScale;
        ba.scores = ix->w_scores.as<float>(); ba.m_stride = row_stride; ba.cand_off = ix->w_candoff.as<int32_t>();
        const int max_tiles = (int)(np_items / tq) + ix->nlist;
        // 2. every score of the nearest lists, then their top-k: the k-th is the query's threshold
        ba.dense = 1; ba.bucket_lo = 0; ba.bucket_hi = ix->nlist;
        HIP_TRY(timed(ix, st, P_BATCH_FIRST, [&] { return launch_batch_scan(ba, ix->d, bits, max_tiles, st); }));
        SelectArgs s1 = sa;
        s1.p_limit = first; s1.out_vals = ix->w_fscores.as<float>(); s1.out_i64 = ix->w_fids.as<int64_t>();
        s1.stride = row_stride; s1.m_bound = (int)row_stride;
        HIP_TRY(timed(ix, st, P_SELECT_TOPK, [&] { return launch_select(1, s1, st); }));
        // 3. the other lists against the thresholds
        ba.dense = 0; ba.bucket_lo = ix->nlist; ba.bucket_hi = 2 * ix->nlist;
        ba.thresh = ix->w_fscores.as<float>() + (k - 1); ba.thresh_stride = k;
        HIP_TRY(timed(ix, st, P_BATCH_SCAN, [&] { return launch_batch_scan(ba, ix->d, bits, max_tiles, st); }));
        // 4. merge; a query whose candidate list overflowed is redone by the exact streaming scan
        MergeArgs ma{};
        ma.first_scores = ix->w_fscores.as<float>(); ma.first_ids = ix->w_fids.as<int64_t>();
        ma.cand_score = ix->w_cscore.as<float>(); ma.cand_slot = ix->w_cslot.as<int64_t>();
        ma.cand_cnt = ix->w_ccnt.as<int32_t>(); ma.cap = cap; ma.ids = labels;
        ma.kappa = kappa;
        ma.z = ix->w_z.as<float>(); ma.z_pitch = ix->dp; ma.d = ix->d; ma.b = bits; ma.cb = cb;
        ma.coarse = ix->w_coarse.as<float>(); ma.np = nprobe; ma.store = codes_store;
        ma.k = k; ma.out_scores = scores_dev + q0 * k; ma.out_ids = ids_dev + q0 * k;
        ma.gate = ix->w_gate.as<int32_t>();
        HIP_TRY(timed(ix, st, P_MERGE, [&] { return launch_merge(ma, cnt, st); }));
        SelectArgs s2 = sa;
        s2.gate = ix->w_gate.as<int32_t>(); s2.gate_rows = (int)gate_rows;
        for (int64_t g0 = 0; g0 < cnt; g0 += gate_rows) {
            s2.gate_begin = (int)g0;
            HIP_TRY(timed(ix, st, P_LIST_SCAN, [&] { return stream_scan(ix->w_gate.as<int32_t>(), (int)g0, 8); }));
            HIP_TRY(timed(ix, st, P_SELECT_TOPK, [&] { return launch_select(1, s2, st); }));
        }
    }
    return IVFTQ_OK;
}

}  // namespace

extern "C" {

ivftq_status ivftq_search(ivftq_index* ix, const float* q_dev, int64_t nq, int nprobe, int k,
                          float* scores_dev, int64_t* ids_dev, void* stream) {
    if (check_index(ix)) return IVFTQ_INVALID_ARG;
    return search_core(ix, q_dev, nq, nprobe, k, ix->cb.as<float>(), ix->store(), ix->b, ix->ids.as<int64_t>(), scores_dev, ids_dev, stream);
}

ivftq_status ivftq_build_coarsened_codebook(int b, int sign_bit, int d, int beta, float* values_out) {
    if (!values_out) return fail(IVFTQ_INVALID_ARG, "values_out is NULL");
    std::vector<double> lv, bd;
    const bool ok = sign_bit ? build_refined_codebook(b, d, lv, bd) : build_codebook(b, d, lv, bd);
    if (!ok) return fail(IVFTQ_INVALID_ARG, "no codebook for b=%d d=%d", b, d);
    if (beta < 1 || beta > b) return fail(IVFTQ_INVALID_ARG, "beta=%d outside [1, %d]", beta, b);
    std::vector<double> out;
    if (!build_coarsened_levels(d, lv, bd, beta, out)) return fail(IVFTQ_INVALID_ARG, "no coarsened codebook for these parameters");
    for (size_t i = 0; i < out.size(); ++i) values_out[i] = (float)out[i];
    return IVFTQ_OK;
}

ivftq_status ivftq_search_cascade(ivftq_index* ix, const float* q_dev, int64_t nq, int nprobe, int k, int beta,
                                  int n_keep, float* scores_dev, int64_t* ids_dev, void* stream) {
    ivftq_status s = check_query_args(ix, q_dev, nq, nprobe);
    if (s != IVFTQ_OK) return s;
    if (ix->metric != IVFTQ_METRIC_COSINE) return fail(IVFTQ_UNSUPPORTED, "the cascade search ranks by the cosine estimate only");
    const int b1 = ix->b - (ix->sign_bit ? 1 : 0);
    if (beta < 1 || beta > b1) return fail(IVFTQ_INVALID_ARG, "beta=%d outside [1, %d]", beta, b1);
    if (k < 1 || k > n_keep) return fail(IVFTQ_INVALID_ARG, "k=%d outside [1, n_keep=%d]", k, n_keep);
    if (n_keep > kMaxK) return fail(IVFTQ_UNSUPPORTED, "n_keep=%d above %d", n_keep, kMaxK);
    if (nq == 0) return IVFTQ_OK;
    if (!scores_dev || !ids_dev) return fail(IVFTQ_INVALID_ARG, "output pointer is NULL");
    hipStream_t st = use_stream(ix, stream);

    // Pass 1 ranks by the top beta bits of every code.  With a plane of exactly those bits the scan reads the plane
    // (beta-bit codes, the coarsened codebook as their table); otherwise it reads the full codes through a table
    // whose entry e holds the value of the merged bin e >> (bits - beta).  Both give the same scores.
    const bool plane = ix->plane_beta == beta;
    const int key = plane ? -beta : beta;
    if (ix->cascade_beta != key) {
        std::vector<double> lv(ix->h_cb.begin(), ix->h_cb.end()), bd(ix->h_tau.begin(), ix->h_tau.end()), cc;
        if (!build_coarsened_levels(ix->d, lv, bd, beta, cc)) return fail(IVFTQ_INVALID_ARG, "no coarsened codebook for these parameters");
        std::vector<float> table(ix->K);
        for (int e = 0; e < ix->K; ++e) table[e] = plane ? (e < (1 << beta) ? (float)cc[e] : 0.f) : (float)cc[e >> (ix->b - beta)];
        HIP_TRY(ix->cb_cascade.ensure((size_t)ix->K * sizeof(float)));
        HIP_TRY(hipMemcpyAsync(ix->cb_cascade.p, table.data(), table.size() * sizeof(float), hipMemcpyHostToDevice, st));
        HIP_TRY(hipStreamSynchronize(st));       // table is a local
        ix->cascade_beta = key;
    }
    HIP_TRY(ix->w_keep.ensure((size_t)nq * n_keep * sizeof(int64_t)));
    HIP_TRY(ix->w_keep_scores.ensure((size_t)nq * n_keep * sizeof(float)));
    // pass 1: the ordinary search on the coarsened values, n_keep slots per query
    s = plane ? search_core(ix, q_dev, nq, nprobe, n_keep, ix->cb_cascade.as<float>(), ix->head_store(), beta, nullptr,
                            ix->w_keep_scores.as<float>(), ix->w_keep.as<int64_t>(), stream)
              : search_core(ix, q_dev, nq, nprobe, n_keep, ix->cb_cascade.as<float>(), ix->store(), ix->b, nullptr,
                            ix->w_keep_scores.as<float>(), ix->w_keep.as<int64_t>(), stream);
    if (s != IVFTQ_OK) return s;
    // pass 2: the kept candidates on the full codes.  Probes, coarse terms and rotated queries are
    // recomputed per chunk by search_core, so they are produced once more here for all queries.
    HIP_TRY(ix->w_probe.ensure((size_t)nq * nprobe * sizeof(int32_t)));
    HIP_TRY(ix->w_coarse.ensure((size_t)nq * nprobe * sizeof(float)));
    HIP_TRY(ix->w_z.ensure((size_t)nq * ix->dp * sizeof(float)));
    const int64_t ldS = round_up(ix->nlist, 4);
    int64_t qc = std::max<int64_t>(1, std::min<int64_t>(ix->ws_limit / (4 * ldS), std::min<int64_t>(nq, 32768)));
    HIP_TRY(ix->w_S.ensure((size_t)qc * ldS * sizeof(float)));
    for (int64_t q0 = 0; q0 < nq; q0 += qc) {
        const int64_t cnt = std::min(qc, nq - q0);
        s = coarse_and_probe(ix, q_dev + q0 * ix->d, cnt, nprobe, ix->w_probe.as<int32_t>() + q0 * nprobe,
                             ix->w_coarse.as<float>() + q0 * nprobe, st);
        if (s != IVFTQ_OK) return s;
    }
    EncodeArgs ea{};
    ea.x = q_dev; ea.n = nq; ea.d = ix->d; ea.b = ix->b;
    ea.pi_h = ix->pi_h.as<uint16_t>(); ea.pi_l = ix->pi_l.as<uint16_t>(); ea.zout = ix->w_z.as<float>();
    HIP_TRY(timed(ix, st, P_ROTATE_Q, [&] { return launch_encode(2, ea, st); }));
    CascadeArgs ca{};
    ca.z = ix->w_z.as<float>(); ca.z_pitch = ix->dp; ca.d = ix->d; ca.b = ix->b;
    ca.cb = ix->cb.as<float>();
    ca.probe = ix->w_probe.as<int32_t>(); ca.coarse = ix->w_coarse.as<float>(); ca.np = nprobe;
    ca.store = ix->store(); ca.ids = ix->ids.as<int64_t>();
    ca.cand = ix->w_keep.as<int64_t>(); ca.n_keep = n_keep; ca.k = k;
    ca.out_scores = scores_dev; ca.out_ids = ids_dev;
    HIP_TRY(timed(ix, st, P_CASCADE, [&] { return launch_cascade_rescore(ca, nq, st); }));
    return IVFTQ_OK;
}

}  // extern "C"
