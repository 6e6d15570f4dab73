// Residual rotation, Lloyd-Max quantisation and bit-packing in one kernel (Section "Architecture",
// Indexing: r = x~ - c~_l, rotate by Pi, normalise Pi r, quantise each coordinate; Bit accounting:
// b*d code bits and a float16 norm per vector), plus the query-side rotation z = Pi q~ (Section
// "Architecture", Search).
//
// The rotation is a d x d contraction on the matrix cores (v_mfma_f32_32x32x16_f16 on split float16
// operands with float32 accumulation, see split_f16.h).  A wavefront owns 32*R rows; their unit
// residuals r^ = r/|r| are the right-hand operand held in registers, 32-row tiles of Pi stream
// through a double-buffered LDS stage as the left-hand operand (one barrier per tile, the next
// tile's global loads in flight during the multiplies).  In tile t a lane holds, for one row, the
// rotated coordinates 32t + 8g + 4*half + {0..3}.
//
// Pi is orthogonal, so |Pi r| = |r| and the quantiser input Pi r / |Pi r| is Pi r^ itself; the
// library only accepts rotations whose defect |Pi Pi^T - I| is at float32 rounding level, which
// bounds the difference at 1e-6 of the coordinate.  Each tile is therefore quantised as soon as its
// multiplies are done and no rotated vector is ever held whole.
//
// Quantiser: code = #{i : rho >= tau_i} through the uniform-grid index of host_math.h (one
// independent 8-byte LDS lookup and one comparison per coordinate, any b; the comparison is taken on
// the accumulator against the boundary times 2^20, an exact rescaling).  Codes are packed in registers
// four at a time.  With b = 4 the two lanes of a row hold the two halves of each 32-bit word and
// exchange them with one lane swap, with b = 8 a lane holds whole words; both store straight to the
// row's slot.  Any other b (and an index that keeps the plane of top bits) merges the pieces into the
// row's words in LDS with ds_or first.  Rows are processed in list order, which makes the stores of
// a wavefront land in consecutive slots.
#include <hip/hip_fp16.h>

#include <algorithm>

#include "kernels.h"
#include "split_f16.h"

namespace ivftq {

namespace {

template <int DP>
struct EncCfg {
    static constexpr int KB = DP / 16;
    static constexpr int NT = DP / 32;
    static constexpr int LDH = DP + 8;                     // halves per LDS row of the Pi tile
    static constexpr int R = DP <= 64 ? 2 : 1;   // 32-row tiles per wavefront (register budget)
    static constexpr int stage_halves = 2 * 32 * LDH;      // hi and lo parts of one 32-row tile of Pi
    static constexpr int PF = (32 * (DP / 8) + 255) / 256; // 16-byte pieces of one part a thread stages
    static constexpr size_t pi_bytes = (size_t)2 * stage_halves * sizeof(uint16_t);
};

inline int pack_pitch(int words) { return (words + 1) | 1; }   // odd and > words: room for a spill word

template <int DP>
size_t encode_lds_bytes(int mode, int pack_b, int cells, int words, int head_words) {
    size_t bytes = EncCfg<DP>::pi_bytes;
    if (mode != 2) bytes += (size_t)cells * 8;
    if (mode == 0 && pack_b == 0) bytes += (size_t)4 * 32 * EncCfg<DP>::R * pack_pitch(words) * 4;
    if (mode == 0 && pack_b == 0 && head_words > 0) bytes += (size_t)4 * 32 * EncCfg<DP>::R * pack_pitch(head_words) * 4;
    return bytes;
}

// MODE 0: encode and store into the lists; 1: encode into flat arrays; 2: rotate queries only.  A template
// parameter, so that each instantiation carries its own path only.  PACK_B (mode 0): 4 or 8 = the index
// stores that many bits per coordinate and no plane of top bits, words are put together in registers;
// 0 = any b, through LDS.
template <int DP, int MODE, int PACK_B>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2)))
void k_encode(EncodeArgs a, int flags) {
    constexpr int mode = MODE;
    constexpr bool via_lds = MODE == 0 && PACK_B == 0;
    using Cfg = EncCfg<DP>;
    constexpr int KB = Cfg::KB, NT = Cfg::NT, R = Cfg::R, LDH = Cfg::LDH, PF = Cfg::PF;
    extern __shared__ unsigned char lds_raw[];
    uint16_t* stage = reinterpret_cast<uint16_t*>(lds_raw);                    // [2][hi,lo][32][LDH]
    float2* grid_s = reinterpret_cast<float2*>(lds_raw + Cfg::pi_bytes);        // [cells] (boundary, index bits)
    uint32_t* pack_s = reinterpret_cast<uint32_t*>(lds_raw + Cfg::pi_bytes + (size_t)a.q_cells * 8);

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, half = lane >> 5, j = lane & 31;
    const int vec4 = flags & 1;          // rows of x can be read 16 bytes at a time
    const bool codes4 = flags & 2;       // rows of codes_flat can be written 4 bytes at a time
    const int d = a.d, b = PACK_B ? PACK_B : a.b;
    const int words = a.store.words;
    const int pitch = (words + 1) | 1;
    const int head_words = (via_lds && a.store.head) ? a.store.head_words : 0;   // top-bit plane kept as well
    const int pitch_h = (head_words + 1) | 1;
    const int beta = b - a.store.head_shift;
    const int64_t pos0 = ((int64_t)blockIdx.x * 4 + wave) * (32 * R);

    // ---- this lane's rows: x~, residual against the assigned centroid, gamma, split unit residual
    half8 bh[R][KB], bl[R][KB];
    int64_t row_of[R];
    int cell_of[R];
    float gamma[R], xnorm[R];
    bool valid[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int64_t pos = pos0 + 32 * r + j;
        valid[r] = pos < a.n;
        row_of[r] = valid[r] ? pos : 0;
        cell_of[r] = -1;
        if (mode == 0 && valid[r]) {
            const int2 oc = a.order_cell[pos];
            row_of[r] = oc.x;
            cell_of[r] = oc.y;
        } else if (mode == 1 && valid[r]) {
            cell_of[r] = a.assign[pos];
        }
        // A position past the end reads row 0 and an unassigned row reads centroid 0: what they compute
        // is never stored, so nothing here is masked by validity.
        float v[KB][8];
        load_row_blocks<KB>(a.x + row_of[r] * (int64_t)d, true, d, vec4, half, v);
        const float n2 = row_norm2<KB>(v);
        const bool good = (n2 > 0.f) && (n2 < __builtin_inff());
        const float inv_n = good ? 1.f / sqrtf(n2) : 0.f;   // one division per row, then multiplies
        gamma[r] = 0.f;
        xnorm[r] = good ? sqrtf(n2) : 0.f;
        if (mode == 2 && a.norm_out && valid[r] && half == 0) a.norm_out[row_of[r]] = xnorm[r];
        float to_unit = inv_n;
        if (mode != 2) {
            const int cell = cell_of[r];
            float c[KB][8];
            load_row_blocks<KB>(a.cent + (int64_t)(cell < 0 ? 0 : cell) * a.cent_pitch, true, DP, 1, half, c);
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int e = 0; e < 8; ++e) v[kb][e] = fmaf(v[kb][e], inv_n, -c[kb][e]);      // r = x~ - c~
            const float g = sqrtf(row_norm2<KB>(v));
            // The rotation acts on the unit residual: the quantiser input does not depend on the scale
            // of r, and a unit vector keeps the split float16 form accurate however small r is.
            to_unit = (g > 1e-30f) ? 1.f / g : 0.f;   // a zero residual quantises as rho = 0
            gamma[r] = cell >= 0 ? g : 0.f;
        }
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int e = 0; e < 8; ++e) v[kb][e] *= to_unit;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                _Float16 h, l;
                split_scaled(v[kb][e], h, l);
                bh[r][kb][e] = h;
                bl[r][kb][e] = l;
            }
    }

    // ---- LDS set-up: quantiser grid, cleared packing words, first tile of Pi
    if (mode != 2)
        for (int e = tid; e < a.q_cells; e += 256) {      // boundaries in accumulator units
            const float2 ent = a.q_grid[e];
            grid_s[e] = make_float2(ent.x * (kSplitScale * kSplitScale), ent.y);
        }
    uint32_t* my_pack = pack_s + (size_t)wave * (32 * R) * pitch;
    uint32_t* my_head = pack_s + (size_t)4 * (32 * R) * pitch + (size_t)wave * (32 * R) * pitch_h;
    if (via_lds) {
        for (int e = lane; e < 32 * R * pitch; e += 64) my_pack[e] = 0u;
        if (head_words)
            for (int e = lane; e < 32 * R * pitch_h; e += 64) my_head[e] = 0u;
    }

    // Staging of one 32-row tile of Pi: thread `tid` moves the 16-byte pieces tid, tid + 256, ...
    uint4 pf_h[PF], pf_l[PF];
#define IVFTQ_FETCH_TILE(T)                                                                          \
    _Pragma("unroll") for (int p = 0; p < PF; ++p) {                                                 \
        int e_ = tid + 256 * p;                                                                      \
        e_ = e_ < 32 * (DP / 8) ? e_ : 32 * (DP / 8) - 1;      /* surplus threads re-read the last piece */ \
        const int64_t src_ = (int64_t)((T) * 32 + e_ / (DP / 8)) * DP + (e_ % (DP / 8)) * 8;         \
        pf_h[p] = *reinterpret_cast<const uint4*>(a.pi_h + src_);                                    \
        pf_l[p] = *reinterpret_cast<const uint4*>(a.pi_l + src_);                                    \
    }
#define IVFTQ_STORE_TILE(BUF)                                                                        \
    _Pragma("unroll") for (int p = 0; p < PF; ++p) {                                                 \
        const int e_ = tid + 256 * p;                                                                \
        if (PF * 256 == 32 * (DP / 8) || e_ < 32 * (DP / 8)) {                                       \
            const int at_ = (BUF) * Cfg::stage_halves + (e_ / (DP / 8)) * LDH + (e_ % (DP / 8)) * 8; \
            *reinterpret_cast<uint4*>(stage + at_) = pf_h[p];                                        \
            *reinterpret_cast<uint4*>(stage + at_ + 32 * LDH) = pf_l[p];                             \
        }                                                                                            \
    }
    IVFTQ_FETCH_TILE(0)
    IVFTQ_STORE_TILE(0)
    __syncthreads();

    constexpr float kUnscale = 1.f / (kSplitScale * kSplitScale);
    const float q_scale = a.q_scale * kUnscale, q_offset = a.q_offset;
    const float q_last = (float)(a.q_cells - 1);

    // mode 0 without LDS: where this lane's rows go.  Lane (j, half) stores half of the words of row j
    // of every tile r.
    uint32_t* direct_dst[R];
    if (MODE == 0 && !via_lds) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int64_t pos = pos0 + 32 * r + j;
            const int cell = cell_of[r];
            const int64_t slot = (valid[r] && cell >= 0) ? a.list_base[cell] + (pos - a.batch_base[cell]) : -1;
            direct_dst[r] = slot >= 0 ? a.store.codes + (slot >> 6) * (int64_t)words * 64 + (slot & 63) : nullptr;
            if (slot >= 0 && half == 0) {
                a.store.gamma[slot] = __half_as_ushort(__float2half_rn(gamma[r]));
                a.store.ids[slot] = a.labels ? a.labels[row_of[r]] : a.label_base + row_of[r];
                if (a.store.xnorm) a.store.xnorm[slot] = xnorm[r];
            }
        }
    }

#pragma unroll
    for (int t = 0; t < NT; ++t) {
        if (t + 1 < NT) { IVFTQ_FETCH_TILE(t + 1) }   // in flight during this tile's multiplies
        const uint16_t* ah_base = stage + (t & 1) * Cfg::stage_halves + j * LDH + 8 * half;
        const uint16_t* al_base = ah_base + 32 * LDH;
        floatx16 acc[R];
        const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const half8 ah = *reinterpret_cast<const half8*>(ah_base + 16 * kb);
            const half8 al = *reinterpret_cast<const half8*>(al_base + 16 * kb);
#pragma unroll
            for (int r = 0; r < R; ++r) acc[r] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh[r][kb], kb ? acc[r] : zero, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < R; ++r) acc[r] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bl[r][kb], acc[r], 0, 0, 0);
#pragma unroll
            for (int r = 0; r < R; ++r) acc[r] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, bh[r][kb], acc[r], 0, 0, 0);
        }
        if (t + 1 < NT) { IVFTQ_STORE_TILE((t + 1) & 1) }   // that buffer was last read before the previous barrier

        if (mode == 2) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (!valid[r]) continue;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 o = make_float4(acc[r][4 * g] * kUnscale, acc[r][4 * g + 1] * kUnscale,
                                                 acc[r][4 * g + 2] * kUnscale, acc[r][4 * g + 3] * kUnscale);
                    const int64_t at = row_of[r] * (int64_t)DP + t * 32 + 8 * g + 4 * half;
                    *reinterpret_cast<float4*>(a.zout + at) = o;
                    if (a.zh_out) {
                        const float z[4] = {o.x, o.y, o.z, o.w};
                        uint16_t h[4], l[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            _Float16 hi, lo;
                            split_scaled(z[e], hi, lo);
                            h[e] = __builtin_bit_cast(uint16_t, hi);
                            l[e] = __builtin_bit_cast(uint16_t, lo);
                        }
                        *reinterpret_cast<uint2*>(a.zh_out + at) = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
                        *reinterpret_cast<uint2*>(a.zl_out + at) = make_uint2(l[0] | ((uint32_t)l[1] << 16), l[2] | ((uint32_t)l[3] << 16));
                    }
                }
            }
        } else {
            // d is within 32 of the padded width: only the last tile can hold padding, and only there can a
            // word lie past the row's last one
            const bool ragged = t == NT - 1 && 32 * t + 32 > d;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                uint32_t chunk[4];                     // the four codes of group g, b bits each
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int c0 = 32 * t + 8 * g + 4 * half;
                    uint32_t code[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float av = acc[r][4 * g + e];
                        const float at = __builtin_amdgcn_fmed3f(fmaf(av, q_scale, q_offset), 0.f, q_last);
                        const float2 ent = grid_s[(int)at];
                        code[e] = (uint32_t)__float_as_int(ent.y) + (av >= ent.x ? 1u : 0u);
                        if (ragged && c0 + e >= d) code[e] = 0u;
                    }
                    if (mode == 1) {
                        if (a.codes_flat && valid[r]) {
                            uint8_t* out = a.codes_flat + row_of[r] * (int64_t)d + c0;
                            if (!ragged && codes4) {
                                *reinterpret_cast<uint32_t*>(out) = code[0] | (code[1] << 8) | (code[2] << 16) | (code[3] << 24);
                            } else {
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    if (c0 + e < d) out[e] = (uint8_t)code[e];
                            }
                        }
                        continue;
                    }
                    // four codes = 4b bits at bit c0*b of the row's little-endian bit string
                    chunk[g] = code[0] | (code[1] << b) | (code[2] << (2 * b)) | (code[3] << (3 * b));
                    if (via_lds) {
                        const int bit = c0 * b;
                        const int sh = bit & 31;
                        uint32_t* wp = my_pack + (32 * r + j) * pitch + (bit >> 5);
                        const uint32_t lo = chunk[g] << sh;
                        const uint32_t hi = sh ? chunk[g] >> (32 - sh) : 0u;
                        if (lo) atomicOr(wp, lo);
                        if (hi) atomicOr(wp + 1, hi);
                        if (head_words) {      // the same four codes cut down to their top beta bits, packed likewise
                            const int hs = a.store.head_shift;
                            const uint32_t ch = (code[0] >> hs) | ((code[1] >> hs) << beta) | ((code[2] >> hs) << (2 * beta)) |
                                                ((code[3] >> hs) << (3 * beta));
                            const int hbit = c0 * beta, hsh = hbit & 31;
                            uint32_t* hp = my_head + (32 * r + j) * pitch_h + (hbit >> 5);
                            const uint32_t hlo = ch << hsh;
                            const uint32_t hhi = hsh ? ch >> (32 - hsh) : 0u;
                            if (hlo) atomicOr(hp, hlo);
                            if (hhi) atomicOr(hp + 1, hhi);
                        }
                    }
                }
                if (MODE == 0 && PACK_B == 4) {
                    // Word 4t + g of a row = group g of half 0 (low 16 bits) and of half 1 (high 16 bits).
                    // v_permlane32_swap(a, b) gives lanes 0..31 (a, a of lane + 32) and lanes 32..63 (b of
                    // lane - 32, b): with a = group g and b = group g + 2 a lane of half h ends up with both
                    // parts of word 4t + g + 2h.
#pragma unroll
                    for (int g = 0; g < 2; ++g) {
                        const auto sw = __builtin_amdgcn_permlane32_swap(chunk[g], chunk[g + 2], false, false);
                        const uint32_t word = sw[0] | (sw[1] << 16);
                        const int w = 4 * t + g + 2 * half;
                        if (direct_dst[r] && (t < NT - 1 || w < words)) direct_dst[r][(int64_t)w * 64] = word;
                    }
                } else if (MODE == 0 && PACK_B == 8) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {      // a group is a whole word: 8t + 2g + half
                        const int w = 8 * t + 2 * g + half;
                        if (direct_dst[r] && (t < NT - 1 || w < words)) direct_dst[r][(int64_t)w * 64] = chunk[g];
                    }
                }
            }
        }
        if (t + 1 < NT) __syncthreads();
    }
    if (mode == 2 || (MODE == 0 && !via_lds)) return;

    if (mode == 1) {
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (valid[r] && half == 0 && a.gamma_flat)
                a.gamma_flat[row_of[r]] = __half_as_ushort(__float2half_rn(gamma[r]));
        return;
    }

    // ---- mode 0: the wavefront's packed words go to the rows' storage slots.  Lane (j, half) stores
    // row 32*half + j when R = 2 (every word), row j when R = 1 (words of parity `half`).
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    __builtin_amdgcn_wave_barrier();
    const int my_r = (R == 2) ? half : 0;
    const bool mine = (R == 2) ? (half ? valid[R - 1] : valid[0]) : valid[0];
    const int64_t my_row = (R == 2 && half) ? row_of[R - 1] : row_of[0];
    const int my_cell = (R == 2 && half) ? cell_of[R - 1] : cell_of[0];
    const int64_t my_pos = pos0 + 32 * my_r + j;
    const float my_gamma = (R == 2 && half) ? gamma[R - 1] : gamma[0];
    const float my_xnorm = (R == 2 && half) ? xnorm[R - 1] : xnorm[0];
    const int64_t slot = (mine && my_cell >= 0) ? a.list_base[my_cell] + (my_pos - a.batch_base[my_cell]) : -1;
    if (slot >= 0) {
        const uint32_t* src = my_pack + (32 * my_r + j) * pitch;
        uint32_t* dst = a.store.codes + (slot >> 6) * (int64_t)words * 64 + (slot & 63);
        if (R == 2) {
            for (int w = 0; w < words; ++w) dst[(int64_t)w * 64] = src[w];
        } else {
            for (int w = half; w < words; w += 2) dst[(int64_t)w * 64] = src[w];
        }
        if (head_words) {
            const uint32_t* hsrc = my_head + (32 * my_r + j) * pitch_h;
            uint32_t* hdst = a.store.head + (slot >> 6) * (int64_t)head_words * 64 + (slot & 63);
            if (R == 2) {
                for (int w = 0; w < head_words; ++w) hdst[(int64_t)w * 64] = hsrc[w];
            } else {
                for (int w = half; w < head_words; w += 2) hdst[(int64_t)w * 64] = hsrc[w];
            }
        }
        if (R == 2 || half == 0) {
            a.store.gamma[slot] = __half_as_ushort(__float2half_rn(my_gamma));
            a.store.ids[slot] = a.labels ? a.labels[my_row] : a.label_base + my_row;
            if (a.store.xnorm) a.store.xnorm[slot] = my_xnorm;
        }
    }
}

#undef IVFTQ_FETCH_TILE
#undef IVFTQ_STORE_TILE

// Encode-and-store for the common shapes (d <= 128 read 16 bytes at a time, 4 or 8 stored bits, no plane
// of top bits): the same arithmetic as k_encode mode 0, organised so that nothing waits on anything else.
// All of Pi (both float16 parts) stays in LDS for the life of the workgroup, so after the one barrier
// that follows its load the four wavefronts run on their own.  A wavefront walks 32-row tiles
// tile, tile + stride, ...; while it multiplies and quantises one tile the rows of its next tile are
// already on their way into registers (their positions were fetched a tile earlier still), so the row
// reads from HBM are in flight all the time instead of once per workgroup start.
template <int DP>
constexpr size_t resident_lds_bytes(int cells) { return (size_t)2 * DP * EncCfg<DP>::LDH * sizeof(uint16_t) + (size_t)cells * 8; }

template <int DP, int PACK_B>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(DP <= 96 ? 3 : 2)))
void k_encode_resident(EncodeArgs a, int64_t tiles) {
    using Cfg = EncCfg<DP>;
    constexpr int KB = Cfg::KB, NT = Cfg::NT, LDH = Cfg::LDH, b = PACK_B;
    extern __shared__ unsigned char lds_raw[];
    uint16_t* pi_hs = reinterpret_cast<uint16_t*>(lds_raw);                   // [DP][LDH] leading parts
    uint16_t* pi_ls = pi_hs + DP * LDH;                                        // [DP][LDH] trailing parts
    float2* grid_s = reinterpret_cast<float2*>(lds_raw + (size_t)2 * DP * LDH * sizeof(uint16_t));
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, half = lane >> 5, j = lane & 31;
    const int d = a.d, words = a.store.words;
    const int last4 = d / 4 - 1;

    for (int e = tid; e < DP * (DP / 8); e += 256) {
        const int r = e / (DP / 8), c8 = e % (DP / 8);
        *reinterpret_cast<uint4*>(pi_hs + r * LDH + c8 * 8) = *reinterpret_cast<const uint4*>(a.pi_h + (int64_t)r * DP + c8 * 8);
        *reinterpret_cast<uint4*>(pi_ls + r * LDH + c8 * 8) = *reinterpret_cast<const uint4*>(a.pi_l + (int64_t)r * DP + c8 * 8);
    }
    for (int e = tid; e < a.q_cells; e += 256) {          // boundaries in accumulator units
        const float2 ent = a.q_grid[e];
        grid_s[e] = make_float2(ent.x * (kSplitScale * kSplitScale), ent.y);
    }
    __syncthreads();

    constexpr float kUnscale = 1.f / (kSplitScale * kSplitScale);
    const float q_scale = a.q_scale * kUnscale, q_offset = a.q_offset;
    const float q_last = (float)(a.q_cells - 1);
    const int64_t stride = (int64_t)gridDim.x * 4;
    int64_t tile = (int64_t)blockIdx.x * 4 + wave;

    // (row, cell) of this lane's position in a tile; a position past the end reads row 0 and stores nothing
    auto position = [&](int64_t t) {
        const int64_t pos = t * 32 + j;
        return (t < tiles && pos < a.n) ? a.order_cell[pos] : make_int2(0, -1);
    };
    // the lane's 16-byte pieces of a row: coordinates 16*kb + 8*half + 4*e (clamped inside the row)
    float4 xr[KB][2];
    auto fetch_row = [&](int row) {
        const float4* q = reinterpret_cast<const float4*>(a.x + (int64_t)row * d);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int i4 = (16 * kb + 8 * half + 4 * e) / 4;
                const bool inside = 16 * kb + 16 <= 16 * KB - 32;
                xr[kb][e] = q[(inside || i4 < last4) ? i4 : last4];
            }
    };
    int2 oc = position(tile);
    fetch_row(oc.x);
    int2 oc_next = position(tile + stride);

    for (; tile < tiles; tile += stride) {
        const int64_t pos = tile * 32 + j;
        const int row = oc.x, cell = oc.y;
        // ---- x~, residual against the assigned centroid, gamma, split unit residual
        float v[KB][8];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int c = 16 * kb + 8 * half + 4 * e;
                const bool in = 16 * kb + 16 <= 16 * KB - 32 || c < d;
                v[kb][4 * e] = in ? xr[kb][e].x : 0.f; v[kb][4 * e + 1] = in ? xr[kb][e].y : 0.f;
                v[kb][4 * e + 2] = in ? xr[kb][e].z : 0.f; v[kb][4 * e + 3] = in ? xr[kb][e].w : 0.f;
            }
        const float n2 = row_norm2<KB>(v);
        const bool good = (n2 > 0.f) && (n2 < __builtin_inff());
        const float inv_n = good ? 1.f / sqrtf(n2) : 0.f;
        float c[KB][8];
        load_row_blocks<KB>(a.cent + (int64_t)(cell < 0 ? 0 : cell) * a.cent_pitch, true, DP, 1, half, c);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int e = 0; e < 8; ++e) v[kb][e] = fmaf(v[kb][e], inv_n, -c[kb][e]);          // r = x~ - c~
        const float g = sqrtf(row_norm2<KB>(v));
        const float to_unit = (g > 1e-30f) ? 1.f / g : 0.f;       // a zero residual quantises as rho = 0
        half8 bh[KB], bl[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                _Float16 h, l;
                const float u = v[kb][e] * to_unit;
                split_scaled(u, h, l);
                bh[kb][e] = h;
                bl[kb][e] = l;
            }
        const int64_t slot = cell >= 0 ? a.list_base[cell] + (pos - a.batch_base[cell]) : -1;
        uint32_t* dst = slot >= 0 ? a.store.codes + (slot >> 6) * (int64_t)words * 64 + (slot & 63) : nullptr;
        if (slot >= 0 && half == 0) {
            a.store.gamma[slot] = __half_as_ushort(__float2half_rn(g));
            a.store.ids[slot] = a.labels ? a.labels[row] : a.label_base + row;
            if (a.store.xnorm) a.store.xnorm[slot] = good ? sqrtf(n2) : 0.f;
        }

        // ---- the next tile's rows set off now and arrive while this tile is multiplied and quantised
        oc = oc_next;
        fetch_row(oc.x);
        oc_next = position(tile + 2 * stride);

        // This lane's place in a tile of Pi is the same for every row tile; hidden from the compiler, which
        // would otherwise read all of Pi into registers once, ahead of the loop, and spill.
        int pi_at = j * LDH + 8 * half;
        asm volatile("" : "+v"(pi_at));
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const uint16_t* ah_base = pi_hs + t * 32 * LDH + pi_at;
            const uint16_t* al_base = pi_ls + t * 32 * LDH + pi_at;
            floatx16 acc;
            const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                const half8 ah = *reinterpret_cast<const half8*>(ah_base + 16 * kb);
                const half8 al = *reinterpret_cast<const half8*>(al_base + 16 * kb);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh[kb], kb ? acc : zero, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bl[kb], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, bh[kb], acc, 0, 0, 0);
            }
            const bool ragged = t == NT - 1 && 32 * t + 32 > d;      // only the last tile can hold padding
            uint32_t chunk[4];
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int c0 = 32 * t + 8 * g4 + 4 * half;
                uint32_t code[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float av = acc[4 * g4 + e];
                    const float at = __builtin_amdgcn_fmed3f(fmaf(av, q_scale, q_offset), 0.f, q_last);
                    const float2 ent = grid_s[(int)at];
                    code[e] = (uint32_t)__float_as_int(ent.y) + (av >= ent.x ? 1u : 0u);
                    if (ragged && c0 + e >= d) code[e] = 0u;
                }
                chunk[g4] = code[0] | (code[1] << b) | (code[2] << (2 * b)) | (code[3] << (3 * b));
            }
            if (PACK_B == 4) {           // see k_encode: a lane of half h ends up with both parts of word 4t + g + 2h
#pragma unroll
                for (int g4 = 0; g4 < 2; ++g4) {
                    const auto sw = __builtin_amdgcn_permlane32_swap(chunk[g4], chunk[g4 + 2], false, false);
                    const int w = 4 * t + g4 + 2 * half;
                    if (dst && (t < NT - 1 || w < words)) dst[(int64_t)w * 64] = sw[0] | (sw[1] << 16);
                }
            } else {
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const int w = 8 * t + 2 * g4 + half;
                    if (dst && (t < NT - 1 || w < words)) dst[(int64_t)w * 64] = chunk[g4];
                }
            }
        }
    }
}

template <int DP, int MODE, int PACK_B>
hipError_t run_mode(const EncodeArgs& a, hipStream_t st) {
    static LdsLimit lim;
    const size_t lds = encode_lds_bytes<DP>(MODE, PACK_B, a.q_cells, a.store.words, a.store.head ? a.store.head_words : 0);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    const hipError_t e = lim.ensure(reinterpret_cast<const void*>(k_encode<DP, MODE, PACK_B>), lds);
    if (e != hipSuccess) return e;
    const int rows_per_wg = 4 * 32 * EncCfg<DP>::R;
    const int64_t blocks = (a.n + rows_per_wg - 1) / rows_per_wg;
    int flags = 0;
    if (a.d % 4 == 0 && reinterpret_cast<uintptr_t>(a.x) % 16 == 0) flags |= 1;
    if (a.d % 4 == 0 && reinterpret_cast<uintptr_t>(a.codes_flat) % 4 == 0) flags |= 2;
    hipLaunchKernelGGL((k_encode<DP, MODE, PACK_B>), dim3((unsigned)blocks), dim3(256), lds, st, a, flags);
    return hipGetLastError();
}

template <int DP, int PACK_B>
hipError_t run_resident(const EncodeArgs& a, hipStream_t st) {
    static LdsLimit lim;
    static int units[16] = {0};         // compute units per device, asked once
    const size_t lds = resident_lds_bytes<DP>(a.q_cells);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    hipError_t e = lim.ensure(reinterpret_cast<const void*>(k_encode_resident<DP, PACK_B>), lds);
    if (e != hipSuccess) return e;
    int dev = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    int cus = (dev >= 0 && dev < 16) ? units[dev] : 0;
    if (cus <= 0) {
        if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
        if (dev >= 0 && dev < 16) units[dev] = cus;
    }
    const int64_t tiles = (a.n + 31) / 32;
    const int64_t resident = (int64_t)cus * (160 * 1024 / lds < 3 ? 160 * 1024 / lds : 3);   // workgroups the chip holds at once
    const int64_t blocks = std::min<int64_t>((tiles + 3) / 4, resident);
    hipLaunchKernelGGL((k_encode_resident<DP, PACK_B>), dim3((unsigned)blocks), dim3(256), lds, st, a, tiles);
    return hipGetLastError();
}

template <int DP>
hipError_t run(int mode, const EncodeArgs& a, hipStream_t st) {
    if (mode == 0) {
        if constexpr (DP <= 128) {
            const bool vec4 = a.d % 4 == 0 && reinterpret_cast<uintptr_t>(a.x) % 16 == 0;
            if (vec4 && !a.store.head && a.n < (int64_t)1 << 31) {
                if (a.b == 4) return run_resident<DP, 4>(a, st);
                if (a.b == 8) return run_resident<DP, 8>(a, st);
            }
        }
        // words put together in registers when a group of four codes is half a word or a whole one
        // and only the codes themselves are stored
        if (a.b == 4 && !a.store.head) return run_mode<DP, 0, 4>(a, st);
        if (a.b == 8 && !a.store.head) return run_mode<DP, 0, 8>(a, st);
        return run_mode<DP, 0, 0>(a, st);
    }
    if (mode == 1) return run_mode<DP, 1, 0>(a, st);
    if (mode == 2) return run_mode<DP, 2, 0>(a, st);
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_encode(int mode, const EncodeArgs& a, hipStream_t st) {
    if (a.n <= 0) return hipSuccess;
    if (mode != 2 && (a.q_cells < 1 || !a.q_grid)) return hipErrorInvalidValue;
    switch (rot_dp(a.d)) {
        case 32: return run<32>(mode, a, st);
        case 64: return run<64>(mode, a, st);
        case 96: return run<96>(mode, a, st);
        case 128: return run<128>(mode, a, st);
        case 160: return run<160>(mode, a, st);
        case 192: return run<192>(mode, a, st);
        case 224: return run<224>(mode, a, st);
        case 256: return run<256>(mode, a, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ivftq
