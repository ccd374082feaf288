// Batched / segmented tolerance check for gfx950 (MI355X): the device code, as templates
// over the set of element types a launch can meet.  evo_check_inst.hip instantiates it once
// per set (one translation unit each, so that they compile side by side).
//
// Functional-correctness constraint g(p) = 0 of EvoEngineer (arXiv 2510.03760,
// Sec. 3.1, Eq. 1) as evaluated by the functional-testing stage of Sec. 4.3, for a
// whole population per launch.  The element rule and the statistics are stated in
// evo.h (evo_stats).
//
// Shape of the kernel.  HBM-bound streaming reduction, no contraction, so no MFMA.
// A wavefront takes one 2 KiB reference tile into registers with two 128-bit loads
// per lane, derives the per-reference-element tolerance and reciprocal once, and
// then streams the same tile of each candidate of its group past it.  Statistics of
// a group live in registers for the whole job and are reduced across lanes once, at
// the end of the job (wavefront shuffles, then LDS across the wavefronts of the
// workgroup, then one partial row per candidate in global scratch).  The last
// workgroup of a segment to finish folds the partial rows in a fixed order, so
// results do not depend on scheduling.
//
// Two code paths per (tile, candidate):
//   fast  -- full, 16-byte aligned tile whose reference elements are all finite;
//            branch-free arithmetic; it is discarded if any |c - r| in the tile is
//            not finite (NaN/Inf candidate, or overflow);
//   exact -- element-at-a-time transcription of the rule with bounds checks; used
//            for ragged tails, unaligned tensors and every tile the fast path
//            rejects.
// Both give identical integers and maxima on the tiles the fast path accepts; the
// sums differ only in summation order (fp32 over 8 non-negative terms in a tree,
// then fp64), which stays far inside the 1e-6 relative budget of evo_stats.

#pragma once

#include <type_traits>

#include "evo_internal.h"
#include "evo_fitness_device.h"
#include "evo_rcp.h"

namespace evo {
namespace {

constexpr float kInf = __builtin_huge_valf();
constexpr float kFltMin = 1.17549435e-38f;
constexpr double kInfD = __builtin_huge_val();
constexpr double kDblMin = 2.2250738585072014e-308;
constexpr float kModerate = 0x1p102f;   // see fast_tiles
constexpr double kModerateD = 0x1p969;   // the binary64 counterpart, see fast_tiles_wide
static_assert(kModerate <= kRecipShortcutBelow, "the reciprocal shortcut must be exact below kModerate");
constexpr int kDepth = EVO_DEPTH;
constexpr uint32_t kRotate = EVO_ROTATE;   // slot rotation per step (odd)

template <uint32_t DT> struct Tile;
template <> struct Tile<EVO_F32> {
    static constexpr int kVec = 4;   // elements per 16-byte vector
    static constexpr int kNV = EVO_NV_F32;    // vectors per lane per tile
    static constexpr int kE = kVec * kNV;
    using elem_t = float;
};
template <> struct Tile<EVO_BF16> {
    static constexpr int kVec = 8;
    static constexpr int kNV = EVO_NV_BF16;
    static constexpr int kE = kVec * kNV;
    using elem_t = uint16_t;
};
template <> struct Tile<EVO_F16> : Tile<EVO_BF16> {};
template <> struct Tile<EVO_I32> : Tile<EVO_F32> {};
template <> struct Tile<EVO_F64> {
    static constexpr int kVec = 2;
    static constexpr int kNV = EVO_NV_F32;
    static constexpr int kE = kVec * kNV;
    using elem_t = double;
};
template <> struct Tile<EVO_I64> : Tile<EVO_F64> {};

template <uint32_t DT> constexpr bool kIsInt = DT == EVO_I32 || DT == EVO_I64;
template <uint32_t DT> constexpr bool kIsWide = DT == EVO_F64 || kIsInt<DT>;   // see fast_tiles_wide

// IEEE binary16 -> binary32 (v_cvt_f32_f16: exact, subnormals included).
__device__ __forceinline__ float half_bits_to_f32(uint16_t h) {
    return (float)__builtin_bit_cast(_Float16, h);
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // one 128-bit load

__device__ __forceinline__ float as_f32(uint32_t w) { return __builtin_bit_cast(float, w); }

__device__ __forceinline__ uint32_t popc64(uint64_t m) { return (uint32_t)__builtin_popcountll(m); }

__device__ __forceinline__ uint64_t ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }

// Widen one 16-byte vector to binary32 values (exact for both element types).
template <uint32_t DT>
__device__ __forceinline__ void widen(const u32x4 &raw, float *out) {
    if constexpr (DT == EVO_F32) {
        out[0] = as_f32(raw.x);
        out[1] = as_f32(raw.y);
        out[2] = as_f32(raw.z);
        out[3] = as_f32(raw.w);
    } else if constexpr (DT == EVO_BF16) {
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            out[2 * k] = as_f32(w[k] << 16);
            out[2 * k + 1] = as_f32(w[k] & 0xffff0000u);
        }
    } else {
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            out[2 * k] = half_bits_to_f32((uint16_t)(w[k] & 0xffffu));
            out[2 * k + 1] = half_bits_to_f32((uint16_t)(w[k] >> 16));
        }
    }
}

template <uint32_t DT>
__device__ __forceinline__ float load_elem(const void *base, uint64_t idx) {
    if constexpr (DT == EVO_F32) {
        return static_cast<const float *>(base)[idx];
    } else if constexpr (DT == EVO_BF16) {
        return as_f32((uint32_t) static_cast<const uint16_t *>(base)[idx] << 16);
    } else {
        return half_bits_to_f32(static_cast<const uint16_t *>(base)[idx]);
    }
}

// Per-lane running statistics of one candidate, plus wave-uniform integers.
struct Acc {
    float max_abs;
    float max_rel;
    double sum_abs;
    double sum_rel;
};

// What the exact path has gathered for one candidate of one wavefront.  It lives in
// LDS (indexed by a run-time candidate number) so that the rarely taken exact path
// never touches the register-resident accumulators of the fast path.
struct ExactAcc {
    double sum_abs, sum_rel;
    float max_abs, max_rel;
    uint32_t n_mismatch, n_excluded, flags, pad;
};

// Wavefront-wide reductions with data-parallel-primitive (DPP) moves: four shifts inside
// each row of 16 lanes (a running combination ends up in the row's last lane), then the
// last lane of every row is broadcast into the next row, then lane 31 into rows 2 and 3, so
// that lane 63 holds the combination of all 64 lanes in a fixed order (the other lanes hold
// partial combinations that nobody reads).  Lanes without a source lane receive 0, the
// neutral element of both uses below (bound_ctrl; every row enabled, so no lane keeps an
// old value and none has to be prepared: that cost one move per step and word before).
// No LDS traffic, one vector instruction per step and 32-bit word.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_word(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
constexpr int kRowShr1 = 0x111, kRowShr2 = 0x112, kRowShr4 = 0x114, kRowShr8 = 0x118;
constexpr int kRowBcast15 = 0x142, kRowBcast31 = 0x143;

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_f64(double v) {
    const uint64_t b = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = dpp_word<CTRL, ROW_MASK>((uint32_t)b);
    const uint32_t hi = dpp_word<CTRL, ROW_MASK>((uint32_t)(b >> 32));
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

// One step of the two reductions (the callers interleave the steps of several values so
// that independent instructions fill the wait states between a write and its DPP read).
// Maxima are taken on the bit patterns: the values are binary32 numbers >= +0 and finite,
// for which the unsigned integer order is the numeric order.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ void reduce_step(uint32_t &max_bits, double &sum) {
    const uint32_t m = dpp_word<CTRL, ROW_MASK>(max_bits);
    max_bits = m > max_bits ? m : max_bits;
    sum += dpp_f64<CTRL, ROW_MASK>(sum);
}

__device__ __forceinline__ float last_lane_f32(uint32_t bits) {
    return as_f32(__builtin_amdgcn_readlane(bits, kLanes - 1));
}
__device__ __forceinline__ double last_lane_f64(double v) {
    const uint64_t b = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)b, kLanes - 1);
    const uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(b >> 32), kLanes - 1);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

#define EVO_WAVE_REDUCE(STEP)            \
    STEP(kRowShr1, 0xf);                 \
    STEP(kRowShr2, 0xf);                 \
    STEP(kRowShr4, 0xf);                 \
    STEP(kRowShr8, 0xf);                 \
    STEP(kRowBcast15, 0xa);              \
    STEP(kRowBcast31, 0xc)

// Lanes -> wavefront for the NC candidates of a group at the end of a job: per candidate two
// maxima (as bit patterns, see reduce_step) and two binary64 sums.  Reducing every candidate
// over all 64 lanes on its own (EVO_WAVE_REDUCE) costs 6 steps x NC candidates x 10
// instructions of which all but one lane's result is thrown away -- 4 us per job for 16
// candidates, on the path behind the last tile.  Here the lanes of a row of 16 split the
// candidates among themselves instead: in each of four steps a lane and its partner (the
// row's mirror image, the half row's mirror image, the quad's other pair, the neighbour)
// exchange halves -- the lower one keeps the first half of the candidates it still holds
// and adds the partner's values for them, the upper one the second half -- so that the data
// per lane halves with every step and lane l ends up with the row's total of one candidate,
// (l % 16) >> (4 - log2 NC).  The four rows are then added through two lane exchanges
// (bpermute; a commutative tree, so all rows hold the same bits), and one lane per candidate
// writes the wavefront's row.  Every order is fixed by the lane numbers.
constexpr int kRowMirror = 0x140, kRowHalfMirror = 0x141, kQuadSwapPairs = 0x4E, kQuadSwapNeighbours = 0xB1;

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_all(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
template <int CTRL>
__device__ __forceinline__ double dpp_all_f64(double v) {
    const uint64_t b = __builtin_bit_cast(uint64_t, v);
    return __builtin_bit_cast(double, ((uint64_t)dpp_all<CTRL>((uint32_t)(b >> 32)) << 32) | dpp_all<CTRL>((uint32_t)b));
}

// One step: L candidates live in x[0 .. L) of every lane; afterwards L / 2 (or the one, summed
// with the partner's, when L == 1).  `low`: this lane is the lower one of its pair.
template <int L, int CTRL>
__device__ __forceinline__ void scatter_step(bool low, uint32_t *ma, uint32_t *mr, double *sa, double *sr) {
    if constexpr (L > 1) {
        constexpr int H = L / 2;
#pragma unroll
        for (int j = 0; j < H; ++j) {
            const uint32_t ma_send = low ? ma[j + H] : ma[j], ma_keep = low ? ma[j] : ma[j + H];
            const uint32_t mr_send = low ? mr[j + H] : mr[j], mr_keep = low ? mr[j] : mr[j + H];
            const double sa_send = low ? sa[j + H] : sa[j], sa_keep = low ? sa[j] : sa[j + H];
            const double sr_send = low ? sr[j + H] : sr[j], sr_keep = low ? sr[j] : sr[j + H];
            const uint32_t ma_got = dpp_all<CTRL>(ma_send), mr_got = dpp_all<CTRL>(mr_send);
            ma[j] = ma_got > ma_keep ? ma_got : ma_keep;
            mr[j] = mr_got > mr_keep ? mr_got : mr_keep;
            sa[j] = sa_keep + dpp_all_f64<CTRL>(sa_send);
            sr[j] = sr_keep + dpp_all_f64<CTRL>(sr_send);
        }
    } else {
        const uint32_t ma_got = dpp_all<CTRL>(ma[0]), mr_got = dpp_all<CTRL>(mr[0]);
        ma[0] = ma_got > ma[0] ? ma_got : ma[0];
        mr[0] = mr_got > mr[0] ? mr_got : mr[0];
        sa[0] += dpp_all_f64<CTRL>(sa[0]);
        sr[0] += dpp_all_f64<CTRL>(sr[0]);
    }
}

__device__ __forceinline__ uint32_t from_lane(uint32_t v, int src_lane) {
    return (uint32_t)__builtin_amdgcn_ds_bpermute(src_lane * 4, (int)v);
}
__device__ __forceinline__ double from_lane_f64(double v, int src_lane) {
    const uint64_t b = __builtin_bit_cast(uint64_t, v);
    return __builtin_bit_cast(double, ((uint64_t)from_lane((uint32_t)(b >> 32), src_lane) << 32) | from_lane((uint32_t)b, src_lane));
}

// ma, mr, sa, sr: NC values per lane (destroyed).  n_mismatch_of_lane: what the row of the
// candidate this lane ends up with gets as its mismatch count (see group_candidate_of_lane).
template <int NC>
__device__ __forceinline__ int group_candidate_of_lane(int lane) {
    constexpr int kShift = NC == 16 ? 0 : NC == 8 ? 1 : NC == 4 ? 2 : NC == 2 ? 3 : 4;
    return (lane & 15) >> kShift;
}
template <int NC>
__device__ __forceinline__ void reduce_group_to_rows(uint32_t *ma, uint32_t *mr, double *sa, double *sr, int lane,
                                                     uint32_t n_mismatch_of_lane, Partial *wpart) {
    static_assert(NC == 1 || NC == 2 || NC == 4 || NC == 8 || NC == 16, "group sizes");
    scatter_step<NC, kRowMirror>((lane & 8) == 0, ma, mr, sa, sr);
    scatter_step<(NC > 1 ? NC / 2 : 1), kRowHalfMirror>((lane & 4) == 0, ma, mr, sa, sr);
    scatter_step<(NC > 2 ? NC / 4 : 1), kQuadSwapPairs>((lane & 2) == 0, ma, mr, sa, sr);
    scatter_step<(NC > 4 ? NC / 8 : 1), kQuadSwapNeighbours>((lane & 1) == 0, ma, mr, sa, sr);
    // rows: with the neighbouring row, then with the other pair of rows
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
        const uint32_t ma_got = from_lane(ma[0], lane ^ off), mr_got = from_lane(mr[0], lane ^ off);
        const double sa_got = from_lane_f64(sa[0], lane ^ off), sr_got = from_lane_f64(sr[0], lane ^ off);
        ma[0] = ma_got > ma[0] ? ma_got : ma[0];
        mr[0] = mr_got > mr[0] ? mr_got : mr[0];
        sa[0] += sa_got;
        sr[0] += sr_got;
    }
    constexpr int kPerCandidate = 16 / NC;   // lanes of a row that hold the same candidate
    if (lane < 16 && (lane & (kPerCandidate - 1)) == 0) {
        Partial p;
        p.n_mismatch = n_mismatch_of_lane;
        p.n_excluded = 0;
        p.sum_abs = sa[0];
        p.sum_rel = sr[0];
        p.max_abs = as_f32(ma[0]);
        p.max_rel = as_f32(mr[0]);
        p.flags = 0;
        p.pad = 0;
        wpart[group_candidate_of_lane<NC>(lane)] = p;
    }
}

// Per-lane counts of one tile (mismatches in the low half, exclusions in the high half: at
// most 16 each, so the halves of the wavefront's total do not meet) and per-lane flags into
// the wavefront's LDS record of the candidate.
__device__ __forceinline__ void settle_counts(ExactAcc *out, int lane, uint32_t counts, uint32_t flags) {
#define EVO_STEP(CTRL_, MASK_) counts += dpp_word<CTRL_, MASK_>(counts)
    EVO_WAVE_REDUCE(EVO_STEP);
#undef EVO_STEP
    const uint32_t total = __builtin_amdgcn_readlane(counts, kLanes - 1);
    const uint32_t nan_flags = EVO_F_CAND_NAN | EVO_F_NAN_SITE_DIFF, inf_flags = EVO_F_CAND_INF | EVO_F_INF_DIFF;
    const uint32_t all_flags = (ballot((flags & nan_flags) != 0) ? nan_flags : 0u) |
                               (ballot((flags & inf_flags) != 0) ? inf_flags : 0u);
    if (lane == 0) {
        out->n_mismatch += total & 0xffffu;
        out->n_excluded += total >> 16;
        out->flags |= all_flags;
    }
}

// Wavefront totals of one exact-path tile into the wavefront's LDS record of the candidate.
__device__ __forceinline__ void exact_commit(ExactAcc *out, int lane, float max_abs, float max_rel,
                                             double sum_abs, double sum_rel, uint32_t n_mismatch,
                                             uint32_t n_excluded, uint32_t flags) {
    uint32_t ma_bits = __builtin_bit_cast(uint32_t, max_abs), mr_bits = __builtin_bit_cast(uint32_t, max_rel);
#define EVO_STEP(CTRL_, MASK_)                            \
    reduce_step<CTRL_, MASK_>(ma_bits, sum_abs);          \
    reduce_step<CTRL_, MASK_>(mr_bits, sum_rel)
    EVO_WAVE_REDUCE(EVO_STEP);
#undef EVO_STEP
    max_abs = last_lane_f32(ma_bits);
    max_rel = last_lane_f32(mr_bits);
    sum_abs = last_lane_f64(sum_abs);
    sum_rel = last_lane_f64(sum_rel);
    if (lane == 0) {
        out->sum_abs += sum_abs;
        out->sum_rel += sum_rel;
        out->max_abs = __builtin_fmaxf(out->max_abs, max_abs);
        out->max_rel = __builtin_fmaxf(out->max_rel, max_rel);
        out->n_mismatch += n_mismatch;
        out->n_excluded += n_excluded;
        out->flags |= flags;
    }
}

// Exact path: the rule of evo.h one element per lane at a time.  Handles elements
// beyond n (ignored), any alignment and every special value.  Results are reduced
// over the wavefront and added to the wavefront's LDS record of the candidate.
template <uint32_t DT>
__device__ __forceinline__ void exact_tile_narrow(const void *ref, const void *cand, uint64_t n,
                                                  uint64_t tile_base, int lane, float atol,
                                                  float rtol, ExactAcc *out) {
    constexpr int kE = Tile<DT>::kE;
    float max_abs = 0.0f, max_rel = 0.0f;
    double sum_abs = 0.0, sum_rel = 0.0;
    uint32_t n_mismatch = 0, n_excluded = 0, flags = 0;
    // four elements per lane at a time: their loads share one memory round trip (the loop
    // stays rolled: unrolling it all raises the register pressure of the whole kernel)
    constexpr int kChunk = 4;
    static_assert(kE % kChunk == 0, "tile elements per lane");
#pragma unroll 1
    for (int k0 = 0; k0 < kE; k0 += kChunk) {
        float rv[kChunk], cv[kChunk];
#pragma unroll
        for (int k = 0; k < kChunk; ++k) {
            const uint64_t idx = tile_base + (uint64_t)((k0 + k) * kLanes + lane);
            rv[k] = 0.0f;
            cv[k] = 0.0f;
            if (idx < n) {
                rv[k] = load_elem<DT>(ref, idx);
                cv[k] = load_elem<DT>(cand, idx);
            }
        }
#pragma unroll
        for (int k = 0; k < kChunk; ++k) {
            const uint64_t idx = tile_base + (uint64_t)((k0 + k) * kLanes + lane);
            const bool inb = idx < n;
            const float r = rv[k], c = cv[k];
            const float ar = __builtin_fabsf(r);
            const float ac = __builtin_fabsf(c);
            const float scaled = rtol * ar;
            const float tol = atol + scaled;
            const bool r_nan = r != r, c_nan = c != c;
            const bool r_inf = ar == kInf, c_inf = ac == kInf;
            const bool both = !r_nan && !c_nan && !r_inf && !c_inf;
            const float d = __builtin_fabsf(c - r);
            const bool match = (c == r) || (both && d <= tol);
            n_mismatch += popc64(ballot(inb && !match));
            n_excluded += popc64(ballot(inb && !both));
            if (ballot(c_nan)) flags |= EVO_F_CAND_NAN;
            if (ballot(c_inf)) flags |= EVO_F_CAND_INF;
            if (ballot(r_nan)) flags |= EVO_F_REF_NAN;
            if (ballot(r_inf)) flags |= EVO_F_REF_INF;
            if (ballot(c_nan != r_nan)) flags |= EVO_F_NAN_SITE_DIFF;
            if (ballot((c_inf || r_inf) && !c_nan && !r_nan && c != r)) flags |= EVO_F_INF_DIFF;
            if (inb && both) {
                float inv = 0.0f;
                if (ar >= kFltMin) inv = 1.0f / ar;
                const float q = d * inv;
                max_abs = d > max_abs ? d : max_abs;
                max_rel = q > max_rel ? q : max_rel;
                sum_abs += (double)d;
                sum_rel += (double)q;
            }
        }
    }
    exact_commit(out, lane, max_abs, max_rel, sum_abs, sum_rel, n_mismatch, n_excluded, flags);
}

// Exact path, binary64 tensors: the same rule with every operation in binary64; the
// maxima are rounded to binary32 when they leave the lane (rounding is monotone).
__device__ __forceinline__ void exact_tile_f64(const void *ref, const void *cand, uint64_t n,
                                               uint64_t tile_base, int lane, float atol,
                                               float rtol, ExactAcc *out) {
    constexpr int kE = Tile<EVO_F64>::kE;
    const double atol_d = (double)atol, rtol_d = (double)rtol;
    double max_abs = 0.0, max_rel = 0.0, sum_abs = 0.0, sum_rel = 0.0;
    uint32_t n_mismatch = 0, n_excluded = 0, flags = 0;
    double rv[kE], cv[kE];
#pragma unroll
    for (int k = 0; k < kE; ++k) {
        const uint64_t idx = tile_base + (uint64_t)(k * kLanes + lane);
        rv[k] = 0.0;
        cv[k] = 0.0;
        if (idx < n) {
            rv[k] = static_cast<const double *>(ref)[idx];
            cv[k] = static_cast<const double *>(cand)[idx];
        }
    }
#pragma unroll
    for (int k = 0; k < kE; ++k) {
        const uint64_t idx = tile_base + (uint64_t)(k * kLanes + lane);
        const bool inb = idx < n;
        const double r = rv[k], c = cv[k];
        const double ar = __builtin_fabs(r);
        const double ac = __builtin_fabs(c);
        const double scaled = rtol_d * ar;
        const double tol = atol_d + scaled;
        const bool r_nan = r != r, c_nan = c != c;
        const bool r_inf = ar == kInfD, c_inf = ac == kInfD;
        const bool both = !r_nan && !c_nan && !r_inf && !c_inf;
        const double d = __builtin_fabs(c - r);
        const bool match = (c == r) || (both && d <= tol);
        n_mismatch += popc64(ballot(inb && !match));
        n_excluded += popc64(ballot(inb && !both));
        if (ballot(c_nan)) flags |= EVO_F_CAND_NAN;
        if (ballot(c_inf)) flags |= EVO_F_CAND_INF;
        if (ballot(r_nan)) flags |= EVO_F_REF_NAN;
        if (ballot(r_inf)) flags |= EVO_F_REF_INF;
        if (ballot(c_nan != r_nan)) flags |= EVO_F_NAN_SITE_DIFF;
        if (ballot((c_inf || r_inf) && !c_nan && !r_nan && c != r)) flags |= EVO_F_INF_DIFF;
        if (inb && both) {
            double inv = 0.0;
            if (ar >= kDblMin) inv = 1.0 / ar;
            const double q = d * inv;
            max_abs = d > max_abs ? d : max_abs;
            max_rel = q > max_rel ? q : max_rel;
            sum_abs += d;
            sum_rel += q;
        }
    }
    exact_commit(out, lane, (float)max_abs, (float)max_rel, sum_abs, sum_rel, n_mismatch, n_excluded,
                 flags);
}

// |c - r| of two signed integers as an exact unsigned integer.
__device__ __forceinline__ uint32_t abs_diff(int32_t c, int32_t r) {
    return c > r ? (uint32_t)c - (uint32_t)r : (uint32_t)r - (uint32_t)c;
}
__device__ __forceinline__ uint64_t abs_diff(int64_t c, int64_t r) {
    return c > r ? (uint64_t)c - (uint64_t)r : (uint64_t)r - (uint64_t)c;
}

// Exact path, integer tensors: equality; |c - r| exact, its maximum rounded to binary32
// when it leaves the lane, its sum in binary64.
template <uint32_t DT>
__device__ __forceinline__ void exact_tile_int(const void *ref, const void *cand, uint64_t n,
                                               uint64_t tile_base, int lane, ExactAcc *out) {
    using elem_t = typename std::conditional<DT == EVO_I32, int32_t, int64_t>::type;
    constexpr int kE = Tile<DT>::kE;
    uint64_t max_d = 0;
    double sum_abs = 0.0;
    uint32_t n_mismatch = 0;
    elem_t rv[kE], cv[kE];
#pragma unroll
    for (int k = 0; k < kE; ++k) {
        const uint64_t idx = tile_base + (uint64_t)(k * kLanes + lane);
        rv[k] = 0;
        cv[k] = 0;
        if (idx < n) {
            rv[k] = static_cast<const elem_t *>(ref)[idx];
            cv[k] = static_cast<const elem_t *>(cand)[idx];
        }
    }
#pragma unroll
    for (int k = 0; k < kE; ++k) {
        const uint64_t d = abs_diff(cv[k], rv[k]);   // 0 beyond n
        n_mismatch += popc64(ballot(d != 0));
        max_d = d > max_d ? d : max_d;
        sum_abs += (double)d;
    }
    exact_commit(out, lane, (float)max_d, 0.0f, sum_abs, 0.0, n_mismatch, 0u, 0u);
}

template <uint32_t DT>
__device__ __forceinline__ void exact_tile(const void *ref, const void *cand, uint64_t n,
                                           uint64_t tile_base, int lane, float atol,
                                           float rtol, ExactAcc *out) {
    if constexpr (kIsInt<DT>) {
        exact_tile_int<DT>(ref, cand, n, tile_base, lane, out);
    } else if constexpr (DT == EVO_F64) {
        exact_tile_f64(ref, cand, n, tile_base, lane, atol, rtol, out);
    } else {
        exact_tile_narrow<DT>(ref, cand, n, tile_base, lane, atol, rtol, out);
    }
}

// 16 bytes from global memory at a wave-uniform base plus a per-lane byte offset.
// STREAM: the data is read once by the whole grid (candidate tiles; the reference tile
// too when no other wavefront shares it), so the load is marked non-temporal and does
// not displace anything in the caches -- measured 7.2 TB/s against 6.3 TB/s for plain
// loads on a read-only sweep of 8 GiB.
template <bool STREAM>
__device__ __forceinline__ u32x4 load16(const char *base, uint32_t lane_off) {
    typedef __attribute__((address_space(1))) const u32x4 global_u32x4;
    global_u32x4 *p = (global_u32x4 *)((__attribute__((address_space(1))) const char *)base + lane_off);
#if EVO_NT_LOADS
    if constexpr (STREAM) return __builtin_nontemporal_load(p);
#endif
    return *p;
}

// The same from a per-lane address.
template <bool STREAM>
__device__ __forceinline__ u32x4 load16_at(uint64_t addr) {
    typedef __attribute__((address_space(1))) const u32x4 global_u32x4;
    global_u32x4 *p = (global_u32x4 *)addr;
#if EVO_NT_LOADS
    if constexpr (STREAM) return __builtin_nontemporal_load(p);
#endif
    return *p;
}

// max(m, |a|, |b|) and max(m, a, b) in one instruction each.  Operands are finite
// whenever the result is used (tiles holding anything else are redone exactly).
__device__ __forceinline__ float max3_abs(float m, float a, float b) {
    float o;
    asm("v_max3_f32 %0, |%1|, |%2|, %3" : "=v"(o) : "v"(a), "v"(b), "v"(m));
    return o;
}
__device__ __forceinline__ float max_abs2(float a, float b) {
    float o;
    asm("v_max_f32_e64 %0, |%1|, |%2|" : "=v"(o) : "v"(a), "v"(b));
    return o;
}
__device__ __forceinline__ float max3(float m, float a, float b) {
    float o;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(o) : "v"(a), "v"(b), "v"(m));
    return o;
}

// |a| + |b| in one instruction (the magnitudes as source modifiers; left to itself the
// compiler first clears the sign bits with one v_and_b32 per operand).
__device__ __forceinline__ float add_abs2(float a, float b) {
    float o;
    asm("v_add_f32_e64 %0, |%1|, |%2|" : "=v"(o) : "v"(a), "v"(b));
    return o;
}

// Pairwise sum of N values (of their magnitudes when ABS), N a power of two >= 2.
template <int N, bool ABS>
__device__ __forceinline__ float tree_sum(const float *v) {
    if constexpr (N == 2) {
        return ABS ? add_abs2(v[0], v[1]) : v[0] + v[1];
    } else {
        return tree_sum<N / 2, ABS>(v) + tree_sum<N / 2, ABS>(v + N / 2);
    }
}

__device__ __forceinline__ const char *uniform_ptr(const void *p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const char *>(((uint64_t)hi << 32) | lo);
}

// The pointer that lane `src` holds in `v`, as a wave-uniform value.
__device__ __forceinline__ const char *lane_ptr(uint64_t v, uint32_t src) {
    const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)v, src);
    const uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(v >> 32), src);
    return reinterpret_cast<const char *>(((uint64_t)hi << 32) | lo);
}

// The tiles of one wavefront.  In step k the wavefront slots of a group block together
// cover one contiguous window of n_slots tiles of every tensor, so that at any moment
// the whole grid reads a few MiB-sized windows (DRAM pages and TLB entries are shared
// by neighbouring workgroups).  The slot -> tile map is rotated from step to step:
// with a fixed map every workgroup would return to the same DRAM channels in every
// window and inherit that channel's service rate for the whole launch.
struct TileWalk {
    uint32_t n_chunks, chunk, tpw, tl;
    __device__ __forceinline__ uint64_t window() const { return (uint64_t)n_chunks * tpw; }
    __device__ __forceinline__ uint64_t at(uint32_t k) const {
        // 32 bits suffice: chunk < n_chunks <= 2^30 and k <= kMaxTilesPerWave
        const uint32_t c = (chunk + k * kRotate) % n_chunks;
        return ((uint64_t)k * n_chunks + c) * tpw + tl;
    }
    // number of steps k = 0, 1, ... whose tile lies below `limit`
    __device__ __forceinline__ uint32_t steps_below(uint64_t limit) const {
        // (a 64-bit division is a few hundred instructions; both operands almost always fit
        // 32 bits, and this is on every job's path before its first load and after its last)
        const uint64_t w = window();
        const uint32_t full = ((limit | w) >> 32) == 0 ? (uint32_t)limit / (uint32_t)w : (uint32_t)(limit / w);
        return full + (at(full) < limit ? 1u : 0u);
    }
};

// Exact path for the FULL, 16-byte-aligned tiles of ONE candidate that the fast path has
// handed back (bit `bit` of redo_w[k] for step k < k_fast): the rule of evo.h, element by
// element, as in exact_tile_narrow, but
//  * on tiles fetched the way the fast path fetches them, four tiles per memory round trip,
//  * with the counts and flags kept per lane (vector compares and selects; no wave-wide
//    ballot per element), and
//  * with one cross-lane reduction for the whole candidate instead of one per tile.
// A candidate that is NaN or Inf throughout -- what a broken kernel tends to produce -- has
// every one of its tiles handed back; with a reduction and eleven ballots per tile that cost
// 2.7 us per tile, 25 % on top of a launch of 16 candidates for each such candidate.
template <uint32_t DT>
__device__ __forceinline__ void exact_candidate_pass(const char *rptr, const char *cptr, const TileWalk walk,
                                                     uint32_t k_fast, uint32_t bit, const uint16_t *redo_w,
                                                     int lane, float atol, float rtol, ExactAcc *out) {
    using TL = Tile<DT>;
    constexpr int kE = TL::kE;
    constexpr int kNV = TL::kNV;
    constexpr int kB = 4;   // tiles per round trip
    constexpr uint64_t kTileBytes = (uint64_t)tile_elems(DT) * sizeof(typename TL::elem_t);
    const uint32_t lane_off = (uint32_t)lane * 16u;
    float max_abs = 0.0f, max_rel = 0.0f;
    double sum_abs = 0.0, sum_rel = 0.0;
    uint32_t n_mismatch = 0, n_excluded = 0, flags = 0;   // of this lane
    for (uint32_t k0 = 0; k0 < k_fast; k0 += (uint32_t)kLanes) {
        const uint32_t kk = k0 + (uint32_t)lane;
        const uint32_t v = kk < k_fast ? (uint32_t)redo_w[kk] : 0u;
        uint64_t hits = ballot(((v >> bit) & 1u) != 0);
        while (hits) {
            uint64_t off[kB];
            bool has[kB];
#pragma unroll
            for (int b = 0; b < kB; ++b) {
                has[b] = hits != 0;
                const uint32_t idx = has[b] ? (uint32_t)__builtin_ctzll(hits) : 0u;
                hits &= hits - 1;   // 0 stays 0
                off[b] = walk.at(k0 + idx) * kTileBytes;
            }
            u32x4 rraw[kB][kNV], craw[kB][kNV];
#pragma unroll
            for (int b = 0; b < kB; ++b) {
                if (has[b]) {
#pragma unroll
                    for (int j = 0; j < kNV; ++j) {
                        rraw[b][j] = load16<false>(rptr + off[b] + j * 1024, lane_off);
                        craw[b][j] = load16<true>(cptr + off[b] + j * 1024, lane_off);
                    }
                }
            }
#pragma unroll
            for (int b = 0; b < kB; ++b) {
                if (!has[b]) continue;
                float r[kE], c[kE];
#pragma unroll
                for (int j = 0; j < kNV; ++j) {
                    widen<DT>(rraw[b][j], &r[j * TL::kVec]);
                    widen<DT>(craw[b][j], &c[j * TL::kVec]);
                }
#pragma unroll
                for (int e = 0; e < kE; ++e) {
                    const float rr = r[e], cc = c[e];
                    const float ar = __builtin_fabsf(rr);
                    const float ac = __builtin_fabsf(cc);
                    const float scaled = rtol * ar;
                    const float tol = atol + scaled;
                    const bool r_nan = rr != rr, c_nan = cc != cc;
                    const bool r_inf = ar == kInf, c_inf = ac == kInf;
                    const bool both = !r_nan && !c_nan && !r_inf && !c_inf;
                    const float d = __builtin_fabsf(cc - rr);
                    const bool match = (cc == rr) || (both && d <= tol);
                    n_mismatch += match ? 0u : 1u;
                    n_excluded += both ? 0u : 1u;
                    flags |= (c_nan ? EVO_F_CAND_NAN : 0u) | (c_inf ? EVO_F_CAND_INF : 0u) |
                             (r_nan ? EVO_F_REF_NAN : 0u) | (r_inf ? EVO_F_REF_INF : 0u) |
                             (c_nan != r_nan ? EVO_F_NAN_SITE_DIFF : 0u) |
                             ((c_inf || r_inf) && !c_nan && !r_nan && cc != rr ? EVO_F_INF_DIFF : 0u);
                    float inv = 0.0f;
                    if (both && ar >= kFltMin) inv = 1.0f / ar;
                    // 0 is the identity of both maxima and both sums (every term is >= +0)
                    const float dm = both ? d : 0.0f;
                    const float qm = both ? d * inv : 0.0f;
                    max_abs = dm > max_abs ? dm : max_abs;
                    max_rel = qm > max_rel ? qm : max_rel;
                    sum_abs += (double)dm;
                    sum_rel += (double)qm;
                }
            }
        }
    }
    // lanes -> wavefront, once: the counts travel as binary64 (exact below 2^53)
    uint32_t ma_bits = __builtin_bit_cast(uint32_t, max_abs), mr_bits = __builtin_bit_cast(uint32_t, max_rel);
    uint32_t zero_a = 0, zero_b = 0;
    double mis = (double)n_mismatch, exc = (double)n_excluded;
#define EVO_STEP(CTRL_, MASK_)                            \
    reduce_step<CTRL_, MASK_>(ma_bits, sum_abs);          \
    reduce_step<CTRL_, MASK_>(mr_bits, sum_rel);          \
    reduce_step<CTRL_, MASK_>(zero_a, mis);               \
    reduce_step<CTRL_, MASK_>(zero_b, exc)
    EVO_WAVE_REDUCE(EVO_STEP);
#undef EVO_STEP
    max_abs = last_lane_f32(ma_bits);
    max_rel = last_lane_f32(mr_bits);
    sum_abs = last_lane_f64(sum_abs);
    sum_rel = last_lane_f64(sum_rel);
    mis = last_lane_f64(mis);
    exc = last_lane_f64(exc);
    uint32_t all_flags = 0;
#pragma unroll
    for (uint32_t f = 1u; f <= EVO_F_INF_DIFF; f <<= 1)
        if (ballot((flags & f) != 0)) all_flags |= f;
    if (lane == 0) {
        out->sum_abs += sum_abs;
        out->sum_rel += sum_rel;
        out->max_abs = __builtin_fmaxf(out->max_abs, max_abs);
        out->max_rel = __builtin_fmaxf(out->max_rel, max_rel);
        out->n_mismatch += (uint32_t)mis;
        out->n_excluded += (uint32_t)exc;
        out->flags |= all_flags;
    }
}

// Fast path of one wavefront over its full tiles walk.at(0), walk.at(1), ... (those below
// t_fend) for a full group of NC candidates.  Straight-line code per candidate apart from the
// commit test; loads run D candidates ahead of the arithmetic, across tile boundaries
// too.  Candidates of a tile that the fast path must not settle (a non-finite or huge
// reference element, overflow) are recorded in redo[tile slot] for the exact path; NaN and
// Inf in a candidate tile over a moderate reference tile are settled on the spot
// (counts, exclusions and flags in xacc).  Ends with the lanes -> wavefront
// reduction into wpart[0 .. NC).
template <uint32_t DT, int NC, bool REF_STREAM, bool PADDED>
__device__ __forceinline__ uint32_t fast_tiles(const char *rptr, const uint64_t *cptr_lds_generic,
                                               const TileWalk walk, uint64_t t_fend,
                                               float atol, float rtol, int lane, bool second_round,
                                               uint32_t n_real, uint16_t *redo, Partial *wpart,
                                               ExactAcc *xacc) {
    using TL = Tile<DT>;
    constexpr int kE = TL::kE;
    constexpr int kNV = TL::kNV;
    constexpr uint64_t kTileBytes = (uint64_t)tile_elems(DT) * sizeof(typename TL::elem_t);
    constexpr int D = NC < kDepth ? NC : kDepth;
    static_assert(kE >= 2 && (kE & (kE - 1)) == 0 && kE <= 16,
                  "pairwise fp32 trees: at most 4 roundings deep keeps the sums inside 1e-6");
    const uint32_t lane_off = (uint32_t)lane * 16u;

    // The NC candidate pointers stay in LDS (cptr_lds[g], one broadcast read per use) and a
    // candidate's address is formed per lane; as NC wave-uniform register pairs they -- and
    // NC wave-uniform mismatch counters -- left no scalar registers for anything else, and
    // the loop spent a sixth of its vector instructions moving scalars in and out of
    // vector lanes.  Mismatches are counted in the wavefront's LDS record (xacc) instead:
    // they are rare.
    Acc acc[NC];
#pragma unroll
    for (int g = 0; g < NC; ++g) acc[g] = Acc{0.0f, 0.0f, 0.0, 0.0};
    uint32_t any_redo = 0;
    // The table's LDS address is kept in a vector register (LDS reads take their address
    // from one; as a wave-uniform value it would be moved there before every read).
    typedef __attribute__((address_space(3))) const uint64_t lds_u64;
    // (plus a per-lane zero that the compiler does not see through: 0 lanes counted below each)
    const uint32_t table_addr = (uint32_t)(uintptr_t)(lds_u64 *)cptr_lds_generic + __builtin_amdgcn_mbcnt_lo(0u, 0u);
    lds_u64 *cptr_lds = (lds_u64 *)(uintptr_t)table_addr;

    const uint32_t k_end = walk.steps_below(t_fend);
    // A single candidate leaves the pipeline above with two tiles in flight (the next
    // tile's reference and candidate), where a group of two or more has three: its loop
    // takes TWO tiles per iteration instead, each in registers of its own, and requests
    // tile k + 2 of both tensors when tile k has been consumed -- three to four tiles in
    // flight.  kTPI = 1 is the plain loop.
    constexpr int kTPI = NC == 1 ? 2 : 1;
    if (k_end > 0) {
        u32x4 ref_raw[kTPI][kNV];
        u32x4 buf[kTPI][D][kNV];
        uint64_t tile_of[kTPI];   // the tile whose data ref_raw[u] / buf[u] hold or await
#pragma unroll
        for (int u = 0; u < kTPI; ++u) {
            tile_of[u] = walk.at((uint32_t)u < k_end ? (uint32_t)u : k_end - 1u);
            const uint64_t off = tile_of[u] * kTileBytes;
            const uint64_t voff = off + lane_off;
#pragma unroll
            for (int j = 0; j < kNV; ++j) ref_raw[u][j] = load16<REF_STREAM>(rptr + off + j * 1024, lane_off);
#pragma unroll
            for (int g = 0; g < D; ++g)
#pragma unroll
                for (int j = 0; j < kNV; ++j) buf[u][g][j] = load16_at<true>(cptr_lds[g] + voff + j * 1024);
        }
        for (uint32_t slot0 = 0; slot0 < k_end; slot0 += (uint32_t)kTPI) {
#pragma unroll
          for (int u = 0; u < kTPI; ++u) {
            const uint32_t slot = slot0 + (uint32_t)u;
            if (kTPI > 1 && slot >= k_end) break;
            // Issue priority, see `second_round` in check_body: raised for two steps,
            // normal for two steps.
            if (second_round) {
                if (slot & 2u) __builtin_amdgcn_s_setprio(1);
                else __builtin_amdgcn_s_setprio(0);
            }
            const uint64_t t = tile_of[u];
            const uint64_t off = t * kTileBytes;
            // the tile these registers take next; at the end of the job tile 0 (a few redundant,
            // in-bounds loads instead of a branch per load: tile 0 of every tensor is what all
            // wavefronts ask for at their end, so it comes from a cache -- the registers are
            // reused right after the loop and must wait for these loads)
            const uint64_t t_next = (slot + (uint32_t)kTPI < k_end) ? walk.at(slot + (uint32_t)kTPI) : 0;
            const uint64_t off_next = t_next * kTileBytes;
            const uint64_t voff = off + lane_off, voff_next = off_next + lane_off;   // per lane
            tile_of[u] = t_next;

            float r[kE], inv[kE];
#pragma unroll
            for (int j = 0; j < kNV; ++j) widen<DT>(ref_raw[u][j], &r[j * TL::kVec]);
#pragma unroll
            for (int j = 0; j < kNV; ++j) ref_raw[u][j] = load16<REF_STREAM>(rptr + off_next + j * 1024, lane_off);
            // One test per reference element serves two shortcuts: below kModerate (2^102, far
            // inside the range where the reciprocal shortcut is exact) the reciprocal needs no
            // division, and a candidate tile without a single number in it can be settled on
            // the spot (see below).  A NaN reference element fails the test too.
            bool huge = false;
#pragma unroll
            for (int e = 0; e < kE; ++e) {
                const float ar = __builtin_fabsf(r[e]);
                inv[e] = ar >= kFltMin ? recip_shortcut(ar) : 0.0f;
                huge = huge || !(ar < kModerate);
            }
            const bool moderate_tile = ballot(huge) == 0;
            if (!moderate_tile) {   // |r| >= 2^102 or NaN somewhere in the tile: true division
#pragma unroll
                for (int e = 0; e < kE; ++e) {
                    const float ar = __builtin_fabsf(r[e]);
                    inv[e] = ar >= kFltMin ? 1.0f / ar : 0.0f;
                }
            }

            // PADDED: the pointer that candidate g's refill starts from -- candidate g + D of this
            // tile or, behind the last real ones, candidate g % D of the next.  (The table's
            // address through an opaque copy: the NC addresses formed from it do not depend
            // on the tile, and kept in registers across the whole loop they are what tips the
            // 16-bit kernels into spilling.)
            auto padded_refill_ptr = [&](int g) -> uint64_t {
                uint32_t table_here = table_addr;
                asm volatile("" : "+v"(table_here));
                lds_u64 *table = (lds_u64 *)(uintptr_t)table_here;
                return table[(uint32_t)(g + D) < n_real ? (uint32_t)(g + D) : (uint32_t)(g % D)];
            };
            uint64_t ptr_ahead = 0;
            if constexpr (PADDED) ptr_ahead = padded_refill_ptr(0);

            uint32_t redo_mask = 0;
#pragma unroll
            for (int g = 0; g < NC; ++g) {
                // PADDED: the group's last NC - n_real candidates are stand-ins; nothing is
                // loaded or computed for them (n_real > NC / 2, so the candidates that the
                // pipeline requests ahead of a tile are always real)
                const bool real = !PADDED || (uint32_t)g < n_real;
                float d[kE], q[kE];
                if (real) {
                    float c[kE];
#pragma unroll
                    for (int j = 0; j < kNV; ++j) widen<DT>(buf[u][g % D][j], &c[j * TL::kVec]);
#pragma unroll
                    for (int e = 0; e < kE; ++e) d[e] = c[e] - r[e];
                }
                // refill the slot: candidate g+D of this tile, or g+D-NC of the next
                if constexpr (!PADDED) {
#pragma unroll
                    for (int j = 0; j < kNV; ++j)
                        buf[u][g % D][j] = load16_at<true>(cptr_lds[(g + D) % NC] + (g + D < NC ? voff : voff_next) +
                                                        j * 1024);
                } else if (real) {
                    // With n_real candidates the slot of the last D of them is free for the
                    // next tile's first D candidates (candidate k uses slot k % D in every
                    // tile): requested here, D real candidates ahead like every other load,
                    // and not when the loop reaches the stand-ins' positions -- which left
                    // each tile's first candidates a full memory latency away (5 candidates
                    // ran at 0.68-0.72 of peak where 4 and 8 reach 0.79).
                    const bool same_tile = (uint32_t)(g + D) < n_real;
                    const uint64_t base = ptr_ahead + (same_tile ? voff : voff_next);
#pragma unroll
                    for (int j = 0; j < kNV; ++j) buf[u][g % D][j] = load16_at<true>(base + j * 1024);
                    // the pointer the NEXT candidate's refill starts from, fetched a candidate
                    // ahead: which one it is depends on n_real, so its LDS read cannot be
                    // placed early by the compiler as in the plain loop, and issued where it
                    // is needed it held every refill back by an LDS round trip
                    if (g + 1 < NC) ptr_ahead = padded_refill_ptr(g + 1);
                }
                if (!real) continue;
#pragma unroll
                for (int e = 0; e < kE; ++e) q[e] = __builtin_fabsf(d[e]) * inv[e];
                // fp32 pairwise trees over the tile's kE non-negative terms (log2 kE
                // roundings deep: 3 for fp32 tiles, 4 for bf16 tiles), then fp64
                const float sa = tree_sum<kE, true>(d);
                const float sr = tree_sum<kE, false>(q);
                const double s_abs = acc[g].sum_abs + (double)sa;
                const double s_rel = acc[g].sum_rel + (double)sr;
                const float chk = sa + sr;
                float t_abs = max_abs2(d[0], d[1]);       // largest |d| of this lane's tile elements
                float m_rel = max3(acc[g].max_rel, q[0], q[1]);
#pragma unroll
                for (int e = 2; e < kE; e += 2) {
                    t_abs = max3_abs(t_abs, d[e], d[e + 1]);
                    m_rel = max3(m_rel, q[e], q[e + 1]);
                }
                const float m_abs = max3(acc[g].max_abs, t_abs, t_abs);
                // The tolerance of an element is at least atol (rtol*|r| >= 0 and rounding
                // is monotone), so a tile whose largest |d| does not exceed atol has no
                // mismatch and the per-element comparison is skipped.  It is taken by the
                // whole wavefront as soon as one lane cannot rule a mismatch out.
                uint32_t mism = 0;
                if (ballot(!(t_abs <= atol)) != 0) {
                    // (rtol through an opaque copy: the tolerances are then worked out here,
                    // where they are needed, and not once per tile for every candidate's sake,
                    // which cost kE vector registers and 2 kE instructions per tile)
                    float rtol_here = rtol;
                    asm volatile("" : "+s"(rtol_here));
#pragma unroll
                    for (int e = 0; e < kE; ++e) {
                        const float scaled = rtol_here * __builtin_fabsf(r[e]);
                        const float tol = atol + scaled;
                        mism += popc64(ballot(!(__builtin_fabsf(d[e]) <= tol)));
                    }
                }
                // Every d and q of the tile is finite and no fp32 partial sum overflowed
                // <=> chk is finite.  (A NaN or Inf reference element makes d non-finite
                // for any candidate value, so it lands here too.)
                if (ballot(!(chk < kInf)) == 0) {
                    acc[g].max_abs = m_abs;
                    acc[g].max_rel = m_rel;
                    acc[g].sum_abs = s_abs;
                    acc[g].sum_rel = s_rel;
                    if (mism != 0 && lane == 0) xacc[g].n_mismatch += mism;
                } else {
                    // What a broken kernel tends to produce: NaN or +-Inf, throughout a tile
                    // or scattered among numbers.  Over reference elements below 2^102 in
                    // magnitude a difference is NaN iff the candidate element is NaN and
                    // infinite iff it is infinite (a finite one cannot carry the difference
                    // past the largest binary32 number: 2^102 is a quarter of its last
                    // place), so such a tile is settled here from the differences alone: an
                    // element whose difference is not a number mismatches and is excluded from
                    // the statistics (0, the identity of both sums and both maxima, takes its
                    // place), the flags follow from which of the two kinds occurred.  Counts
                    // and flags are kept per lane and combined once per tile.
                    bool settled = false;
                    // (through an opaque copy: the compiler otherwise duplicates the candidates'
                    // code along "the tile is moderate" and "it is not", which costs the loop
                    // its register allocation)
                    uint32_t moderate_here = __builtin_amdgcn_readfirstlane(moderate_tile ? 1u : 0u);
                    asm volatile("" : "+s"(moderate_here));
                    if (moderate_here != 0u) {
                        float rtol_here = rtol;
                        asm volatile("" : "+s"(rtol_here));
                        uint32_t counts = 0;   // mismatches | exclusions << 16
                        uint32_t flags = 0;
#pragma unroll
                        for (int e = 0; e < kE; ++e) {
                            const float scaled = rtol_here * __builtin_fabsf(r[e]);
                            const float tol = atol + scaled;
                            const float ad = __builtin_fabsf(d[e]);
                            counts += (ad <= tol) ? 0u : 1u;          // NaN and Inf included
                            const bool is_number = ad < kInf;
                            counts += is_number ? 0u : 0x10000u;
                            flags |= (ad == kInf) ? (uint32_t)(EVO_F_CAND_INF | EVO_F_INF_DIFF) : 0u;
                            flags |= (ad != ad) ? (uint32_t)(EVO_F_CAND_NAN | EVO_F_NAN_SITE_DIFF) : 0u;
                            d[e] = is_number ? ad : 0.0f;
                            q[e] = is_number ? q[e] : 0.0f;
                            if (kE > 8 && (e & 3) == 3) __builtin_amdgcn_sched_barrier(0);   // (register pressure)
                        }
                        const float sa_n = tree_sum<kE, false>(d);
                        const float sr_n = tree_sum<kE, false>(q);
                        const float chk_n = sa_n + sr_n;
                        // (still not finite: a sum or a relative error that overflows binary32
                        // -- left to the exact path)
                        if (ballot(!(chk_n < kInf)) == 0) {
                            float ta_n = max3(0.0f, d[0], d[1]);
                            float mr_n = max3(acc[g].max_rel, q[0], q[1]);
#pragma unroll
                            for (int e = 2; e < kE; e += 2) {
                                ta_n = max3(ta_n, d[e], d[e + 1]);
                                mr_n = max3(mr_n, q[e], q[e + 1]);
                            }
                            acc[g].max_abs = max3(acc[g].max_abs, ta_n, ta_n);
                            acc[g].max_rel = mr_n;
                            acc[g].sum_abs += (double)sa_n;
                            acc[g].sum_rel += (double)sr_n;
                            settle_counts(&xacc[g], lane, counts, flags);
                            settled = true;
                        }
                    }
                    if (!settled) redo_mask |= 1u << g;
                }
            }
            if (lane == 0) redo[slot] = (uint16_t)redo_mask;
            any_redo |= redo_mask;
          }
        }
    }

    __builtin_amdgcn_s_setprio(0);
    // Lanes -> wavefront (the mismatch counts are in xacc), see reduce_group_to_rows.
    uint32_t ma_bits[NC], mr_bits[NC];
    double sum_a[NC], sum_r[NC];
#pragma unroll
    for (int g = 0; g < NC; ++g) {
        ma_bits[g] = __builtin_bit_cast(uint32_t, acc[g].max_abs);
        mr_bits[g] = __builtin_bit_cast(uint32_t, acc[g].max_rel);
        sum_a[g] = acc[g].sum_abs;
        sum_r[g] = acc[g].sum_rel;
    }
    reduce_group_to_rows<NC>(ma_bits, mr_bits, sum_a, sum_r, lane, 0u, wpart);
    return any_redo;
}

// Pairwise sum of N binary64 values (of their magnitudes when ABS), N a power of two.
template <int N, bool ABS>
__device__ __forceinline__ double tree_sum_f64(const double *v) {
    if constexpr (N == 1) {
        return ABS ? __builtin_fabs(v[0]) : v[0];
    } else {
        return tree_sum_f64<N / 2, ABS>(v) + tree_sum_f64<N / 2, ABS>(v + N / 2);
    }
}

__device__ __forceinline__ uint64_t u64_of(uint32_t lo, uint32_t hi) { return ((uint64_t)hi << 32) | lo; }

// Fast path for the 64-bit and integer element types (EVO_F64, EVO_I32, EVO_I64): the
// load pipeline of fast_tiles with the arithmetic of those types.  Kept apart from
// fast_tiles so that the register allocation of the binary32 loop is not touched.
//   EVO_F64  as fast_tiles with every operation in binary64 (correctly rounded division
//            for the reciprocal); a tile's maxima are rounded to binary32 when they are
//            folded into the running ones.
//   integers |c - r| as an exact unsigned integer; running maximum as an integer (kept in
//            the two 32-bit words of the accumulator's maxima), sum of the exactly
//            converted differences in binary64; nothing is ever left to the exact path.
template <uint32_t DT, int NC, bool REF_STREAM, bool PADDED>
__device__ __forceinline__ uint32_t fast_tiles_wide(const char *rptr, uint64_t cand_ptr_of_lane,
                                                    const TileWalk walk, uint64_t t_fend,
                                                    float atol, float rtol, int lane,
                                                    bool second_round, uint32_t n_real,
                                                    uint16_t *redo, Partial *wpart, ExactAcc *xacc) {
    using TL = Tile<DT>;
    constexpr bool kInt = kIsInt<DT>;
    constexpr int kE = TL::kE;
    constexpr int kNV = TL::kNV;
    constexpr uint64_t kTileBytes = (uint64_t)tile_elems(DT) * elem_bytes(DT);
    constexpr int D = NC < kDepth ? NC : kDepth;
    const uint32_t lane_off = (uint32_t)lane * 16u;
    const double atol_d = (double)atol, rtol_d = (double)rtol;

    Acc acc[NC];
    uint32_t n_mismatch[NC];
    const char *cptr[NC];
#pragma unroll
    for (int g = 0; g < NC; ++g) {
        acc[g] = Acc{0.0f, 0.0f, 0.0, 0.0};   // integers: the two maxima hold one 64-bit integer, 0
        n_mismatch[g] = 0;
        cptr[g] = lane_ptr(cand_ptr_of_lane, g);
    }
    uint32_t any_redo = 0;

    const uint32_t k_end = walk.steps_below(t_fend);
    if (k_end > 0) {
        u32x4 ref_raw[kNV];
        u32x4 buf[D][kNV];
        {
            const uint64_t off = walk.at(0) * kTileBytes;
#pragma unroll
            for (int j = 0; j < kNV; ++j) ref_raw[j] = load16<REF_STREAM>(rptr + off + j * 1024, lane_off);
#pragma unroll
            for (int g = 0; g < D; ++g)
#pragma unroll
                for (int j = 0; j < kNV; ++j) buf[g][j] = load16<true>(cptr[g] + off + j * 1024, lane_off);
        }
        uint64_t t = walk.at(0);
        for (uint32_t slot = 0; slot < k_end; ++slot) {
            if (second_round) {   // issue priority, as in fast_tiles
                if (slot & 2u) __builtin_amdgcn_s_setprio(1);
                else __builtin_amdgcn_s_setprio(0);
            }
            const uint64_t off = t * kTileBytes;
            const uint64_t t_next = (slot + 1 < k_end) ? walk.at(slot + 1) : t;
            const uint64_t off_next = t_next * kTileBytes;

            // this tile's reference elements, then the request for the next tile's
            u32x4 rw[kNV];
#pragma unroll
            for (int j = 0; j < kNV; ++j) rw[j] = ref_raw[j];
#pragma unroll
            for (int j = 0; j < kNV; ++j) ref_raw[j] = load16<REF_STREAM>(rptr + off_next + j * 1024, lane_off);
            double r[kInt ? 1 : kE], inv[kInt ? 1 : kE];
            bool moderate_tile = false;   // every |r| of the tile below kModerateD (and none NaN)
            if constexpr (!kInt) {
#pragma unroll
                for (int j = 0; j < kNV; ++j) {
                    r[2 * j] = __builtin_bit_cast(double, u64_of(rw[j].x, rw[j].y));
                    r[2 * j + 1] = __builtin_bit_cast(double, u64_of(rw[j].z, rw[j].w));
                }
                bool huge = false;
#pragma unroll
                for (int e = 0; e < kE; ++e) {
                    const double ar = __builtin_fabs(r[e]);
                    inv[e] = ar >= kDblMin ? 1.0 / ar : 0.0;
                    huge = huge || !(ar < kModerateD);
                }
                moderate_tile = ballot(huge) == 0;
            }

            uint32_t redo_mask = 0;
#pragma unroll
            for (int g = 0; g < NC; ++g) {
                const bool real = !PADDED || (uint32_t)g < n_real;   // see fast_tiles
                u32x4 cw[kNV];
#pragma unroll
                for (int j = 0; j < kNV; ++j) cw[j] = buf[g % D][j];
                // refill the slot: candidate g+D of this tile, or g+D-NC of the next
                if (!PADDED || (uint32_t)((g + D) % NC) < n_real) {
#pragma unroll
                    for (int j = 0; j < kNV; ++j)
                        buf[g % D][j] = load16<true>(cptr[(g + D) % NC] + (g + D < NC ? off : off_next) + j * 1024,
                                               lane_off);
                }
                if (!real) continue;
                if constexpr (DT == EVO_F64) {
                    double d[kE], q[kE];
#pragma unroll
                    for (int j = 0; j < kNV; ++j) {
                        d[2 * j] = __builtin_bit_cast(double, u64_of(cw[j].x, cw[j].y)) - r[2 * j];
                        d[2 * j + 1] = __builtin_bit_cast(double, u64_of(cw[j].z, cw[j].w)) - r[2 * j + 1];
                    }
#pragma unroll
                    for (int e = 0; e < kE; ++e) q[e] = __builtin_fabs(d[e]) * inv[e];
                    const double sa = tree_sum_f64<kE, true>(d);
                    const double sr = tree_sum_f64<kE, false>(q);
                    const double chk = sa + sr;
                    double t_abs = __builtin_fabs(d[0]), t_rel = q[0];
#pragma unroll
                    for (int e = 1; e < kE; ++e) {
                        t_abs = __builtin_fmax(t_abs, __builtin_fabs(d[e]));
                        t_rel = __builtin_fmax(t_rel, q[e]);
                    }
                    uint32_t mism = 0;
                    if (ballot(!(t_abs <= atol_d)) != 0) {   // see fast_tiles
#pragma unroll
                        for (int e = 0; e < kE; ++e) {
                            const double scaled = rtol_d * __builtin_fabs(r[e]);
                            const double tol = atol_d + scaled;
                            mism += popc64(ballot(!(__builtin_fabs(d[e]) <= tol)));
                        }
                    }
                    if (ballot(!(chk < kInfD)) == 0) {
                        const float ta = (float)t_abs, tr = (float)t_rel;   // +Inf beyond binary32
                        acc[g].max_abs = max3(acc[g].max_abs, ta, ta);
                        acc[g].max_rel = max3(acc[g].max_rel, tr, tr);
                        acc[g].sum_abs += sa;
                        acc[g].sum_rel += sr;
                        n_mismatch[g] += mism;
                    } else {
                        // As in fast_tiles: over a moderate reference tile (below 2^969 a finite
                        // candidate element cannot carry the difference past the largest
                        // binary64 number: that is a quarter of its last place) a tile that
                        // holds NaN or +-Inf is settled from the differences alone -- an
                        // element whose difference is not a number mismatches and is excluded.
                        bool settled = false;
                        uint32_t moderate_here = __builtin_amdgcn_readfirstlane(moderate_tile ? 1u : 0u);
                        asm volatile("" : "+s"(moderate_here));   // see fast_tiles
                        if (moderate_here != 0u) {
                            uint32_t counts = 0;   // mismatches | exclusions << 16
                            uint32_t flags = 0;
#pragma unroll
                            for (int e = 0; e < kE; ++e) {
                                const double scaled = rtol_d * __builtin_fabs(r[e]);
                                const double tol = atol_d + scaled;
                                const double ad = __builtin_fabs(d[e]);
                                counts += (ad <= tol) ? 0u : 1u;
                                const bool is_number = ad < kInfD;
                                counts += is_number ? 0u : 0x10000u;
                                flags |= (ad == kInfD) ? (uint32_t)(EVO_F_CAND_INF | EVO_F_INF_DIFF) : 0u;
                                flags |= (ad != ad) ? (uint32_t)(EVO_F_CAND_NAN | EVO_F_NAN_SITE_DIFF) : 0u;
                                d[e] = is_number ? ad : 0.0;
                                q[e] = is_number ? q[e] : 0.0;
                            }
                            const double sa_n = tree_sum_f64<kE, false>(d);
                            const double sr_n = tree_sum_f64<kE, false>(q);
                            const double chk_n = sa_n + sr_n;
                            if (ballot(!(chk_n < kInfD)) == 0) {   // else: overflow, exact path
                                double ta_n = d[0], tr_n = q[0];
#pragma unroll
                                for (int e = 1; e < kE; ++e) {
                                    ta_n = __builtin_fmax(ta_n, d[e]);
                                    tr_n = __builtin_fmax(tr_n, q[e]);
                                }
                                const float ta = (float)ta_n, tr = (float)tr_n;
                                acc[g].max_abs = max3(acc[g].max_abs, ta, ta);
                                acc[g].max_rel = max3(acc[g].max_rel, tr, tr);
                                acc[g].sum_abs += sa_n;
                                acc[g].sum_rel += sr_n;
                                settle_counts(&xacc[g], lane, counts, flags);
                                settled = true;
                            }
                        }
                        if (!settled) redo_mask |= 1u << g;
                    }
                } else if constexpr (DT == EVO_I32) {
                    const uint32_t rr[kE] = {rw[0].x, rw[0].y, rw[0].z, rw[0].w, rw[1].x, rw[1].y, rw[1].z, rw[1].w};
                    const uint32_t cc[kE] = {cw[0].x, cw[0].y, cw[0].z, cw[0].w, cw[1].x, cw[1].y, cw[1].z, cw[1].w};
                    static_assert(kNV == 2, "element lists above");
                    // Integer outputs are mostly equal to the reference: a tile without a
                    // single differing bit changes nothing and costs one XOR per element.
                    uint32_t any_bits = 0;
#pragma unroll
                    for (int e = 0; e < kE; ++e) any_bits |= cc[e] ^ rr[e];
                    if (ballot(any_bits != 0) != 0) {
                        uint32_t du[kE];
                        uint32_t t_max = 0;
                        double sa = 0.0;
#pragma unroll
                        for (int e = 0; e < kE; ++e) {
                            du[e] = abs_diff((int32_t)cc[e], (int32_t)rr[e]);
                            t_max = du[e] > t_max ? du[e] : t_max;
                            sa += (double)du[e];
                        }
                        uint32_t mism = 0;
#pragma unroll
                        for (int e = 0; e < kE; ++e) mism += popc64(ballot(du[e] != 0));
                        const uint32_t run = __builtin_bit_cast(uint32_t, acc[g].max_abs);
                        acc[g].max_abs = __builtin_bit_cast(float, t_max > run ? t_max : run);
                        acc[g].sum_abs += sa;
                        n_mismatch[g] += mism;
                    }
                } else {
                    static_assert(kNV == 2 && kE == 4, "element lists below");
                    const uint64_t rr[kE] = {u64_of(rw[0].x, rw[0].y), u64_of(rw[0].z, rw[0].w),
                                             u64_of(rw[1].x, rw[1].y), u64_of(rw[1].z, rw[1].w)};
                    const uint64_t cc[kE] = {u64_of(cw[0].x, cw[0].y), u64_of(cw[0].z, cw[0].w),
                                             u64_of(cw[1].x, cw[1].y), u64_of(cw[1].z, cw[1].w)};
                    uint64_t any_bits = 0;   // as for 32-bit integers
#pragma unroll
                    for (int e = 0; e < kE; ++e) any_bits |= cc[e] ^ rr[e];
                    if (ballot(any_bits != 0) != 0) {
                        uint64_t du[kE];
                        uint64_t t_max = 0;
                        double sa = 0.0;
#pragma unroll
                        for (int e = 0; e < kE; ++e) {
                            du[e] = abs_diff((int64_t)cc[e], (int64_t)rr[e]);
                            t_max = du[e] > t_max ? du[e] : t_max;
                            sa += (double)du[e];
                        }
                        uint32_t mism = 0;
#pragma unroll
                        for (int e = 0; e < kE; ++e) mism += popc64(ballot(du[e] != 0));
                        const uint64_t run = u64_of(__builtin_bit_cast(uint32_t, acc[g].max_abs),
                                                    __builtin_bit_cast(uint32_t, acc[g].max_rel));
                        const uint64_t top = t_max > run ? t_max : run;
                        acc[g].max_abs = __builtin_bit_cast(float, (uint32_t)top);
                        acc[g].max_rel = __builtin_bit_cast(float, (uint32_t)(top >> 32));
                        acc[g].sum_abs += sa;
                        n_mismatch[g] += mism;
                    }
                }
            }
            if (lane == 0) redo[slot] = (uint16_t)redo_mask;
            any_redo |= redo_mask;
            t = t_next;
        }
    }
    __builtin_amdgcn_s_setprio(0);

    // Lanes -> wavefront, as in fast_tiles.  Integer maxima become binary32 values first
    // (rounded to nearest even: monotone, so the order of rounding and maximum is free).
    uint32_t ma_bits[NC], mr_bits[NC];
    double sum_a[NC], sum_r[NC];
    uint32_t my_mismatches = 0;   // the count of the candidate this lane will write the row of
#pragma unroll
    for (int g = 0; g < NC; ++g) {
        ma_bits[g] = __builtin_bit_cast(uint32_t, acc[g].max_abs);
        mr_bits[g] = __builtin_bit_cast(uint32_t, acc[g].max_rel);
        if constexpr (DT == EVO_I32) {
            ma_bits[g] = __builtin_bit_cast(uint32_t, (float)ma_bits[g]);
        } else if constexpr (DT == EVO_I64) {
            ma_bits[g] = __builtin_bit_cast(uint32_t, (float)u64_of(ma_bits[g], mr_bits[g]));
            mr_bits[g] = 0;
        }
        sum_a[g] = acc[g].sum_abs;
        sum_r[g] = acc[g].sum_rel;
        my_mismatches = group_candidate_of_lane<NC>(lane) == g ? n_mismatch[g] : my_mismatches;
    }
    reduce_group_to_rows<NC>(ma_bits, mr_bits, sum_a, sum_r, lane, my_mismatches, wpart);
    return any_redo;
}

__device__ __forceinline__ void write_stats(evo_stats *dst, const Partial &a, uint64_t n_elems);

// One job: a chunk of tiles of one segment for up to kWaves candidate groups.
// SKIP: instantiate the fast path a second time for groups that end in stand-ins, without
// their loads and arithmetic (off in the all-types kernel, where the stand-ins are loaded --
// their pointer is the reference's -- and evaluated like candidates: same results, and the
// largest translation unit stays a quarter of the compile time).
template <uint32_t DT, bool SKIP>
__device__ __forceinline__ void run_job(const SegDesc &sd, const uint64_t *ptr_table, uint32_t job_local,
                        uint32_t job_global, float atol, float rtol, bool second_round,
                        Partial *partials, ExactAcc (*exact_acc)[kG],
                        Partial (*wave_part)[kG], uint16_t (*redo)[kMaxTilesPerWave],
                        uint64_t (*cand_lds)[kG], evo_stats *stats) {
    constexpr uint32_t kTileElems = tile_elems(DT);
    const int lane = (int)(threadIdx.x & (kLanes - 1));
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    const uint32_t gpw = sd.gpw;
    const uint32_t tpw = kWaves / gpw;                 // tile slots per workgroup
    const uint32_t gl = wave % gpw;                    // group slot inside the job
    const uint32_t tl = wave / gpw;                    // tile slot inside the job
    const uint32_t gblock = job_local / sd.n_chunks;
    const uint32_t chunk = job_local - gblock * sd.n_chunks;
    const uint32_t group = gblock * gpw + gl;
    Group grp = group_of(sd.P, group);
    grp.cand0 = __builtin_amdgcn_readfirstlane(grp.cand0);
    grp.nc = __builtin_amdgcn_readfirstlane(group < sd.n_groups ? grp.nc : 0u);
    const uint32_t nc = grp.nc;

    const uint64_t n = sd.n;
    const uint64_t n_full = n / kTileElems;                         // full tiles
    const uint64_t n_tiles = (n + kTileElems - 1) / kTileElems;     // with the ragged one
    // Workgroups whose indices are congruent modulo 8 run on one XCD, and so do the chunks
    // of a segment whose numbers are congruent modulo 8.  The chunks of such a class are
    // placed side by side in the window, so that each XCD (each L2) streams one contiguous
    // eighth of it.  Dealt round-robin instead, every address that an XCD touches during
    // one step has the same bits 11..13 whenever a workgroup's share of the window is a
    // single tile (four candidate groups side by side): 12 % slower on 64 bf16 candidates
    // of 32 MiB each, 3 % on the ragged fp32 mix, no difference with four tiles per
    // workgroup.
#if EVO_XCD_BLOCKS
    const uint32_t per_class = sd.n_chunks / 8u, longer = sd.n_chunks % 8u, cls = chunk % 8u;
    const uint32_t place = cls * per_class + (cls < longer ? cls : longer) + chunk / 8u;
#else
    const uint32_t place = chunk;
#endif
    const TileWalk walk{sd.n_chunks, place, tpw, tl};

    if (lane < kG) {
        exact_acc[wave][lane] = ExactAcc{0.0, 0.0, 0.0f, 0.0f, 0u, 0u, 0u, 0u};
        wave_part[wave][lane] = Partial{0u, 0u, 0.0, 0.0, 0.0f, 0.0f, 0u, 0u};
    }

    // Lane g fetches the pointer of candidate g of the group: one memory round trip
    // for the whole group.  Vector loads need every tensor 16-byte aligned.
    const char *rptr = uniform_ptr(sd.ref);
    uint64_t cand_ptr_of_lane = 0;
    if ((uint32_t)lane < nc) {
        typedef __attribute__((address_space(1))) const uint64_t global_u64;
        cand_ptr_of_lane = ((global_u64 *)(uintptr_t)ptr_table)[sd.ptr0 + grp.cand0 + lane];
    }
    const bool vec_ok = ((uintptr_t)rptr & 15u) == 0 && ballot((cand_ptr_of_lane & 15u) != 0) == 0;
    // the same pointers in LDS, for fast_tiles (written and read by this wavefront only)
    if (lane < kG) cand_lds[wave][lane] = cand_ptr_of_lane;

    // the segment's last group may end in stand-ins (SegDesc::n_pad)
    const uint32_t n_real = __builtin_amdgcn_readfirstlane(group + 1 == sd.n_groups ? nc - sd.n_pad : nc);
    uint32_t any_redo = 0;
    if (vec_ok && nc > 0) {
        uint16_t *rd = redo[wave];
        Partial *wp = wave_part[wave];
        // the reference tile is shared by the workgroup's wavefronts iff gpw > 1
#define EVO_TILES(FN_, NC_)                                                                    \
    any_redo = (gpw == 1)                                                                      \
        ? FN_<DT, NC_, true, false>(rptr, cand_ptr_of_lane, walk, n_full, atol, rtol, lane,     \
                                    second_round, n_real, rd, wp, exact_acc[wave])              \
        : FN_<DT, NC_, false, false>(rptr, cand_ptr_of_lane, walk, n_full, atol, rtol, lane,    \
                                     second_round, n_real, rd, wp, exact_acc[wave])
#define EVO_TILES_PADDED(FN_, NC_)                                                             \
    any_redo = FN_<DT, NC_, true, (SKIP && NC_ >= 4)>(rptr, cand_ptr_of_lane, walk, n_full, atol, rtol, \
                                                      lane, second_round, n_real, rd, wp, exact_acc[wave])
#define EVO_TILES_LDS(FN_, NC_)                                                                \
    any_redo = (gpw == 1)                                                                      \
        ? FN_<DT, NC_, true, false>(rptr, cand_lds[wave], walk, n_full, atol, rtol, lane,       \
                                    second_round, n_real, rd, wp, exact_acc[wave])              \
        : FN_<DT, NC_, false, false>(rptr, cand_lds[wave], walk, n_full, atol, rtol, lane,      \
                                     second_round, n_real, rd, wp, exact_acc[wave])
#define EVO_TILES_PADDED_LDS(FN_, NC_)                                                         \
    any_redo = FN_<DT, NC_, true, (SKIP && NC_ >= 4)>(rptr, cand_lds[wave], walk, n_full, atol, rtol, \
                                                      lane, second_round, n_real, rd, wp, exact_acc[wave])
        // A segment that is a single group with stand-ins (so gpw == 1) skips them.  Beside
        // full groups the workgroup ends with its full groups anyway, and the stand-ins
        // are loaded (cache hits) and evaluated like candidates.
        const bool skip = SKIP && sd.n_groups == 1 && n_real < nc;
#define EVO_FAST(NC_)                                                                          \
    if constexpr (kIsWide<DT>) {                                                               \
        if (NC_ >= 4 && skip) { EVO_TILES_PADDED(fast_tiles_wide, NC_); }                      \
        else { EVO_TILES(fast_tiles_wide, NC_); }                                              \
    } else {                                                                                   \
        if (NC_ >= 4 && skip) { EVO_TILES_PADDED_LDS(fast_tiles, NC_); }                       \
        else { EVO_TILES_LDS(fast_tiles, NC_); }                                               \
    }
        switch (nc) {
#if EVO_KG > 8
            case 16: EVO_FAST(16); break;
#endif
            case 8: EVO_FAST(8); break;
            case 4: EVO_FAST(4); break;
            case 2: EVO_FAST(2); break;
            default: EVO_FAST(1); break;
        }
#undef EVO_FAST
#undef EVO_TILES
#undef EVO_TILES_PADDED
#undef EVO_TILES_LDS
#undef EVO_TILES_PADDED_LDS
    }

    // Exact path over whatever is left: tiles the fast path flagged, the ragged last
    // tile of the segment, and everything when some tensor is not 16-byte aligned.
    if (nc > 0) {
        const uint32_t all_mask = (1u << n_real) - 1u;   // stand-ins are never evaluated
        const uint32_t k_all = walk.steps_below(n_tiles);
        auto one_by_one = [&](uint64_t t, uint32_t m) {
            while (m) {
                const int g = __builtin_ctz(m);
                m &= m - 1;
                exact_tile<DT>(rptr, lane_ptr(cand_ptr_of_lane, (uint32_t)g), n,
                               t * (uint64_t)kTileElems, lane, atol, rtol, &exact_acc[wave][g]);
            }
        };
        if (vec_ok) {
            const uint32_t k_fast = walk.steps_below(n_full);   // the steps the fast path took
            if (any_redo) {
                if constexpr (!kIsWide<DT>) {
                    // candidate by candidate
                    uint32_t cm = __builtin_amdgcn_readfirstlane(any_redo & all_mask);
                    while (cm) {
                        const uint32_t g = (uint32_t)__builtin_ctz(cm);
                        cm &= cm - 1;
                        exact_candidate_pass<DT>(rptr, lane_ptr(cand_ptr_of_lane, g), walk, k_fast, g,
                                                 redo[wave], lane, atol, rtol, &exact_acc[wave][g]);
                    }
                } else {
                    // The list of flagged tiles is scanned 64 steps at a time, and a tile's
                    // number (a division) is only worked out for the flagged ones: step by
                    // step, the scan alone took 0.4 us per step, 400 us after a 2^30-element
                    // launch.
                    for (uint32_t k0 = 0; k0 < k_fast; k0 += (uint32_t)kLanes) {
                        const uint32_t kk = k0 + (uint32_t)lane;
                        const uint32_t v = kk < k_fast ? (uint32_t)redo[wave][kk] & all_mask : 0u;
                        uint64_t hits = ballot(v != 0);
                        while (hits) {
                            const uint32_t b = (uint32_t)__builtin_ctzll(hits);
                            hits &= hits - 1;
                            one_by_one(walk.at(k0 + b), __builtin_amdgcn_readlane(v, b));
                        }
                    }
                }
            }
            // the ragged tile: only the last step of the walk can land on it
            if (k_all > k_fast) one_by_one(walk.at(k_all - 1), all_mask);
        } else {
            for (uint32_t k = 0; k < k_all; ++k) one_by_one(walk.at(k), all_mask);
        }
        if ((uint32_t)lane < nc) {
            const ExactAcc x = exact_acc[wave][lane];
            Partial p = wave_part[wave][lane];
            p.n_mismatch += x.n_mismatch;
            p.n_excluded += x.n_excluded;
            p.sum_abs += x.sum_abs;
            p.sum_rel += x.sum_rel;
            p.max_abs = __builtin_fmaxf(p.max_abs, x.max_abs);
            p.max_rel = __builtin_fmaxf(p.max_rel, x.max_rel);
            p.flags |= x.flags;
            wave_part[wave][lane] = p;
        }
    }
    __syncthreads();

    // Wavefronts -> workgroup, in wave order, one thread per (group slot, candidate).
    if (threadIdx.x < (uint32_t)kRowsPerJob) {
        const uint32_t slot = threadIdx.x / kG;     // group slot
        const uint32_t gi = threadIdx.x % kG;
        if (slot < gpw) {
            Partial out = wave_part[slot][gi];      // tile slot 0
            for (uint32_t k = 1; k < tpw; ++k) {
                const Partial &o = wave_part[k * gpw + slot][gi];
                out.n_mismatch += o.n_mismatch;
                out.n_excluded += o.n_excluded;
                out.sum_abs += o.sum_abs;
                out.sum_rel += o.sum_rel;
                out.max_abs = __builtin_fmaxf(out.max_abs, o.max_abs);
                out.max_rel = __builtin_fmaxf(out.max_rel, o.max_rel);
                out.flags |= o.flags;
            }
            if (sd.n_jobs == 1 && sd.n_cases <= 1) {
                // The segment was this one job (small tensors: the call is bound by latency,
                // and tickets with their folds would double it): the row is final and goes
                // straight into the caller's evo_stats.  One group block: the group is the slot.
                const Group gr = group_of(sd.P, slot);
                const uint32_t p = gr.cand0 + gi;
                if (gi < gr.nc && p < sd.P - sd.n_pad) write_stats(&stats[sd.stats_row0 + p], out, sd.n);
            } else {
                // published by the release of the ticket this workgroup takes next
                partials[(uint64_t)job_global * kRowsPerJob + slot * kG + gi] = out;
            }
        }
    }
}

// Reduction tree over the jobs of a segment.  Level 1: the jobs of a group block are
// taken kFold consecutive chunks at a time; the last workgroup of such a bundle to finish
// adds the bundle's rows (in chunk order) into one second-level row per candidate.
// Level 2: the last bundle of the segment to be folded adds the second-level rows (in
// bundle order) and writes the evo_stats rows.  Every order is a function of the launch
// geometry only, so the sums are reproducible; and no workgroup ever has to read more
// than a few dozen rows per candidate after the last tile has been streamed.
constexpr uint32_t kFold = 16;
#ifndef EVO_ONE_LEVEL_ROWS
#define EVO_ONE_LEVEL_ROWS 8
#endif
constexpr uint32_t kOneLevelRows = EVO_ONE_LEVEL_ROWS;   // see check_body

__device__ __forceinline__ void add_row(Partial &a, const uint64_t (&w)[6]) {
    a.n_mismatch += w[0];
    a.n_excluded += w[1];
    a.sum_abs += __builtin_bit_cast(double, w[2]);
    a.sum_rel += __builtin_bit_cast(double, w[3]);
    a.max_abs = __builtin_fmaxf(a.max_abs, as_f32((uint32_t)w[4]));
    a.max_rel = __builtin_fmaxf(a.max_rel, as_f32((uint32_t)(w[4] >> 32)));
    a.flags |= (uint32_t)w[5];
}

__device__ __forceinline__ void add_partial(Partial &a, const Partial &o) {
    a.n_mismatch += o.n_mismatch;
    a.n_excluded += o.n_excluded;
    a.sum_abs += o.sum_abs;
    a.sum_rel += o.sum_rel;
    a.max_abs = __builtin_fmaxf(a.max_abs, o.max_abs);
    a.max_rel = __builtin_fmaxf(a.max_rel, o.max_rel);
    a.flags |= o.flags;
}

// One 48-byte row, written by another workgroup (possibly through another XCD's L2), as three
// plain 16-byte loads.  What makes them see the writer's data is the acquire of the ticket
// that thread 0 drew before (it invalidates this compute unit's L1 and the stale lines of
// this XCD's L2) and the workgroup barrier behind it; no line of these rows can come back
// stale afterwards, because rows that share a cache line have one writer, and it had released
// them before that ticket could be the last.  As six device-scope 8-byte loads -- each of
// which goes to memory on its own -- the rows of a fold took 5 us to arrive.
__device__ __forceinline__ void load_row(const Partial *row, uint64_t (&w)[6]) {
    typedef __attribute__((address_space(1))) const u32x4 global_u32x4;
    global_u32x4 *src = (global_u32x4 *)(uintptr_t)row;
#pragma unroll
    for (int q = 0; q < 3; ++q) {
        const u32x4 v = src[q];
        w[2 * q] = u64_of(v.x, v.y);
        w[2 * q + 1] = u64_of(v.z, v.w);
    }
}

// Level 1: rows of chunks [first, first + count) of group block `gblock` -> one row per
// candidate slot in rows1[bundle].  Thread t: slot row t % 64, quarter t / 64 of the bundle.
__device__ __forceinline__ void fold_bundle(const SegDesc &sd, uint32_t gblock, uint32_t first, uint32_t count,
                            const Partial *rows0, Partial *row1, Partial *fold) {
    static_assert(kRowsPerJob <= 64 && kThreads == 256 && kFold == 16, "thread layout");
    const uint32_t slot_row = threadIdx.x % 64u;
    const uint32_t quarter = threadIdx.x / 64u;
    Partial a{};
    if (slot_row < (uint32_t)kRowsPerJob) {
        uint64_t w[4][6];
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) {
            const uint32_t ch = first + min(quarter * 4u + k, count - 1u);
            const uint64_t job = (uint64_t)sd.job0 + (uint64_t)gblock * sd.n_chunks + ch;
            load_row(rows0 + job * kRowsPerJob + slot_row, w[k]);
        }
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k)
            if (quarter * 4u + k < count) add_row(a, w[k]);
    }
    fold[threadIdx.x] = a;
    __syncthreads();
    if (quarter == 0 && slot_row < (uint32_t)kRowsPerJob) {
        for (uint32_t k = 1; k < 4; ++k) add_partial(a, fold[threadIdx.x + 64u * k]);
        row1[slot_row] = a;   // published by the release of the segment ticket
    }
    __syncthreads();
}

// Level 2.  Thread layout: the candidates of a pass are consecutive threads (their rows of one
// unit are neighbours in memory, so a wavefront's load touches a contiguous run of rows
// instead of 64 different cache lines: the level took 7 us before, with a candidate's R
// ranges side by side), and thread group k of the R groups takes the k-th range of the
// candidate's `units` second-level rows; the R results are then added by a fixed tree.
// A segment that stands alone writes its evo_stats rows; one that is a case of a case
// group leaves one row per candidate in case_rows for write_case_group.
__device__ __forceinline__ void write_stats(evo_stats *dst, const Partial &a, uint64_t n_elems) {
    evo_stats s;
    s.n_mismatch = a.n_mismatch;
    s.n_finite = n_elems - a.n_excluded;
    s.sum_abs_err = a.sum_abs;
    s.sum_rel_err = a.sum_rel;
    s.max_abs_err = a.max_abs;
    s.max_rel_err = a.max_rel;
    s.flags = a.flags;
    s.valid = a.n_mismatch == 0 ? 1u : 0u;
    s.median_ms = 0.0f;
    s.mean_ms = 0.0f;
    s.speedup = 0.0f;
    s.fitness = 0.0f;
    s.n_elems_lo = (uint32_t)(n_elems & 0xffffffffu);
    s.n_elems_hi = (uint32_t)(n_elems >> 32);
    *dst = s;
}

__device__ __forceinline__ void finalize_segment(const SegDesc &sd, const Partial *rows1, uint32_t units,
                                 evo_stats *stats, Partial *case_rows, Partial *fold) {
    uint32_t pc = 1;
    while (pc < sd.P && pc < (uint32_t)kThreads) pc <<= 1;   // candidates per pass (power of 2)
    const uint32_t R = kThreads / pc;                          // chunk ranges per candidate
    const uint32_t per = (units + R - 1) / R;
    const uint32_t ci = threadIdx.x % pc;
    const uint32_t ri = threadIdx.x / pc;

    for (uint32_t p0 = 0; p0 < sd.P; p0 += pc) {
        const uint32_t p = p0 + ci;
        Partial a{};
        if (p < sd.P) {
            uint32_t group, gi;
            locate(sd.P, p, &group, &gi);
            const uint32_t gblock = group / sd.gpw;
            const uint32_t slot = group - gblock * sd.gpw;
            const uint32_t ch_lo = ri * per;
            const uint32_t ch_hi = min(ch_lo + per, units);
            // Rows are fetched eight at a time so that their loads overlap; they are
            // added in bundle order.
            constexpr uint32_t kBatch = 8;
            for (uint32_t ch = ch_lo; ch < ch_hi; ch += kBatch) {
                uint64_t w[kBatch][6];
#pragma unroll
                for (uint32_t k = 0; k < kBatch; ++k) {
                    const uint32_t c2 = min(ch + k, ch_hi - 1);
                    const uint64_t unit = (uint64_t)sd.job0 + (uint64_t)gblock * units + c2;
                    load_row(rows1 + unit * kRowsPerJob + slot * kG + gi, w[k]);
                }
#pragma unroll
                for (uint32_t k = 0; k < kBatch; ++k)
                    if (ch + k < ch_hi) add_row(a, w[k]);
            }
        }
        fold[threadIdx.x] = a;
        __syncthreads();
        // The R ranges of a candidate are added pairwise (range k with range k + stride, a fixed
        // tree): one thread adding them one after the other took 4 us per segment with few
        // candidates, where R is 64 to 256.
        for (uint32_t stride = R >> 1; stride >= 1; stride >>= 1) {
            if (ri < stride) {
                add_partial(a, fold[threadIdx.x + stride * pc]);
                fold[threadIdx.x] = a;
            }
            __syncthreads();
        }
        if (ri == 0 && p < sd.P - sd.n_pad) {
            if (sd.n_cases <= 1) {
                write_stats(&stats[sd.stats_row0 + p], a, sd.n);
            } else {
                case_rows[sd.ptr0 + p] = a;   // published by the release of the case-group ticket
            }
        }
        __syncthreads();
    }
}

// Level 3 (case groups only): candidate p over all cases of the group, cases added in
// case order.
__device__ __forceinline__ void write_case_group(const SegDesc *descs, const SegDesc &sd, const Partial *case_rows,
                                 evo_stats *stats) {
    for (uint32_t p = threadIdx.x; p < sd.P - sd.n_pad; p += kThreads) {
        Partial a{};
        uint64_t n_elems = 0;
        for (uint32_t k = 0; k < sd.n_cases; ++k) {
            const SegDesc &dk = descs[sd.case0 + k];
            uint64_t w[6];
            load_row(case_rows + dk.ptr0 + p, w);
            add_row(a, w);
            n_elems += dk.n;
        }
        write_stats(&stats[sd.stats_row0 + p], a, n_elems);
    }
}

// kFoldCasesDirect: the rows of all jobs of all K cases of a group in one workgroup.  A thread
// per (candidate, case, range of the case's jobs) adds its rows in job order (at most
// kDirectRowsPerThread, fetched together), the ranges of a (candidate, case) are added by a
// fixed tree in LDS, and the cases of a candidate are merged in case order.
__device__ __forceinline__ void finalize_cases_direct(const SegDesc *descs, const SegDesc &sd,
                                                      const Partial *rows, evo_stats *stats, Partial *fold) {
    const uint32_t K = sd.n_cases;
    uint32_t Kp = 1, pc = 1;
    while (Kp < K) Kp <<= 1;
    while (pc < sd.P) pc <<= 1;
    const uint32_t R = (uint32_t)kThreads / (Kp * pc);   // >= 1: the host chose this mode
    const uint32_t ci = threadIdx.x % pc;
    const uint32_t ki = (threadIdx.x / pc) % Kp;
    const uint32_t ri = threadIdx.x / (pc * Kp);
    Partial a{};
    if (ki < K && ci < sd.P) {
        const SegDesc &dk = descs[sd.case0 + ki];
        uint32_t group, gi;
        locate(dk.P, ci, &group, &gi);
        const uint32_t gblock = group / dk.gpw;
        const uint32_t slot = group - gblock * dk.gpw;
        const uint32_t units = dk.n_chunks;
        const uint32_t per = (units + R - 1) / R;
        const uint32_t ch_lo = ri * per;
        const uint32_t ch_hi = min(ch_lo + per, units);
        if (ch_lo < ch_hi) {
            uint64_t w[kDirectRowsPerThread][6];
#pragma unroll
            for (uint32_t k = 0; k < kDirectRowsPerThread; ++k) {
                const uint32_t c2 = min(ch_lo + k, ch_hi - 1);
                const uint64_t unit = (uint64_t)dk.job0 + (uint64_t)gblock * units + c2;
                load_row(rows + unit * kRowsPerJob + slot * kG + gi, w[k]);
            }
#pragma unroll
            for (uint32_t k = 0; k < kDirectRowsPerThread; ++k)
                if (ch_lo + k < ch_hi) add_row(a, w[k]);
        }
    }
    fold[threadIdx.x] = a;
    __syncthreads();
    for (uint32_t stride = R >> 1; stride >= 1; stride >>= 1) {
        if (ri < stride) {
            add_partial(a, fold[threadIdx.x + stride * pc * Kp]);
            fold[threadIdx.x] = a;
        }
        __syncthreads();
    }
    if (threadIdx.x < pc && ci < sd.P - sd.n_pad) {   // range 0 of case 0: the candidate's writer
        Partial m{};
        uint64_t n_elems = 0;
        for (uint32_t k = 0; k < K; ++k) {
            add_partial(m, fold[ci + k * pc]);
            n_elems += descs[sd.case0 + k].n;
        }
        write_stats(&stats[sd.stats_row0 + ci], m, n_elems);
    }
}

// DTS = set of element types (bit 1 << evo_dtype) this instantiation can meet.  A launch
// whose segments all have one element type gets a kernel that holds only that type's
// code, so that its register allocation is not the worst case over all types.
// job / total_jobs: this workgroup's job and the number of jobs of the launch (the grid may
// hold other workgroups too, see evo_evaluate_kernel).  Returns true, in every thread, in a
// workgroup that has just written evo_stats rows.
template <uint32_t DTS>
__device__ __forceinline__ bool check_body(const SegDesc *descs, const uint64_t *ptr_table,
                                           uint32_t S, uint32_t n_first,
                                           uint32_t job, uint32_t total_jobs,
                                           Partial *partials, uint32_t *tickets, evo_stats *stats) {
    // Which segment does this workgroup belong to?  (job0 is ascending.)
    uint32_t lo = 0, hi = S;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (descs[mid].job0 <= job) lo = mid; else hi = mid;
    }
    const uint32_t s = lo;
    const SegDesc sd = descs[s];
    const uint32_t job_local = job - sd.job0;
    const float atol = sd.atol, rtol = sd.rtol;   // the segment's tolerance (set by the host's policy)

    // Workgroups are placed one per compute unit first; those numbered n_first (the number
    // of compute units) and above then share a compute unit, SIMD by SIMD, with one of the
    // first round.  The instruction arbiter of a SIMD prefers its older wavefront, so in a
    // launch that keeps the vector ALUs busy (16-bit element types) the second round would
    // trail the first by 15-25 % and the launch would end with it.  Wavefronts of the
    // second round therefore raise their issue priority every other pair of steps
    // (s_setprio; results do not depend on it), which splits the ALU time evenly.
    const bool second_round = blockIdx.x >= n_first;

    __shared__ ExactAcc exact_acc[kWaves][kG];
    __shared__ Partial wave_part[kWaves][kG];
    __shared__ uint16_t redo[kWaves][kMaxTilesPerWave];
    __shared__ uint64_t cand_lds[kWaves][kG];
    constexpr bool kSkip = (DTS & (DTS - 1u)) == 0;   // one element type: see run_job
    if constexpr ((DTS & (1u << EVO_BF16)) != 0) {
        if (sd.dtype == EVO_BF16 || DTS == (1u << EVO_BF16))
            run_job<EVO_BF16, kSkip>(sd, ptr_table, job_local, job, atol, rtol, second_round, partials, exact_acc,
                             wave_part, redo, cand_lds, stats);
    }
    if constexpr ((DTS & (1u << EVO_F16)) != 0) {
        if (sd.dtype == EVO_F16 || DTS == (1u << EVO_F16))
            run_job<EVO_F16, kSkip>(sd, ptr_table, job_local, job, atol, rtol, second_round, partials, exact_acc,
                             wave_part, redo, cand_lds, stats);
    }
    if constexpr ((DTS & (1u << EVO_F32)) != 0) {
        if (sd.dtype == EVO_F32 || DTS == (1u << EVO_F32))
            run_job<EVO_F32, kSkip>(sd, ptr_table, job_local, job, atol, rtol, second_round, partials, exact_acc,
                             wave_part, redo, cand_lds, stats);
    }
    if constexpr ((DTS & (1u << EVO_F64)) != 0) {
        if (sd.dtype == EVO_F64 || DTS == (1u << EVO_F64))
            run_job<EVO_F64, kSkip>(sd, ptr_table, job_local, job, atol, rtol, second_round, partials, exact_acc,
                             wave_part, redo, cand_lds, stats);
    }
    if constexpr ((DTS & (1u << EVO_I32)) != 0) {
        if (sd.dtype == EVO_I32 || DTS == (1u << EVO_I32))
            run_job<EVO_I32, kSkip>(sd, ptr_table, job_local, job, atol, rtol, second_round, partials, exact_acc,
                             wave_part, redo, cand_lds, stats);
    }
    if constexpr ((DTS & (1u << EVO_I64)) != 0) {
        if (sd.dtype == EVO_I64 || DTS == (1u << EVO_I64))
            run_job<EVO_I64, kSkip>(sd, ptr_table, job_local, job, atol, rtol, second_round, partials, exact_acc,
                             wave_part, redo, cand_lds, stats);
    }

    // Two tickets: the bundle of kFold chunks this job belongs to, then the segment (see
    // fold_bundle).  Second-level rows and tickets follow the first-level ones in the same
    // buffers; all counters re-arm themselves.
    //
    // Ordering.  Rows are written with plain stores by many threads; the workgroup barrier
    // orders them before thread 0's ticket, an acquire-release read-modify-write at device
    // scope, whose release makes everything that happened before it in the workgroup
    // visible to the other XCDs.  The workgroup that draws the last ticket acquires through
    // the same operation, hands that on to its other threads through the next barrier, and
    // reads the rows with plain loads (see load_row).  There is no separate fence: each
    // one is a write-back and invalidation of the whole L2 of the XCD and was measured at
    // 2-10 us, on a path that nothing overlaps once the last tile has been streamed.
    __shared__ uint32_t is_last;
    __shared__ Partial fold[kThreads];
    Partial *rows1 = partials + (uint64_t)total_jobs * kRowsPerJob;
    uint32_t *seg_tickets = tickets + total_jobs;
    const uint32_t gblock = job_local / sd.n_chunks;
    const uint32_t chunk = job_local - gblock * sd.n_chunks;
    const uint32_t units = (sd.n_chunks + kFold - 1) / kFold;        // bundles per group block
    const uint32_t bundle = sd.job0 + gblock * units + chunk / kFold; // unique in the launch
    const uint32_t first = (chunk / kFold) * kFold;
    const uint32_t count = min(kFold, sd.n_chunks - first);
    __syncthreads();
    if (sd.n_jobs == 1 && sd.n_cases <= 1) return true;   // run_job has written the evo_stats rows
    Partial *case_rows = rows1 + (uint64_t)total_jobs * kRowsPerJob;
    if (sd.fold_mode == kFoldCasesDirect) {
        // A small case group: one ticket for all jobs of all its cases (they are numbered
        // consecutively), and the last one folds everything.
        uint32_t *group_ticket = seg_tickets + S + sd.case0;
        if (threadIdx.x == 0) {
            const SegDesc &d_first = descs[sd.case0], &d_last = descs[sd.case0 + sd.n_cases - 1];
            const uint32_t group_jobs = d_last.job0 + d_last.n_jobs - d_first.job0;
            const uint32_t prev = __hip_atomic_fetch_add(group_ticket, 1u, __ATOMIC_ACQ_REL,
                                                         __HIP_MEMORY_SCOPE_AGENT);
            is_last = (prev == group_jobs - 1) ? 1u : 0u;
        }
        __syncthreads();
        if (!is_last) return false;
        finalize_cases_direct(descs, sd, partials, stats, fold);
        if (threadIdx.x == 0)
            __hip_atomic_store(group_ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return true;
    }
    // A segment whose jobs' rows one workgroup can add in a few batches per thread (at most
    // kOneLevelRows per thread in finalize_segment's layout, i.e. one batch of loads: up to 128
    // jobs of 16 candidates, 512 of 4, any number of a single one) skips the first level: every job takes the segment's ticket, and the last one
    // adds the jobs' rows directly, in job order.  That is one ticket round trip and one fold
    // less on the path that nothing overlaps (2-3 us of a 25-45 us launch).  With more rows per
    // thread the single fold takes longer than the two levels it replaces (measured with 32:
    // the ragged eight-shape mix 0.71 -> 0.72 ms, 2^23 x 16 114 -> 117 us).
    uint32_t pc = 1;
    while (pc < sd.P && pc < (uint32_t)kThreads) pc <<= 1;
    const bool one_level = (uint64_t)sd.n_chunks * pc <= (uint64_t)kOneLevelRows * kThreads;
    if (one_level) {
        if (threadIdx.x == 0) {
            const uint32_t prev = __hip_atomic_fetch_add(&seg_tickets[s], 1u, __ATOMIC_ACQ_REL,
                                                         __HIP_MEMORY_SCOPE_AGENT);
            is_last = (prev == sd.n_jobs - 1) ? 1u : 0u;
        }
        __syncthreads();
        if (!is_last) return false;
        finalize_segment(sd, partials, sd.n_chunks, stats, case_rows, fold);
    } else {
        if (threadIdx.x == 0) {
            const uint32_t prev = __hip_atomic_fetch_add(&tickets[bundle], 1u, __ATOMIC_ACQ_REL,
                                                         __HIP_MEMORY_SCOPE_AGENT);
            is_last = (prev == count - 1) ? 1u : 0u;
        }
        __syncthreads();
        if (!is_last) return false;
        fold_bundle(sd, gblock, first, count, partials, rows1 + (uint64_t)bundle * kRowsPerJob, fold);
        if (threadIdx.x == 0) {
            __hip_atomic_store(&tickets[bundle], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint32_t n_bundles = units * ((sd.n_groups + sd.gpw - 1) / sd.gpw);
            const uint32_t prev = __hip_atomic_fetch_add(&seg_tickets[s], 1u, __ATOMIC_ACQ_REL,
                                                         __HIP_MEMORY_SCOPE_AGENT);
            is_last = (prev == n_bundles - 1) ? 1u : 0u;
        }
        __syncthreads();
        if (!is_last) return false;
        finalize_segment(sd, rows1, units, stats, case_rows, fold);
    }
    if (threadIdx.x == 0)
        __hip_atomic_store(&seg_tickets[s], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (sd.n_cases <= 1) return true;

    // The segment is one case of a case group: third ticket, and the last case merges.
    uint32_t *case_tickets = seg_tickets + S;
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t prev = __hip_atomic_fetch_add(&case_tickets[sd.case0], 1u, __ATOMIC_ACQ_REL,
                                                     __HIP_MEMORY_SCOPE_AGENT);
        is_last = (prev == sd.n_cases - 1) ? 1u : 0u;
    }
    __syncthreads();
    if (!is_last) return false;
    write_case_group(descs, sd, case_rows, stats);
    if (threadIdx.x == 0)
        __hip_atomic_store(&case_tickets[sd.case0], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return true;
}

template <uint32_t DTS>
__global__ void __launch_bounds__(kThreads, EVO_WAVES_PER_EU)
evo_check_kernel(const SegDesc *__restrict__ descs, const uint64_t *__restrict__ ptr_table,
                 uint32_t S, uint32_t n_first,
                 Partial *__restrict__ partials, uint32_t *__restrict__ tickets,
                 evo_stats *__restrict__ stats) {
    (void)check_body<DTS>(descs, ptr_table, S, n_first, blockIdx.x, gridDim.x, partials, tickets,
                          stats);
}

// Same kernel with the table inside the kernel argument block.  The block is read in
// place through the kernel-argument segment pointer (the table is the first argument,
// at offset 0); naming the by-value parameter would make the compiler copy all of it
// into per-lane scratch memory.
template <uint32_t DTS>
__global__ void __launch_bounds__(kThreads, EVO_WAVES_PER_EU)
evo_check_kernel_inline(const InlineTable /*read via the segment pointer*/, uint32_t S,
                        uint32_t n_first, Partial *__restrict__ partials,
                        uint32_t *__restrict__ tickets, evo_stats *__restrict__ stats) {
    const InlineTable *tab = (const InlineTable *)__builtin_amdgcn_kernarg_segment_ptr();
    (void)check_body<DTS>(tab->descs, tab->ptrs, S, n_first, blockIdx.x, gridDim.x, partials,
                          tickets, stats);
}

// The whole evaluation of a population in one launch: the check of evo_check_kernel_inline
// and the timing reduction of evo_fitness_kernel.  The LAST P + 1 workgroups of the grid
// reduce the timing rows: they are dispatched when the first check jobs end and run, a few
// microseconds each, on compute units that would otherwise idle while the slowest check jobs
// finish (in front of the check jobs, 257 of them delayed a 512-job launch by 10-15 us); the
// others are check jobs.  Speedup, fitness and the population figures need every median and
// every valid flag: each timing workgroup and every workgroup that writes evo_stats rows (one
// per case group, else one per segment; `writers` in all) take a ticket, and whoever draws
// the last of the P + 1 + writers does the rest.
struct FitArgs {
    const float *timings;
    const float *baseline;
    evo_pop_summary *summary;
    float *base;          // two floats of scratch: baseline median and mean
    float *rows;          // P (median, mean) pairs of scratch
    uint32_t *ticket;     // zero between launches
    uint32_t P, T, reducer;
    uint32_t writers;     // workgroups whose check_body returns true
};

template <uint32_t DTS>
__global__ void __launch_bounds__(kThreads, EVO_WAVES_PER_EU)
evo_evaluate_kernel(const InlineTable /*read via the segment pointer*/, uint32_t S,
                    uint32_t n_first, Partial *__restrict__ partials,
                    uint32_t *__restrict__ tickets, evo_stats *__restrict__ stats, const FitArgs fit) {
    const InlineTable *tab = (const InlineTable *)__builtin_amdgcn_kernarg_segment_ptr();
    const uint32_t n_rows = fit.P + 1;
    const uint32_t n_jobs = gridDim.x - n_rows;
    bool last;
    if (blockIdx.x >= n_jobs) {
        // the pairs go to scratch: the evo_stats rows are written whole, later, by the check
        last = fitness_row_and_ticket(fit.timings, fit.baseline, blockIdx.x - n_jobs, fit.P, fit.T, stats,
                                      fit.rows, fit.base, fit.ticket, n_rows + fit.writers - 1u);
    } else {
        if (!check_body<DTS>(tab->descs, tab->ptrs, S, n_first, blockIdx.x, n_jobs, partials,
                             tickets, stats))
            return;
        __shared__ uint32_t drew_last;
        __syncthreads();   // every row of this workgroup is written before thread 0's release
        if (threadIdx.x == 0) {
            const uint32_t prev = __hip_atomic_fetch_add(fit.ticket, 1u, __ATOMIC_ACQ_REL,
                                                         __HIP_MEMORY_SCOPE_AGENT);
            drew_last = (prev == n_rows + fit.writers - 1u) ? 1u : 0u;
        }
        __syncthreads();
        last = drew_last != 0;
    }
    if (!last) return;
    fitness_finish(fit.P, fit.reducer, stats, fit.summary, fit.base, fit.rows);
    if (threadIdx.x == 0) __hip_atomic_store(fit.ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace

// The launchers of the instantiation for the element-type set DTS (declared in
// evo_internal.h; one translation unit per set, see evo_check_inst.hip).
template <uint32_t DTS>
hipError_t launch_check_for(const SegDesc *d_descs, const uint64_t *d_ptrs, uint32_t S,
                            uint32_t total_jobs, uint32_t n_first,
                            Partial *partials, uint32_t *tickets, evo_stats *stats,
                            hipStream_t stream) {
    hipLaunchKernelGGL(evo_check_kernel<DTS>, dim3(total_jobs), dim3(kThreads), 0, stream, d_descs,
                       d_ptrs, S, n_first, partials, tickets, stats);
    return hipGetLastError();
}

template <uint32_t DTS>
hipError_t launch_check_inline_for(const InlineTable &tab, uint32_t S, uint32_t total_jobs,
                                   uint32_t n_first, Partial *partials,
                                   uint32_t *tickets, evo_stats *stats, hipStream_t stream) {
    hipLaunchKernelGGL(evo_check_kernel_inline<DTS>, dim3(total_jobs), dim3(kThreads), 0, stream,
                       tab, S, n_first, partials, tickets, stats);
    return hipGetLastError();
}

template <uint32_t DTS>
hipError_t launch_evaluate_for(const InlineTable &tab, uint32_t S, uint32_t total_jobs,
                               uint32_t n_first, Partial *partials, uint32_t *tickets,
                               evo_stats *stats, const FitLaunch &f, hipStream_t stream) {
    const FitArgs fit{f.timings, f.baseline, f.summary, f.base, f.rows, f.ticket, f.P, f.T, f.reducer,
                      f.writers};
    hipLaunchKernelGGL(evo_evaluate_kernel<DTS>, dim3(total_jobs + f.P + 1), dim3(kThreads), 0, stream,
                       tab, S, n_first, partials, tickets, stats, fit);
    return hipGetLastError();
}

}  // namespace evo
