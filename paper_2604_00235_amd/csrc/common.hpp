// Shared device-side helpers for the MAC-Attention kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mac {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kHeadDim = 128;      // d; a K or V row is 256 bytes = 16 chunks of 16 bytes
constexpr int kTileTokens = 32;    // tokens per MFMA tile of the attention kernel (two 16-token sub-tiles)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float bits_to_float(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t float_to_bits(float f) { return __builtin_bit_cast(uint32_t, f); }

// v_perm_b32: result bytes 0..3 are picked from the 8 bytes {hi_src(4..7), lo_src(0..3)} by the selector.
__device__ __forceinline__ uint32_t perm(uint32_t hi_src, uint32_t lo_src, uint32_t sel) {
    return __builtin_amdgcn_perm(hi_src, lo_src, sel);
}
// (lo16(first), lo16(second)) and (hi16(first), hi16(second)) packed into one dword, first in the low half
__device__ __forceinline__ uint32_t pack_lo16(uint32_t first, uint32_t second) { return perm(second, first, 0x05040100u); }
__device__ __forceinline__ uint32_t pack_hi16(uint32_t first, uint32_t second) { return perm(second, first, 0x07060302u); }

// fp32 -> bf16 bits, round to nearest even; NaN stays NaN
__device__ __forceinline__ uint16_t float_to_bf16_rne(float f) {
    const uint32_t u = float_to_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }   // v_exp_f32; exp2(-inf) = 0

// ---- cross-lane helpers (wave64).  Reductions inside a 16-lane row use DPP (no shared-memory round trip as a
// bpermute-based shuffle has); rows are combined with v_readlane.  Lane-wise exchanges between rows use the
// row-swap instructions of this chip: v_permlane16_swap exchanges the odd rows of its first operand with the even
// rows of its second, v_permlane32_swap the upper half of the first with the lower half of the second.
template <int kCtrl>
__device__ __forceinline__ float dpp_f32(float v) {
    return bits_to_float((uint32_t)__builtin_amdgcn_update_dpp((int)float_to_bits(v), (int)float_to_bits(v), kCtrl, 0xf, 0xf, false));
}
constexpr int kDppQuadSwap1 = 0xB1, kDppQuadSwap2 = 0x4E, kDppRowHalfMirror = 0x141, kDppRowMirror = 0x140;
constexpr int kDppRowRor8 = 0x128;        // lane ^ 8 inside a row of 16
#define MAC_WAVE_REDUCE(NAME, OP)                                                                    \
    __device__ __forceinline__ float NAME(float v) {                                                 \
        v = OP(v, dpp_f32<kDppQuadSwap1>(v));                                                        \
        v = OP(v, dpp_f32<kDppQuadSwap2>(v));                                                        \
        v = OP(v, dpp_f32<kDppRowHalfMirror>(v));                                                    \
        v = OP(v, dpp_f32<kDppRowMirror>(v));                      /* every lane: its row's result */ \
        const float r0 = bits_to_float((uint32_t)__builtin_amdgcn_readlane((int)float_to_bits(v), 0));   \
        const float r1 = bits_to_float((uint32_t)__builtin_amdgcn_readlane((int)float_to_bits(v), 16));  \
        const float r2 = bits_to_float((uint32_t)__builtin_amdgcn_readlane((int)float_to_bits(v), 32));  \
        const float r3 = bits_to_float((uint32_t)__builtin_amdgcn_readlane((int)float_to_bits(v), 48));  \
        return OP(OP(r0, r1), OP(r2, r3));                                                           \
    }
__device__ __forceinline__ float op_add(float a, float b) { return a + b; }
MAC_WAVE_REDUCE(wave_min_f32, fminf)
MAC_WAVE_REDUCE(wave_max_f32, fmaxf)
MAC_WAVE_REDUCE(wave_sum_f32, op_add)      // rows in fixed order: reproducible
#undef MAC_WAVE_REDUCE

// x[l] + x[l ^ 16] and x[l] + x[l ^ 32], lane-wise
__device__ __forceinline__ float add_xor16(float x) {
    const auto r = __builtin_amdgcn_permlane16_swap(float_to_bits(x), float_to_bits(x), false, false);
    return bits_to_float(r[0]) + bits_to_float(r[1]);
}
__device__ __forceinline__ float add_xor32(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(float_to_bits(x), float_to_bits(x), false, false);
    return bits_to_float(r[0]) + bits_to_float(r[1]);
}
__device__ __forceinline__ float max_xor16(float x) {
    const auto r = __builtin_amdgcn_permlane16_swap(float_to_bits(x), float_to_bits(x), false, false);
    return fmaxf(bits_to_float(r[0]), bits_to_float(r[1]));
}
__device__ __forceinline__ float max_xor32(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(float_to_bits(x), float_to_bits(x), false, false);
    return fmaxf(bits_to_float(r[0]), bits_to_float(r[1]));
}
__device__ __forceinline__ double add_xor16(double x) {
    const uint64_t u = __builtin_bit_cast(uint64_t, x);
    const auto lo = __builtin_amdgcn_permlane16_swap((uint32_t)u, (uint32_t)u, false, false);
    const auto hi = __builtin_amdgcn_permlane16_swap((uint32_t)(u >> 32), (uint32_t)(u >> 32), false, false);
    return __builtin_bit_cast(double, ((uint64_t)hi[0] << 32) | lo[0]) + __builtin_bit_cast(double, ((uint64_t)hi[1] << 32) | lo[1]);
}
__device__ __forceinline__ double add_xor32(double x) {
    const uint64_t u = __builtin_bit_cast(uint64_t, x);
    const auto lo = __builtin_amdgcn_permlane32_swap((uint32_t)u, (uint32_t)u, false, false);
    const auto hi = __builtin_amdgcn_permlane32_swap((uint32_t)(u >> 32), (uint32_t)(u >> 32), false, false);
    return __builtin_bit_cast(double, ((uint64_t)hi[0] << 32) | lo[0]) + __builtin_bit_cast(double, ((uint64_t)hi[1] << 32) | lo[1]);
}
__device__ __forceinline__ double readlane_f64(double x, int l) {      // l uniform
    const uint64_t u = __builtin_bit_cast(uint64_t, x);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)u, l), hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(u >> 32), l);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

// sum over the wave of a double, the same in every lane (rows by DPP, the four rows in fixed order)
template <int kCtrl>
__device__ __forceinline__ double dpp_f64(double v) {
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)u, (int)(uint32_t)u, kCtrl, 0xf, 0xf, false);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)(u >> 32), (int)(uint32_t)(u >> 32), kCtrl, 0xf, 0xf, false);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ double wave_sum_f64(double v) {
    v += dpp_f64<kDppQuadSwap1>(v);
    v += dpp_f64<kDppQuadSwap2>(v);
    v += dpp_f64<kDppRowHalfMirror>(v);
    v += dpp_f64<kDppRowMirror>(v);
    return (readlane_f64(v, 0) + readlane_f64(v, 16)) + (readlane_f64(v, 32) + readlane_f64(v, 48));
}
// inclusive prefix sum over the lanes of a wave: shifts inside each 16-lane row (DPP, zeros shifted in), then the totals
// of the rows before
template <int kShift>
__device__ __forceinline__ int dpp_row_shr(int v) { return __builtin_amdgcn_update_dpp(0, v, 0x110 + kShift, 0xf, 0xf, true); }
__device__ __forceinline__ int wave_scan_incl_i32(int v, int lane) {
    v += dpp_row_shr<1>(v);
    v += dpp_row_shr<2>(v);
    v += dpp_row_shr<4>(v);
    v += dpp_row_shr<8>(v);
    const int r0 = __builtin_amdgcn_readlane(v, 15), r1 = __builtin_amdgcn_readlane(v, 31), r2 = __builtin_amdgcn_readlane(v, 47);
    return v + (lane >= 16 ? r0 : 0) + (lane >= 32 ? r1 : 0) + (lane >= 48 ? r2 : 0);
}

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// head_start[] holds, per (request, head), the first key of the head's fresh range; this flag is set when the per-head
// matcher has already finished the head's whole step (hit with a short fresh range): the split-K attention kernel and
// the merge kernel then skip the head.  Starts are below 2^30.
constexpr int kHeadDone = 0x40000000;

// Result of scanning one slice of a head's query-ring window: the nearest entry of the slice.
struct MatchPartial {
    double d2;      // squared distance, +inf if the slice has no candidate
    int32_t np;     // length n_p at which the entry was created, -1 if none
    int32_t j;      // ring entry index, -1 if none
};

// lexicographic order of candidates: smaller distance first, then the more recent entry
__device__ __forceinline__ bool better(double d2, int np, double od2, int onp) {
    return d2 < od2 || (d2 == od2 && np > onp);
}

// Where the per-slice results of the match kernel live and how to turn them into the decision.
struct MatchView {
    const MatchPartial* part;   // [batch*Hq] nearest entry of each head's window; nullptr = no matching (full decode)
    int32_t band;               // B
    int32_t max_gap;            // distance cap on n - n_p; 0 = none
    double T2;                  // (double)T * (double)T, times G when one reuse point is chosen per KV group
};

struct MatchDecision {
    double d2;      // nearest squared distance over the whole window (+inf if it is empty)
    int32_t np;     // matched n_p, or -1 on a miss
    int32_t j;      // matched ring entry, or -1
    int32_t start;  // first key this head has to recompute: max(0, n_p - B) on a hit, 0 on a miss
};

// Acceptance of the nearest candidate (d2, np) of a whole window at length n: threshold, then the optional distance cap.
__device__ __forceinline__ bool match_accept(const MatchView& mv, double d2, int np, int n) {
    return np >= 1 && d2 < mv.T2 && (mv.max_gap <= 0 || n - np <= mv.max_gap);
}

// Nearest entry of a head's whole window from the slice results of the group matcher (paper Sec. 4.2 K1 "final
// reducer").  One wave handles up to 64 / n_split consecutive heads at once: lane l holds slice l % n_split of head
// bh0 + l / n_split (n_split is a power of two <= 64), one coalesced 16-byte load per lane, then a butterfly inside
// each n_split-lane segment.  On return every lane of a segment holds its head's nearest entry; lanes of segments
// >= cnt hold none.  Must be called by all 64 lanes of the wave.
__device__ __forceinline__ MatchPartial match_nearest_wave(const MatchPartial* slices, int S, int bh0, int cnt, int lane) {
    const int seg = lane >> (31 - __builtin_clz(S));         // S is a power of two
    MatchPartial c{INFINITY, -1, -1};
    if (seg < cnt) c = slices[(int64_t)bh0 * S + lane];
    for (int off = S >> 1; off > 0; off >>= 1) {
        const double od2 = __shfl_xor(c.d2, off);
        const int onp = __shfl_xor(c.np, off);
        const int oj = __shfl_xor(c.j, off);
        if (better(od2, onp, c.d2, c.np)) { c.d2 = od2; c.np = onp; c.j = oj; }
    }
    return c;
}

// The decision of a head from the nearest entry of its window (Eq. (accept)): threshold, then the optional distance cap.
__device__ __forceinline__ MatchDecision decide(const MatchView& mv, const MatchPartial& c, int n) {
    MatchDecision r{c.d2, -1, -1, 0};
    if (match_accept(mv, c.d2, c.np, n)) {
        r.np = c.np;
        r.j = c.j;
        r.start = c.np - mv.band > 0 ? c.np - mv.band : 0;
    }
    return r;
}

}  // namespace mac
