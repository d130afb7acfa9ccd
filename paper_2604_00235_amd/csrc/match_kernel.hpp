// Pre-RoPE squared-L2 distances over the query ring: the arithmetic shared by the matchers, and the matcher that
// picks one reuse point per KV group (gfx950, wave64).  The per-head matcher of the paper lives in hit_kernel.hpp.
//
// Paper: Eq. (accept) and Sec. 3.2.3 (single streaming pass over the last W queries), Sec. 3.5 step 1,
// Sec. 4.2 "K1" (at most one reuse point per (request, head), then the threshold).
// For request b (ring set slot_ids[b]) and query head h, over the ring entries created at lengths
// n_p in [max(1, n - W), n - 1]:  d2_j = sum_i (q_i - ring_j,i)^2,  j* = argmin (ties -> larger n_p),
// hit iff d2_j* < T^2.  On a hit the head's fresh range starts at s_h = max(0, n_p - B), else at 0.
//
// Arithmetic.  The decision has to agree with an fp64 evaluation of the exact bf16 inputs, so each
// difference is formed in fp64 (exact) and squared/accumulated with fp64 FMAs; the result is within a few
// ulp(fp64) of the true real value, so decisions differ from any other fp64 evaluation only for candidates
// that tie to ~1e-15 relative (the per-head matcher resolves those in index order, see hit_kernel.hpp; the group
// matcher below does not: it is a variant beyond the paper's rule).
//
// Access pattern.  A head's window is contiguous in the ring ([slot][head][entry][d]).  Sixteen lanes own one 256-byte
// row, one 16-byte chunk each, so a load instruction of a wave fetches four whole rows.  Rows are loaded without
// waiting for their n_p tag (the ring memory always exists; an entry outside the window is simply discarded), which
// removes one dependent memory round trip.  The 16 partial sums of a row are combined with four cross-lane adds, the
// per-lane running (d2, n_p) minimum with a shuffle butterfly and one exchange through shared memory between the waves.
#pragma once
#include "common.hpp"

namespace mac {

struct MatchParams {
    const int32_t* slot_ids;     // [batch]
    const int32_t* kv_lens;      // [batch]
    const uint16_t* q_pre;       // [batch, Hq, d] bf16
    const uint16_t* ring_q;      // [slots, Hq, W, 128] bf16
    const int32_t* ring_npos;    // [slots, Hq, W]; 0 = empty entry (the heads of a request carry the same tags)
    MatchPartial* slices;        // [batch*Hq, n_split] nearest entry of each window slice (group matcher)
    MatchPartial* part;          // [batch*Hq] nearest entry of the whole window (written by the finalize kernel)
    int32_t* head_start;         // [batch*Hq] start of each head's fresh range (written by the finalize kernel)
    unsigned long long* st_steps;   // [2]: decode steps, head-steps (device-side so that graph replays count too)
    int32_t batch, Hq, W, max_kv_len;
    int32_t head_dim;            // d of the caller's q_pre rows (ring rows are 128 wide, zero beyond d)
    int32_t n_split;             // window slices per group = gridDim.z of the group matcher (power of two <= 64)
    int32_t rows_per_split;      // multiple of 16 with rows_per_split * G <= kMatchGroupItems
    int32_t G;                   // heads per KV group
    MatchView mv;                // threshold, band and distance cap of the acceptance rule (part unused)
};

// start of the fresh range of a head whose nearest window entry is (d2, np): max(0, np - B) on a hit, else 0;
// clamped to the start of the last-B band like everywhere else
__device__ __forceinline__ int head_start(const MatchView& mv, double d2, int np, int n) {
    const int nb = n - mv.band > 0 ? n - mv.band : 0;
    const int s = match_accept(mv, d2, np, n) ? (np - mv.band > 0 ? np - mv.band : 0) : 0;
    return s < nb ? s : nb;
}

__device__ __forceinline__ double bf16_lo_to_f64(uint32_t pair) { return (double)bits_to_float(pair << 16); }
__device__ __forceinline__ double bf16_hi_to_f64(uint32_t pair) { return (double)bits_to_float(pair & 0xffff0000u); }

// Sums over the 16 lanes of a row of the wave (DPP), the same in each of them
__device__ __forceinline__ float row_sum_f32(float v) {
    v += dpp_f32<kDppQuadSwap1>(v);
    v += dpp_f32<kDppQuadSwap2>(v);
    v += dpp_f32<kDppRowHalfMirror>(v);
    return v + dpp_f32<kDppRowMirror>(v);
}
__device__ __forceinline__ double row_sum_f64(double v) {
    v += dpp_f64<kDppQuadSwap1>(v);
    v += dpp_f64<kDppQuadSwap2>(v);
    v += dpp_f64<kDppRowHalfMirror>(v);
    return v + dpp_f64<kDppRowMirror>(v);
}
// One lane's share of a squared distance in fp64: a 16-byte chunk of the query against the same chunk of a ring row
__device__ __forceinline__ double sq_dist_chunk(const u32x4& q, const u32x4& v) {
    double s0 = 0.0, s1 = 0.0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const double d0 = bf16_lo_to_f64(q[e]) - bf16_lo_to_f64(v[e]);
        const double d1 = bf16_hi_to_f64(q[e]) - bf16_hi_to_f64(v[e]);
        s0 = fma(d0, d0, s0);
        s1 = fma(d1, d1, s1);
    }
    return s0 + s1;
}

constexpr int kMatchThreads = 256;

// One reuse point per KV group: candidates are ranked by D2_j = sum over the group's heads of d2_{h,j} (the squared
// distance of the group's concatenated queries), summed in head order.  One work-group per (KV group, request,
// window slice).  The (row, head) pairs of the slice are dealt to the 64 quads, so all ring loads are independent;
// the per-pair distances meet in shared memory, then thread r sums row r over the heads and the argmin proceeds as
// in the per-head matcher.  The slice result is written for every head of the group, so the consumers need no change.
constexpr int kMatchGroupItems = 4096;   // (row, head) pairs per work-group: 32 KB of shared memory

__global__ __launch_bounds__(kMatchThreads) void match_group_kernel(const MatchParams p) {
    const int g = blockIdx.x, b = blockIdx.y, sp = blockIdx.z;
    const int tid = threadIdx.x;
    const int G = p.G, W = p.W;
    const int n = clampi(p.kv_lens[b], 0, p.max_kv_len);
    const int64_t slot = p.slot_ids[b];
    const int32_t* npos = p.ring_npos + (slot * p.Hq + g * G) * W;       // tags of the group's first head
    const int np_lo = max(1, n - W), np_hi = n - 1;
    const int j_begin = sp * p.rows_per_split;
    const int rows = max(0, min(W, j_begin + p.rows_per_split) - j_begin);
    const int items = rows * G;                                  // <= kMatchGroupItems (host)
    __shared__ double s_pair[kMatchGroupItems];

    // 16 lanes per (row, head) pair, one 16-byte chunk of the ring row and of the head's query each, so that a load
    // instruction takes four whole rows (the access pattern a compute unit pulls fastest); eight pairs per lane and
    // trip, their loads issued before the arithmetic.  Pair i is (row i / G, head i % G): i < 4096 and G <= 32, so the
    // quotient comes exactly out of a single-precision multiplication.
    constexpr int kPairsPerPass = kMatchThreads / 16, kUnroll = 8;
    const int pl = tid >> 4, ch = tid & 15;
    const float inv_g = 1.0f / (float)G;
    for (int i0 = 0; i0 < items; i0 += kUnroll * kPairsPerPass) {
        u32x4 qv[kUnroll], v[kUnroll];
#pragma unroll
        for (int t = 0; t < kUnroll; ++t) {
            const int i = i0 + t * kPairsPerPass + pl;
            const int ic = i < items ? i : items - 1;            // keeps the loads of idle lanes inside the slice
            const int r = (int)(((float)ic + 0.5f) * inv_g), h = g * G + (ic - r * G);
            qv[t] = 8 * ch < p.head_dim ? *reinterpret_cast<const u32x4*>(p.q_pre + ((int64_t)b * p.Hq + h) * p.head_dim + 8 * ch)
                                        : u32x4{0u, 0u, 0u, 0u};
            v[t] = *reinterpret_cast<const u32x4*>(p.ring_q + ((slot * p.Hq + h) * W + j_begin + r) * (int64_t)kHeadDim + 8 * ch);
        }
#pragma unroll
        for (int t = 0; t < kUnroll; ++t) {
            const int i = i0 + t * kPairsPerPass + pl;
            const double d2 = row_sum_f64(sq_dist_chunk(qv[t], v[t]));
            if (i < items && ch == 0) s_pair[i] = d2;
        }
    }
    __syncthreads();

    double best_d2 = INFINITY;
    int best_np = -1, best_j = -1;
    for (int r = tid; r < rows; r += kMatchThreads) {
        const int j = j_begin + r;
        const int np = npos[j];
        double D = 0.0;
        for (int hh = 0; hh < G; ++hh) D += s_pair[r * G + hh];
        if (np >= np_lo && np <= np_hi && better(D, np, best_d2, best_np)) { best_d2 = D; best_np = np; best_j = j; }
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const double od2 = __shfl_xor(best_d2, off);
        const int onp = __shfl_xor(best_np, off);
        const int oj = __shfl_xor(best_j, off);
        if (better(od2, onp, best_d2, best_np)) { best_d2 = od2; best_np = onp; best_j = oj; }
    }
    constexpr int kWaves = kMatchThreads / 64;
    __shared__ double s_d2[kWaves];
    __shared__ int s_np[kWaves], s_j[kWaves];
    if ((tid & 63) == 0) { s_d2[tid >> 6] = best_d2; s_np[tid >> 6] = best_np; s_j[tid >> 6] = best_j; }
    __syncthreads();
    if (tid == 0 && g == 0 && b == 0 && sp == 0) {
        atomicAdd(&p.st_steps[0], 1ull);
        atomicAdd(&p.st_steps[1], (unsigned long long)gridDim.x * gridDim.y * G);
    }
    if (tid < G) {
        best_d2 = s_d2[0]; best_np = s_np[0]; best_j = s_j[0];
        for (int w = 1; w < kWaves; ++w)
            if (better(s_d2[w], s_np[w], best_d2, best_np)) { best_d2 = s_d2[w]; best_np = s_np[w]; best_j = s_j[w]; }
        p.slices[((int64_t)b * p.Hq + g * G + tid) * p.n_split + sp] = MatchPartial{best_d2, best_np, best_j};
    }
}

// Final reducer of the group matcher: one wave per head combines the head's slice results into the nearest entry of
// the whole window and stores it with the start of the head's fresh range, the form the attention and merge kernels
// read (the per-head matcher writes the same two records itself).
__global__ __launch_bounds__(256) void match_group_finalize_kernel(const MatchParams p) {
    const int lane = threadIdx.x & 63;
    const int bh = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (bh >= p.batch * p.Hq) return;
    const int b = bh / p.Hq;
    const int n = clampi(p.kv_lens[b], 0, p.max_kv_len);
    const MatchPartial c = match_nearest_wave(p.slices, p.n_split, bh, 1, lane);
    if (lane == 0) {
        p.part[bh] = c;
        p.head_start[bh] = head_start(p.mv, c.d2, c.np, n);
    }
}

}  // namespace mac
