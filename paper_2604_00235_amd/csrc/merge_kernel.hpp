// Complete (log-domain merge) and rectify-append (ring write-back) (gfx950).
//
// Merge, per (request b, query head h) -- paper Sec. 3.1 (summaries over disjoint sets add), Eq. (rect-merge),
// Sec. 4.2 "K2 (3) Merge":  in a fixed order
//     rect = prefix (ring summary of the matched entry, on a hit)  (+)  partials of the mid chunks [s_h, n-B)
//     out  = rect  (+)  partials of the band chunks [n-B, n)
// where (O_a, L_a) (+) (O_b, L_b) = ((e^{L_a} O_a + e^{L_b} O_b)/(e^{L_a} + e^{L_b}), ln(e^{L_a} + e^{L_b})),
// evaluated relative to the largest LSE so no exponent overflows; the empty summary is (0, -inf).
// `rect` is this step's total without the last-B band (Fig. 1(c)), built add-only so nothing cancels.
//
// Write-back, per (b, h) -- Sec. 4.1, Sec. 4.2 "K3": ring entry (n-1) mod W of the request's ring set gets the
// pre-RoPE query, the rectified summary row and its ln-LSE; the entry's n_p tag is set to n.  It runs after the
// merge of the same head because the overwritten entry (n_p = n - W) is still a candidate of this step.
//
// A head whose whole step the per-head matcher has finished (hit with a short fresh range, see hit_kernel.hpp) is
// flagged in head_start[]: its work-group leaves at once.
//
// Both steps exist as kernels of their own (merge_kernel, writeback_kernel: one work-group per (head, request))
// and fused in merge_writeback_kernel (one launch less per step; the default).  Folding them further into the
// attention kernel ("last work-group of a group merges") was tried and dropped: the device-scope release fence
// every work-group then needs writes back the XCD's L2 and cost 25-100 % of the attention kernel's time.
#pragma once
#include "common.hpp"

namespace mac {

struct WritebackParams {
    const int32_t* kv_lens;
    const int32_t* slot_ids;
    const uint16_t* q_pre;       // [batch, Hq, d] bf16
    const float* rect_O;         // staging [batch*Hq, 128] (separate-kernel mode only)
    const float* rect_lse;       // [batch*Hq]
    uint16_t* ring_q;            // [slots, Hq, W, 128]
    float* ring_O;               // [slots, Hq, W, 128]
    float* ring_lse;             // [slots, Hq, W]
    int32_t* ring_npos;          // [slots, Hq, W]: every head carries its own n_p tags
    const int32_t* head_start;   // [batch*Hq] or null: heads flagged kHeadDone were appended by the matcher already
    int32_t Hq, W, max_kv_len;
    int32_t head_dim;            // d of the caller's q_pre rows; ring rows are 128 wide, zero beyond d
};

struct MergeParams {
    const int32_t* kv_lens;
    const int32_t* slot_ids;     // null for full decode
    MatchView mv;                // per-head match results; part == nullptr for full decode
    const int32_t* head_start;   // [batch*Hq] or null: heads flagged kHeadDone are finished, their work-group leaves
    int32_t emit_decision;       // 1: this kernel reports the decisions (caller outputs, counters); 0: the matcher did
    int32_t* out_match_pos;      // optional caller outputs [batch*Hq] (MAC mode)
    double* out_match_d2;
    unsigned long long* st_hits; // per (b, h) accumulators, touched only by that (b, h)'s work-group; null for full decode
    unsigned long long* st_gap;
    double* st_skip;
    const float* ring_O;         // [slots, Hq, W, 128]
    const float* ring_lse;       // [slots, Hq, W]
    const float* part_O;         // [batch*Hq, n_slots, 128]
    const float* part_lse;       // [batch*Hq, n_slots]
    void* out;                   // [batch, Hq, d] fp32, or bf16 when out_bf16
    int32_t out_bf16;
    int32_t head_dim;            // d of `out` (the partials and the rings are 128 wide)
    float* out_lse;              // optional [batch, Hq]
    float* rect_O;               // staging for a separate write-back kernel [batch*Hq, 128]; may be null
    float* rect_lse;             // [batch*Hq]
    int32_t Hq, G, W, band, n_mid_slots, n_slots, max_kv_len;
    int32_t chunk_fixed;         // > 0: tokens per work item of the attention kernel, fixed by the caller;
    const int32_t* step_chunk;   // 0: read here what the attention kernel chose for this step
    int32_t* pending;            // the matcher's count of heads left to the split-K path: cleared here for the next step; or null
};

// 256 threads per (request, head).  Thread (c = tid/32, q = tid%32) accumulates the partials
// x = first + c, first + c + 8, ... for the four output columns 4q..4q+3 in a single pass, with weights relative
// to the largest LSE that lane has seen; the 8 lane summaries are combined in a fixed order through LDS, so the
// result is bitwise reproducible.  Two summaries are kept: the rect part (prefix + mid chunks) and the band part.
constexpr int kMergeThreads = 256;
constexpr int kMergeLanes = 8;      // chunks summed in parallel

struct MergeSmem {
    float acc[2][kMergeLanes][kHeadDim];   // [rect part | band part][chunk lane][column]
    float m[2][kMergeLanes];               // running maximum of the LSEs each lane has seen
    float z[2][kMergeLanes];               // sum of weights relative to that maximum
};

// One chunk lane's running summary of four output columns: weights relative to the largest LSE seen so far.
struct LaneMerge {
    float M = -INFINITY, Z = 0.f;
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    // branch-free, so that the loads of later chunks are not held back: an empty summary (L = -inf) gets weight 0
    __device__ __forceinline__ void add(const f32x4 o, float L) {
        const float Mn = fmaxf(M, L);
        const float a = M == -INFINITY ? 0.f : __expf(M - Mn);
        const float w = L == -INFINITY ? 0.f : __expf(L - Mn);
        acc = acc * a + o * w;
        Z = Z * a + w;
        M = Mn;
    }
};

// Ring append of one head by threads d < 128 (values of the rectified summary passed in registers).
__device__ __forceinline__ void writeback_head(const WritebackParams& p, int b, int h, int d, float rect_o, float rect_l) {
    const int n = clampi(p.kv_lens[b], 0, p.max_kv_len);
    if (n < 1) return;
    const int bh = b * p.Hq + h;
    const int64_t slot = p.slot_ids[b];
    const int j = (n - 1) % p.W;
    const int64_t e = (slot * p.Hq + h) * p.W + j;
    p.ring_q[e * kHeadDim + d] = d < p.head_dim ? p.q_pre[(int64_t)bh * p.head_dim + d] : (uint16_t)0;
    p.ring_O[e * kHeadDim + d] = rect_o;
    if (d == 0) {
        p.ring_lse[e] = rect_l;
        p.ring_npos[e] = n;
    }
}

// Merge of one head by a 256-thread work-group; with `do_wb` it also appends to the ring.
// Contains __syncthreads: every thread of the work-group must call it.
__device__ __forceinline__ void merge_head(const MergeParams& p, const WritebackParams& wb, bool do_wb, int b, int h,
                                           MergeSmem& sm) {
    const int tid = threadIdx.x;
    const int c = tid >> 5, q = tid & 31;
    const int bh = b * p.Hq + h;
    if (bh == 0 && threadIdx.x == 0 && p.pending != nullptr) *p.pending = 0;
    if (p.head_start != nullptr && (p.head_start[bh] & kHeadDone)) return;     // the whole work-group: before any barrier
    const int n = clampi(p.kv_lens[b], 0, p.max_kv_len);
    const int nb = n - p.band > 0 ? n - p.band : 0;
    const int C = p.chunk_fixed > 0 ? p.chunk_fixed : *p.step_chunk;
    MatchDecision md{INFINITY, -1, -1, 0};
    if (p.mv.part != nullptr) md = decide(p.mv, p.mv.part[bh], n);
    const int s = clampi(md.start, 0, nb);
    const int64_t pbase = (int64_t)bh * p.n_slots;

    // chunks of this head: mid slots [x0, x1) (those with a non-empty part of [s, nb)), band slots [y0, y1)
    const int x0 = s / C, x1 = (nb + C - 1) / C;
    const int y0 = p.n_mid_slots, y1 = nb < n ? p.n_mid_slots + ((n + C - 1) / C - nb / C) : p.n_mid_slots;
    int64_t pre = -1;                                    // ring entry of the reused prefix, if any
    if (md.j >= 0) pre = ((int64_t)p.slot_ids[b] * p.Hq + h) * p.W + md.j;

    // single pass over this lane's chunks (all loads are independent of one another)
    LaneMerge r, bnd;
    const f32x4 zero4 = f32x4{0.f, 0.f, 0.f, 0.f};
    if (c == 0 && pre >= 0) {
        const float L = p.ring_lse[pre];
        const f32x4 o = *reinterpret_cast<const f32x4*>(p.ring_O + pre * kHeadDim + 4 * q);
        r.add(L == -INFINITY ? zero4 : o, L);
    }
    // four chunks per trip, loads first (clamped to a slot of this head, then masked)
    constexpr int kU = 4;
    for (int x = x0 + c; x < x1; x += kU * kMergeLanes) {
        f32x4 o[kU];
        float L[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int xu = x + u * kMergeLanes;
            const int xc = min(xu, x1 - 1);
            o[u] = *reinterpret_cast<const f32x4*>(p.part_O + (pbase + xc) * kHeadDim + 4 * q);
            L[u] = p.part_lse[pbase + xc];
            // nothing of this head in the chunk (or past the last chunk): identity
            if (xu >= x1 || max(s, xu * C) >= min(nb, (xu + 1) * C)) { L[u] = -INFINITY; }
            if (L[u] == -INFINITY) o[u] = zero4;
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) r.add(o[u], L[u]);
    }
    for (int y = y0 + c; y < y1; y += kMergeLanes) {
        const float L = p.part_lse[pbase + y];
        const f32x4 o = *reinterpret_cast<const f32x4*>(p.part_O + (pbase + y) * kHeadDim + 4 * q);
        bnd.add(L == -INFINITY ? zero4 : o, L);
    }
    *reinterpret_cast<f32x4*>(&sm.acc[0][c][4 * q]) = r.acc;
    *reinterpret_cast<f32x4*>(&sm.acc[1][c][4 * q]) = bnd.acc;
    if (q == 0) { sm.m[0][c] = r.M; sm.z[0][c] = r.Z; sm.m[1][c] = bnd.M; sm.z[1][c] = bnd.Z; }
    __syncthreads();                                     // also orders the prefix reads before the ring write below
    if (tid < kHeadDim) {
        const int d = tid;
        float M_r = -INFINITY, M_b = -INFINITY;
#pragma unroll
        for (int k = 0; k < kMergeLanes; ++k) { M_r = fmaxf(M_r, sm.m[0][k]); M_b = fmaxf(M_b, sm.m[1][k]); }
        float S_r = 0.f, Z_r = 0.f, S_b = 0.f, Z_b = 0.f;
#pragma unroll
        for (int k = 0; k < kMergeLanes; ++k) {
            const float fr = sm.z[0][k] > 0.f ? __expf(sm.m[0][k] - M_r) : 0.f;     // an empty lane has m = -inf
            const float fb = sm.z[1][k] > 0.f ? __expf(sm.m[1][k] - M_b) : 0.f;
            S_r += sm.acc[0][k][d] * fr; Z_r += sm.z[0][k] * fr;
            S_b += sm.acc[1][k][d] * fb; Z_b += sm.z[1][k] * fb;
        }
        // rect = prefix (+) mid chunks: this step's total without the last-B band
        const float rect_o = Z_r > 0.f ? S_r / Z_r : 0.f;
        const float rect_l = Z_r > 0.f ? M_r + logf(Z_r) : -INFINITY;
        if (p.rect_O != nullptr) {
            p.rect_O[(int64_t)bh * kHeadDim + d] = rect_o;
            if (d == 0) p.rect_lse[bh] = rect_l;
        }
        // out = rect (+) band
        const float M_o = fmaxf(M_r, M_b);
        float o = 0.f, lse = -INFINITY;
        if (M_o != -INFINITY) {
            const float fr = expf(M_r - M_o), fb = expf(M_b - M_o);     // exp(-inf) = 0 for an empty part
            const float Z = fr * Z_r + fb * Z_b;
            o = (fr * S_r + fb * S_b) / Z;
            lse = M_o + logf(Z);
        }
        if (d < p.head_dim) {
            if (p.out_bf16) static_cast<uint16_t*>(p.out)[(int64_t)bh * p.head_dim + d] = float_to_bf16_rne(o);
            else static_cast<float*>(p.out)[(int64_t)bh * p.head_dim + d] = o;
        }
        if (d == 0 && p.out_lse != nullptr) p.out_lse[bh] = lse;
        if (do_wb) writeback_head(wb, b, h, d, rect_o, rect_l);
    }

    // The decision, for the caller and the counters (acceptance, reuse gap, skipped-prefix fraction).
    if (p.mv.part != nullptr && p.emit_decision && tid < 64) {
        if (tid == 0) {
            if (p.out_match_pos) p.out_match_pos[bh] = md.np;
            if (p.out_match_d2) p.out_match_d2[bh] = md.d2;
            if (md.np >= 0) {          // one writer per address and step: the atomics only make the adds fire-and-forget
                atomicAdd(&p.st_hits[bh], 1ull);
                atomicAdd(&p.st_gap[bh], (unsigned long long)(n - md.np));
                atomicAdd(&p.st_skip[bh], (double)md.start / (double)n);
            }
        }
    }

    __syncthreads();                                     // shared memory is reused by the next head
}

__global__ __launch_bounds__(kMergeThreads) void merge_kernel(const MergeParams p) {
    __shared__ MergeSmem sm;
    const WritebackParams none{};
    merge_head(p, none, false, blockIdx.y, blockIdx.x, sm);
}

__global__ __launch_bounds__(kMergeThreads) void merge_writeback_kernel(const MergeParams p, const WritebackParams wb) {
    __shared__ MergeSmem sm;
    merge_head(p, wb, true, blockIdx.y, blockIdx.x, sm);
}

__global__ __launch_bounds__(128) void writeback_kernel(const WritebackParams p) {
    const int h = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
    const int bh = b * p.Hq + h;
    if (p.head_start != nullptr && (p.head_start[bh] & kHeadDone)) return;
    writeback_head(p, b, h, d, p.rect_O[(int64_t)bh * kHeadDim + d], p.rect_lse[bh]);
}

}  // namespace mac
