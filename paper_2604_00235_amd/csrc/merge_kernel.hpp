// Complete (log-domain merge) and rectify-append (ring write-back) kernels (gfx950).
//
// Merge, per (request b, query head h) -- paper Sec. 3.1 (summaries over disjoint sets add), Eq. (rect-merge),
// Sec. 4.2 "K2 (3) Merge":  in fixed ascending order
//     rect = prefix (ring summary of the matched entry, on a hit)  (+)  partials of the mid chunks [s_h, n-B)
//     out  = rect  (+)  partials of the band chunks [n-B, n)
// where (O_a, L_a) (+) (O_b, L_b) = ((e^{L_a} O_a + e^{L_b} O_b)/(e^{L_a} + e^{L_b}), ln(e^{L_a} + e^{L_b})),
// evaluated with a running maximum so no exponent overflows; the empty summary is (0, -inf).
// `rect` is this step's total without the last-B band (Fig. 1(c)), built add-only so nothing cancels.
//
// Write-back, per (b, h) -- Sec. 4.1, Sec. 4.2 "K3": ring entry (n-1) mod W of the request's ring set gets the
// pre-RoPE query, the rectified summary row and its ln-LSE; the entry's n_p tag is set to n.  It runs after the
// merge in stream order because the overwritten entry (n_p = n - W) is still a candidate of this step.
#pragma once
#include "common.hpp"

namespace mac {

struct MergeParams {
    const int32_t* kv_lens;
    const int32_t* slot_ids;     // null for full decode
    const int32_t* m_j;          // [batch*Hq] matched ring entry or -1; null for full decode
    const int32_t* m_start;      // [batch*Hq] s_h; null for full decode (all 0)
    const float* ring_O;         // [slots, Hq, W, 128]
    const float* ring_lse;       // [slots, Hq, W]
    const float* part_O;         // [batch*Hq, n_slots, 128]
    const float* part_lse;       // [batch*Hq, n_slots]
    float* out;                  // [batch, Hq, 128]
    float* out_lse;              // optional [batch, Hq]
    float* rect_O;               // staging for the write-back [batch*Hq, 128]; null for full decode
    float* rect_lse;             // [batch*Hq]
    unsigned long long* st_read; // per (b, kv head) accumulators; null for full decode
    unsigned long long* st_full;
    int32_t Hq, G, W, band, chunk, n_mid_slots, n_slots, max_kv_len;
};

struct RunningMerge {
    float M = -INFINITY, Z = 0.f, acc = 0.f;
    __device__ __forceinline__ void add(float o, float L) {
        if (L == -INFINITY) return;                // empty summary: identity
        const float Mn = fmaxf(M, L);
        const float a = expf(M - Mn), bw = expf(L - Mn);
        acc = acc * a + o * bw;
        Z = Z * a + bw;
        M = Mn;
    }
    __device__ __forceinline__ float value() const { return Z > 0.f ? acc / Z : 0.f; }
    __device__ __forceinline__ float lse() const { return Z > 0.f ? M + logf(Z) : -INFINITY; }
};

__global__ __launch_bounds__(128) void merge_kernel(const MergeParams p) {
    const int h = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
    const int bh = b * p.Hq + h;
    const int n = clampi(p.kv_lens[b], 0, p.max_kv_len);
    const int nb = n - p.band > 0 ? n - p.band : 0;
    const int C = p.chunk;
    const int s = p.m_start ? clampi(p.m_start[bh], 0, nb) : 0;

    RunningMerge r;
    if (p.m_j != nullptr) {
        const int j = p.m_j[bh];
        if (j >= 0) {
            const int64_t e = ((int64_t)p.slot_ids[b] * p.Hq + h) * p.W + j;
            r.add(p.ring_O[e * kHeadDim + d], p.ring_lse[e]);
        }
    }
    const int64_t pbase = (int64_t)bh * p.n_slots;
    for (int x = s / C; x * C < nb; ++x) {
        if (max(s, x * C) >= min(nb, (x + 1) * C)) continue;     // nothing of this head in the chunk
        r.add(p.part_O[(pbase + x) * kHeadDim + d], p.part_lse[pbase + x]);
    }
    if (p.rect_O != nullptr) {
        p.rect_O[(int64_t)bh * kHeadDim + d] = r.value();
        if (d == 0) p.rect_lse[bh] = r.lse();
    }
    const int cb = nb / C;
    for (int k = 0; (cb + k) * C < n && nb < n; ++k) {
        const int x = p.n_mid_slots + k;
        r.add(p.part_O[(pbase + x) * kHeadDim + d], p.part_lse[pbase + x]);
    }
    p.out[(int64_t)bh * kHeadDim + d] = r.value();
    if (d == 0 && p.out_lse != nullptr) p.out_lse[bh] = r.lse();

    // KV tokens streamed by this step for the KV group (read once per group from its smallest start)
    if (p.st_read != nullptr && d == 0 && (h % p.G) == 0) {
        int gs = nb;
        for (int i = 0; i < p.G; ++i) gs = min(gs, clampi(p.m_start[bh + i], 0, nb));
        const int bg = bh / p.G;
        p.st_read[bg] += (unsigned long long)(n - gs);
        p.st_full[bg] += (unsigned long long)n;
    }
}

struct WritebackParams {
    const int32_t* kv_lens;
    const int32_t* slot_ids;
    const uint16_t* q_pre;       // [batch, Hq, 128] bf16
    const float* rect_O;         // [batch*Hq, 128]
    const float* rect_lse;       // [batch*Hq]
    uint16_t* ring_q;            // [slots, Hq, W, 128]
    float* ring_O;               // [slots, Hq, W, 128]
    float* ring_lse;             // [slots, Hq, W]
    int32_t* ring_npos;          // [slots, W]
    int32_t Hq, W, max_kv_len;
};

__global__ __launch_bounds__(128) void writeback_kernel(const WritebackParams p) {
    const int h = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
    const int bh = b * p.Hq + h;
    const int n = clampi(p.kv_lens[b], 0, p.max_kv_len);
    if (n < 1) return;
    const int64_t slot = p.slot_ids[b];
    const int j = (n - 1) % p.W;
    const int64_t e = (slot * p.Hq + h) * p.W + j;
    p.ring_q[e * kHeadDim + d] = p.q_pre[(int64_t)bh * kHeadDim + d];
    p.ring_O[e * kHeadDim + d] = p.rect_O[(int64_t)bh * kHeadDim + d];
    if (d == 0) {
        p.ring_lse[e] = p.rect_lse[bh];
        if (h == 0) p.ring_npos[slot * p.W + j] = n;
    }
}

}  // namespace mac
