// Match, and the whole hit path of a head whose fresh range is short, in one kernel (gfx950, wave64).
//
// Paper: Eq. (accept), Sec. 3.2.3 and Sec. 3.5 step 1 (match: one streaming pass over the last W pre-RoPE queries,
// nearest entry, threshold), then for a hit Sec. 3.5 steps 2-3 (amend: attention over the band and tail
// [max(0, n_p - B), n) under the current post-RoPE query, Eq. (rect-recomp); complete: merge with the cached prefix
// summary, Eq. (rect-merge)) and Fig. 1(c) / Sec. 4.2 "K3" (rectify-append).  The paper runs these as three kernels
// with a host-side planner in between (Table "fine_grained_latency": match 9 us + load balance 29-31 us + attention
// 25 us at a 1 % KV budget); its hit path is launch- and plan-bound.  Here one work-group per (request, query head)
// does all of it for the common case:
//
//   1. match: scan the head's whole window of the query ring (fp64 differences and FMAs, see match_kernel.hpp for the
//      arithmetic), argmin with ties to the larger n_p, threshold and optional distance cap.  The decision, the head's
//      counters and the caller's match_pos / match_d2 are written here.
//   2. if the head hits and its fresh range [s, n), s = max(0, n_p - B), has at most `fused_span` tokens, the same
//      work-group computes the two summaries the method needs -- mid = [s, n-B) and band = [n-B, n) -- with plain
//      fp32 VALU arithmetic (a few hundred tokens of one head: no matrix cores needed), forms
//      rect = prefix (+) mid and out = rect (+) band, writes the output and appends (q~, rect) to the ring.  The head
//      is then marked done: the split-K attention kernel and the merge kernel that follow skip it.
//   3. any other head (miss, or a hit with a long tail) only gets its start stored; it is served by the split-K
//      attention kernel (per KV group, matrix cores) and the merge kernel as before.
//
// K/V of a fused head are read per head, not per KV group, so a group's rows are read G times; the heads of a group
// are placed on the same XCD and run at about the same time, so the repeats are served by that XCD's L2.  The
// bytes are small next to the query ring the same work-group has just scanned (W x 256 B per head against
// (gap + B) x 512 B per group).
//
// Nothing here synchronises across work-groups: a head's ring entries (queries, summaries, n_p tags) are read and
// written by that head's work-group only, the prefix entry is in registers before the append can overwrite it.
#pragma once
#include "common.hpp"
#include "match_kernel.hpp"

namespace mac {

constexpr int kHitMaxSpan = 2048;            // largest fresh range finished here: its logits sit in shared memory

struct HitParams {
    // match
    const int32_t* slot_ids;     // [batch]
    const int32_t* kv_lens;      // [batch]
    const uint16_t* q_pre;       // [batch, Hq, 128] bf16
    uint16_t* ring_q;            // [slots, Hq, W, 128] bf16
    float* ring_O;               // [slots, Hq, W, 128]
    float* ring_lse;             // [slots, Hq, W]
    int32_t* ring_npos;          // [slots, Hq, W]; 0 = empty entry
    MatchPartial* part;          // [batch*Hq] nearest entry of the head's window (one slice)
    int32_t* head_start;         // [batch*Hq] start of the head's fresh range, | kHeadDone if finished here
    unsigned long long* st_steps;   // [2]: decode steps, head-steps
    unsigned long long* st_hits; // per (b, h) accumulators
    unsigned long long* st_gap;
    double* st_skip;
    unsigned long long* st_fused;   // per (b, h): K/V tokens read by the fused path
    int32_t* out_match_pos;      // optional caller outputs [batch*Hq]
    double* out_match_d2;
    MatchView mv;                // threshold, band, distance cap (part / n_split unused)
    int32_t batch, Hq, G, W, max_kv_len;
    int32_t fused_span;          // largest fresh range finished here, 0 = none, <= kHitMaxSpan
    // fused hit path
    const uint16_t* q_rope;      // [batch, Hq, 128] bf16
    const uint16_t* kv_pages;
    int64_t stride_page, stride_kv, stride_head, stride_tok;
    const int32_t* block_table;
    int32_t bt_stride, page_shift;
    float scale_log2;
    void* out;                   // [batch, Hq, 128] fp32 or bf16
    int32_t out_bf16;
    float* out_lse;              // optional
};

__device__ __forceinline__ float bf16_lo_to_f32(uint32_t pair) { return bits_to_float(pair << 16); }
__device__ __forceinline__ float bf16_hi_to_f32(uint32_t pair) { return bits_to_float(pair & 0xffff0000u); }

// (O_a, L_a) (+) (O_b, L_b) for one output column, natural-log LSEs, empty = (0, -inf)
__device__ __forceinline__ void merge2(float oa, float la, float ob, float lb, float& o, float& l) {
    const float M = fmaxf(la, lb);
    if (M == -INFINITY) { o = 0.f; l = -INFINITY; return; }
    const float wa = la == -INFINITY ? 0.f : __expf(la - M), wb = lb == -INFINITY ? 0.f : __expf(lb - M);
    const float Z = wa + wb;
    o = (wa * (la == -INFINITY ? 0.f : oa) + wb * (lb == -INFINITY ? 0.f : ob)) / Z;
    l = M + logf(Z);
}

template <int NT>      // threads per work-group: 256, or 1024 when there are few heads and a large window
__global__ __launch_bounds__(NT) void hit_kernel(const HitParams p) {
    constexpr int NW = NT / 64;
    constexpr int kRows = NT / 4;                              // ring rows (or K rows) per pass: a quad per 256-byte row
    constexpr int kPasses = 2;                                 // passes in flight
    // Work-groups are dealt to the 8 XCDs in turn: the G heads of a KV group take ids that are 8 apart.
    const int id = blockIdx.x, xcd = id & 7, k = id >> 3;
    const int G = p.G, Hkv = p.Hq / G;
    const int kq = k / G;
    const int grp = kq * 8 + xcd;
    if (grp >= p.batch * Hkv) return;
    const int b = grp / Hkv, g = grp - b * Hkv, h = g * G + (k - kq * G);
    const int tid = threadIdx.x, quad = tid >> 2, sub = tid & 3, lane = tid & 63, w = tid >> 6;
    const int bh = b * p.Hq + h;
    const int n = clampi(p.kv_lens[b], 0, p.max_kv_len);
    const int64_t slot = p.slot_ids[b];
    const int W = p.W;
    const int64_t ring_row0 = (slot * p.Hq + h) * W;

    __shared__ double s_d2[NW];
    __shared__ int s_np[NW], s_j[NW];
    __shared__ float s_logit[kHitMaxSpan];
    __shared__ int s_pid[kHitMaxSpan / 16 + 2];
    __shared__ float s_red[2][NW][2];                          // [max | sum][wave][mid | band]
    __shared__ float s_acc[NW][2][kHeadDim];
    // Page ids of the last fused_span tokens, which hold every fresh range this kernel may finish: requested before
    // the match, needed after it (the barrier of the match result also publishes them).
    const int first_page = max(0, n - p.fused_span) >> p.page_shift;
    if (p.fused_span > 0 && n > 0) {
        const int n_pages = ((n - 1) >> p.page_shift) - first_page + 1;
        for (int i = tid; i < n_pages; i += NT) s_pid[i] = p.block_table[(int64_t)b * p.bt_stride + first_page + i];
    }
    double best_d2 = INFINITY;
    int best_np = -1, best_j = -1;
    {
        // ---- 1. match (same scan as the one-slice case of the window-slice design: rows loaded without waiting for
        // their n_p tag, several passes in flight)
        double q[32];
        load_query_f64(p.q_pre + (int64_t)bh * kHeadDim + 8 * sub, q);
        const uint16_t* ring = p.ring_q + ring_row0 * kHeadDim + 8 * sub;
        const int32_t* npos = p.ring_npos + ring_row0;
        const int np_lo = max(1, n - W), np_hi = n - 1;
        auto row_of = [&](int j0, int& j, int& np, u32x4 (&v)[4]) {
            j = j0 + quad;
            const int jc = j < W ? j : W - 1;                  // keep the speculative loads inside the ring
            np = npos[jc];
            const uint16_t* rp = ring + (int64_t)jc * kHeadDim;
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = *reinterpret_cast<const u32x4*>(rp + 32 * i);
        };
        auto take = [&](int j, int np, const u32x4 (&v)[4]) {
            const bool valid = j < W && np >= np_lo && np <= np_hi;
            double d2 = lane_sq_dist(q, v);
            d2 += __shfl_xor(d2, 1);
            d2 += __shfl_xor(d2, 2);
            if (valid && better(d2, np, best_d2, best_np)) { best_d2 = d2; best_np = np; best_j = j; }
        };
        int j0 = 0;
        for (; j0 + (kPasses - 1) * kRows < W; j0 += kPasses * kRows) {
            int jj[kPasses], nn[kPasses];
            u32x4 vv[kPasses][4];
#pragma unroll
            for (int t = 0; t < kPasses; ++t) row_of(j0 + t * kRows, jj[t], nn[t], vv[t]);
#pragma unroll
            for (int t = 0; t < kPasses; ++t) take(jj[t], nn[t], vv[t]);
        }
        for (; j0 < W; j0 += kRows) {
            int ja, npa;
            u32x4 va[4];
            row_of(j0, ja, npa, va);
            take(ja, npa, va);
        }
#pragma unroll
        for (int off = 4; off < 64; off <<= 1) {               // all 4 lanes of a quad hold the same triple
            const double od2 = __shfl_xor(best_d2, off);
            const int onp = __shfl_xor(best_np, off);
            const int oj = __shfl_xor(best_j, off);
            if (better(od2, onp, best_d2, best_np)) { best_d2 = od2; best_np = onp; best_j = oj; }
        }
        if (lane == 0) { s_d2[w] = best_d2; s_np[w] = best_np; s_j[w] = best_j; }
        __syncthreads();
        best_d2 = s_d2[0]; best_np = s_np[0]; best_j = s_j[0];
#pragma unroll
        for (int ww = 1; ww < NW; ++ww)
            if (better(s_d2[ww], s_np[ww], best_d2, best_np)) { best_d2 = s_d2[ww]; best_np = s_np[ww]; best_j = s_j[ww]; }
    }

    // ---- 2. decision (every thread holds the same values)
    const bool hit = match_accept(p.mv, best_d2, best_np, n);
    const int nb = n - p.mv.band > 0 ? n - p.mv.band : 0;      // the band is [nb, n)
    const int s = head_start(p.mv, best_d2, best_np, n);       // max(0, n_p - B) on a hit, else 0; never above nb
    const int cnt = n - s;
    const bool fuse = hit && cnt <= p.fused_span;
    if (tid == 0) {
        if (id == 0) {
            atomicAdd(&p.st_steps[0], 1ull);
            atomicAdd(&p.st_steps[1], (unsigned long long)p.batch * p.Hq);
        }
        p.part[bh] = MatchPartial{best_d2, best_np, best_j};
        p.head_start[bh] = s | (fuse ? kHeadDone : 0);
        if (p.out_match_pos) p.out_match_pos[bh] = hit ? best_np : -1;
        if (p.out_match_d2) p.out_match_d2[bh] = best_d2;
        if (hit) {                      // one writer per address and step: the atomics only make the adds fire-and-forget
            atomicAdd(&p.st_hits[bh], 1ull);
            atomicAdd(&p.st_gap[bh], (unsigned long long)(n - best_np));
            atomicAdd(&p.st_skip[bh], (double)s / (double)n);
            if (fuse) atomicAdd(&p.st_fused[bh], (unsigned long long)cnt);
        }
    }
    if (!fuse) return;

    // ---- 3. the hit path of this head: summaries of [s, nb) and [nb, n), merge with the prefix, append.
    // Everything it reads is requested in one go (the page ids were fetched before the match): K rows, the first V
    // rows, the query and the prefix summary share one memory round trip.
    const int page_mask = (1 << p.page_shift) - 1;
    const uint16_t* kv_g = p.kv_pages + (int64_t)g * p.stride_head;
    auto row_ptr = [&](int r) {                                // K row of the r-th token of the fresh range
        const int t = s + r;
        return kv_g + (int64_t)s_pid[(t >> p.page_shift) - first_page] * p.stride_page + (int64_t)(t & page_mask) * p.stride_tok;
    };
    // the reused prefix summary: in registers before anything of this head's ring is overwritten
    const int64_t pre = ring_row0 + best_j;
    float pre_o = 0.f, pre_l = -INFINITY;
    if (tid < kHeadDim) {
        pre_l = p.ring_lse[pre];
        pre_o = p.ring_O[pre * kHeadDim + tid];
    }
    u32x4 qv[4];                                               // this lane's 32 elements of the post-RoPE query
    {
        const uint16_t* qp = p.q_rope + (int64_t)bh * kHeadDim + 8 * sub;
#pragma unroll
        for (int i = 0; i < 4; ++i) qv[i] = *reinterpret_cast<const u32x4*>(qp + 32 * i);
    }
    // weighted sums of V rows: 16 lanes cover a 256-byte row, a wave takes 4 rows per load; the first kVPre rows of
    // every thread are requested now
    constexpr int kRowGroups = NT / 16, kVPre = 8;
    const int col = tid & 15, rg = tid >> 4;
    u32x4 vpre[kVPre];
    // logits (log2 domain), a quad per K row
    for (int r0 = 0; r0 < cnt; r0 += 2 * kRows) {
        u32x4 kk[2][4];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint16_t* rp = row_ptr(min(r0 + u * kRows + quad, cnt - 1)) + 8 * sub;
#pragma unroll
            for (int i = 0; i < 4; ++i) kk[u][i] = *reinterpret_cast<const u32x4*>(rp + 32 * i);
        }
        if (r0 == 0) {
#pragma unroll
            for (int u = 0; u < kVPre; ++u)
                vpre[u] = *reinterpret_cast<const u32x4*>(row_ptr(min(u * kRowGroups + rg, cnt - 1)) + p.stride_kv + 8 * col);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            float d0 = 0.f, d1 = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    d0 = fmaf(bf16_lo_to_f32(qv[i][e]), bf16_lo_to_f32(kk[u][i][e]), d0);
                    d1 = fmaf(bf16_hi_to_f32(qv[i][e]), bf16_hi_to_f32(kk[u][i][e]), d1);
                }
            float dot = d0 + d1;
            dot += __shfl_xor(dot, 1);
            dot += __shfl_xor(dot, 2);
            const int r = r0 + u * kRows + quad;
            if (sub == 0 && r < cnt) s_logit[r] = dot * p.scale_log2;
        }
    }
    __syncthreads();
    // maxima and sums of the two parts, in a fixed order
    const int nbr = nb - s;                                    // rows [0, nbr) are the mid part, [nbr, cnt) the band
    float mx0 = -INFINITY, mx1 = -INFINITY;
    for (int r = tid; r < cnt; r += NT) {
        const float l = s_logit[r];
        if (r < nbr) mx0 = fmaxf(mx0, l); else mx1 = fmaxf(mx1, l);
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        mx0 = fmaxf(mx0, __shfl_xor(mx0, off));
        mx1 = fmaxf(mx1, __shfl_xor(mx1, off));
    }
    if (lane == 0) { s_red[0][w][0] = mx0; s_red[0][w][1] = mx1; }
    __syncthreads();
    float M0 = s_red[0][0][0], M1 = s_red[0][0][1];
#pragma unroll
    for (int ww = 1; ww < NW; ++ww) { M0 = fmaxf(M0, s_red[0][ww][0]); M1 = fmaxf(M1, s_red[0][ww][1]); }
    float z0 = 0.f, z1 = 0.f;
    for (int r = tid; r < cnt; r += NT) {
        const bool mid = r < nbr;
        const float pw = exp2_fast(s_logit[r] - (mid ? M0 : M1));
        s_logit[r] = pw;
        if (mid) z0 += pw; else z1 += pw;
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        z0 += __shfl_xor(z0, off);
        z1 += __shfl_xor(z1, off);
    }
    if (lane == 0) { s_red[1][w][0] = z0; s_red[1][w][1] = z1; }
    __syncthreads();
    float Z0 = 0.f, Z1 = 0.f;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) { Z0 += s_red[1][ww][0]; Z1 += s_red[1][ww][1]; }
    {
        float a0[8], a1[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) a0[j] = a1[j] = 0.f;
        auto add_row = [&](int r, const u32x4& v) {
            const float pw = r < cnt ? s_logit[r] : 0.f;
            const float w0 = r < nbr ? pw : 0.f, w1 = pw - w0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float lo = bf16_lo_to_f32(v[e]), hi = bf16_hi_to_f32(v[e]);
                a0[2 * e] = fmaf(w0, lo, a0[2 * e]);
                a0[2 * e + 1] = fmaf(w0, hi, a0[2 * e + 1]);
                a1[2 * e] = fmaf(w1, lo, a1[2 * e]);
                a1[2 * e + 1] = fmaf(w1, hi, a1[2 * e + 1]);
            }
        };
#pragma unroll
        for (int u = 0; u < kVPre; ++u) add_row(u * kRowGroups + rg, vpre[u]);
        for (int r0 = kVPre * kRowGroups; r0 < cnt; r0 += 4 * kRowGroups) {
            u32x4 vv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                vv[u] = *reinterpret_cast<const u32x4*>(row_ptr(min(r0 + u * kRowGroups + rg, cnt - 1)) + p.stride_kv + 8 * col);
#pragma unroll
            for (int u = 0; u < 4; ++u) add_row(r0 + u * kRowGroups + rg, vv[u]);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {                          // lanes l, l^16, l^32, l^48 hold the same columns
            a0[j] += __shfl_xor(a0[j], 16);
            a0[j] += __shfl_xor(a0[j], 32);
            a1[j] += __shfl_xor(a1[j], 16);
            a1[j] += __shfl_xor(a1[j], 32);
        }
        if (lane < 16) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                s_acc[w][0][8 * col + j] = a0[j];
                s_acc[w][1][8 * col + j] = a1[j];
            }
        }
    }
    __syncthreads();
    if (tid < kHeadDim) {
        const int d = tid;
        float S0 = 0.f, S1 = 0.f;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) { S0 += s_acc[ww][0][d]; S1 += s_acc[ww][1][d]; }
        const float o_mid = Z0 > 0.f ? S0 / Z0 : 0.f, l_mid = Z0 > 0.f ? (M0 + __log2f(Z0)) * kLn2 : -INFINITY;
        const float o_band = Z1 > 0.f ? S1 / Z1 : 0.f, l_band = Z1 > 0.f ? (M1 + __log2f(Z1)) * kLn2 : -INFINITY;
        float rect_o, rect_l, o, lse;
        merge2(pre_o, pre_l, o_mid, l_mid, rect_o, rect_l);    // this step's total without the last-B band
        merge2(rect_o, rect_l, o_band, l_band, o, lse);
        if (p.out_bf16) {
            static_cast<uint16_t*>(p.out)[(int64_t)bh * kHeadDim + d] = float_to_bf16_rne(o);
        } else {
            static_cast<float*>(p.out)[(int64_t)bh * kHeadDim + d] = o;
        }
        if (d == 0 && p.out_lse != nullptr) p.out_lse[bh] = lse;
        // rectify-append into entry (n - 1) mod W of this head
        const int jn = (n - 1) % W;
        const int64_t e = ring_row0 + jn;
        p.ring_q[e * kHeadDim + d] = p.q_pre[(int64_t)bh * kHeadDim + d];
        p.ring_O[e * kHeadDim + d] = rect_o;
        if (d == 0) {
            p.ring_lse[e] = rect_l;
            p.ring_npos[e] = n;
        }
    }
}

}  // namespace mac
