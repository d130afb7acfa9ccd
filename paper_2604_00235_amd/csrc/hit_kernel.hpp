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
//   1. match: the head's whole window of the query ring, in three tiers.
//      (a) Filter in fp32: ring rows are read four whole rows per load instruction (1 KiB contiguous; one compute unit
//          pulls that pattern ~3x faster than 16 rows x 64 bytes per instruction, the layout a matrix-core operand
//          needs, which is why the filter does not use the matrix cores: measured 110 against 36 GB/s from the
//          caches).  Each lane forms its 16-byte chunk's share of |r_j|^2 - 2 q.r_j with v_dot2c_f32_bf16 for the 16
//          rows it holds a chunk of, a butterfly over the 16 lanes of a row of the wave completes one row's sum per
//          lane, and f_j = |q|^2 + |r_j|^2 - 2 q.r_j carries a proven bound |f_j - d2_j| <= eps_j (bf16 products are
//          exact in fp32; only the accumulation rounds).  U = min_j (f_j + eps_j) over the work-group bounds the
//          nearest distance from above.
//      (b) Rows with f_j - eps_j <= U -- typically one -- are evaluated in fp64 (exact differences, fp64 FMAs) in the
//          registers they were loaded into; argmin with ties to the larger n_p.
//      (c) Two fp64 evaluations of one distance agree to ~2^-46 relative.  If the runner-up, or the threshold, lies
//          within 2^-40 of the winner, the rows in question are summed once more in index order without FMAs, the
//          plain left-to-right sum a reference takes, so that the decision is the same bit for bit by construction.
//      An fp64 scan of every row (the first version of this kernel) kept a compute unit's VALU busy for 5 us per 1024
//      rows of one head; a filter on the matrix cores was bound by the operand layout's access pattern (256 KB of one
//      head in 8.2 us); this one scans them in 3.5 us.
//      The decision, the head's counters and the caller's match_pos / match_d2 are written here.
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
// Error bound of the filter, relative to |q|^2 + |r|^2: the three dot products are sums of 128 exact bf16 x bf16 products
// accumulated in fp32 (128 x 2^-23 each, against (|q| + |r|)^2 <= 2 (|q|^2 + |r|^2) in total: 3.1e-5), taken four
// times over to be independent of how the dot instruction and the butterfly order and round their partial sums
// (measured for v_dot2c_f32_bf16 chains of 128 products: 9.4e-8 of the sum of the products' magnitudes).
constexpr float kFilterEps = 1.25e-4f;
constexpr float kFilterTiny = 1e-30f;        // below this |q|^2 + |r|^2 single products may underflow: no bound claimed
constexpr double kTieRel = 0x1p-40;          // two fp64 evaluations of one distance differ by far less than this

struct HitParams {
    // match
    const int32_t* slot_ids;     // [batch]
    const int32_t* kv_lens;      // [batch]
    const uint16_t* q_pre;       // [batch, Hq, d] bf16
    uint16_t* ring_q;            // [slots, Hq, W, 128] bf16
    float* ring_O;               // [slots, Hq, W, 128]
    float* ring_lse;             // [slots, Hq, W]
    int32_t* ring_npos;          // [slots, Hq, W]; 0 = empty entry
    MatchPartial* part;          // [batch*Hq] nearest entry of the head's window (one slice)
    int32_t* head_start;         // [batch*Hq] start of the head's fresh range, | kHeadDone if finished here
    int32_t* pending;            // [1] number of heads of this step left to the split-K path (the merge kernel clears it)
    unsigned long long* st_steps;   // [2]: decode steps, head-steps
    unsigned long long* st_hits; // per (b, h) accumulators
    unsigned long long* st_gap;
    double* st_skip;
    unsigned long long* st_fused;   // per (b, h): K/V tokens read by the fused path
    int32_t* out_match_pos;      // optional caller outputs [batch*Hq]
    double* out_match_d2;
    MatchView mv;                // threshold, band, distance cap (part / n_split unused)
    int32_t batch, Hq, G, W, max_kv_len;
    int32_t head_dim;            // d of the caller's tensors (32, 64, 96, 128); ring rows are 128 wide, zero beyond d
    int32_t fused_span;          // largest fresh range finished here, 0 = none, <= kHitMaxSpan
    // fused hit path
    const uint16_t* q_rope;      // [batch, Hq, d] bf16
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

// Partial squared distance of one lane in fp64: four 16-byte chunks of the query against the same chunks of a ring row,
// both as packed bf16.  The query is widened here, per call, rather than once per work-group: 32 doubles would cost
// 64 registers for the whole kernel (the empty asm statement keeps the compiler from doing just that).
__device__ __forceinline__ double sq_dist_packed(const u32x4 (&q)[4], const u32x4 (&v)[4]) {
    double s0 = 0.0, s1 = 0.0;
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint32_t qw = q[c][e];
            asm volatile("" : "+v"(qw));
            const double d0 = bf16_lo_to_f64(qw) - bf16_lo_to_f64(v[c][e]);
            const double d1 = bf16_hi_to_f64(qw) - bf16_hi_to_f64(v[c][e]);
            s0 = fma(d0, d0, s0);
            s1 = fma(d1, d1, s1);
        }
    return s0 + s1;
}

// Sum of eight products of bf16 pairs, accumulated in fp32 (v_dot2c_f32_bf16: two exact products and the accumulator
// per instruction).  The pairs are taken out of the 8-element vector with shuffles: going through the 32-bit words
// (bit_cast of x[e]) makes this compiler use the first word four times.
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
__device__ __forceinline__ float dot8_bf16(const u32x4& x, const u32x4& y) {
    const bf16x8 vx = __builtin_bit_cast(bf16x8, x), vy = __builtin_bit_cast(bf16x8, y);
    float acc = 0.f;
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(vx, vx, 0, 1), __builtin_shufflevector(vy, vy, 0, 1), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(vx, vx, 2, 3), __builtin_shufflevector(vy, vy, 2, 3), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(vx, vx, 4, 5), __builtin_shufflevector(vy, vy, 4, 5), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(vx, vx, 6, 7), __builtin_shufflevector(vy, vy, 6, 7), acc, false);
    return acc;
}
// NT = threads per work-group: 256, or 1024 when there are few heads and a large window.  kLean (256 threads only): fewer
// loads in flight per wave (half a block of the window, five K/V rows), which fits five work-groups on a compute unit
// instead of four: for launches with more heads than the chip holds work-groups.
template <int NT, bool kLean>
__global__ __launch_bounds__(NT, NT == 256 ? (kLean ? 5 : 4) : 1) void hit_kernel(const HitParams p) {
    constexpr int NW = NT / 64;
    constexpr int kRows = NT / 4;                              // ring rows per pass of the near-tie scan: a quad per 256-byte row
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

    __shared__ double s_d2[NW], s_second[NW];
    __shared__ int s_np[NW], s_j[NW];
    __shared__ float s_u[2][NW];
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
    // ---- 1. match, in three tiers (see the head of this file): fp32 filter, fp64 evaluation of the candidates
    // it leaves, and -- only for candidates that tie to rounding -- the sum in index order.
    const uint16_t* ring_h = p.ring_q + ring_row0 * kHeadDim;
    const int D = p.head_dim;                                  // the caller's rows; everything in here is 128 wide, zero beyond D
    const uint16_t* q_h = p.q_pre + (int64_t)bh * D;
    const u32x4 kZero4 = u32x4{0u, 0u, 0u, 0u};
    const int32_t* npos = p.ring_npos + ring_row0;
    const int np_lo = max(1, n - W), np_hi = n - 1;
    double best_d2 = INFINITY, second_d2 = INFINITY;           // nearest candidate and the distance of the next one
    int best_np = -1, best_j = -1;
    {
        // A load instruction takes four whole rows (1 KiB contiguous: lane = 16 x (row of the four) + 16-byte chunk of
        // the row): the pattern one compute unit pulls fastest (~110 GB/s from the caches against ~36 GB/s with 16 rows
        // x 64 bytes per instruction, the layout a matrix-core operand would need).  A wave holds a block of 64 rows
        // in 16 such loads; each lane forms its chunk's share of |r|^2 - 2 q.r for the 16 rows it has a chunk of,
        // and a butterfly over the 16 lanes of a row of the wave (partners lane ^ 8, ^ 7, ^ 2, ^ 1: the exchanges
        // DPP offers) leaves every lane with the complete sum of one row -- the row it "owns" below.
        const int rsub = lane >> 4, ch = lane & 15;
        const bool bA = (ch & 8) != 0, bB = (ch & 4) != 0, bC = (((ch >> 1) ^ (ch >> 2)) & 1) != 0, bD = ((ch ^ (ch >> 2)) & 1) != 0;
        constexpr int kLoads = kLean ? 8 : 16;                 // loads (of four rows) per block of the window and wave
        const int own_i = (kLean ? 0 : 8 * (int)bA) + 4 * (int)bB + 2 * (int)bC + (int)bD;    // load number of the row this lane owns
        const bool owner = !kLean || !bA;                      // (with 8 loads per block each row's sum ends up in two lanes)
        const u32x4 qc = 8 * ch < D ? *reinterpret_cast<const u32x4*>(q_h + 8 * ch) : kZero4;      // this lane's chunk of the query
        const float qq = row_sum_f32(dot8_bf16(qc, qc));       // |q|^2 (the same in every lane)
        float U = INFINITY;                                    // smallest upper bound the work-group has seen so far
        const int n_blocks = (W + 4 * kLoads - 1) / (4 * kLoads);
        int parity = 0;
        for (int base = 0; base < n_blocks; base += NW, parity ^= 1) {       // the same trip count in every wave
            const int row0 = 4 * kLoads * (base + w);
            u32x4 a[kLoads];
#pragma unroll
            for (int i = 0; i < kLoads; ++i) {
                const int row = min(row0 + 4 * i + rsub, W - 1);           // keeps the loads inside the ring
                a[i] = *reinterpret_cast<const u32x4*>(ring_h + (int64_t)row * kHeadDim + 8 * ch);
            }
            const int own = row0 + 4 * own_i + rsub;
            const int tag = npos[min(own, W - 1)];
            float part[kLoads];                                // this lane's chunk of |r|^2 - 2 q.r, per load
#pragma unroll
            for (int i = 0; i < kLoads; ++i) part[i] = fmaf(-2.f, dot8_bf16(a[i], qc), dot8_bf16(a[i], a[i]));
            float s8[8], s4[4], s2[2];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if constexpr (kLean) s8[k] = part[k] + dpp_f32<kDppRowRor8>(part[k]);
                else s8[k] = (bA ? part[k + 8] : part[k]) + dpp_f32<kDppRowRor8>(bA ? part[k] : part[k + 8]);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) s4[k] = (bB ? s8[k + 4] : s8[k]) + dpp_f32<kDppRowHalfMirror>(bB ? s8[k] : s8[k + 4]);
#pragma unroll
            for (int k = 0; k < 2; ++k) s2[k] = (bC ? s4[k + 2] : s4[k]) + dpp_f32<kDppQuadSwap2>(bC ? s4[k] : s4[k + 2]);
            const float rr2sd = (bD ? s2[1] : s2[0]) + dpp_f32<kDppQuadSwap1>(bD ? s2[0] : s2[1]);      // |r|^2 - 2 q.r of row `own`
            const bool valid = owner && own < W && tag >= np_lo && tag <= np_hi;
            // |f - d2| <= kFilterEps (|q|^2 + |r|^2), and |r|^2 <= (sqrt(d2) + |q|)^2 <= 2 d2 + 2 |q|^2
            const float f = qq + rr2sd, eps = 1.001f * kFilterEps * (2.f * fmaxf(f, 0.f) + 3.f * qq);
            float up = f + eps, lower = f - eps;
            // overflow, or magnitudes so small that products underflow: decided in fp64
            if (!(fabsf(f) < INFINITY) || qq < kFilterTiny) { lower = -INFINITY; up = INFINITY; }
            if (!valid) lower = INFINITY;
            else U = fminf(U, up);
            U = wave_min_f32(U);
            if (lane == 0) s_u[parity][w] = U;
            __syncthreads();
#pragma unroll
            for (int ww = 0; ww < NW; ++ww) U = fminf(U, s_u[parity][ww]);
            // tier 2: rows the filter cannot rule out are evaluated in fp64 where they sit (load i, the 16 lanes of the
            // owner's row of the wave)
            const bool cand = lower <= U && lower < INFINITY;
            if (__builtin_amdgcn_ballot_w64(cand) != 0) {
#pragma unroll
                for (int i = 0; i < kLoads; ++i) {
                    if (__builtin_amdgcn_ballot_w64(cand && own_i == i) == 0) continue;
                    const double d2 = row_sum_f64(sq_dist_chunk(qc, a[i]));
                    if (cand && own_i == i) {
                        if (better(d2, tag, best_d2, best_np)) { second_d2 = best_d2; best_d2 = d2; best_np = tag; best_j = own; }
                        else second_d2 = fmin(second_d2, d2);
                    }
                }
            }
        }
    }
    // Block-wide (nearest, next) of the lanes' candidates: few lanes hold one, so a wave walks over those lanes with
    // v_readlane instead of a 64-lane butterfly; the waves' results meet in shared memory.  Every thread gets the result.
    auto reduce_best = [&](double& d2, int& np, int& j, double& second, bool holds) {
        double bd = INFINITY, bs = INFINITY;
        int bnp = -1, bj = -1;
        unsigned long long mask = __builtin_amdgcn_ballot_w64(holds);
        while (mask != 0) {                                    // wave-uniform
            const int l = __builtin_ctzll(mask);
            mask &= mask - 1;
            const double od = readlane_f64(d2, l), os = readlane_f64(second, l);
            const int onp = __builtin_amdgcn_readlane(np, l), oj = __builtin_amdgcn_readlane(j, l);
            if (better(od, onp, bd, bnp)) { bs = fmin(bd, os); bd = od; bnp = onp; bj = oj; }
            else bs = fmin(fmin(bs, os), od);
        }
        __syncthreads();                                       // the arrays may still be read from an earlier call
        if (lane == 0) { s_d2[w] = bd; s_np[w] = bnp; s_j[w] = bj; s_second[w] = bs; }
        __syncthreads();
        d2 = s_d2[0]; np = s_np[0]; j = s_j[0]; second = s_second[0];
#pragma unroll
        for (int ww = 1; ww < NW; ++ww) {
            if (better(s_d2[ww], s_np[ww], d2, np)) { second = fmin(d2, s_second[ww]); d2 = s_d2[ww]; np = s_np[ww]; j = s_j[ww]; }
            else second = fmin(fmin(second, s_second[ww]), s_d2[ww]);
        }
    };
    reduce_best(best_d2, best_np, best_j, second_d2, best_np >= 0);
    // tier 3: two fp64 evaluations of one distance agree to ~2^-46 relative, so the order of two candidates, or of the
    // nearest one and the threshold, can depend on the evaluation only if they lie closer than that.  Then the window
    // is scanned once more in fp64 (a quad per row) and the rows in question are summed, one lane each, in index order
    // without fused multiply-adds: the plain left-to-right sum that a reference evaluation of Eq. (accept) takes, so
    // that the decision is the same bit for bit.  (Exact duplicates in the window come here too, and fall to the
    // tie-break as before.)
    if (best_np >= 0 && (second_d2 <= best_d2 * (1.0 + kTieRel) || fabs(best_d2 - p.mv.T2) <= kTieRel * p.mv.T2)) {
        const double bound = best_d2 * (1.0 + kTieRel);
        double e_d2 = INFINITY, e_second = INFINITY;
        int e_np = -1, e_j = -1;
        u32x4 qs[4];                                           // the query in the quad layout: chunks sub, sub + 4, ...
#pragma unroll
        for (int i = 0; i < 4; ++i) qs[i] = 8 * sub + 32 * i < D ? *reinterpret_cast<const u32x4*>(q_h + 8 * sub + 32 * i) : kZero4;
        for (int r0 = 0; r0 < W; r0 += kRows) {
            const int r = r0 + quad, rc = min(r, W - 1);
            u32x4 v[4];
            const uint16_t* rp = ring_h + (int64_t)rc * kHeadDim;
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = *reinterpret_cast<const u32x4*>(rp + 8 * sub + 32 * i);
            const int np = npos[rc];
            double d2 = sq_dist_packed(qs, v);
            d2 += __shfl_xor(d2, 1);
            d2 += __shfl_xor(d2, 2);
            if (r < W && np >= np_lo && np <= np_hi && d2 <= bound) {
                double e = 0.0;
                for (int i = 0; i < D; ++i) {
                    const double diff = __dsub_rn((double)bits_to_float((uint32_t)q_h[i] << 16), (double)bits_to_float((uint32_t)rp[i] << 16));
                    e = __dadd_rn(e, __dmul_rn(diff, diff));
                }
                if (better(e, np, e_d2, e_np)) { e_second = e_d2; e_d2 = e; e_np = np; e_j = r; }
                else e_second = fmin(e_second, e);
            }
        }
        reduce_best(e_d2, e_np, e_j, e_second, sub == 0 && e_np >= 0);       // the 4 lanes of a quad hold the same values
        best_d2 = e_d2; best_np = e_np; best_j = e_j;
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
        if (!fuse) atomicAdd(p.pending, 1);
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
    // K and V rows are read alike: 16 lanes cover a 256-byte row, a wave takes 4 whole rows per load instruction (the
    // pattern a compute unit pulls fastest, see the match above); the first kVPre V rows of every thread are requested
    // together with its first K rows.
    constexpr int kRowGroups = NT / 16, kKPass = NT == 256 ? (kLean ? 5 : 9) : 8, kVPre = kKPass;   // (256 threads: one pass for B + 1 = 129 rows; lean: 65)
    const int col = tid & 15, rg = tid >> 4;
    const u32x4 qk = 8 * col < D ? *reinterpret_cast<const u32x4*>(p.q_rope + (int64_t)bh * D + 8 * col) : kZero4;    // this lane's chunk of the post-RoPE query
    const int colc = min(col, (D >> 3) - 1);                   // lanes past the end of a K/V row re-read its last 16 bytes
    u32x4 vpre[kVPre];
    // logits (log2 domain): each lane its chunk's share (v_dot2c_f32_bf16), summed over the 16 lanes of the row
    for (int r0 = 0; r0 < cnt; r0 += kKPass * kRowGroups) {
        u32x4 kk[kKPass];
#pragma unroll
        for (int u = 0; u < kKPass; ++u)
            kk[u] = *reinterpret_cast<const u32x4*>(row_ptr(min(r0 + u * kRowGroups + rg, cnt - 1)) + 8 * colc);
        if (r0 == 0) {
#pragma unroll
            for (int u = 0; u < kVPre; ++u)
                vpre[u] = *reinterpret_cast<const u32x4*>(row_ptr(min(u * kRowGroups + rg, cnt - 1)) + p.stride_kv + 8 * colc);
        }
#pragma unroll
        for (int u = 0; u < kKPass; ++u) {
            const float dot = row_sum_f32(dot8_bf16(kk[u], qk));
            const int r = r0 + u * kRowGroups + rg;
            if (col == 0 && r < cnt) s_logit[r] = dot * p.scale_log2;
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
    mx0 = wave_max_f32(mx0);
    mx1 = wave_max_f32(mx1);
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
    z0 = wave_sum_f32(z0);
    z1 = wave_sum_f32(z1);
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
                vv[u] = *reinterpret_cast<const u32x4*>(row_ptr(min(r0 + u * kRowGroups + rg, cnt - 1)) + p.stride_kv + 8 * colc);
#pragma unroll
            for (int u = 0; u < 4; ++u) add_row(r0 + u * kRowGroups + rg, vv[u]);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {                          // lanes l, l^16, l^32, l^48 hold the same columns
            a0[j] = add_xor32(add_xor16(a0[j]));
            a1[j] = add_xor32(add_xor16(a1[j]));
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
        if (d < D) {
            if (p.out_bf16) static_cast<uint16_t*>(p.out)[(int64_t)bh * D + d] = float_to_bf16_rne(o);
            else static_cast<float*>(p.out)[(int64_t)bh * D + d] = o;
        }
        if (d == 0 && p.out_lse != nullptr) p.out_lse[bh] = lse;
        // rectify-append into entry (n - 1) mod W of this head
        const int jn = (n - 1) % W;
        const int64_t e = ring_row0 + jn;
        p.ring_q[e * kHeadDim + d] = d < D ? p.q_pre[(int64_t)bh * D + d] : (uint16_t)0;
        p.ring_O[e * kHeadDim + d] = rect_o;
        if (d == 0) {
            p.ring_lse[e] = rect_l;
            p.ring_npos[e] = n;
        }
    }
}

}  // namespace mac
