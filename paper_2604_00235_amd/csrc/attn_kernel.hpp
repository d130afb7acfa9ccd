// Band+tail / full split-K decode attention over a paged bf16 KV cache (gfx950, wave64, MFMA).
//
// What it computes (paper Sec. 2 "Notation", Sec. 3.1, Eq. (rect-recomp)): for one KV group (request b,
// kv head g) and one work item = a token range [lo, hi), for every query head h of the group that is served here the
// attention summary of the keys [max(lo, s_h), hi) under the post-RoPE query:  O = sum_t p_t V_t / sum_t p_t,
// LSE = ln sum_t e^{scale q.K_t}.  The summaries of all work items are merged by the merge kernel.
// KV is streamed once per KV group, from the smallest start among the group's heads (Sec. 5.8); heads that
// start later mask the tokens before their own start.  Heads the per-head matcher has already finished (hits with a
// short fresh range, see hit_kernel.hpp) are not served: a group all of whose heads are finished has no work items.
//
// Work items.  The fresh range [gs, n) of a group is cut at n - B (the last-B band, whose summary must stay
// separate because the stored rectified summary excludes it, Fig. 1(c)) and on a global grid of C tokens: "mid" items
// are the chunks x = floor(gs/C) .. ceil((n-B)/C) - 1, [x C, (x+1) C) clipped to [gs, n-B); "band" items the chunks from
// floor((n-B)/C) on, clipped to [n-B, n).  A mid item writes its partial to slot x of its heads' rows, the k-th band
// item to slot n_mid_slots + k.  C and the list of items are derived on the device by the planner at the head of the
// kernel (below).
//
// Mapping to the hardware.  A work-group is 4 waves; wave w takes the 32-token tiles w, w+4, ... of the chunk
// (those that intersect the work item) and keeps its own online-softmax state; the 4 states are merged
// through LDS at the end.
// Per tile and wave, with lane l = (r = l%16, kg = l/16):
//   S = K Q^T by v_mfma_f32_16x16x32_bf16:  A = K rows (lane: row 4(r%4) + r/4 of a 16-token sub-tile,
//       8 contiguous d elements 32c+8kg.. of k-step c), B = Q^T (lane: head r, same d elements).  Output: lane
//       holds head r and the scores of tokens 4i+kg (i<4) of the sub-tile.  K is loaded from global memory
//       directly in this layout (16 rows x 64 contiguous bytes per instruction; the four k-steps cover each
//       256-byte row once).
//   O += P V by the same MFMA:  A = P (lane: head r, 8 tokens = its own 2x4 scores, so the QK output is
//       used in place), B = V (lane: 8 d-columns 8r..8r+7 of the same 8 tokens 4i+kg).  With that token
//       labelling V load i of a sub-tile reads rows 4i..4i+3, one per quarter-wave: 1 KiB contiguous per
//       instruction.  The 8 rows are transposed in registers with v_perm_b32 into 8 operands, one per
//       column offset j; operand j produces output columns d = 8r + j.
//       (Supplying K rows in natural order makes the V loads 4 separate 256-byte rows per instruction; measured
//       with load-only probes, that combination streams ~4 % slower at this occupancy.)
//   P is fp32 on the VALU (max, exp2, sum) and enters the MFMA as two bf16 terms hi + lo (truncation split,
//       relative error 2^-16), because a single bf16 P would cost ~1e-3 relative output error.
// Heads beyond G in the 16-row head tile, and heads that are not served, carry zero queries; their results are never
// stored.  Cross-row maxima and sums use the row-swap instructions of this chip (v_permlane16_swap / v_permlane32_swap).
//
// Memory.  Every K/V byte is used once per KV group, so the tiles are read with non-temporal loads (the stream
// then neither displaces the query ring from the last-level cache nor pays for allocating lines it will not reuse:
// measured 327 us against 366 us on 4 x 8 groups of 131072 tokens) into two register tiles per wave; the loads of
// the next tile are in flight while the current one is computed.  K/V never pass through shared memory: both
// operand layouts are reachable with 16-byte global loads, and a round trip through shared memory for a coalesced
// K image (tried with ds_write/ds_read and with loads that write shared memory directly) costs more than the
// better access pattern returns.
#pragma once
#include "common.hpp"

namespace mac {

struct AttnParams {
    const int32_t* kv_lens;      // [batch]
    const int32_t* head_start;   // [batch*Hq + 32] first key of each head's fresh range, | kHeadDone if the matcher has
                                 // finished the head; null = full decode (every head starts at 0)
    const uint16_t* q_rope;      // [batch, Hq, d] bf16
    const uint16_t* kv_pages;    // paged cache, bf16
    int64_t stride_page, stride_kv, stride_head, stride_tok;   // elements
    const int32_t* block_table;  // [batch, bt_stride]
    int32_t bt_stride;
    float* part_O;               // [batch*Hq, n_slots, 128] normalised partial outputs
    float* part_lse;             // [batch*Hq, n_slots]      natural-log LSE of each partial
    int32_t batch, Hq, G;
    int32_t head_dim;            // d of the caller's tensors: 32, 64, 96 or 128 (rows are widened to 128 in here)
    int32_t page_shift;          // log2(page_size)
    int32_t band;                // B; 0 for full decode (no band work items)
    int32_t chunk_fixed;         // > 0: tokens per work item fixed by the caller (multiple of 32, <= 4096);
                                 // 0: chosen per launch from the work the step has, within [chunk_min, 8192]
    int32_t chunk_min;           // multiple of 32; the partial slots are laid out for it
    int32_t n_mid_slots, n_slots;
    int32_t n_cu;                 // compute units of the device: the planner makes work items in multiples of it
    int32_t max_kv_len;
    float scale_log2;            // sm_scale * log2(e)
    const int32_t* pending;      // [1] heads the matcher left to this kernel, or null: 0 = nothing to do, leave at once
    int32_t* step_chunk;         // [1] tokens per work item of this launch, for the merge kernel (chunk_fixed == 0)
    unsigned long long* st_read; // [batch*Hkv] KV tokens the method streams per group (from the smallest start of all
                                 // its heads); null for full decode
    unsigned long long* st_full; // [batch*Hkv] KV tokens a full decode would stream
    unsigned long long* st_split;   // [batch*Hkv] KV tokens this kernel streams (heads the matcher finished excluded)
};

// A K/V tile in registers: k[sub-tile][k-step] are the A operands of S = K Q^T; v[4*sub-tile + i] holds 8 d-columns of
// token 16*sub + 4i + kg.

// Fresh ranges of one KV group: n, band start, smallest / largest start among the heads this kernel serves (gs, gmax),
// smallest start among all heads (gs_all: what the method streams per KV group, Sec. 5.8 -- a counter only).
struct GroupSpan {
    int n, nb, gs, gmax, gs_all;
    bool any;                    // some head of the group is served by this kernel
};

__device__ __forceinline__ GroupSpan group_span(const AttnParams& p, int b, int hbase) {
    GroupSpan s;
    s.n = clampi(p.kv_lens[b], 0, p.max_kv_len);
    s.nb = s.n - p.band > 0 ? s.n - p.band : 0;              // the band is [nb, n)
    s.gs = 0; s.gmax = 0; s.gs_all = 0;
    s.any = true;
    if (p.head_start != nullptr) {
        // (the array is padded by 32 entries, so that blocks of 16 loads can be issued without a bound check)
        s.gs = s.nb; s.gs_all = s.nb;
        s.any = false;
        for (int i0 = 0; i0 < p.G; i0 += 16) {
            int t[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) t[j] = p.head_start[hbase + i0 + j];
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (i0 + j < p.G) {
                    const int sv = min(t[j] & (kHeadDone - 1), s.nb);
                    s.gs_all = min(s.gs_all, sv);
                    if (!(t[j] & kHeadDone)) {
                        s.any = true;
                        s.gs = min(s.gs, sv);
                        s.gmax = max(s.gmax, sv);
                    }
                }
        }
    }
    return s;
}

constexpr int kAttnChunkMax = 8192;      // tokens per work item at most (a wave's page ids sit one per lane in two registers)
constexpr int kAttnChunkPref = 2048;     // the planner makes fewer items rather than shorter ones

template <int HT> struct AttnCaps { static constexpr int kMaxGroups = HT == 1 ? 2048 : 256; };

template <int HT, bool kFullDim>
__device__ __forceinline__ void attn_item(const AttnParams& p, int C, int q, bool is_band, int item_k, int n, int gs,
                                          float (&s_O)[4][HT * 16 * kHeadDim], float (&s_m)[4][HT * 16],
                                          float (&s_l)[4][HT * 16], char* s_q, int (&s_skip)[HT * 16]);

// The planner of the paper (Sec. 4.2 K2 (1), App. B.2 "Load balancing": work-groups in proportion to span) runs inside
// the kernel: every work-group derives the same list of work items from kv_lens and the heads' starts -- one thread
// per KV group for the group's range, then, after one barrier, every wave by itself: the step's total span, from it
// the tokens per item (the rule is stated where it is applied, below), the prefix sums of the groups' item counts --
// and takes the item blockIdx.x (and blockIdx.x + gridDim.x, ... should there be more items than work-groups).  The
// host launches as many work-groups as the same rule makes items for max_kv_len tokens per group: normally one item
// per work-group, handed out by the hardware dispatcher as earlier work-groups finish.  A step whose heads were all
// finished by the matcher costs one load per work-group.
// HT = number of 16-head tiles: 1 (G <= 16) or 2 (G <= 32).  kFullDim = the head dimension is 128; otherwise (32, 64, 96)
// the kernel works on rows widened to 128: the queries are padded with zeros, K loads of the missing k-steps and V loads of
// the missing columns re-read the row's last valid 64 / 16 bytes (so that the loads of a tile stay the same in number), and
// the columns d .. 127 of the partial results are never looked at by anyone.
template <int HT, bool kFullDim>
__global__ __launch_bounds__(256, 2) void attn_kernel(const AttnParams p) {
    // Shared memory.  s_O carries the waves' states to the merge at the end.  With two head tiles (HT == 2) a wave
    // keeps only one tile's output accumulators in registers: during the stream s_O[w] holds both tiles'
    // accumulators in register layout ([tile][column block j][lane] x 16 B: conflict-free) and each tile is loaded,
    // updated and stored back per K/V tile.  The queries (B operands of S = K Q^T) sit in s_q, rows padded to 272 B
    // so that the 16 rows read by one instruction fall into different banks.
    __shared__ __attribute__((aligned(16))) float s_O[4][HT * 16 * kHeadDim];
    __shared__ __attribute__((aligned(16))) float s_m[4][HT * 16];
    __shared__ __attribute__((aligned(16))) float s_l[4][HT * 16];
    constexpr int kQRowBytes = 2 * kHeadDim + 16;
    __shared__ __attribute__((aligned(16))) char s_q[HT * 16 * kQRowBytes];
    __shared__ int s_skip[HT * 16];
    constexpr int kCap = AttnCaps<HT>::kMaxGroups;
    __shared__ int s_prefix[kCap], s_bprefix[kCap];          // mid / band work items before group q inside its block of 64 groups
    __shared__ int s_blk[2][kCap / 64];                      // mid / band work items of each block of 64 groups
    __shared__ int s_gs[kCap], s_n[kCap];                    // start of the group's range (-1: nothing to do), kv_len
    __shared__ double s_red[2][4];
    // every head was finished by the matcher: only the first work-group stays, for the per-group counters
    if (p.pending != nullptr && *p.pending == 0 && blockIdx.x != 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int Hkv = p.Hq / p.G, NG = p.batch * Hkv;
    const int P = gridDim.x;
    // Up to 64 KV groups every wave derives the whole plan by itself (one group per lane, no barrier after the first);
    // beyond that the four waves share the groups (thread t takes t, t + 256, ...: a wave always holds 64
    // consecutive groups) and meet through shared memory.  Totals up to 2^41 tokens are exact in double precision.
    const bool coop = NG > 64;
    const int first = coop ? tid : lane, stride = coop ? 256 : 64;
    int parity = 0;
    auto total_of = [&](double v) {                          // the same total in every thread
        v = wave_sum_f64(v);
        if (coop) {
            if (lane == 0) s_red[parity][wv] = v;
            __syncthreads();
            v = (s_red[parity][0] + s_red[parity][1]) + (s_red[parity][2] + s_red[parity][3]);
            parity ^= 1;
        }
        return v;
    };

    // ---- plan: the groups' ranges (one thread per group); the first work-group also keeps the per-group counters
    for (int q = tid; q < NG; q += 256) {
        const int b = q / Hkv, g = q - b * Hkv;
        const GroupSpan s = group_span(p, b, b * p.Hq + g * p.G);
        const bool work = s.any && s.n > s.gs;
        s_gs[q] = work ? s.gs : -1;
        s_n[q] = s.n;
        if (blockIdx.x == 0 && p.st_read != nullptr) {       // one writer per address and step: fire-and-forget adds
            atomicAdd(&p.st_read[q], (unsigned long long)(s.n - s.gs_all));
            atomicAdd(&p.st_full[q], (unsigned long long)s.n);
            if (s.any) atomicAdd(&p.st_split[q], (unsigned long long)(s.n - s.gs));
        }
    }
    __syncthreads();
    double tok = 0.0, busy = 0.0;                            // the step's span, and the groups that have any
    for (int q = first; q < NG; q += stride)
        if (s_gs[q] >= 0) { tok += (double)(s_n[q] - s_gs[q]); busy += 1.0; }
    tok = total_of(tok);
    busy = total_of(busy);
    if (tok == 0.0) return;
    // ---- plan: tokens per item
    // Measured on 256 compute units (two work-groups resident on each), 32 groups of equal length: what counts is
    // that the number of items is a whole multiple of the number of compute units (each then streams the same bytes;
    // whether one or two of its work-groups are busy matters little), that items stay at or above ~2048 tokens (an
    // item's prologue and epilogue cost several microseconds in which its slot streams nothing) and that work-groups
    // are handed their item by the dispatcher rather than looping over a fixed share (a compute unit favours its
    // older work-group: with fixed shares the younger one is left alone at the end).  So: as many items as 4 per
    // compute unit, fewer (3, 2, 1 per unit) while that keeps them at 2048 tokens, more only to keep them within the
    // cap or because there are more groups with work than that (each has an item of its own anyway).
    // (Divisions by C: exact, by a double-precision reciprocal and one correction step; an integer division costs ~40
    // instructions here and the plan has four per group.)
    auto div_by = [](int x, int c, double rc) {
        const int qt = __double2int_rz(__int2double_rn(x) * rc);
        const int r = x - qt * c;
        return qt + (r >= c ? 1 : 0) - (r < 0 ? 1 : 0);
    };
    auto mid_items_of = [&](int q, int c, double rc) {       // chunks of [gs, n-B) on the global grid of c tokens
        const int gs = s_gs[q], n = s_n[q];
        const int nb = n - p.band > 0 ? n - p.band : 0;
        return (gs >= 0 && nb > gs) ? div_by(nb + c - 1, c, rc) - div_by(gs, c, rc) : 0;
    };
    auto band_items_of = [&](int q, int c, double rc) {      // chunks of the band [n-B, n) on the same grid
        const int gs = s_gs[q], n = s_n[q];
        const int nb = n - p.band > 0 ? n - p.band : 0;
        return (gs >= 0 && n > nb) ? div_by(n + c - 1, c, rc) - div_by(nb, c, rc) : 0;
    };
    int C = p.chunk_fixed;
    if (C == 0) {
        const double U = (double)p.n_cu;
        double N = floor(tok / ((double)kAttnChunkPref * U)) * U;
        N = N < U ? U : (N > 4.0 * U ? 4.0 * U : N);
        if (N * kAttnChunkMax < tok) N = ceil(tok / (U * kAttnChunkMax)) * U;
        if (N < busy) N = ceil(busy / U) * U;
        auto chunk_for = [&](double items) {
            const int c = ((int)ceil(tok / items) + 31) & ~31;
            return c < p.chunk_min ? p.chunk_min : c;
        };
        C = chunk_for(N);
        for (int tries = 0; tries < 6; ++tries) {
            if (C > kAttnChunkMax) { N += U; C = chunk_for(N); }
            const double rc = 1.0 / (double)C;
            double items = 0.0;
            for (int q = first; q < NG; q += stride) items += (double)mid_items_of(q, C, rc);
            items = total_of(items);
            if (items <= N || C >= kAttnChunkMax) break;
            // too many by `items - N`: lengthen every item by its share of their tokens
            C += ((int)ceil((items - N) * (double)C / N) + 31) & ~31;
        }
        if (C > kAttnChunkMax) C = kAttnChunkMax;
    }
    C = __builtin_amdgcn_readfirstlane(C);                   // uniform values in scalar registers: what derives from them stays there
    const double rC = 1.0 / (double)C;
    // ---- plan: the list of work items.  It holds the mid items of all groups first, then the band items (at most B
    // tokens each).  Two levels of prefix sums: inside each block of 64 groups (shared memory, one entry per group),
    // and over the blocks (at most 32: one per lane, kept in registers by every wave).
    const int nblk = (NG + 63) >> 6;
    for (int q0 = 0; q0 < NG; q0 += stride) {
        const int q = q0 + first;                            // (64 consecutive groups in a wave)
        const int cm = q < NG ? mid_items_of(q, C, rC) : 0, cb = q < NG ? band_items_of(q, C, rC) : 0;
        const int im = wave_scan_incl_i32(cm, lane), ib = wave_scan_incl_i32(cb, lane);
        if (q < NG) { s_prefix[q] = im - cm; s_bprefix[q] = ib - cb; }
        if (lane == 63) { s_blk[0][q >> 6] = im; s_blk[1][q >> 6] = ib; }
    }
    if (coop) __syncthreads();
    int off_m = lane < nblk ? s_blk[0][lane] : 0, off_b = lane < nblk ? s_blk[1][lane] : 0;   // -> items before block `lane`
    off_m = wave_scan_incl_i32(off_m, lane) - off_m;
    off_b = wave_scan_incl_i32(off_b, lane) - off_b;
    const int total_mid = __builtin_amdgcn_readlane(off_m, nblk - 1) + __builtin_amdgcn_readfirstlane(s_blk[0][nblk - 1]);
    const int total = total_mid + __builtin_amdgcn_readlane(off_b, nblk - 1) + __builtin_amdgcn_readfirstlane(s_blk[1][nblk - 1]);
    if (tid == 0 && blockIdx.x == 0 && p.step_chunk != nullptr) *p.step_chunk = C;

    // ---- work items: normally one per work-group (the grid is sized by the same rule); the loop serves launches with a
    // caller-fixed item size or more items than the grid's cap.  Handing the items out one by one from a counter to
    // resident work-groups (requested before an item's epilogue, so that its latency is hidden) was measured against
    // fixed shares with 2 to 8 items per work-group and was never faster (32 groups of 131072 tokens: 337 us at 2, 360 us
    // at 8; fixed shares 337 us; one item per dispatched work-group 332 us).
    for (int item = blockIdx.x; item < total; item += P) {
        const bool is_band = item >= total_mid;
        const int pos = is_band ? item - total_mid : item;
        // the block, then the group inside it: the last one whose items start at or before `pos`
        const int off = is_band ? off_b : off_m;
        const int j = __popcll(__builtin_amdgcn_ballot_w64(lane < nblk && off <= pos)) - 1;
        const int qq = 64 * j + lane;
        const int before = qq < NG ? (is_band ? s_bprefix[qq] : s_prefix[qq]) + __builtin_amdgcn_readlane(off, j) : 0x7fffffff;
        const int r = __popcll(__builtin_amdgcn_ballot_w64(before <= pos)) - 1;
        const int q = 64 * j + r;
        const int k = pos - __builtin_amdgcn_readlane(before, r);      // index among the group's mid (or band) items
        const int n = __builtin_amdgcn_readfirstlane(s_n[q]), gs = __builtin_amdgcn_readfirstlane(s_gs[q]);
        attn_item<HT, kFullDim>(p, C, q, is_band, k, n, gs, s_O, s_m, s_l, s_q, s_skip);
        __syncthreads();
    }
}

// One work item: the `item_k`-th mid (or band) item of KV group q with C tokens per item.  Contains barriers: called by
// the whole work-group.
template <int HT, bool kFullDim>
__device__ __forceinline__ void attn_item(const AttnParams& p, const int C, const int q, const bool is_band, const int item_k, const int n,
                                          const int gs, float (&s_O)[4][HT * 16 * kHeadDim], float (&s_m)[4][HT * 16],
                                          float (&s_l)[4][HT * 16], char* s_q, int (&s_skip)[HT * 16]) {
    constexpr int kQRowBytes = 2 * kHeadDim + 16;
    const int Hkv = p.Hq / p.G;
    const int b = q / Hkv, g = q - b * Hkv;
    // (the thread index passes through an empty asm statement: what is derived from it is then computed per work
    // item instead of being kept in registers across the loop over work items, where none are to spare)
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave index as a scalar: tile positions and page bases stay in SGPRs
    const int r16 = l & 15, kg = l >> 4;
    const int G = p.G;
    const int tiles_per_chunk = C >> 5;
    const int hbase = b * p.Hq + g * G;
    const int nb = n - p.band > 0 ? n - p.band : 0;          // the band is [nb, n)
    // chunk index on the global grid of C tokens, the item's token range, and its partial slot
    const bool is_mid = !is_band;
    const int x = (is_mid ? gs : nb) / C + item_k;
    const int lo = is_mid ? max(gs, x * C) : max(nb, x * C);
    const int hi = is_mid ? min(nb, (x + 1) * C) : min(n, (x + 1) * C);
    const int slot = is_mid ? x : p.n_mid_slots + item_k;
    if (lo >= hi) return;                                    // (the plan lists no empty item)

    // Page ids of this wave's 16-token sub-tiles, one per lane and register: lane i of register j <-> (k = 32j + i/2,
    // sub-tile i%2), where the wave's k-th tile of the chunk is chunk_tile0 + w + 4k.
    const int pk = l >> 1, pu = l & 1;
    const int chunk_tile0 = x * tiles_per_chunk;
    int mypid[2] = {0, 0};
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int tok = (chunk_tile0 + w + 4 * (pk + 32 * j)) * kTileTokens + 16 * pu;
        if (w + 4 * (pk + 32 * j) < tiles_per_chunk)
            mypid[j] = p.block_table[(int64_t)b * p.bt_stride + min(tok >> p.page_shift, p.bt_stride - 1)];
    }
    int my_start[HT];                                        // start of the head this lane holds in each head tile,
#pragma unroll                                               // | kHeadDone if the head needs nothing (or does not exist)
    for (int ht = 0; ht < HT; ++ht) {
        my_start[ht] = (ht * 16 + r16 < G) ? 0 : kHeadDone;
        if (p.head_start != nullptr && ht * 16 + r16 < G) my_start[ht] = p.head_start[hbase + ht * 16 + r16];
    }
    // largest start among the heads served here: tiles at or above it need no start mask
    int gmax = 0;
#pragma unroll
    for (int ht = 0; ht < HT; ++ht)
        if (!(my_start[ht] & kHeadDone)) gmax = max(gmax, min(my_start[ht], nb));
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) gmax = max(gmax, __shfl_xor(gmax, off));
    const int maxstart = max(__builtin_amdgcn_readfirstlane(gmax), lo);

    // per-lane head data for each head tile: first token this head attends to
    int hstart[HT];
    // a head that needs nothing here (finished by the matcher, or padding of the head tile) gets a zero query and no
    // mask; its rows of the result are never stored
#pragma unroll
    for (int ht = 0; ht < HT; ++ht) {
        const bool skip = (my_start[ht] & kHeadDone) != 0;
        hstart[ht] = skip ? lo : max(lo, min(my_start[ht], nb));
        if (w == 0 && kg == 0) s_skip[ht * 16 + r16] = skip ? 1 : 0;
    }
    // Queries: HT * 16 rows x 16 chunks of 16 B, HT per thread; rows of heads that need nothing are zero.  The loads are
    // issued here and stored to shared memory only after the first K/V tile has been requested (below), so that the
    // wait for them overlaps that tile's latency.
    u32x4 qv[HT];
    int qflag[HT];
#pragma unroll
    for (int t = 0; t < HT; ++t) {
        const int idx = tid + 256 * t, row = idx >> 4, ch = idx & 15;
        const int rowc = row < G ? row : 0;
        qflag[t] = p.head_start != nullptr ? p.head_start[hbase + rowc] : 0;
        const int chc = kFullDim ? ch : min(ch, (p.head_dim >> 3) - 1);
        qv[t] = *reinterpret_cast<const u32x4*>(p.q_rope + (int64_t)(hbase + rowc) * (kFullDim ? kHeadDim : p.head_dim) + 8 * chc);
    }
    auto stage_queries = [&]() {
#pragma unroll
        for (int t = 0; t < HT; ++t) {
            const int idx = tid + 256 * t, row = idx >> 4, ch = idx & 15;
            const bool skip = row >= G || (qflag[t] & kHeadDone) || (!kFullDim && 8 * ch >= p.head_dim);
            *reinterpret_cast<u32x4*>(s_q + row * kQRowBytes + 16 * ch) = skip ? u32x4{0u, 0u, 0u, 0u} : qv[t];
        }
        if constexpr (HT == 2) {
            // this wave's accumulators of both tiles start at zero
            char* acc_img = reinterpret_cast<char*>(&s_O[w][0]);
#pragma unroll
            for (int i = 0; i < 16; ++i) *reinterpret_cast<f32x4*>(acc_img + 1024 * i + 16 * l) = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        __syncthreads();
    };

    // this wave's tiles of the chunk that intersect [lo, hi): k = k_first .. k_last
    const int tt_lo = lo >> 5, tt_hi = (hi - 1) >> 5;
    const int d_lo = tt_lo - chunk_tile0 - w, d_hi = tt_hi - chunk_tile0 - w;
    const int k_first = d_lo > 0 ? (d_lo + 3) >> 2 : 0;
    const int k_end = d_hi >= 0 ? (d_hi >> 2) + 1 : 0;        // one past the last; <= 64 because chunk <= 8192
    // A sub-tile wholly past the end (only the second one of a request's last tile can be) has no table entry of its
    // own: it re-reads the tile's first sub-tile, whose rows are real data of this request (its scores are masked, but
    // its V rows still enter the P V product with weight 0, so they must be finite: no page the request does not own is
    // ever touched).
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int first_sub = __shfl(mypid[j], l & ~1);
        if ((chunk_tile0 + w + 4 * (pk + 32 * j)) * kTileTokens + 16 * pu >= n) mypid[j] = first_sub;
    }
    const int page_mask = (1 << p.page_shift) - 1;
    const uint16_t* kv_g = p.kv_pages + (int64_t)g * p.stride_head;

    // All 16 loads of a tile are issued unconditionally (rows past the end re-read the last valid row, whose
    // scores are masked): with a fixed number of loads per tile the compiler can wait for exactly the older
    // tile's loads and leave the prefetched tile in flight.
    // The page base of a sub-tile is wave-uniform (scalar registers); each lane adds a 32-bit byte offset that does
    // not depend on the tile: its row times the token stride (clamped to the last valid row with one v_min) plus its
    // 16-byte column.  So a load costs one or two vector instructions of address arithmetic.
    const int krow = 4 * (r16 & 3) + (r16 >> 2);               // sub-tile row this lane supplies to S = K Q^T
    const uint32_t tok_bytes = (uint32_t)p.stride_tok * 2u;    // host checks stride_tok < 2^26
    const uint32_t k_row_b = (uint32_t)krow * tok_bytes, k_col_b = 16u * (uint32_t)kg;
    uint32_t v_row_b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) v_row_b[i] = (uint32_t)(4 * i + kg) * tok_bytes;
    const uint32_t v_col_b = 16u * (uint32_t)(kFullDim ? r16 : min(r16, (p.head_dim >> 3) - 1));
    const int k_steps = kFullDim ? 4 : p.head_dim >> 5;          // k-steps of 32 elements that the rows really have
    // base address of sub-tile u of the wave's k-th tile (rows past the end fold back, see above) and its row limit
    auto sub_tile = [&](int k, int u, uint32_t& lim_b) {
        const int t0 = (chunk_tile0 + w + 4 * k) * kTileTokens;
        const bool past = t0 + 16 * u >= n;                   // then u == 1 and t0 < n: the tile intersects [lo, hi)
        const int tb = past ? t0 : t0 + 16 * u;
        lim_b = (uint32_t)min(15, n - 1 - tb) * tok_bytes;    // last valid row, in bytes
        const int pid = k < 32 ? __builtin_amdgcn_readlane(mypid[0], 2 * k + u) : __builtin_amdgcn_readlane(mypid[1], 2 * (k - 32) + u);
        return reinterpret_cast<const char*>(kv_g + (int64_t)pid * p.stride_page + (int64_t)(tb & page_mask) * p.stride_tok);
    };
    auto load_k = [&](int k, u32x4 (&K)[2][4]) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            uint32_t lim_b;
            const char* kp = sub_tile(k, u, lim_b) + (min(k_row_b, lim_b) + k_col_b);
#pragma unroll
            for (int c = 0; c < 4; ++c)
                K[u][c] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kp + 64 * (kFullDim ? c : min(c, k_steps - 1))));
        }
    };
    auto load_v = [&](int k, u32x4 (&V)[8]) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            uint32_t lim_b;
            const char* vbase = sub_tile(k, u, lim_b) + 2 * p.stride_kv;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                V[4 * u + i] = __builtin_nontemporal_load(
                    reinterpret_cast<const u32x4*>(vbase + (min(v_row_b[i], lim_b) + v_col_b)));
        }
    };

    // online-softmax state of this wave: running max (log2 domain), this lane's share of the running sum,
    // and the unnormalised output: acc[ht][j][i] = O[head ht*16 + 4kg + i][d = 8*r16 + j]
    float m_run[HT], l_run[HT];
    f32x4 acc[8];                                             // HT == 2: the tile being updated, see s_O above
#pragma unroll
    for (int ht = 0; ht < HT; ++ht) {
        m_run[ht] = -INFINITY;
        l_run[ht] = 0.f;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};

    bf16x8 qreg[4];                                           // HT == 1: this lane's B operands of S = K Q^T (set below)
    // scores of the wave's k-th tile for every head tile: sc[ht][4u + i] = scale * q_head . K_token, log2 domain, masked
    auto qk = [&](int k, const u32x4 (&K)[2][4], float (&sc)[HT][8]) {
        const int t0 = (chunk_tile0 + w + 4 * k) * kTileTokens;
        const bool need_mask = (t0 < maxstart) || (t0 + kTileTokens > hi);   // wave-uniform
        // With two head tiles the queries come from shared memory (row = head, 16-byte chunk 4c + kg of k-step c), read
        // again for every tile: 32 registers that are not to spare there.  One head tile keeps them in registers.
        if constexpr (HT == 2) asm volatile("" ::: "memory");
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) {
            bf16x8 qop[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if constexpr (HT == 1) qop[c] = qreg[c];
                else qop[c] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(
                                  s_q + (ht * 16 + r16) * kQRowBytes + 64 * c + 16 * kg));
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, K[u][c]), qop[c], s, 0, 0, 0);
#pragma unroll
                for (int i = 0; i < 4; ++i) sc[ht][4 * u + i] = s[i] * p.scale_log2;
            }
            if (need_mask) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int tok = t0 + 16 * (e >> 2) + 4 * (e & 3) + kg;
                    if (tok < hstart[ht] || tok >= hi) sc[ht][e] = -INFINITY;
                }
            }
        }
    };
    // softmax update and O += P V of the wave's k-th tile, one head tile after the other
    auto pv = [&](const u32x4 (&V)[8], const float (&sc)[HT][8]) {
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) {
            char* const acc_img = reinterpret_cast<char*>(&s_O[w][0]) + 8192 * ht + 16 * l;
            if constexpr (HT == 2) {
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] = *reinterpret_cast<const f32x4*>(acc_img + 1024 * j);
            }
            float tmax = sc[ht][0];
#pragma unroll
            for (int e = 1; e < 8; ++e) tmax = fmaxf(tmax, sc[ht][e]);
            tmax = max_xor32(max_xor16(tmax));
            const float m_new = fmaxf(m_run[ht], tmax);
            const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = exp2_fast(m_run[ht] - m_safe);
            float pw[8];
            float psum = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                pw[e] = exp2_fast(sc[ht][e] - m_safe);
                psum += pw[e];
            }
            l_run[ht] = l_run[ht] * alpha + psum;
            if (__builtin_amdgcn_ballot_w64(m_new > m_run[ht]) != 0) {     // some head's max moved: rescale O
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float a = __shfl(alpha, 4 * kg + i);             // lane 4kg+i holds head 4kg+i
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[j][i] *= a;
                }
            }
            m_run[ht] = m_new;
            // P = hi + lo, both bf16 by truncation
            uint32_t hb[8], lb[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t bits = float_to_bits(pw[e]);
                hb[e] = bits;
                lb[e] = float_to_bits(pw[e] - bits_to_float(bits & 0xffff0000u));
            }
            u32x4 a_hi, a_lo;
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                a_hi[q4] = pack_hi16(hb[2 * q4], hb[2 * q4 + 1]);
                a_lo[q4] = pack_hi16(lb[2 * q4], lb[2 * q4 + 1]);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int c = j >> 1;
                u32x4 bj;
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    bj[q4] = (j & 1) ? pack_hi16(V[2 * q4][c], V[2 * q4 + 1][c]) : pack_lo16(V[2 * q4][c], V[2 * q4 + 1][c]);
                const bf16x8 bop = __builtin_bit_cast(bf16x8, bj);
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a_hi), bop, acc[j], 0, 0, 0);
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a_lo), bop, acc[j], 0, 0, 0);
            }
            if constexpr (HT == 2) {
#pragma unroll
                for (int j = 0; j < 8; ++j) *reinterpret_cast<f32x4*>(acc_img + 1024 * j) = acc[j];
                // one tile after the other: interleaving them would need both accumulator sets in registers again
                asm volatile("" ::: "memory");
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    float sc[HT][8];
    int k = k_first;
    if constexpr (HT == 1) {
        // Two-deep software pipeline over whole tiles: the next tile's 16 loads are in flight while the current one
        // is computed.  The steady-state loop has no conditional loads; the last one or two tiles are peeled.
        u32x4 ka[2][4], va[8], kb[2][4], vb[8];
        if (k < k_end) { load_k(k, ka); load_v(k, va); }
        stage_queries();
#pragma unroll
        for (int c = 0; c < 4; ++c)
            qreg[c] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(s_q + r16 * kQRowBytes + 64 * c + 16 * kg));
        for (; k + 2 < k_end; k += 2) {
            load_k(k + 1, kb); load_v(k + 1, vb);
            qk(k, ka, sc); pv(va, sc);
            load_k(k + 2, ka); load_v(k + 2, va);
            qk(k + 1, kb, sc); pv(vb, sc);
        }
        if (k_end - k == 2) {
            load_k(k + 1, kb); load_v(k + 1, vb);
            qk(k, ka, sc); pv(va, sc);
            qk(k + 1, kb, sc); pv(vb, sc);
        } else if (k_end - k == 1) {
            qk(k, ka, sc); pv(va, sc);
        }
    } else {
        // Two head tiles leave no room for two whole K/V tiles: K and V are pipelined separately.  While the scores of
        // tile k are formed from K(k), K(k+1) is in flight; its V(k+1) is requested when K(k)'s registers are free and
        // arrives during the softmax and P V of tile k.  Three half-tiles are live at any time instead of four.
        // (Loads past the wave's last tile re-read that tile: every load stays unconditional.)
        u32x4 ka[2][4], va[8], kb[2][4], vb[8];
        const int k_last = k_end - 1;
        if (k < k_end) { load_k(k, ka); load_v(k, va); }
        stage_queries();
        for (; k + 2 <= k_end; k += 2) {
            load_k(k + 1, kb);
            qk(k, ka, sc);
            __builtin_amdgcn_sched_barrier(0);
            load_v(k + 1, vb);
            pv(va, sc);
            load_k(min(k + 2, k_last), ka);
            qk(k + 1, kb, sc);
            __builtin_amdgcn_sched_barrier(0);
            load_v(min(k + 2, k_last), va);
            pv(vb, sc);
        }
        if (k < k_end) {
            qk(k, ka, sc);
            pv(va, sc);
        }
    }

    // ---- the four waves' states meet in shared memory and leave as one normalised partial per head.
    // The accumulators are stored as they sit in the registers ("image" of a wave: [tile][j][lane] x 16 B, lane
    // 16 kg + r16 holding O[heads 4kg .. 4kg+3][d = 8 r16 + j]; with two head tiles the images are there already).
    // Then each wave takes blocks of four heads (tile ht, kg): lane (jq, r) sums the four images' entries
    // (j = 2jq, 2jq+1; lane 16 kg + r) with the heads' weights, which gives it two adjacent columns of the four
    // heads, so that the 64 lanes together store whole 512-byte rows.
    if constexpr (HT == 1) {
        char* const img = reinterpret_cast<char*>(&s_O[w][0]) + 16 * l;
#pragma unroll
        for (int j = 0; j < 8; ++j) *reinterpret_cast<f32x4*>(img + 1024 * j) = acc[j];
    }
#pragma unroll
    for (int ht = 0; ht < HT; ++ht) {
        const float lsum = add_xor32(add_xor16(l_run[ht]));
        if (kg == 0) {
            s_m[w][ht * 16 + r16] = m_run[ht];
            s_l[w][ht * 16 + r16] = lsum;
        }
    }
    __syncthreads();
    for (int u = w; u < HT * 4; u += 4) {
        const int ht = u >> 2, kgu = u & 3, h0 = ht * 16 + 4 * kgu;
        if (h0 >= G) continue;
        f32x4 mw[4], lw[4], wgt[4];
#pragma unroll
        for (int ww = 0; ww < 4; ++ww) {
            mw[ww] = *reinterpret_cast<const f32x4*>(&s_m[ww][h0]);
            lw[ww] = *reinterpret_cast<const f32x4*>(&s_l[ww][h0]);
        }
        float lse[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float M = fmaxf(fmaxf(mw[0][i], mw[1][i]), fmaxf(mw[2][i], mw[3][i]));
            float f[4], L = 0.f;
#pragma unroll
            for (int ww = 0; ww < 4; ++ww) {
                f[ww] = M == -INFINITY ? 0.f : exp2_fast(mw[ww][i] - M);
                L += lw[ww][i] * f[ww];
            }
            const float inv = L > 0.f ? 1.f / L : 0.f;
#pragma unroll
            for (int ww = 0; ww < 4; ++ww) wgt[ww][i] = f[ww] * inv;
            lse[i] = L > 0.f ? (M + __log2f(L)) * kLn2 : -INFINITY;
        }
        const int jq = l >> 4, r = l & 15;
        f32x4 o[2];
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            o[jj] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ww = 0; ww < 4; ++ww) {
                const f32x4 v = *reinterpret_cast<const f32x4*>(reinterpret_cast<const char*>(&s_O[ww][0]) + 8192 * ht +
                                                                1024 * (2 * jq + jj) + 16 * (16 * kgu + r));
                o[jj] += v * wgt[ww];
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int h = h0 + i;
            if (h >= G || s_skip[h]) continue;
            const int64_t row = (int64_t)(hbase + h) * p.n_slots + slot;
            *reinterpret_cast<f32x2*>(p.part_O + row * kHeadDim + 8 * r + 2 * jq) = f32x2{o[0][i], o[1][i]};
            if (l == 0) p.part_lse[row] = lse[i];
        }
    }
}

}  // namespace mac
