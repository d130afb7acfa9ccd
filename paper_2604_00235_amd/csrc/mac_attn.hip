// Host side of libmacattn: context, argument validation, kernel launches, counters.  C ABI in include/mac_attn.h.
#include "../../include/mac_attn.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "attn_kernel.hpp"
#include "hit_kernel.hpp"
#include "match_kernel.hpp"
#include "merge_kernel.hpp"

// Split-K partials of mac_attn_full_decode_static: one copy per GPU the library runs on, held until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress; kernels get the address it returns.
static __device__ __align__(256) unsigned char scratch[MAC_ATTN_STATIC_SCRATCH_BYTES];

namespace {

thread_local std::string g_last_hip_error;

int hip_fail(hipError_t e, const char* what) {
    g_last_hip_error = std::string(what) + ": " + hipGetErrorString(e);
    return e == hipErrorOutOfMemory ? MAC_ATTN_ERR_OOM : MAC_ATTN_ERR_HIP;
}

#define HIP_TRY(expr)                                        \
    do {                                                     \
        hipError_t e_ = (expr);                              \
        if (e_ != hipSuccess) return hip_fail(e_, #expr);    \
    } while (0)

// Address of this GPU's copy of `scratch`, looked up once per device (each GPU holds the array at an address of
// its own).  `device` must be the current device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(int device, void** out) {
    if (device < 0 || device >= kMaxDevices) return MAC_ATTN_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device] == nullptr) {
        void* ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (ptr == nullptr) return MAC_ATTN_ERR_HIP;
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return MAC_ATTN_OK;
}

// Every device buffer of a context lies between two guard zones of this many bytes holding kGuardByte;
// mac_attn_check_guards reports a write that strayed into one.
constexpr int64_t kGuardBytes = 256;
constexpr int kGuardByte = 0xA5;
constexpr int kNumBuffers = 12;

// Largest fresh range (tokens) of a hit that the per-head matcher finishes itself (see hit_kernel.hpp) by default
constexpr int kDefaultFusedSpan = 1024;

// Tokens per work item of the attention kernel.  With chunk_tokens = 0 the kernel chooses them per launch from the
// work the step has (see attn_kernel.hpp), never below this minimum, for which the partial slots are laid out: 256
// tokens, and at least 32 tokens per head of the group, so that the partial a work item writes (516 B per head) stays
// small next to the K/V it reads (512 B per token).
int min_chunk(int heads_per_group) {
    int chunk = 256;
    while (chunk < 32 * heads_per_group) chunk *= 2;
    return chunk;
}

// Fixed tokens per work item for mac_attn_full_decode_static when the caller gives none: a full-length step should
// have about 2000 work items, within [512, 2048], and at least 64 tokens per head of the group.
int default_chunk(int64_t groups, int64_t max_kv_len, int heads_per_group) {
    const int64_t target = groups * max_kv_len / 2048;
    int chunk = 512;
    while (chunk < 2048 && chunk * 2 <= target) chunk *= 2;
    while (chunk < 2048 && chunk < 64 * heads_per_group) chunk *= 2;
    return chunk;
}

constexpr int64_t kPlanBytes = 256;      // ints: [0] tokens per work item the attention kernel chose at its last launch,
                                         // [16] heads of the current step that the matcher left to the split-K path

struct Layout {            // derived sizes, pure host arithmetic
    int G, chunk_fixed, chunk_min, n_mid_slots, n_band_slots, n_slots, page_shift, max_split;
    int64_t ring_q_bytes, ring_O_bytes, ring_lse_bytes, ring_npos_bytes;
    int64_t part_O_bytes, part_lse_bytes, slices_bytes, match_bytes, rect_bytes, stats_bytes, head_start_bytes;
    int64_t total() const {
        return ring_q_bytes + ring_O_bytes + ring_lse_bytes + ring_npos_bytes + part_O_bytes + part_lse_bytes +
               slices_bytes + match_bytes + rect_bytes + stats_bytes + head_start_bytes + kPlanBytes +
               2 * kGuardBytes * kNumBuffers;
    }
};

int validate_config(const mac_attn_config* c, Layout* L) {
    if (c == nullptr) return MAC_ATTN_ERR_INVALID_ARG;
    if (c->device < 0 || c->max_slots < 1 || c->max_batch < 1 || c->max_batch > c->max_slots) return MAC_ATTN_ERR_INVALID_ARG;
    if (c->num_q_heads < 1 || c->num_kv_heads < 1 || c->num_q_heads % c->num_kv_heads != 0) return MAC_ATTN_ERR_INVALID_ARG;
    if (c->window < 1 || c->band < 0 || c->max_kv_len < 1 || c->page_size < 1) return MAC_ATTN_ERR_INVALID_ARG;
    if (!(c->threshold >= 0.f) || !std::isfinite(c->sm_scale)) return MAC_ATTN_ERR_INVALID_ARG;   // rejects NaN; +inf T is legal
    if (c->chunk_tokens < 0 || (c->fuse_epilogue != 0 && c->fuse_epilogue != 1)) return MAC_ATTN_ERR_INVALID_ARG;
    if (c->max_gap < 0 || (c->group_match != 0 && c->group_match != 1) || (c->out_dtype != 0 && c->out_dtype != 1))
        return MAC_ATTN_ERR_INVALID_ARG;
    if (c->fused_hit_span < -1 || c->fused_hit_span > mac::kHitMaxSpan) return MAC_ATTN_ERR_INVALID_ARG;
    if (c->max_kv_len >= mac::kHeadDone) return MAC_ATTN_ERR_INVALID_ARG;
    if (c->head_dim < 1) return MAC_ATTN_ERR_INVALID_ARG;
    // rows are widened to 128 elements inside the library: d = 32, 64, 96 or 128
    if (c->head_dim > mac::kHeadDim || c->head_dim % 32 != 0) return MAC_ATTN_ERR_UNSUPPORTED;
    const int G = c->num_q_heads / c->num_kv_heads;
    if (G > 32) return MAC_ATTN_ERR_UNSUPPORTED;
    if (c->page_size < 16 || (c->page_size & (c->page_size - 1)) != 0) return MAC_ATTN_ERR_UNSUPPORTED;
    if (c->window > 4096) return MAC_ATTN_ERR_UNSUPPORTED;
    const int chunk = c->chunk_tokens == 0 ? min_chunk(G) : c->chunk_tokens;
    if (chunk % mac::kTileTokens != 0 || chunk < 32 || chunk > 4096) return MAC_ATTN_ERR_INVALID_ARG;
    if ((int64_t)c->max_batch * c->num_q_heads > (1 << 24)) return MAC_ATTN_ERR_INVALID_ARG;
    // the attention kernel plans its work items with one list entry per KV group in shared memory
    const int64_t max_groups = G <= 16 ? mac::AttnCaps<1>::kMaxGroups : mac::AttnCaps<2>::kMaxGroups;
    if ((int64_t)c->max_batch * c->num_kv_heads > max_groups) return MAC_ATTN_ERR_UNSUPPORTED;
    L->G = G;
    L->chunk_fixed = c->chunk_tokens;
    L->chunk_min = chunk;
    L->n_mid_slots = (c->max_kv_len + chunk - 1) / chunk;
    const int band_span = c->band < c->max_kv_len ? c->band : c->max_kv_len;
    L->n_band_slots = band_span == 0 ? 0 : (band_span + chunk - 1) / chunk + 1;
    L->n_slots = L->n_mid_slots + L->n_band_slots;
    int sh = 0;
    while ((1 << sh) < c->page_size) ++sh;
    L->page_shift = sh;
    const int64_t entries = (int64_t)c->max_slots * c->num_q_heads * c->window;
    const int64_t bh = (int64_t)c->max_batch * c->num_q_heads;
    L->ring_q_bytes = entries * mac::kHeadDim * 2;
    L->ring_O_bytes = entries * mac::kHeadDim * 4;
    L->ring_lse_bytes = entries * 4;
    L->ring_npos_bytes = entries * 4;
    L->part_O_bytes = bh * L->n_slots * mac::kHeadDim * 4;
    L->part_lse_bytes = bh * L->n_slots * 4;
    L->max_split = 64;                                      // window slices of the group matcher (power of two)
    L->slices_bytes = c->group_match ? bh * L->max_split * (int64_t)sizeof(mac::MatchPartial) : 16;
    L->match_bytes = bh * (int64_t)sizeof(mac::MatchPartial);
    L->rect_bytes = bh * (mac::kHeadDim + 1) * 4;
    // counters: hits, gap, skip, fused tokens per (b, h); read, full, split tokens per (b, g); steps, head-steps
    L->stats_bytes = bh * 4 * 8 + (int64_t)c->max_batch * c->num_kv_heads * 3 * 8 + 2 * 8;
    L->head_start_bytes = (bh + 32) * 4;                    // padded: read in blocks of 16 without a bound check
    return MAC_ATTN_OK;
}

struct TimedCall {
    hipEvent_t ev[5];
    bool ran[4];
};

}  // namespace

struct mac_attn_ctx {
    mac_attn_config cfg;
    Layout L;
    float sm_scale;
    double T2;
    // rings
    uint16_t* ring_q = nullptr;
    float* ring_O = nullptr;
    float* ring_lse = nullptr;
    int32_t* ring_npos = nullptr;
    // per-step scratch
    float* part_O = nullptr;
    float* part_lse = nullptr;
    mac::MatchPartial* m_slices = nullptr; // [bh, n_split] nearest entry per window slice (group matcher only)
    mac::MatchPartial* m_part = nullptr;   // [bh] nearest entry of each head's window
    int32_t* plan = nullptr;               // [0] tokens per work item of the last attention launch
    int32_t n_cu = 256;                    // compute units of the device
    int32_t grid_attn = 1024;              // work-groups of the attention kernel at most: four per compute unit (two are resident)
    int32_t fused_span = 0;                // largest fresh range the per-head matcher finishes itself (0 = none)
    int32_t* head_start = nullptr;         // [max_batch*Hq + 32] fresh-range start per head (| kHeadDone), written by the matchers
    float* rect = nullptr;        // [bh*128] rows then [bh] lse
    // counters
    unsigned long long* stats = nullptr;
    hipStream_t last_stream = nullptr;
    // allocations as returned by hipMalloc (the pointers above point kGuardBytes into them) and their payload sizes
    void* raw[kNumBuffers] = {};
    int64_t payload[kNumBuffers] = {};
    // timing
    bool timing = false;
    std::vector<TimedCall> timed;
    std::vector<hipEvent_t> event_pool;
};

namespace {

int ensure_device(const mac_attn_ctx* ctx) {
    int cur = -1;
    HIP_TRY(hipGetDevice(&cur));
    if (cur != ctx->cfg.device) HIP_TRY(hipSetDevice(ctx->cfg.device));
    return MAC_ATTN_OK;
}

int validate_args(const mac_attn_ctx* ctx, const mac_attn_step_args* a, bool need_pre) {
    if (ctx == nullptr || a == nullptr) return MAC_ATTN_ERR_INVALID_ARG;
    if (a->batch < 1 || a->batch > ctx->cfg.max_batch) return MAC_ATTN_ERR_INVALID_ARG;
    if (a->kv_lens == nullptr || a->q_rope == nullptr || a->kv_pages == nullptr || a->block_table == nullptr ||
        a->out == nullptr)
        return MAC_ATTN_ERR_INVALID_ARG;
    if (need_pre && (a->q_pre == nullptr || a->slot_ids == nullptr)) return MAC_ATTN_ERR_INVALID_ARG;
    const int64_t need_pages = ((int64_t)ctx->cfg.max_kv_len + ctx->cfg.page_size - 1) / ctx->cfg.page_size;
    if (a->block_table_stride < need_pages) return MAC_ATTN_ERR_INVALID_ARG;
    const int64_t st[4] = {a->stride_page, a->stride_kv, a->stride_head, a->stride_tok};
    for (int64_t s : st)
        if (s <= 0 || (s % 8) != 0) return MAC_ATTN_ERR_INVALID_ARG;
    // the kernels form row offsets inside a 16-token sub-tile in 32 bits
    if (a->stride_tok < ctx->cfg.head_dim || a->stride_tok >= (1 << 26)) return MAC_ATTN_ERR_INVALID_ARG;
    // 16-byte vector loads: base pointers must be 16-byte aligned
    if ((reinterpret_cast<uintptr_t>(a->kv_pages) & 15u) || (reinterpret_cast<uintptr_t>(a->q_rope) & 15u)) return MAC_ATTN_ERR_INVALID_ARG;
    if (need_pre && (reinterpret_cast<uintptr_t>(a->q_pre) & 15u)) return MAC_ATTN_ERR_INVALID_ARG;
    return MAC_ATTN_OK;
}

hipEvent_t take_event(mac_attn_ctx* ctx, int* rc) {
    if (!ctx->event_pool.empty()) {
        hipEvent_t e = ctx->event_pool.back();
        ctx->event_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    hipError_t err = hipEventCreate(&e);
    if (err != hipSuccess) *rc = hip_fail(err, "hipEventCreate");
    return e;
}

struct Timer {          // brackets the kernels of one call with events when timing is on
    mac_attn_ctx* ctx;
    hipStream_t stream;
    TimedCall tc{};
    bool on;
    int rc = MAC_ATTN_OK;
    Timer(mac_attn_ctx* c, hipStream_t s) : ctx(c), stream(s), on(c->timing) {
        if (!on) return;
        for (int i = 0; i < 5 && rc == MAC_ATTN_OK; ++i) tc.ev[i] = take_event(ctx, &rc);
        for (bool& r : tc.ran) r = false;
        if (rc == MAC_ATTN_OK) mark(0);
    }
    void mark(int i) {
        if (!on || rc != MAC_ATTN_OK) return;
        hipError_t e = hipEventRecord(tc.ev[i], stream);
        if (e != hipSuccess) rc = hip_fail(e, "hipEventRecord");
    }
    void done(int kernel) {   // kernel 0..3 just launched
        if (!on) return;
        tc.ran[kernel] = true;
        mark(kernel + 1);
    }
    void skip(int kernel) {
        if (!on) return;
        mark(kernel + 1);
    }
    void finish() {
        if (on && rc == MAC_ATTN_OK) {
            ctx->timed.push_back(tc);
            kept = true;
        }
    }
    ~Timer() {               // a call that failed on the way: its events go back to the pool
        if (!on || kept) return;
        for (hipEvent_t e : tc.ev)
            if (e != nullptr) ctx->event_pool.push_back(e);
    }
    bool kept = false;
};

mac::MatchView match_view(const mac_attn_ctx* ctx, bool mac_mode) {
    mac::MatchView mv;
    mv.part = mac_mode ? ctx->m_part : nullptr;
    mv.band = ctx->cfg.band;
    mv.T2 = ctx->T2;
    mv.max_gap = ctx->cfg.max_gap;
    return mv;
}

int launch_attention(mac_attn_ctx* ctx, const mac_attn_step_args* a, bool mac_mode, hipStream_t stream) {
    const mac_attn_config& c = ctx->cfg;
    const Layout& L = ctx->L;
    mac::AttnParams p;
    p.kv_lens = a->kv_lens;
    p.head_start = mac_mode ? ctx->head_start : nullptr;
    p.q_rope = static_cast<const uint16_t*>(a->q_rope);
    p.kv_pages = static_cast<const uint16_t*>(a->kv_pages);
    p.stride_page = a->stride_page;
    p.stride_kv = a->stride_kv;
    p.stride_head = a->stride_head;
    p.stride_tok = a->stride_tok;
    p.block_table = a->block_table;
    p.bt_stride = a->block_table_stride;
    p.part_O = ctx->part_O;
    p.part_lse = ctx->part_lse;
    p.batch = a->batch;
    p.Hq = c.num_q_heads;
    p.G = L.G;
    p.page_shift = L.page_shift;
    p.band = mac_mode ? c.band : 0;
    p.chunk_fixed = L.chunk_fixed;
    p.chunk_min = L.chunk_min;
    p.n_mid_slots = L.n_mid_slots;
    p.n_slots = L.n_slots;
    p.n_cu = ctx->n_cu;
    p.max_kv_len = c.max_kv_len;
    p.scale_log2 = ctx->sm_scale * mac::kLog2e;
    p.step_chunk = ctx->plan;
    p.pending = (mac_mode && !c.group_match) ? ctx->plan + 16 : nullptr;
    const int64_t bh = (int64_t)c.max_batch * c.num_q_heads;
    const int64_t bg = (int64_t)c.max_batch * c.num_kv_heads;
    p.st_read = mac_mode ? ctx->stats + 4 * bh : nullptr;
    p.st_full = mac_mode ? ctx->stats + 4 * bh + bg : nullptr;
    p.st_split = mac_mode ? ctx->stats + 4 * bh + 2 * bg : nullptr;
    // One work-group per work item the planner can make for this batch (its rule, applied to max_kv_len tokens per
    // group: a step with less work makes fewer items, never more mid items), plus one per group for the band; the
    // kernel loops should a fixed item size make more.  A grid much larger than the item list would cost: work-groups
    // without an item still derive the plan before they leave, the last of them when everything else has finished.
    const int64_t groups = (int64_t)a->batch * c.num_kv_heads;
    int64_t max_items = groups * (mac_mode ? L.n_slots : L.n_mid_slots);
    if (L.chunk_fixed == 0) {
        const int64_t tok = groups * c.max_kv_len, U = ctx->n_cu;
        int64_t N = tok / mac::kAttnChunkPref / U * U;
        N = std::min<int64_t>(std::max<int64_t>(N, U), 4 * U);
        if (N * mac::kAttnChunkMax < tok) N = (tok + U * mac::kAttnChunkMax - 1) / (U * mac::kAttnChunkMax) * U;
        N = std::max(std::min<int64_t>(N, ctx->grid_attn), groups);        // at least one work-group per KV group
        max_items = std::min(max_items, N + (mac_mode ? groups : 0));
    } else {
        max_items = std::min<int64_t>(max_items, ctx->grid_attn);
    }
    const dim3 grid((unsigned)std::max<int64_t>(max_items, 1)), block(256);
    p.head_dim = c.head_dim;
    const bool full_dim = c.head_dim == mac::kHeadDim;
    if (L.G <= 16) {
        if (full_dim) hipLaunchKernelGGL((mac::attn_kernel<1, true>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((mac::attn_kernel<1, false>), grid, block, 0, stream, p);
    } else {
        if (full_dim) hipLaunchKernelGGL((mac::attn_kernel<2, true>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((mac::attn_kernel<2, false>), grid, block, 0, stream, p);
    }
    HIP_TRY(hipGetLastError());
    return MAC_ATTN_OK;
}

mac::MergeParams merge_params(mac_attn_ctx* ctx, const mac_attn_step_args* a, bool mac_mode, bool stage_rect) {
    const mac_attn_config& c = ctx->cfg;
    const Layout& L = ctx->L;
    const int64_t bh = (int64_t)c.max_batch * c.num_q_heads;
    mac::MergeParams p;
    p.kv_lens = a->kv_lens;
    p.slot_ids = mac_mode ? a->slot_ids : nullptr;
    p.mv = match_view(ctx, mac_mode);
    p.head_start = mac_mode ? ctx->head_start : nullptr;
    p.emit_decision = c.group_match;                     // per-head matching reports its decisions itself
    p.out_match_pos = mac_mode ? a->match_pos : nullptr;
    p.out_match_d2 = mac_mode ? a->match_d2 : nullptr;
    p.st_hits = mac_mode ? ctx->stats : nullptr;
    p.st_gap = mac_mode ? ctx->stats + bh : nullptr;
    p.st_skip = mac_mode ? reinterpret_cast<double*>(ctx->stats + 2 * bh) : nullptr;
    p.ring_O = ctx->ring_O;
    p.ring_lse = ctx->ring_lse;
    p.part_O = ctx->part_O;
    p.part_lse = ctx->part_lse;
    p.out = a->out;
    p.out_bf16 = ctx->cfg.out_dtype;
    p.out_lse = a->out_lse;
    p.rect_O = stage_rect ? ctx->rect : nullptr;
    p.rect_lse = stage_rect ? ctx->rect + bh * mac::kHeadDim : nullptr;
    p.Hq = c.num_q_heads;
    p.G = L.G;
    p.W = c.window;
    p.band = mac_mode ? c.band : 0;
    p.chunk_fixed = L.chunk_fixed;
    p.step_chunk = ctx->plan;
    p.pending = (mac_mode && !c.group_match) ? ctx->plan + 16 : nullptr;
    p.n_mid_slots = L.n_mid_slots;
    p.n_slots = L.n_slots;
    p.max_kv_len = c.max_kv_len;
    p.head_dim = c.head_dim;
    return p;
}

mac::WritebackParams writeback_params(mac_attn_ctx* ctx, const mac_attn_step_args* a) {
    const mac_attn_config& c = ctx->cfg;
    const int64_t bh = (int64_t)c.max_batch * c.num_q_heads;
    mac::WritebackParams p;
    p.kv_lens = a->kv_lens;
    p.slot_ids = a->slot_ids;
    p.q_pre = static_cast<const uint16_t*>(a->q_pre);
    p.rect_O = ctx->rect;
    p.rect_lse = ctx->rect + bh * mac::kHeadDim;
    p.ring_q = ctx->ring_q;
    p.ring_O = ctx->ring_O;
    p.ring_lse = ctx->ring_lse;
    p.ring_npos = ctx->ring_npos;
    p.head_start = ctx->head_start;
    p.Hq = c.num_q_heads;
    p.W = c.window;
    p.max_kv_len = c.max_kv_len;
    p.head_dim = c.head_dim;
    return p;
}

// with_writeback: the merge kernel also appends to the ring (one launch less), else it stages the rectified
// summary for writeback_kernel.
int launch_merge(mac_attn_ctx* ctx, const mac_attn_step_args* a, bool mac_mode, bool with_writeback, hipStream_t stream) {
    const mac::MergeParams p = merge_params(ctx, a, mac_mode, /*stage_rect=*/mac_mode && !with_writeback);
    dim3 grid(ctx->cfg.num_q_heads, a->batch), block(mac::kMergeThreads);
    if (with_writeback) {
        const mac::WritebackParams wb = writeback_params(ctx, a);
        hipLaunchKernelGGL(mac::merge_writeback_kernel, grid, block, 0, stream, p, wb);
    } else {
        hipLaunchKernelGGL(mac::merge_kernel, grid, block, 0, stream, p);
    }
    HIP_TRY(hipGetLastError());
    return MAC_ATTN_OK;
}

}  // namespace

extern "C" {

const char* mac_attn_strerror(int code) {
    switch (code) {
        case MAC_ATTN_OK: return "ok";
        case MAC_ATTN_ERR_INVALID_ARG: return "invalid argument";
        case MAC_ATTN_ERR_UNSUPPORTED: return "unsupported configuration";
        case MAC_ATTN_ERR_HIP: return "HIP runtime error";
        case MAC_ATTN_ERR_OOM: return "out of device memory";
        case MAC_ATTN_ERR_CORRUPT: return "a guard zone around a device buffer of the context was overwritten";
        case MAC_ATTN_ERR_TOO_LARGE:
            return "the call needs more split-K workspace than the static buffer of mac_attn_full_decode_static holds";
        default: return "unknown error code";
    }
}

const char* mac_attn_last_hip_error(void) { return g_last_hip_error.c_str(); }

int64_t mac_attn_ring_entry_bytes(int32_t head_dim) {
    if (head_dim < 1) return MAC_ATTN_ERR_INVALID_ARG;
    if (head_dim > mac::kHeadDim || head_dim % 32 != 0) return MAC_ATTN_ERR_UNSUPPORTED;
    return (int64_t)mac::kHeadDim * 2 + (int64_t)mac::kHeadDim * 4 + 4;      // rows are stored 128 wide whatever d is
}

int64_t mac_attn_device_bytes(const mac_attn_config* cfg) {
    Layout L;
    const int rc = validate_config(cfg, &L);
    if (rc != MAC_ATTN_OK) return rc;
    return L.total();
}

void mac_attn_destroy(mac_attn_ctx* ctx) {
    if (ctx == nullptr) return;
    int cur = -1;
    if (hipGetDevice(&cur) == hipSuccess && cur != ctx->cfg.device) (void)hipSetDevice(ctx->cfg.device);
    (void)hipDeviceSynchronize();
    for (void* b : ctx->raw)
        if (b != nullptr) (void)hipFree(b);
    for (TimedCall& t : ctx->timed)
        for (hipEvent_t e : t.ev) (void)hipEventDestroy(e);
    for (hipEvent_t e : ctx->event_pool) (void)hipEventDestroy(e);
    delete ctx;
}

int mac_attn_init(const mac_attn_config* cfg, mac_attn_ctx** out_ctx) {
    if (out_ctx == nullptr) return MAC_ATTN_ERR_INVALID_ARG;
    Layout L;
    int rc = validate_config(cfg, &L);
    if (rc != MAC_ATTN_OK) return rc;
    int ndev = 0;
    HIP_TRY(hipGetDeviceCount(&ndev));
    if (cfg->device >= ndev) return MAC_ATTN_ERR_INVALID_ARG;
    HIP_TRY(hipSetDevice(cfg->device));
    {   // set-up of mac_attn_full_decode_static on this device, so that its first call has nothing left to look up
        void* unused = nullptr;
        if ((rc = static_scratch(cfg->device, &unused)) != MAC_ATTN_OK) return rc;
    }
    mac_attn_ctx* ctx = new (std::nothrow) mac_attn_ctx();
    if (ctx == nullptr) return MAC_ATTN_ERR_OOM;
    ctx->cfg = *cfg;
    ctx->L = L;
    ctx->sm_scale = cfg->sm_scale > 0.f ? cfg->sm_scale : 1.0f / std::sqrt((float)cfg->head_dim);
    ctx->T2 = (double)cfg->threshold * (double)cfg->threshold;
    if (cfg->group_match) ctx->T2 = ctx->T2 * (double)L.G;      // concatenated group query: D^2 < G T^2
    {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, cfg->device) != hipSuccess) cus = 0;
        ctx->n_cu = cus > 0 ? cus : 256;
        ctx->grid_attn = 4 * ctx->n_cu;
    }
    ctx->fused_span = cfg->fused_hit_span == 0 ? kDefaultFusedSpan : (cfg->fused_hit_span < 0 ? 0 : cfg->fused_hit_span);
    struct { void** p; int64_t bytes; bool zero; } allocs[] = {
        {reinterpret_cast<void**>(&ctx->ring_q), L.ring_q_bytes, true},
        {reinterpret_cast<void**>(&ctx->ring_O), L.ring_O_bytes, true},
        {reinterpret_cast<void**>(&ctx->ring_lse), L.ring_lse_bytes, true},
        {reinterpret_cast<void**>(&ctx->ring_npos), L.ring_npos_bytes, true},
        {reinterpret_cast<void**>(&ctx->part_O), L.part_O_bytes, false},
        {reinterpret_cast<void**>(&ctx->part_lse), L.part_lse_bytes, false},
        {reinterpret_cast<void**>(&ctx->m_slices), L.slices_bytes, true},
        {reinterpret_cast<void**>(&ctx->m_part), L.match_bytes, true},
        {reinterpret_cast<void**>(&ctx->plan), kPlanBytes, true},
        {reinterpret_cast<void**>(&ctx->rect), L.rect_bytes, true},
        {reinterpret_cast<void**>(&ctx->stats), L.stats_bytes, true},
        {reinterpret_cast<void**>(&ctx->head_start), L.head_start_bytes, true},
    };
    static_assert(sizeof(allocs) / sizeof(allocs[0]) == kNumBuffers, "kNumBuffers");
    for (int i = 0; i < kNumBuffers; ++i) {
        auto& a = allocs[i];
        char* base = nullptr;
        hipError_t e = hipMalloc(reinterpret_cast<void**>(&base), (size_t)(a.bytes + 2 * kGuardBytes));
        if (e == hipSuccess) {
            ctx->raw[i] = base;
            ctx->payload[i] = a.bytes;
            *a.p = base + kGuardBytes;
            e = hipMemset(base, kGuardByte, (size_t)kGuardBytes);
            if (e == hipSuccess) e = hipMemset(base + kGuardBytes + a.bytes, kGuardByte, (size_t)kGuardBytes);
            if (e == hipSuccess && a.zero) e = hipMemset(*a.p, 0, (size_t)a.bytes);
        }
        if (e != hipSuccess) {
            rc = hip_fail(e, "hipMalloc/hipMemset");
            mac_attn_destroy(ctx);
            return rc;
        }
    }
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        rc = hip_fail(e, "hipDeviceSynchronize");
        mac_attn_destroy(ctx);
        return rc;
    }
    *out_ctx = ctx;
    return MAC_ATTN_OK;
}

int mac_attn_full_decode(mac_attn_ctx* ctx, const mac_attn_step_args* args, void* hip_stream) {
    int rc = validate_args(ctx, args, /*need_pre=*/false);
    if (rc != MAC_ATTN_OK) return rc;
    if ((rc = ensure_device(ctx)) != MAC_ATTN_OK) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    ctx->last_stream = stream;
    Timer t(ctx, stream);
    if (t.rc != MAC_ATTN_OK) return t.rc;
    t.skip(0);
    if ((rc = launch_attention(ctx, args, false, stream)) != MAC_ATTN_OK) return rc;
    t.done(1);
    if ((rc = launch_merge(ctx, args, false, false, stream)) != MAC_ATTN_OK) return rc;
    t.done(2);
    t.skip(3);
    t.finish();
    return t.rc;
}

int mac_attn_full_decode_static(const mac_attn_static_geometry* geo, const mac_attn_step_args* args, void* hip_stream) {
    if (geo == nullptr || args == nullptr) return MAC_ATTN_ERR_INVALID_ARG;
    // a context on the stack (nothing is allocated): the configuration of a full decode, and the static array as its
    // split-K workspace
    mac_attn_ctx tmp;
    mac_attn_config& c = tmp.cfg;
    std::memset(&c, 0, sizeof(c));
    c.device = geo->device;
    c.max_slots = c.max_batch = args->batch;
    c.num_q_heads = geo->num_q_heads;
    c.num_kv_heads = geo->num_kv_heads;
    c.head_dim = geo->head_dim;
    c.page_size = geo->page_size;
    c.window = 1;
    c.sm_scale = geo->sm_scale;
    c.max_kv_len = geo->max_kv_len;
    c.chunk_tokens = geo->chunk_tokens;
    c.out_dtype = geo->out_dtype;
    if (c.chunk_tokens == 0 && c.num_kv_heads > 0 && c.num_q_heads > 0)      // fixed tokens per work item (see the header)
        c.chunk_tokens = default_chunk((int64_t)args->batch * c.num_kv_heads, c.max_kv_len, c.num_q_heads / c.num_kv_heads);
    int rc = validate_config(&c, &tmp.L);
    if (rc != MAC_ATTN_OK) return rc;
    if ((rc = validate_args(&tmp, args, /*need_pre=*/false)) != MAC_ATTN_OK) return rc;
    const Layout& L = tmp.L;
    const int64_t bh = (int64_t)args->batch * c.num_q_heads;
    // band = 0, so the layout has no band work items: a head's partials are n_mid_slots rows apart
    const int64_t part_O_bytes = bh * L.n_mid_slots * mac::kHeadDim * 4, part_lse_bytes = bh * L.n_mid_slots * 4;
    if (kPlanBytes + part_O_bytes + part_lse_bytes > (int64_t)MAC_ATTN_STATIC_SCRATCH_BYTES) return MAC_ATTN_ERR_TOO_LARGE;
    int ndev = 0;
    HIP_TRY(hipGetDeviceCount(&ndev));
    if (c.device >= ndev) return MAC_ATTN_ERR_INVALID_ARG;
    if ((rc = ensure_device(&tmp)) != MAC_ATTN_OK) return rc;
    void* base = nullptr;
    if ((rc = static_scratch(c.device, &base)) != MAC_ATTN_OK) return rc;
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c.device) != hipSuccess) cus = 0;
    tmp.n_cu = cus > 0 ? cus : 256;
    tmp.grid_attn = 4 * tmp.n_cu;
    tmp.sm_scale = c.sm_scale > 0.f ? c.sm_scale : 1.0f / std::sqrt((float)c.head_dim);
    tmp.T2 = 0.0;
    // Layout of the array: a word for the attention kernel's plan first (unused with fixed work items), then the
    // partials.  Every partial the merge reads is written by this call's attention kernel first: nothing is cleared.
    tmp.plan = static_cast<int32_t*>(base);
    tmp.part_O = reinterpret_cast<float*>(static_cast<char*>(base) + kPlanBytes);
    tmp.part_lse = reinterpret_cast<float*>(static_cast<char*>(base) + kPlanBytes + part_O_bytes);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if ((rc = launch_attention(&tmp, args, false, stream)) != MAC_ATTN_OK) return rc;
    return launch_merge(&tmp, args, false, false, stream);
}

int mac_attn_decode_step(mac_attn_ctx* ctx, const mac_attn_step_args* args, void* hip_stream) {
    int rc = validate_args(ctx, args, /*need_pre=*/true);
    if (rc != MAC_ATTN_OK) return rc;
    if ((rc = ensure_device(ctx)) != MAC_ATTN_OK) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    ctx->last_stream = stream;
    const mac_attn_config& c = ctx->cfg;
    const int64_t bh = (int64_t)c.max_batch * c.num_q_heads;
    Timer t(ctx, stream);
    if (t.rc != MAC_ATTN_OK) return t.rc;

    // 1. match; per head it also finishes the heads that hit with a short fresh range
    const int64_t bg = (int64_t)c.max_batch * c.num_kv_heads;
    unsigned long long* st_steps = ctx->stats + 4 * bh + 3 * bg;
    if (!c.group_match) {
        mac::HitParams p;
        p.slot_ids = args->slot_ids;
        p.kv_lens = args->kv_lens;
        p.q_pre = static_cast<const uint16_t*>(args->q_pre);
        p.ring_q = ctx->ring_q;
        p.ring_O = ctx->ring_O;
        p.ring_lse = ctx->ring_lse;
        p.ring_npos = ctx->ring_npos;
        p.part = ctx->m_part;
        p.head_start = ctx->head_start;
        p.pending = ctx->plan + 16;
        p.st_steps = st_steps;
        p.st_hits = ctx->stats;
        p.st_gap = ctx->stats + bh;
        p.st_skip = reinterpret_cast<double*>(ctx->stats + 2 * bh);
        p.st_fused = ctx->stats + 3 * bh;
        p.out_match_pos = args->match_pos;
        p.out_match_d2 = args->match_d2;
        p.mv = match_view(ctx, true);
        p.batch = args->batch;
        p.Hq = c.num_q_heads;
        p.G = ctx->L.G;
        p.W = c.window;
        p.max_kv_len = c.max_kv_len;
        p.head_dim = c.head_dim;
        p.fused_span = ctx->fused_span;
        p.q_rope = static_cast<const uint16_t*>(args->q_rope);
        p.kv_pages = static_cast<const uint16_t*>(args->kv_pages);
        p.stride_page = args->stride_page;
        p.stride_kv = args->stride_kv;
        p.stride_head = args->stride_head;
        p.stride_tok = args->stride_tok;
        p.block_table = args->block_table;
        p.bt_stride = args->block_table_stride;
        p.page_shift = ctx->L.page_shift;
        p.scale_log2 = ctx->sm_scale * mac::kLog2e;
        p.out = args->out;
        p.out_bf16 = c.out_dtype;
        p.out_lse = args->out_lse;
        // one work-group per head; the heads of a KV group are 8 ids apart (same XCD), groups padded to a multiple of 8
        const int groups = args->batch * c.num_kv_heads;
        const int grid = ((groups + 7) / 8) * 8 * ctx->L.G;
        // few heads and a window of several 64-row passes: 1024-thread work-groups scan it in fewer round trips
        const int64_t heads = (int64_t)args->batch * c.num_q_heads;
        if (heads <= 128 && c.window > 256)
            hipLaunchKernelGGL((mac::hit_kernel<1024, false>), dim3(grid), dim3(1024), 0, stream, p);
        else if (heads > 4 * (int64_t)ctx->n_cu)      // more heads than four work-groups per compute unit: the lean variant fits five
            hipLaunchKernelGGL((mac::hit_kernel<256, true>), dim3(grid), dim3(256), 0, stream, p);
        else
            hipLaunchKernelGGL((mac::hit_kernel<256, false>), dim3(grid), dim3(256), 0, stream, p);
        HIP_TRY(hipGetLastError());
        t.done(0);
    } else {
        mac::MatchParams p;
        p.slot_ids = args->slot_ids;
        p.kv_lens = args->kv_lens;
        p.q_pre = static_cast<const uint16_t*>(args->q_pre);
        p.ring_q = ctx->ring_q;
        p.ring_npos = ctx->ring_npos;
        p.slices = ctx->m_slices;
        p.part = ctx->m_part;
        p.head_start = ctx->head_start;
        p.st_steps = st_steps;
        p.batch = args->batch;
        p.Hq = c.num_q_heads;
        p.W = c.window;
        p.max_kv_len = c.max_kv_len;
        p.head_dim = c.head_dim;
        p.G = ctx->L.G;
        // window slices: a power of two, enough work-groups to fill the chip at small batch; a slice holds at most
        // kMatchGroupItems (row, head) pairs and at least 16 rows
        int split = 1;
        const int64_t groups = (int64_t)args->batch * c.num_kv_heads;
        auto rows_of = [&](int sp) { return (((c.window + sp - 1) / sp + 15) / 16) * 16; };
        while (split * 2 <= 64 && (rows_of(split) * p.G > mac::kMatchGroupItems ||
                                   (split * groups < 512 && (c.window + split * 2 - 1) / (split * 2) >= 16)))
            split *= 2;
        p.rows_per_split = rows_of(split);
        p.n_split = split;
        p.mv = match_view(ctx, true);
        dim3 grid(c.num_kv_heads, args->batch, split), block(mac::kMatchThreads);
        hipLaunchKernelGGL(mac::match_group_kernel, grid, block, 0, stream, p);
        HIP_TRY(hipGetLastError());
        // final reducer: nearest entry of the whole window and the fresh-range start of every head
        const int heads = args->batch * c.num_q_heads;
        hipLaunchKernelGGL(mac::match_group_finalize_kernel, dim3((heads + 3) / 4), dim3(256), 0, stream, p);
        HIP_TRY(hipGetLastError());
        t.done(0);
    }
    // 2. band + tail (or full) attention, split-K partials
    if ((rc = launch_attention(ctx, args, true, stream)) != MAC_ATTN_OK) return rc;
    t.done(1);
    if (c.fuse_epilogue) {
        // 3 + 4. complete and rectify-append in one kernel
        if ((rc = launch_merge(ctx, args, true, true, stream)) != MAC_ATTN_OK) return rc;
        t.done(2);
        t.skip(3);
    } else {
        // 3. complete: log-domain merge with the reused prefix
        if ((rc = launch_merge(ctx, args, true, false, stream)) != MAC_ATTN_OK) return rc;
        t.done(2);
        // 4. rectify-append
        const mac::WritebackParams p = writeback_params(ctx, args);
        dim3 grid(c.num_q_heads, args->batch), block(128);
        hipLaunchKernelGGL(mac::writeback_kernel, grid, block, 0, stream, p);
        HIP_TRY(hipGetLastError());
        t.done(3);
    }
    t.finish();
    return t.rc;
}

int mac_attn_check_guards(mac_attn_ctx* ctx) {
    if (ctx == nullptr) return MAC_ATTN_ERR_INVALID_ARG;
    int rc = ensure_device(ctx);
    if (rc != MAC_ATTN_OK) return rc;
    HIP_TRY(hipDeviceSynchronize());
    unsigned char host[2 * kGuardBytes];
    for (int i = 0; i < kNumBuffers; ++i) {
        const char* base = static_cast<const char*>(ctx->raw[i]);
        HIP_TRY(hipMemcpy(host, base, (size_t)kGuardBytes, hipMemcpyDeviceToHost));
        HIP_TRY(hipMemcpy(host + kGuardBytes, base + kGuardBytes + ctx->payload[i], (size_t)kGuardBytes, hipMemcpyDeviceToHost));
        for (unsigned char v : host)
            if (v != kGuardByte) return MAC_ATTN_ERR_CORRUPT;
    }
    return MAC_ATTN_OK;
}

int mac_attn_stats(mac_attn_ctx* ctx, mac_attn_stats_t* out, int reset) {
    if (ctx == nullptr || out == nullptr) return MAC_ATTN_ERR_INVALID_ARG;
    int rc = ensure_device(ctx);
    if (rc != MAC_ATTN_OK) return rc;
    HIP_TRY(hipDeviceSynchronize());          // steps may have been replayed from a graph on any stream
    const mac_attn_config& c = ctx->cfg;
    const int64_t bh = (int64_t)c.max_batch * c.num_q_heads, bg = (int64_t)c.max_batch * c.num_kv_heads;
    std::vector<unsigned long long> host((size_t)(4 * bh + 3 * bg + 2));
    HIP_TRY(hipMemcpy(host.data(), ctx->stats, (size_t)ctx->L.stats_bytes, hipMemcpyDeviceToHost));
    mac_attn_stats_t s;
    std::memset(&s, 0, sizeof(s));
    s.steps = host[(size_t)(4 * bh + 3 * bg)];
    s.head_steps = host[(size_t)(4 * bh + 3 * bg + 1)];
    for (int64_t i = 0; i < bh; ++i) {          // fixed order: the double sum is reproducible
        s.hits += host[(size_t)i];
        s.sum_gap += host[(size_t)(bh + i)];
        double f;
        std::memcpy(&f, &host[(size_t)(2 * bh + i)], 8);
        s.sum_skip_frac += f;
        s.kv_tokens_fused += host[(size_t)(3 * bh + i)];
    }
    s.misses = s.head_steps - s.hits;
    for (int64_t i = 0; i < bg; ++i) {
        s.kv_tokens_read += host[(size_t)(4 * bh + i)];
        s.kv_tokens_full += host[(size_t)(4 * bh + bg + i)];
        s.kv_tokens_split += host[(size_t)(4 * bh + 2 * bg + i)];
    }
    *out = s;
    if (reset) {
        HIP_TRY(hipMemset(ctx->stats, 0, (size_t)ctx->L.stats_bytes));
    }
    return MAC_ATTN_OK;
}

int mac_attn_reset(mac_attn_ctx* ctx, const int32_t* slot_ids, int32_t n) {
    if (ctx == nullptr) return MAC_ATTN_ERR_INVALID_ARG;
    int rc = ensure_device(ctx);
    if (rc != MAC_ATTN_OK) return rc;
    HIP_TRY(hipDeviceSynchronize());
    const int W = ctx->cfg.window;
    if (slot_ids == nullptr || n <= 0) {
        HIP_TRY(hipMemset(ctx->ring_npos, 0, (size_t)ctx->L.ring_npos_bytes));
    } else {
        for (int i = 0; i < n; ++i)
            if (slot_ids[i] < 0 || slot_ids[i] >= ctx->cfg.max_slots) return MAC_ATTN_ERR_INVALID_ARG;
        const int64_t per_slot = (int64_t)ctx->cfg.num_q_heads * W;
        for (int i = 0; i < n; ++i) HIP_TRY(hipMemset(ctx->ring_npos + (int64_t)slot_ids[i] * per_slot, 0, (size_t)per_slot * 4));
    }
    HIP_TRY(hipDeviceSynchronize());
    return MAC_ATTN_OK;
}

int mac_attn_ring_peek(mac_attn_ctx* ctx, int32_t slot, int32_t j, int32_t h, uint16_t* q_pre, float* summary,
                       float* lse, int32_t* n_p) {
    if (ctx == nullptr) return MAC_ATTN_ERR_INVALID_ARG;
    const mac_attn_config& c = ctx->cfg;
    if (slot < 0 || slot >= c.max_slots || j < 0 || j >= c.window || h < 0 || h >= c.num_q_heads) return MAC_ATTN_ERR_INVALID_ARG;
    int rc = ensure_device(ctx);
    if (rc != MAC_ATTN_OK) return rc;
    HIP_TRY(hipDeviceSynchronize());
    const int64_t e = ((int64_t)slot * c.num_q_heads + h) * c.window + j;
    if (q_pre) HIP_TRY(hipMemcpy(q_pre, ctx->ring_q + e * mac::kHeadDim, (size_t)c.head_dim * 2, hipMemcpyDeviceToHost));
    if (summary) HIP_TRY(hipMemcpy(summary, ctx->ring_O + e * mac::kHeadDim, (size_t)c.head_dim * 4, hipMemcpyDeviceToHost));
    if (lse) HIP_TRY(hipMemcpy(lse, ctx->ring_lse + e, 4, hipMemcpyDeviceToHost));
    if (n_p) HIP_TRY(hipMemcpy(n_p, ctx->ring_npos + e, 4, hipMemcpyDeviceToHost));
    return MAC_ATTN_OK;
}

int mac_attn_set_timing(mac_attn_ctx* ctx, int enable) {
    if (ctx == nullptr) return MAC_ATTN_ERR_INVALID_ARG;
    ctx->timing = enable != 0;
    return MAC_ATTN_OK;
}

int mac_attn_kernel_us(mac_attn_ctx* ctx, double sum_us[4], int64_t* n_calls) {
    if (ctx == nullptr || sum_us == nullptr || n_calls == nullptr) return MAC_ATTN_ERR_INVALID_ARG;
    int rc = ensure_device(ctx);
    if (rc != MAC_ATTN_OK) return rc;
    for (int k = 0; k < 4; ++k) sum_us[k] = 0.0;
    *n_calls = (int64_t)ctx->timed.size();
    for (TimedCall& t : ctx->timed) {
        HIP_TRY(hipEventSynchronize(t.ev[4]));      // the call's last event, on whatever stream the call was made
        for (int k = 0; k < 4; ++k) {
            if (t.ran[k]) {
                float ms = 0.f;
                HIP_TRY(hipEventElapsedTime(&ms, t.ev[k], t.ev[k + 1]));
                sum_us[k] += 1000.0 * ms;
            }
        }
        for (hipEvent_t e : t.ev) ctx->event_pool.push_back(e);
    }
    ctx->timed.clear();
    return MAC_ATTN_OK;
}

}  // extern "C"
