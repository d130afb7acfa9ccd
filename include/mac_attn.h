/*
 * mac_attn.h -- C ABI of the MAC-Attention decode-attention operator for AMD MI355X (gfx950).
 *
 * One decode step of the operator, per (request, query head) (paper Sec. 3.5, Fig. 1, Sec. 4.2):
 *   match    : pre-RoPE squared-L2 nearest neighbour of the current query among the last W cached
 *              queries of the request, accepted iff distance < T (Eq. (accept), Sec. 3.2.3);
 *   amend    : on a hit at entry n_p, recompute attention over the band and tail [max(0, n_p - B), n)
 *              under the current post-RoPE query (Eq. (rect-recomp));
 *   complete : merge it with the cached rectified prefix summary in the log domain (Eq. (rect-merge));
 *              on a miss run full attention over [0, n) (Sec. 3.2.1: outputs identical to the baseline);
 *   append   : store the pre-RoPE query and this step's rectified summary (its total without the last B
 *              keys) into ring slot (n - 1) mod W (Fig. 1(c), Sec. 4.1, Sec. 4.2 "K3").
 *
 * Conventions
 *   - All pointers named "device" are HIP device pointers on the context's GPU; "host" pointers are
 *     ordinary host memory.  No torch types cross this boundary.
 *   - n = kv_len of a request INCLUDING the current token: the caller has already appended the current
 *     token's post-RoPE K and V to the paged cache (the attention sum runs over t <= m, Sec. 2).
 *   - bf16 tensors are passed as raw 16-bit patterns.
 *   - Every entry point returns 0 on success or a negative MAC_ATTN_ERR_* code; nothing throws or aborts.
 *   - mac_attn_decode_step / mac_attn_full_decode only enqueue work on the given stream: no host
 *     synchronisation, no device-to-host copy.  The library borrows the argument buffers until the stream
 *     has executed the enqueued work.  One context must not be used from two streams/threads at once.
 *   - Device-resident values (kv_lens, slot_ids, block_table) cannot be validated by the host; kv_len is
 *     clamped to [0, max_kv_len] on the device, slot ids and page ids must be in range.  Only the pages
 *     block_table lists for the first ceil(kv_len / page_size) logical pages of a request are read, and of the
 *     last one only the rows below kv_len: other pages and rows may hold anything (NaN included).
 */
#ifndef MAC_ATTN_H
#define MAC_ATTN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MAC_ATTN_OK               0
#define MAC_ATTN_ERR_INVALID_ARG (-1)   /* null pointer, out-of-range size, inconsistent geometry        */
#define MAC_ATTN_ERR_UNSUPPORTED (-2)   /* valid request this build cannot serve (e.g. head_dim 256) */
#define MAC_ATTN_ERR_HIP         (-3)   /* a HIP runtime call failed; see mac_attn_last_hip_error        */
#define MAC_ATTN_ERR_OOM         (-4)   /* device allocation failed                                      */
#define MAC_ATTN_ERR_CORRUPT     (-5)   /* mac_attn_check_guards found an overwritten guard zone         */
#define MAC_ATTN_ERR_TOO_LARGE   (-6)   /* mac_attn_full_decode_static: the call needs more than
                                           MAC_ATTN_STATIC_SCRATCH_BYTES of split-K workspace            */

typedef struct mac_attn_ctx mac_attn_ctx;   /* opaque: owns rings, split-K workspace and counters */

/* Geometry and hyper-parameters, fixed for the life of a context (one context per layer). */
typedef struct mac_attn_config {
    int32_t device;        /* HIP device ordinal                                                          */
    int32_t max_slots;     /* number of per-request ring sets (>= 1)                                      */
    int32_t max_batch;     /* largest batch of one call (1 .. max_slots)                                  */
    int32_t num_q_heads;   /* Hq                                                                          */
    int32_t num_kv_heads;  /* Hkv; Hq % Hkv == 0, group size G = Hq/Hkv in 1 .. 32                        */
    int32_t head_dim;      /* d: 32, 64, 96 or 128 (q, out and K/V rows have d elements; inside the library
                              rows are widened to 128, so rings and workspace do not shrink with d); other
                              values are MAC_ATTN_ERR_UNSUPPORTED                                          */
    int32_t page_size;     /* tokens per KV page: a power of two >= 16                                    */
    int32_t window;        /* W >= 1 (paper's K), at most 4096                                            */
    int32_t band;          /* B >= 0 (paper's r)                                                          */
    float   threshold;     /* T: absolute pre-RoPE L2 distance (paper: sqrt(2d)(1 - tau));
                              hit iff d^2 < (double)T * (double)T, strict                                 */
    float   sm_scale;      /* softmax scale, 1/sqrt(head_dim) in the paper; <= 0 selects that default     */
    int32_t max_kv_len;    /* upper bound of kv_len; sizes the split-K workspace and the launch grids     */
    int32_t chunk_tokens;  /* tokens per split-K work item: multiple of 32 in [32, 4096]; 0 = chosen per launch,
                              on the device, from the span the step really has (the planner of Sec. 4.2 K2 (1):
                              work in proportion to span), within [max(256, 32 G), 8192]                    */
    int32_t fuse_epilogue; /* 1: the merge kernel also appends to the ring (decode_step = 3 launches);
                              0: write-back runs as a kernel of its own (4 launches)                      */
    int32_t max_gap;       /* distance cap of the appendix on prefill ("Recommendations" (i)): the nearest
                              candidate is accepted only if also n - n_p <= max_gap; 0 = no cap           */
    int32_t group_match;   /* 0: one reuse point per query head (the paper's matching, Sec. 4);
                              1: one per KV group: candidates are ranked by the squared distance of the
                              group's concatenated pre-RoPE queries, D^2 = sum over the group's heads of
                              d^2, hit iff D^2 < G * T^2; match_pos / match_d2 of every head of the group
                              carry the group's n_p / D^2.  Removes the skew inside a group (Sec. 5.8)     */
    int32_t out_dtype;     /* type of `out`: 0 = fp32, 1 = bf16 (rounded to nearest even)                 */
    int32_t fused_hit_span;/* per-head matching only: a head that hits and whose fresh range [max(0, n_p - B), n)
                              has at most this many tokens is finished by the match kernel's own work-group
                              (attention over the range, merge with the prefix, ring append: Sec. 3.5 steps 1-3
                              in one launch).  0 = default (1024), -1 = never, at most 2048                  */
} mac_attn_config;

/* Arguments of one decode step for a batch of requests. */
typedef struct mac_attn_step_args {
    int32_t        batch;              /* host value, 1 .. max_batch                                      */
    const int32_t* slot_ids;           /* device [batch]: request -> ring set, distinct, in [0, max_slots) */
    const int32_t* kv_lens;            /* device [batch]: n, including the current token                  */
    const void*    q_pre;              /* device bf16 [batch, Hq, d]: pre-RoPE query (match + ring);
                                          ignored by mac_attn_full_decode (may be null there)             */
    const void*    q_rope;             /* device bf16 [batch, Hq, d]: post-RoPE query (attention)         */
    const void*    kv_pages;           /* device bf16, caller-owned paged cache holding post-RoPE K and V.
                                          Element (page p, kv in {0=K,1=V}, kv head g, token r, dim i) is
                                          at p*stride_page + kv*stride_kv + g*stride_head + r*stride_tok + i */
    int64_t        stride_page, stride_kv, stride_head, stride_tok;   /* in elements; multiples of 8;
                                                                          the d elements of a row are contiguous;
                                                                          d <= stride_tok < 2^26                  */
    const int32_t* block_table;        /* device [batch, block_table_stride]: physical page of logical page */
    int32_t        block_table_stride; /* >= ceil(max_kv_len / page_size)                                 */
    void*          out;                /* device fp32 (or bf16, see out_dtype) [batch, Hq, d]: output     */
    float*         out_lse;            /* optional device fp32 [batch, Hq]: natural-log LSE of the output */
    int32_t*       match_pos;          /* optional device [batch, Hq]: matched n_p, or -1 on a miss
                                          (written by mac_attn_decode_step only)                          */
    double*        match_d2;           /* optional device [batch, Hq]: nearest squared distance, +inf when
                                          the window is empty (mac_attn_decode_step only)                 */
} mac_attn_step_args;

/* Counters since init or the last reset (definitions: Sec. 5.3 "Setup and metrics", Sec. 5.8, App. B.3). */
typedef struct mac_attn_stats_t {
    uint64_t steps;            /* calls of mac_attn_decode_step                                            */
    uint64_t head_steps;       /* sum of batch * Hq over those calls                                       */
    uint64_t hits, misses;     /* per (request, head) match decisions                                      */
    uint64_t sum_gap;          /* sum over hits of n - n_p                                                 */
    uint64_t kv_tokens_read;   /* sum over (request, kv head) of n - min over the group's heads of start   */
    uint64_t kv_tokens_full;   /* sum over (request, kv head) of n: what full attention would stream       */
    double   sum_skip_frac;    /* sum over (request, head) of (n_p - B)_+ / n, misses counted as 0         */
    uint64_t kv_tokens_split;  /* what the split-K attention kernel streamed: sum over (request, kv head) of
                                  n - min start over the group's heads that the match kernel did not finish    */
    uint64_t kv_tokens_fused;  /* what the match kernel's hit path read: sum over the heads it finished of
                                  n - start (per head, mostly from cache: a group's heads read the same rows)  */
} mac_attn_stats_t;

/* Create a context: allocates the rings (empty), the split-K workspace and the counters on cfg->device.
 * Sec. 4.1 (per-request rings of capacity W).  *out_ctx is set only on success. */
int mac_attn_init(const mac_attn_config* cfg /*host*/, mac_attn_ctx** out_ctx /*host*/);

/* One MAC decode step (match -> band+tail or full attention -> merge -> ring append), Sec. 3.5 / Sec. 4.2.
 * hip_stream is a hipStream_t (null = the default stream). */
int mac_attn_decode_step(mac_attn_ctx* ctx, const mac_attn_step_args* args /*host*/, void* hip_stream);

/* Plain full decode attention over [0, n) with the same split-K kernels (the miss path, and the baseline
 * the speed-up is reported against); reads and changes no ring state.  Sec. 2, Sec. 3.2.1. */
int mac_attn_full_decode(mac_attn_ctx* ctx, const mac_attn_step_args* args /*host*/, void* hip_stream);

/* Full decode for callers that cannot allocate device memory or create a context (code under HIP graph capture,
 * serving loops and harnesses that forbid hipMalloc): the same kernels and the same result as
 * mac_attn_full_decode, but with no context -- the geometry comes in `geo`, and the split-K partials go to a
 * static device array of MAC_ATTN_STATIC_SCRATCH_BYTES that every GPU the library runs on holds until the process
 * ends.  The call allocates nothing (no hipMalloc / hipFree, no context) and only enqueues two kernels on the stream.
 *   workspace needed = 256 + batch * Hq * ceil(max_kv_len / chunk) * 516 bytes, chunk = geo->chunk_tokens, or for 0
 *   a fixed size derived from batch * Hkv * max_kv_len on the host (a power of two in [512, 2048], at least 64 G:
 *   the item size is not chosen per launch here, so that the layout of the array is known before the launch);
 *   a call that needs more returns MAC_ATTN_ERR_TOO_LARGE and enqueues nothing.
 * Arguments as for mac_attn_full_decode (args->q_pre, slot_ids, match_* are ignored).  Nothing in the array has to
 * survive between calls and nothing is cleared: every partial a call reads it has written itself.  All calls on one
 * GPU share that GPU's array, so calls that overlap in time on one GPU (two streams, two threads) race; calls on
 * one stream are ordered and safe. */
#define MAC_ATTN_STATIC_SCRATCH_BYTES (16u << 20)
typedef struct mac_attn_static_geometry {
    int32_t device;        /* HIP device ordinal (made current by the call), 0 .. 63                              */
    int32_t num_q_heads;   /* Hq                                                                                  */
    int32_t num_kv_heads;  /* Hkv; Hq % Hkv == 0, G = Hq/Hkv <= 32                                                */
    int32_t head_dim;      /* 32, 64, 96 or 128                                                                   */
    int32_t page_size;     /* tokens per KV page: a power of two >= 16                                            */
    float   sm_scale;      /* softmax scale; <= 0 selects 1/sqrt(head_dim)                                        */
    int32_t max_kv_len;    /* upper bound of kv_len: fixes the launch grid and the workspace layout               */
    int32_t chunk_tokens;  /* tokens per split-K work item: multiple of 32 in [32, 4096], or 0 for the default    */
    int32_t out_dtype;     /* 0 = fp32, 1 = bf16                                                                  */
} mac_attn_static_geometry;
int mac_attn_full_decode_static(const mac_attn_static_geometry* geo /*host*/, const mac_attn_step_args* args /*host*/,
                                void* hip_stream);

/* Wait for all work on the context's device (steps may have been replayed from a captured graph on any stream),
 * then read the counters into *out; reset != 0 clears them.  The counters are the quantities the paper reports per
 * run: acceptance (hit) rate and skipped-prefix ratio (Sec. 5.3 "Setup and metrics"), reuse gap and KV tokens read
 * when a KV group streams from the smallest start among its heads (Sec. 5.8), and the match / miss tallies App. B.3
 * recommends monitoring. */
int mac_attn_stats(mac_attn_ctx* ctx, mac_attn_stats_t* out /*host*/, int reset);

/* Empty the rings of the given ring sets (a new request takes over the slot); null/n <= 0 = all sets.
 * Sec. 4.1: the rings are per request, indexed by the request's own length, so a slot handed to a new request must
 * start with no entries (its first step misses).  Waits for all work on the context's device first. */
int mac_attn_reset(mac_attn_ctx* ctx, const int32_t* slot_ids /*host*/, int32_t n);

/* Test/diagnostic accessor: copy ring entry j (0 <= j < W) of ring set `slot`, head h, to host buffers
 * (any may be null): q_pre bf16 bits [d], summary row fp32 [d], ln-LSE, and the entry's n_p (0 = empty).
 * Waits for all work on the context's device first. */
int mac_attn_ring_peek(mac_attn_ctx* ctx, int32_t slot, int32_t j, int32_t h,
                       uint16_t* q_pre /*host*/, float* summary /*host*/, float* lse /*host*/, int32_t* n_p /*host*/);

/* Diagnostic: every device buffer of the context (rings, workspace, counters) lies between two 256-byte guard
 * zones filled with a pattern at init.  Waits for all work on the context's device, reads the zones back and
 * returns MAC_ATTN_ERR_CORRUPT if a kernel wrote into one, else 0.  (Not part of the paper's operator.) */
int mac_attn_check_guards(mac_attn_ctx* ctx);

/* Bytes of ring state per (ring set, head, entry): bf16 query + fp32 summary row + fp32 ln-LSE
 * (Sec. 5.9 "Auxiliary HBM overhead").  Rows are stored 128 elements wide whatever head_dim is (772 bytes), so a
 * head_dim below 128 pays for the padding; MAC_ATTN_ERR_UNSUPPORTED for a head_dim the library does not take.
 * Pure host arithmetic. */
int64_t mac_attn_ring_entry_bytes(int32_t head_dim);

/* Device bytes a context with this configuration allocates (rings + workspace + counters), or a negative
 * error code.  Pure host arithmetic; needs no GPU. */
int64_t mac_attn_device_bytes(const mac_attn_config* cfg /*host*/);

/* Per-kernel timing with HIP events recorded on the call's own stream.  While enabled, every
 * decode_step/full_decode call brackets each of its kernels with events.  mac_attn_kernel_us waits for
 * the stream, adds up the elapsed times of all calls recorded since the previous query into
 * sum_us[0]=match, [1]=attention, [2]=merge, [3]=write-back (microseconds), stores the number of calls in
 * *n_calls, and forgets them.  Off by default (the events add a little work to the stream). */
int mac_attn_set_timing(mac_attn_ctx* ctx, int enable);
int mac_attn_kernel_us(mac_attn_ctx* ctx, double sum_us[4] /*host*/, int64_t* n_calls /*host*/);

void mac_attn_destroy(mac_attn_ctx* ctx);

/* Static description of an error code; and the text of the last HIP error seen by this library in the
 * calling thread ("" if none). */
const char* mac_attn_strerror(int code);
const char* mac_attn_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MAC_ATTN_H */
