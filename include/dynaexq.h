/*
 * dynaexq.h -- C ABI of the MI355X (gfx950) hot path of DynaExq
 * (arXiv 2511.15015): the routed MoE expert forward over a per-(layer,
 * expert) table of stable handles, each expert either a resident bf16
 * version or a group-quantized int4 version, plus the control pieces around
 * it (hotness counting, budget-feasible top-n selection, the demotion
 * quantizer, publication of new versions between forward passes).
 *
 * Conventions for every call
 *   - "dev" pointers are HIP device pointers on the context's GPU, "host"
 *     pointers are ordinary host memory, "pinned" is page-locked host memory.
 *   - Tensors are caller-allocated and caller-owned; the library keeps no
 *     reference past the call, except for the targets of published handles,
 *     which must stay valid while they are published.
 *   - Device work is enqueued on the compute stream given to dx_create and is
 *     asynchronous to the host unless the call returns host data.
 *   - Errors are return codes; a failing call has no side effect.  The text of
 *     the last error of a context is available from dx_last_error.
 *   - bf16 is the 16-bit truncated-fp32 format; tensors are row-major.
 */
#ifndef DYNAEXQ_H
#define DYNAEXQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dx_ctx dx_ctx; /* opaque, owned by the library */

typedef enum {
    DX_OK = 0,
    DX_ERR_INVALID = 1, /* bad argument: null pointer, id/shape out of range, K % group != 0 ... */
    DX_ERR_BUDGET = 2,  /* the byte budget / high-precision capacity does not admit the request */
    DX_ERR_BUSY = 3,    /* the expert is in transition, or the producer of a version has not finished */
    DX_ERR_NOMEM = 4,   /* host or device allocation failed, or a pool has no free block */
    DX_ERR_HIP = 5      /* a HIP runtime call failed */
} dx_status;

/* numeric format of one stored expert version (Sec. 3.2: an expert keeps
 * several stored versions of the same operator, one per numeric format) */
typedef enum { DX_FMT_BF16 = 0, DX_FMT_INT4G = 1, DX_FMT_INT2G = 2 } dx_fmt;

/* residency state of an expert entry (Sec. 3.2, "Residency states") */
typedef enum {
    DX_STATE_EMPTY = 0,      /* no version published yet */
    DX_STATE_RESIDENT_HI = 1,
    DX_STATE_RESIDENT_LO = 2,
    DX_STATE_PROMOTING = 3,  /* hi version being materialised; handle still resolves to the old one */
    DX_STATE_DEMOTING = 4    /* lo version being materialised; handle still resolves to the old one */
} dx_state;

typedef struct {
    int32_t L;            /* MoE layers */
    int32_t E;            /* routed experts per layer */
    int32_t d;            /* hidden size (multiple of 32) */
    int32_t f;            /* expert intermediate size (multiple of 32) */
    int32_t top_k;        /* experts per token, 1..min(E,64) */
    int32_t group;        /* int4 group size along K: 32, 64 or 128; d and f are multiples of it */
    int32_t shared_f;     /* intermediate size of the always-bf16 shared expert, 0 = none */
    int32_t max_tokens;   /* largest T a call will pass; sizes the scratch buffers */
    int32_t window_steps; /* informational: forward passes per hotness window */
    uint32_t alpha_q16;   /* EMA factor alpha * 65536, 0 <= alpha_q16 < 65536 (Sec. 3.5) */
    int32_t route_updates_hotness; /* != 0: dx_route itself adds `counts` to the layer's window counters
                                      (the router trace tap of Sec. 4); do not also call dx_hotness_update */
    int32_t hi_fmt;       /* precision pair (Sec. 4): DX_FMT_BF16 = bf16 high / int4 low (default),
                             DX_FMT_INT4G = int4 high / int2 low (needs group 64 or 128).  Sets b_hi and
                             b_lo of the budget rule and which formats count as Resident-Hi. */
    uint64_t budget_bytes;    /* expert-weight budget of the whole stack, steady state */
    uint64_t transient_bytes; /* extra bytes in-flight transitions may hold on top of it */
} dx_config;

/* Device-visible expert handle (Sec. 3.2, "Expert entries and stable
 * handles").  The table entry's address is the handle's identity and never
 * changes; its contents are the "active pointer" plus quantization
 * parameters and are replaced as a whole by dx_swap_handle.
 *   bf16:  w_gate, w_up [f,d] bf16, w_down [d,f] bf16, s_* = NULL
 *   int4:  w_gate, w_up [f,d/2] u8, w_down [d,f/2] u8 (element 2i in the low
 *          nibble of byte i, two's complement), s_gate, s_up [f,d/group]
 *          bf16, s_down [d,f/group] bf16.
 *   int2:  w_gate, w_up [f,d/4] u8, w_down [d,f/4] u8 (element 4i in the two
 *          low bits of byte i, two's complement), scales as for int4.
 * All pointers 16-byte aligned. */
typedef struct {
    const void *w_gate, *w_up, *w_down;
    const void *s_gate, *s_up, *s_down;
    uint32_t fmt;     /* dx_fmt */
    uint32_t version; /* increases with every publication */
    uint64_t reserved;
} dx_handle; /* 64 bytes */

typedef struct {
    uint64_t promotions_issued, promotions_published;
    uint64_t demotions_issued, demotions_published;
    uint64_t h2d_bytes;            /* bytes copied from pinned host memory by promotions */
    uint64_t quantize_read_bytes;  /* bf16 bytes read by demotion quantize kernels */
    uint64_t quantize_write_bytes; /* int4 + scale bytes they wrote */
    uint64_t reserved_bytes;       /* budget tracker: bytes currently reserved */
    uint64_t peak_reserved_bytes;
    uint64_t deferred;             /* transitions refused by admission control */
    uint64_t in_flight;            /* transitions issued and not yet published */
    uint64_t peak_in_flight;
    uint64_t queued;               /* requests waiting in the update queue */
} dx_stats;

/* ------------------------------------------------------------------ context */
/* Creates a context on the current HIP device.  `hip_compute_stream` is a
 * hipStream_t (NULL = the null stream).  Allocates the handle tables
 * (L*E routed + L shared entries), the window counters, the routing and
 * forward scratch for max_tokens, a migration stream and two side streams
 * (all at default priority).  A context is not thread-safe: one host thread
 * at a time.  DX_ERR_INVALID for a configuration outside the supported
 * range: E <= 1024, top_k <= min(E, 64), group in {32, 64, 128} dividing d, f
 * and shared_f, d, f, shared_f multiples of 32, an expert matrix smaller than
 * 4 GiB (d * max(f, shared_f) * 2 bytes), max_tokens * (top_k + 1) < 2^31. */
dx_status dx_create(const dx_config *cfg, void *hip_compute_stream, dx_ctx **out);
void dx_destroy(dx_ctx *ctx);
const char *dx_last_error(const dx_ctx *ctx);
const char *dx_status_str(dx_status s);

/* ----------------------------------------------------------- the hot path */
/* Router top-k and token permutation (Sec. 3.1: the router's top-k expert
 * ids of a request are the indices into the handle table).  logits: dev fp32 [T,E].  Outputs, all dev:
 *   topk_ids int32 [T,k]  the k largest logits, largest first, ties to the lower index
 *   topk_w   fp32  [T,k]  softmax over those k logits
 *   counts   int32 [E]    pairs routed to each expert
 *   offsets  int32 [E+1]  exclusive prefix sum of counts
 *   perm     int32 [T*k]  pair indices p = t*k + j grouped by expert, increasing inside a segment
 * 0 <= T <= max_tokens.  Logits must be finite.  With route_updates_hotness
 * set in the configuration the call also performs dx_hotness_update(counts). */
dx_status dx_route(dx_ctx *ctx, int layer, const float *logits, int T,
                   int32_t *topk_ids, float *topk_w,
                   int32_t *counts, int32_t *offsets, int32_t *perm);

/* dx_route followed by dx_moe_forward on the same arrays, as one call: same
 * arguments, same outputs (ids, weights, counts, offsets, perm and y), same
 * hotness update.  For decode batches (T <= 64, E <= 512, top_k <= 16, shapes
 * that fit the streaming kernels' fast path) the gate/up kernel routes in its
 * own prologue (every block repeats the small routing computation of Sec. 3.1
 * and keeps it in LDS; the first block writes the arrays out), which saves the
 * routing kernel and its round trip through memory; otherwise the two calls
 * run one after the other.  table as in dx_moe_forward. */
dx_status dx_route_forward(dx_ctx *ctx, int layer, const dx_handle *handle_table,
                           const float *logits /* dev [T,E] */, const void *x_bf16 /* dev [T,d] */, int T,
                           int32_t *topk_ids, float *topk_w, int32_t *counts, int32_t *offsets, int32_t *perm,
                           void *y_bf16 /* dev [T,d] */);

/* dx_route for callers that cannot allocate device memory or create a context
 * (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): the same kernels and the same outputs as dx_route, with the
 * routing scratch (per-chunk token masks and segment bases) in a static
 * device array of DX_ROUTE_STATIC_MAX_ENTRIES entries (768 KiB per GPU, held
 * until the process ends) instead of a context's buffers.  The call allocates
 * nothing, frees nothing and needs no context; it runs on the current device,
 * on hip_stream (NULL = the null stream), and never touches hotness counters.
 * Limits: 1 <= E <= 1024, 1 <= top_k <= min(E, 64), T >= 0 and
 * ceil(T/64) * E <= DX_ROUTE_STATIC_MAX_ENTRIES (T = 8192 at E = 512, 4096 at
 * E = 1024); anything beyond returns DX_ERR_INVALID with nothing launched, and
 * dx_route_static_last_error() gives the reason (per thread).  All calls on one
 * GPU share that GPU's array: calls that may overlap on one GPU (different
 * streams without ordering between them) race; calls on one stream do not. */
#define DX_ROUTE_STATIC_MAX_ENTRIES 65536
dx_status dx_route_static(const float *logits /* dev [T,E] */, int T, int E, int top_k,
                          int32_t *topk_ids, float *topk_w,
                          int32_t *counts, int32_t *offsets, int32_t *perm, void *hip_stream);
const char *dx_route_static_last_error(void);

/* The router's linear gate in front of dx_route (Sec. 2.1: the router scores
 * every expert for every token; Sec. 3.1 consumes its top-k):
 *   logits[t,e] = sum_c x[t,c] * w_router[e,c] (+ bias[e])
 * x_bf16 dev [T,d], w_router dev bf16 [E,d] row-major, bias dev fp32 [E] or
 * NULL, logits dev fp32 [T,E].  bf16 products accumulated in fp32 on the
 * matrix cores in a fixed order.  0 <= T <= max_tokens. */
dx_status dx_router_logits(dx_ctx *ctx, const void *x_bf16, const void *w_router, const float *bias,
                           int T, float *logits);

/* Mixed-precision expert execution (Sec. 3.2: every selected expert's handle
 * is resolved to its active version and that version's quantization
 * parameters, and the kernel for that format runs).
 *   y[t] = sum_j topk_w[t,j] * W_down( silu(W_gate x[t]) * (W_up x[t]) )  of expert topk_ids[t,j]
 *          (+ the layer's shared expert, weight 1, when shared_f > 0)
 * handle_table: dev, E entries of this layer; NULL = the context's own table
 * for `layer`.  x_bf16 dev [T,d]; y_bf16 dev [T,d]; routing arrays as written
 * by dx_route for the same T.  Weights are read through the handles as they
 * are when the kernels run on the compute stream.
 * Stream order: the call is asynchronous and ordered on the compute stream.
 * Above 128 tokens it forks part of its kernels onto two side streams of the
 * context and joins them before the combine, so the work is still complete
 * in compute-stream order (and can be captured in a HIP graph with the
 * compute stream as origin).  The H and O scratch buffers belong to the
 * context: calls on one context must not overlap. */
dx_status dx_moe_forward(dx_ctx *ctx, int layer, const dx_handle *handle_table,
                         const void *x_bf16, int T,
                         const int32_t *topk_ids, const float *topk_w,
                         const int32_t *offsets, const int32_t *perm, void *y_bf16);

/* Hotness counters (Sec. 3.5, "Hotness Estimation"): c[layer,e] += counts[e].
 * counts: dev int32 [E]. */
dx_status dx_hotness_update(dx_ctx *ctx, int layer, const int32_t *counts);

/* End of an update interval (Sec. 3.5): S <- alpha*S + (1-alpha)*c for every
 * (layer, expert), then c <- 0.  S is kept on the host in units of 2^-16
 * counts: S <- floor((alpha_q16*S + (65536-alpha_q16)*c*65536) / 65536).
 * Synchronises the compute stream.  scores_out: host uint64 [L*E] or NULL. */
dx_status dx_window_end(dx_ctx *ctx, uint64_t *scores_out);

/* Budget-feasible selection (Sec. 3.5, "Budget-feasible Selection"):
 * n = the largest count with n*b_hi + (E-n)*b_lo <= budget_bytes (this
 * layer's share), H = the n experts with the largest score S, ties to the
 * lower index, written to out_ids (host, capacity E) in rank order.
 * DX_ERR_BUDGET and *out_n = 0 when even the all-int4 layer does not fit. */
dx_status dx_select_resident(dx_ctx *ctx, int layer, uint64_t budget_bytes,
                             int32_t *out_ids, int32_t *out_n);

/* The same rule as two pure host functions (no context, no device). */
uint64_t dx_expert_bytes(int d, int f, int group, int fmt);
int dx_budget_capacity(uint64_t budget_bytes, int E, uint64_t b_hi, uint64_t b_lo); /* -1: infeasible */
dx_status dx_select_topn(const uint64_t *scores, int E, int n, int32_t *out_ids);

/* Hysteresis (Sec. 3.5, "Hysteresis for Stability"), pure host functions.
 * cur: E flags (non-zero = member of the current high-precision set), n: the
 * capacity, out_ids: host int32, capacity n, the new set in rank order (score
 * descending, ties to the lower index).
 *   dx_select_hysteresis: an outsider replaces the lowest-ranked member only
 *     if its score exceeds that member's by more than margin (same units as
 *     the scores, 2^-16 counts); repeated until the best outsider no longer
 *     does.  Empty places (fewer than n members) are filled with the best
 *     outsiders, a set above n first sheds its lowest-ranked members.
 *   dx_select_rank_slack: a member keeps its place while it ranks inside the
 *     top n + slack; freed and empty places go to the best outsiders.
 * margin = 0 / slack = 0 give exactly dx_select_topn.  DX_ERR_INVALID for a
 * null pointer, n outside 0..E or a negative slack. */
dx_status dx_select_hysteresis(const uint64_t *scores, int E, const uint8_t *cur, int n, uint64_t margin,
                               int32_t *out_ids);
dx_status dx_select_rank_slack(const uint64_t *scores, int E, const uint8_t *cur, int n, int slack,
                               int32_t *out_ids);

/* dx_select_resident with hysteresis against the layer's current set (the
 * experts that are Resident-Hi or Promoting): n from the budget as above,
 * then dx_select_rank_slack if rank_slack > 0, else dx_select_hysteresis
 * with margin_q16. */
dx_status dx_select_resident_stable(dx_ctx *ctx, int layer, uint64_t budget_bytes, uint64_t margin_q16,
                                    int rank_slack, int32_t *out_ids, int32_t *out_n);

/* Candidates for residency change (Sec. 3.5): promote = H \ H_cur,
 * demote = H_cur \ H, where H_cur is the set of experts of `layer` that are
 * Resident-Hi or Promoting.  Outputs host int32, capacity E each, ascending. */
dx_status dx_plan_transitions(dx_ctx *ctx, int layer, const int32_t *target_ids, int n_target,
                              int32_t *promote, int32_t *n_promote,
                              int32_t *demote, int32_t *n_demote);

/* Demotion quantizer: one matrix bf16 [rows,K] (dev) -> packed int4 u8
 * [rows,K/2] + bf16 scales [rows,K/group] (dev).  Per group of `group`
 * consecutive elements along K: scale = bf16_rne(absmax/7) in fp32,
 * q = clamp(rint(w/scale), -8, 7) (IEEE divide, half to even), 0 when the
 * scale is 0.  The paper prepares both versions offline (Sec. 4
 * Implementation); this kernel produces the low-precision version on device.
 * hip_stream: hipStream_t to run on, NULL = the compute stream. */
dx_status dx_quantize_expert(dx_ctx *ctx, const void *w_bf16, int rows, int K, int group,
                             void *q_out, void *s_out, void *hip_stream);

/* The same for the low tier of the int4 / int2 pair (Sec. 4): packed 2-bit
 * codes u8 [rows,K/4] + bf16 scales [rows,K/group]; scale =
 * bf16_rne(absmax/1), q = clamp(rint(w/scale), -2, 1) -- the int4 rule with
 * q_max = 2^(bits-1) - 1.  group 32, 64 or 128. */
dx_status dx_quantize_expert_int2(dx_ctx *ctx, const void *w_bf16, int rows, int K, int group,
                                  void *q_out, void *s_out, void *hip_stream);

/* Publication (Sec. 3.2, "Non-blocking switching semantics"): replaces the
 * handle of (layer, expert) with *new_version (host pointer to a struct
 * holding dev pointers).  The write is ordered on the compute stream, so it
 * lands between forward passes.  producer_event: hipEvent_t recorded after
 * the work that fills the new version, or NULL when it is already complete;
 * DX_ERR_BUSY if that event has not completed.  expert == E addresses the
 * layer's shared expert. */
dx_status dx_swap_handle(dx_ctx *ctx, int layer, int expert, const dx_handle *new_version,
                         void *producer_event);

/* ------------------------------------------------------- table inspection */
const dx_handle *dx_handle_table(dx_ctx *ctx, int layer); /* dev pointer, E entries */
dx_status dx_get_handle(dx_ctx *ctx, int layer, int expert, dx_handle *out); /* host copy */
dx_status dx_get_formats(dx_ctx *ctx, uint8_t *fmt_out /* host [L*E], dx_fmt; 255 = empty */);
dx_status dx_get_states(dx_ctx *ctx, uint8_t *state_out /* host [L*E], dx_state */);
dx_status dx_get_counters(dx_ctx *ctx, int64_t *counters_out /* host [L*E] */); /* syncs the compute stream */
dx_status dx_get_stats(dx_ctx *ctx, dx_stats *out);
/* Where a weight pool of Sec. 3.3 lives: which = 0 pool_hi, 1 pool_lo; *base dev (NULL before
 * dx_pools_create), blocks of *block_bytes bytes, *n_blocks of them, block i at base + i * block_bytes.
 * For inspection and tests (e.g. filling free blocks with a poison pattern); the memory stays the
 * library's. */
dx_status dx_get_pool(dx_ctx *ctx, int which, void **base, uint64_t *block_bytes, int32_t *n_blocks);

/* Per-kernel timing of dx_moe_forward with HIP events on the compute stream
 * (measurement aid, off by default).  While enabled, every forward call
 * (dx_moe_forward, dx_route_forward) times its kernels: decode batches attach
 * events to each kernel's own dispatch (start and stop stamps of the launch),
 * larger batches record events around the concurrent kernel chains.
 * dx_get_profile synchronises the compute stream, adds the elapsed times of all
 * calls since the last read and clears them.  Keep profiling off while the
 * compute stream is being captured into a graph (timing events do not belong
 * in a captured graph). */
typedef struct {
    uint64_t calls;     /* forward calls accumulated */
    double gate_up_ms;  /* summed duration of the gate/up + SwiGLU kernel */
    double down_ms;     /* summed duration of the down-projection kernel */
    double combine_ms;  /* summed duration of the combine kernel (0 when fused away) */
    double empty_ms;    /* summed elapsed time between two events recorded back to back with nothing
                           between them: what an event pair itself adds to each figure above */
} dx_profile;
dx_status dx_set_profiling(dx_ctx *ctx, int enable);
/* Measurement aid: a streaming read of `bytes` bytes of device memory
 * (whole MiB, 16-byte aligned) on the compute stream, in the launch shape of the
 * decode kernels (one 512-thread block per compute unit, eight 16-byte loads in
 * flight per thread, whole lines per load instruction, non-temporal hint: the
 * fastest read this device was found to do).  Nothing is written.  Timed by the caller, it gives the
 * bandwidth a read-only kernel reaches on this device, next to which the
 * benchmark reports what the expert kernels achieve. */
dx_status dx_probe_read(dx_ctx *ctx, const void *buf /* dev */, uint64_t bytes);
dx_status dx_get_profile(dx_ctx *ctx, dx_profile *out);

/* ------------------------------------------- pools and transitions (Sec. 3.3, 3.4) */
/* One-time carve-out of the two weight pools: hi_blocks blocks of b_hi bytes
 * and lo_blocks blocks of b_lo bytes (each rounded up to 256), with
 * constant-time free lists, plus one bf16-sized staging block. */
dx_status dx_pools_create(dx_ctx *ctx, int hi_blocks, int lo_blocks);

/* Synchronous set-up: materialise (layer, expert) in `fmt` from bf16 master
 * matrices gate [f,d], up [f,d], down [d,f] (`src_on_device` != 0: dev
 * pointers, else host) into a pool block and publish it.  For int4 the
 * masters are quantized on device.  fmt is one of the two tiers of the
 * context's precision pair.  expert == E installs the shared expert (bf16
 * only, intermediate size shared_f). */
dx_status dx_expert_install(dx_ctx *ctx, int layer, int expert, int fmt,
                            const void *gate, const void *up, const void *down, int src_on_device);

/* Quantized precision pair (hi_fmt = DX_FMT_INT4G): where the pre-packed
 * version of (layer, expert) in `fmt` (the pair's high or low tier) lives in
 * pinned host memory: packed codes of gate, up, down and their bf16 scales, in
 * the layouts of dx_handle.  Promotions and demotions of such a context copy
 * these versions (no repacking on the way, Sec. 3.4); the pointers must stay
 * valid while the context lives. */
dx_status dx_register_host_packed(dx_ctx *ctx, int layer, int expert, int fmt,
                                  const void *q_gate, const void *q_up, const void *q_down,
                                  const void *s_gate, const void *s_up, const void *s_down);

/* Promotion (Sec. 3.4, "Update/Evict procedure"): reserve b_hi from the
 * budget tracker, take a block of pool_hi, copy the bf16 masters from pinned
 * host memory on the migration stream, record a completion event.  The
 * handle keeps resolving to the int4 version until dx_migrate_poll publishes.
 * DX_ERR_BUDGET: reservation refused (nothing started); DX_ERR_BUSY: the
 * expert is not Resident-Lo; DX_ERR_NOMEM: pool_hi has no free block.
 * With a quantized precision pair the three pointers are ignored (may be
 * NULL) and the registered packed high-tier version is copied instead. */
dx_status dx_promote_async(dx_ctx *ctx, int layer, int expert,
                           const void *pinned_gate, const void *pinned_up, const void *pinned_down);

/* Demotion: take a block of pool_lo and run the quantizer on the migration
 * stream over the resident bf16 version; the handle keeps resolving to bf16
 * until published.  DX_ERR_BUSY: the expert is not Resident-Hi.  With a
 * quantized precision pair no bf16 version is resident: the registered
 * packed low-tier version is copied from pinned host memory instead. */
dx_status dx_demote_async(dx_ctx *ctx, int layer, int expert);

/* Publish every transition whose completion event has fired, in issue order
 * (wait != 0: block until all in-flight transitions have completed).  The
 * handle is swapped on the compute stream; the old version's block returns
 * to its pool and is reused only after the compute stream has passed the
 * swap.  Call between forward passes. */
dx_status dx_migrate_poll(dx_ctx *ctx, int wait, int *n_published);

/* ---------------------------- transition queue and worker step (Sec. 3.4) */
/* "Asynchronous queues and backpressure" as a deterministic step function the
 * serving loop calls between forward passes (no thread of its own).
 *
 * dx_register_host_master: where the pre-packed bf16 master of (layer,
 *   expert) lives in pinned host memory (gate [f,d], up [f,d], down [d,f]);
 *   the pointers must stay valid while the context lives.  Queued promotions
 *   copy from there.
 * dx_transitions_limits: at most max_inflight transitions between issue and
 *   publication (0 = no bound): bounds the migration traffic that competes
 *   with the forward pass.
 * dx_transitions_enqueue: append requests to the update queue, demotions
 *   first, then promotions (ids of `layer`, host int32).  A request cancels a
 *   queued request for the same expert in the other direction; duplicates are
 *   dropped.
 * dx_transitions_pump: (1) publish every completed transition
 *   (dx_migrate_poll without waiting); (2) walk the queue in order and issue
 *   up to max_issue requests, each only if its admission check passes now: a
 *   promotion needs a free place among the layer's high-precision experts,
 *   b_hi bytes under budget + transient and a free pool_hi block; a demotion
 *   needs b_lo bytes and a free pool_lo block.  A request that does not pass
 *   stays queued (backpressure) and later requests are considered, so that
 *   when capacity is tight the demotions that free it overtake the
 *   promotions that wait for it.  Requests whose expert is already in (or on
 *   its way to) the requested precision are dropped; requests whose expert
 *   is in the opposite transition wait.  Outputs may be NULL. */
dx_status dx_register_host_master(dx_ctx *ctx, int layer, int expert,
                                  const void *pinned_gate, const void *pinned_up, const void *pinned_down);
dx_status dx_transitions_limits(dx_ctx *ctx, int max_inflight);
dx_status dx_transitions_enqueue(dx_ctx *ctx, int layer, const int32_t *promote, int n_promote,
                                 const int32_t *demote, int n_demote);
dx_status dx_transitions_pump(dx_ctx *ctx, int max_issue, int32_t *n_issued, int32_t *n_published,
                              int32_t *n_queued);

#ifdef __cplusplus
}
#endif
#endif /* DYNAEXQ_H */
