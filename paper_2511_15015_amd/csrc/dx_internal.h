// Internal declarations shared by the translation units of libdynaexq.so.
#pragma once

#include <hip/hip_runtime.h>

#include <array>
#include <cstdint>
#include <cstdio>
#include <deque>
#include <string>
#include <vector>

#include "dynaexq.h"

typedef uint16_t dx_bf16; // bit pattern

struct dx_block_pool {
    char *base = nullptr;
    size_t block_bytes = 0;
    int n_blocks = 0;
    std::vector<int> free_list;           // LIFO of free block indices
    std::vector<hipEvent_t> reuse_after;  // per block: compute-stream event to pass before reuse (or null)
    void *block_ptr(int i) const { return base + (size_t)i * block_bytes; }
};

struct dx_entry {
    uint8_t state = DX_STATE_EMPTY;
    int8_t pool = -1;        // -1: caller-owned memory, 0: pool_hi, 1: pool_lo
    int32_t block = -1;      // block index of the published version
    int32_t next_block = -1; // block being filled by an in-flight transition
    dx_handle h{};           // host mirror of the published handle
};

struct dx_packed_host {
    const void *p[6] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr}; // q_gate q_up q_down s_gate s_up s_down
};

struct dx_request {
    int layer, expert;
    bool promote;
};

struct dx_transition {
    int layer, expert;
    bool promote;
    hipEvent_t done;
};

// Timing events of one profiled forward call.  ev[0..3]: before gate/up, after it, after down, after
// combine; ev[7], ev[4]: two records back to back (what an event pair itself adds).  Decode batches set
// per_kernel: there ev[0]/ev[1], ev[5]/ev[2] and ev[6]/ev[3] are the start and stop stamps of the three
// kernels' own dispatches (attached to the launches), not records between them.  Prefill: records around
// the chain on the caller's stream.
struct dx_marks {
    hipEvent_t ev[8];
    bool per_kernel;
};

struct dx_ctx {
    dx_config cfg{};
    int device = 0;
    int n_cu = 0; // compute units of the device: size of the persistent grids
    hipStream_t compute = nullptr;
    hipStream_t mig = nullptr;
    // side streams and fork/join events of the prefill forward pass (independent kernel chains)
    hipStream_t aux[2] = {nullptr, nullptr};
    hipEvent_t fork = nullptr, join[2] = {nullptr, nullptr};
    std::string err;

    // handle tables: routed [L*E] then shared [L]
    dx_handle *d_table = nullptr;
    std::vector<dx_entry> entries; // L*E routed + L shared

    // hotness
    unsigned long long *d_counters = nullptr; // [L*E]
    long long *h_counters = nullptr;          // pinned [L*E]
    std::vector<uint64_t> scores;             // host S, Q16

    // routing scratch (chunks of 64 tokens)
    int n_chunks_max = 0;
    unsigned long long *d_mask = nullptr; // [n_chunks_max, E]
    int32_t *d_chunk_base = nullptr;      // [n_chunks_max, E]

    // forward scratch
    dx_bf16 *d_h = nullptr; // [max_tokens*(k+1), fmax]
    float *d_o = nullptr;   // [max_tokens*(k+1), d]
    int fmax = 0;

    // pools / budget tracker / transitions
    dx_block_pool pool_hi, pool_lo;
    char *staging = nullptr;
    uint64_t b_hi = 0, b_lo = 0, b_shared = 0;
    uint64_t reserved = 0;
    std::vector<int> hi_count; // per layer: Resident-Hi + Promoting
    int n_hi_cap = 0;          // per-layer capacity from the budget rule
    std::deque<dx_transition> inflight;
    std::deque<dx_request> update_q;                       // waiting promotions and demotions, in arrival order
    std::vector<std::array<const void *, 3>> host_master; // per routed entry: pinned bf16 gate/up/down or nulls
    int max_inflight = 0;                                  // 0: unbounded
    // quantized precision pair: pre-packed versions in pinned host memory, [0] high tier, [1] low tier
    std::vector<dx_packed_host> host_packed[2];
    std::vector<hipEvent_t> event_pool;
    dx_stats stats{};

    // optional per-kernel timing of the forward pass
    bool profiling = false;
    std::vector<hipEvent_t> timing_pool;           // free timing-enabled events
    std::vector<dx_marks> marks;                   // one per profiled forward call
};

#define DX_FAIL(ctx, code, ...)                                   \
    do {                                                          \
        char _buf[512];                                           \
        snprintf(_buf, sizeof _buf, __VA_ARGS__);                 \
        if (ctx) (ctx)->err = _buf;                               \
        return (code);                                            \
    } while (0)

#define DX_HIP(ctx, call)                                                                  \
    do {                                                                                   \
        hipError_t _e = (call);                                                            \
        if (_e != hipSuccess)                                                              \
            DX_FAIL(ctx, DX_ERR_HIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(_e), \
                    __FILE__, __LINE__);                                                   \
    } while (0)

// ---- kernel launchers (each validates nothing; callers validate) ----------
// dx_route.hip
hipError_t dxk_route(const float *logits, int T, int E, int k, int32_t *ids, float *w, int32_t *counts,
                     int32_t *offsets, int32_t *perm, unsigned long long *mask, int32_t *chunk_base,
                     unsigned long long *hotness /* window counters of the layer, or null */, hipStream_t s);
hipError_t dxk_router_gemm(const dx_bf16 *x, const dx_bf16 *w_r, const float *bias, int T, int E, int d, float *logits,
                           hipStream_t s);
hipError_t dxk_hotness_add(unsigned long long *counters, const int32_t *counts, int E, hipStream_t s);
hipError_t dxk_fill_u64(unsigned long long *p, size_t n, unsigned long long v, hipStream_t s);
hipError_t dxk_store_handle(dx_handle *slot, const dx_handle &h, hipStream_t s);
hipError_t dxk_probe_read(const void *buf, size_t bytes, int n_cu, hipStream_t s); // bytes: whole MiB are read

// dx_quantize.hip
hipError_t dxk_quantize(const dx_bf16 *w, int rows, int K, int group, uint8_t *q, dx_bf16 *sc, hipStream_t s);
hipError_t dxk_quantize2(const dx_bf16 *w, int rows, int K, int group, uint8_t *q, dx_bf16 *sc, hipStream_t s); // 2-bit

// dx_moe_decode.hip / dx_moe_prefill.hip
struct dx_fwd_args {
    const dx_handle *table;  // E routed entries of the layer
    const dx_handle *shared; // one entry or null
    const dx_bf16 *x;
    dx_bf16 *y;
    const int32_t *ids;
    const float *w;
    const int32_t *offsets;
    const int32_t *perm;
    dx_bf16 *h;  // scratch [T*k (+T), fmax]
    float *o;    // scratch [T*k (+T), d]: fp32, or bf16 in the same allocation when o_bf16
    int T, E, k, d, f, group, shared_f, fmax;
    int m_small; // experts with at most this many tokens take the streaming kernels, the others the tiled ones
    int o_bf16;  // O rows are bf16 (prefill: halves the traffic between the down kernels and the combine), else fp32
    int m_big;   // non-zero: the leading multiple of 256 rows of a bf16 expert takes the 256 x 256 tile kernel
    int big_int4; // non-zero (with m_big): so does the leading multiple of 256 rows of an int4 expert
};
// Decode batches that the gate/up kernel routes itself (dx_route_forward): what its first block reads and
// writes on top of dx_fwd_args (whose ids, w, offsets and perm point at the same arrays for the kernels
// that follow)
constexpr int DX_ROUTED_MAX_TOKENS = 64, DX_ROUTED_MAX_EXPERTS = 512, DX_ROUTED_MAX_TOPK = 16;
struct dx_route_io {
    const float *logits; // [T, E]
    int32_t *ids;        // [T, k]
    float *w;            // [T, k]
    int32_t *counts;     // [E]
    int32_t *offsets;    // [E + 1]
    int32_t *perm;       // [T * k]
    unsigned long long *hotness; // the layer's window counters, or null
};
// Side streams for the prefill pass: its kernel chains (streamed small experts; 128-row tiles; 256-row
// tiles) touch disjoint rows of H and O and run concurrently between `fork` and the joins.
struct dx_fwd_streams {
    hipStream_t aux[2];
    hipEvent_t fork, join[2];
};
hipError_t dxk_moe_forward(const dx_fwd_args &a, int n_cu, hipStream_t s, const dx_fwd_streams *side, dx_marks *marks);
// Routing and forward pass in one call.  Returns true in *routed when the gate/up kernel did the routing
// (small decode batches whose shapes fit); otherwise nothing was launched and the caller runs dxk_route
// and dxk_moe_forward.
hipError_t dxk_route_forward(const dx_fwd_args &a, const dx_route_io &r, int n_cu, hipStream_t s, dx_marks *marks,
                             bool *routed);
// dx_moe_prefill.hip: gate/up then down for the experts above a.m_small tokens.  The 256-row tile
// kernels (when a.m_big) go to s_big, the 128-row ones to s_tiled (the two may be the same stream).
hipError_t dxk_moe_forward_tiled(const dx_fwd_args &a, hipStream_t s_big, hipStream_t s_tiled,
                                 hipEvent_t *mark_after_gate_up);
