// Host side of libdynaexq.so: context, handle table (Versioned Expert
// Residency, Sec. 3.2), hotness window and selection (Sec. 3.5), weight pools
// and budget tracker (Sec. 3.3), and the transition pipeline on a migration
// stream (Sec. 3.4).  All device arithmetic lives in the kernel files.
#include "dx_internal.h"

#include <algorithm>
#include <cstring>
#include <new>

namespace {

thread_local std::string g_create_err;

bool valid_layer(const dx_ctx *c, int layer) { return layer >= 0 && layer < c->cfg.L; }

// index of an entry: routed (layer, e<E) or shared (layer, e==E)
int entry_index(const dx_ctx *c, int layer, int expert)
{
    if (expert == c->cfg.E) return c->cfg.L * c->cfg.E + layer;
    return layer * c->cfg.E + expert;
}

bool valid_expert(const dx_ctx *c, int expert, bool allow_shared)
{
    if (expert >= 0 && expert < c->cfg.E) return true;
    return allow_shared && c->cfg.shared_f > 0 && expert == c->cfg.E;
}

size_t round256(size_t b) { return (b + 255) & ~(size_t)255; }

dx_status get_event(dx_ctx *c, hipEvent_t *ev)
{
    if (!c->event_pool.empty()) {
        *ev = c->event_pool.back();
        c->event_pool.pop_back();
        return DX_OK;
    }
    DX_HIP(c, hipEventCreateWithFlags(ev, hipEventDisableTiming));
    return DX_OK;
}

// carve a handle out of a pool block; layouts: hi = [gate|up|down] bf16,
// lo = [q_gate|q_up|q_down|s_gate|s_up|s_down]
dx_handle handle_in_block(const dx_ctx *c, void *block, int fmt, int f)
{
    const size_t d = c->cfg.d, g = c->cfg.group, ff = f;
    char *p = static_cast<char *>(block);
    dx_handle h{};
    h.fmt = fmt;
    if (fmt == DX_FMT_BF16) {
        h.w_gate = p;
        h.w_up = p + ff * d * 2;
        h.w_down = p + 2 * ff * d * 2;
    } else {
        const size_t qm = ff * d / (fmt == DX_FMT_INT2G ? 4 : 2), sm = ff * d / g * 2;
        h.w_gate = p;
        h.w_up = p + qm;
        h.w_down = p + 2 * qm;
        h.s_gate = p + 3 * qm;
        h.s_up = p + 3 * qm + sm;
        h.s_down = p + 3 * qm + 2 * sm;
    }
    return h;
}

dx_status pool_take(dx_ctx *c, dx_block_pool &pool, hipStream_t user, int *block)
{
    if (pool.free_list.empty()) DX_FAIL(c, DX_ERR_NOMEM, "weight pool has no free block");
    const int b = pool.free_list.back();
    pool.free_list.pop_back();
    if (pool.reuse_after[b]) {
        // the block was released by a publication; the stream that will write it
        // must first pass the point where the compute stream stopped reading it
        hipError_t e = hipStreamWaitEvent(user, pool.reuse_after[b], 0);
        if (e != hipSuccess) {
            pool.free_list.push_back(b);
            DX_FAIL(c, DX_ERR_HIP, "hipStreamWaitEvent: %s", hipGetErrorString(e));
        }
        c->event_pool.push_back(pool.reuse_after[b]);
        pool.reuse_after[b] = nullptr;
    }
    *block = b;
    return DX_OK;
}

void pool_give(dx_block_pool &pool, int block, hipEvent_t after)
{
    pool.reuse_after[block] = after;
    pool.free_list.push_back(block);
}

void track_reserve(dx_ctx *c, uint64_t bytes)
{
    c->reserved += bytes;
    c->stats.reserved_bytes = c->reserved;
    c->stats.peak_reserved_bytes = std::max(c->stats.peak_reserved_bytes, c->reserved);
}

void track_release(dx_ctx *c, uint64_t bytes)
{
    c->reserved -= std::min(bytes, c->reserved);
    c->stats.reserved_bytes = c->reserved;
}

// write the entry's handle to the device table, ordered on the compute stream
dx_status publish(dx_ctx *c, int idx, const dx_handle &h)
{
    dx_entry &en = c->entries[idx];
    dx_handle nh = h;
    nh.version = en.h.version + 1;
    nh.reserved = 0;
    DX_HIP(c, dxk_store_handle(c->d_table + idx, nh, c->compute));
    en.h = nh;
    return DX_OK;
}

} // namespace

// ------------------------------------------------------------- pure host rule
extern "C" uint64_t dx_expert_bytes(int d, int f, int group, int fmt)
{
    if (d <= 0 || f <= 0 || group <= 0) return 0;
    const uint64_t params = 3ull * (uint64_t)d * (uint64_t)f;
    if (fmt == DX_FMT_BF16) return params * 2ull;
    if (fmt == DX_FMT_INT2G) return params / 4ull + (params / (uint64_t)group) * 2ull;
    return params / 2ull + (params / (uint64_t)group) * 2ull;
}

extern "C" int dx_budget_capacity(uint64_t budget, int E, uint64_t b_hi, uint64_t b_lo)
{
    if (E <= 0 || b_hi <= b_lo) return -1;
    const uint64_t floor_bytes = (uint64_t)E * b_lo;
    if (budget < floor_bytes) return -1;
    const uint64_t n = (budget - floor_bytes) / (b_hi - b_lo);
    return n > (uint64_t)E ? E : (int)n;
}

extern "C" dx_status dx_select_topn(const uint64_t *scores, int E, int n, int32_t *out_ids)
{
    if (!scores || E <= 0 || n < 0 || n > E || (n > 0 && !out_ids)) return DX_ERR_INVALID;
    std::vector<int32_t> order(E);
    for (int e = 0; e < E; ++e) order[e] = e;
    std::partial_sort(order.begin(), order.begin() + n, order.end(), [&](int32_t a, int32_t b) {
        return scores[a] != scores[b] ? scores[a] > scores[b] : a < b;
    });
    for (int i = 0; i < n; ++i) out_ids[i] = order[i];
    return DX_OK;
}

namespace {

// members (best first) and outsiders (best first) of the flagged set, brought to exactly n members:
// a larger set sheds its lowest-ranked members, a smaller one takes the best outsiders
void split_by_rank(const uint64_t *scores, int E, const uint8_t *cur, int n, std::vector<int32_t> &members,
                   std::vector<int32_t> &outsiders)
{
    auto above = [&](int32_t a, int32_t b) { return scores[a] != scores[b] ? scores[a] > scores[b] : a < b; };
    std::vector<int32_t> order(E);
    for (int e = 0; e < E; ++e) order[e] = e;
    std::sort(order.begin(), order.end(), above);
    members.clear();
    outsiders.clear();
    for (int32_t e : order) (cur[e] ? members : outsiders).push_back(e);
    if ((int)members.size() > n) {
        outsiders.insert(outsiders.end(), members.begin() + n, members.end());
        members.resize(n);
        std::sort(outsiders.begin(), outsiders.end(), above);
    } else if ((int)members.size() < n) {
        const size_t take = n - members.size();
        members.insert(members.end(), outsiders.begin(), outsiders.begin() + take);
        outsiders.erase(outsiders.begin(), outsiders.begin() + take);
        std::sort(members.begin(), members.end(), above);
    }
}

void emit_in_rank_order(const uint64_t *scores, std::vector<int32_t> &members, int32_t *out_ids)
{
    std::sort(members.begin(), members.end(),
              [&](int32_t a, int32_t b) { return scores[a] != scores[b] ? scores[a] > scores[b] : a < b; });
    for (size_t i = 0; i < members.size(); ++i) out_ids[i] = members[i];
}

} // namespace

extern "C" dx_status dx_select_hysteresis(const uint64_t *scores, int E, const uint8_t *cur, int n, uint64_t margin,
                                          int32_t *out_ids)
{
    if (!scores || !cur || E <= 0 || n < 0 || n > E || (n > 0 && !out_ids)) return DX_ERR_INVALID;
    std::vector<int32_t> members, outsiders;
    split_by_rank(scores, E, cur, n, members, outsiders);
    // i-th worst member against i-th best outsider: the exchanges are a prefix of these pairs
    for (size_t i = 0; i < members.size() && i < outsiders.size(); ++i) {
        int32_t &m = members[members.size() - 1 - i];
        const int32_t o = outsiders[i];
        const bool beats = margin ? (scores[o] > scores[m] && scores[o] - scores[m] > margin)
                                  : (scores[o] != scores[m] ? scores[o] > scores[m] : o < m);
        if (!beats) break;
        m = o;
    }
    emit_in_rank_order(scores, members, out_ids);
    return DX_OK;
}

extern "C" dx_status dx_select_rank_slack(const uint64_t *scores, int E, const uint8_t *cur, int n, int slack,
                                          int32_t *out_ids)
{
    if (!scores || !cur || E <= 0 || n < 0 || n > E || slack < 0 || (n > 0 && !out_ids)) return DX_ERR_INVALID;
    // members outside the top n + slack lose their flag, then the set is brought back to n
    std::vector<int32_t> order(E);
    for (int e = 0; e < E; ++e) order[e] = e;
    std::sort(order.begin(), order.end(),
              [&](int32_t a, int32_t b) { return scores[a] != scores[b] ? scores[a] > scores[b] : a < b; });
    std::vector<uint8_t> keep(E, 0);
    const long wide = std::min<long>((long)n + slack, E);
    for (long r = 0; r < wide; ++r) keep[order[r]] = cur[order[r]] != 0;
    std::vector<int32_t> members, outsiders;
    split_by_rank(scores, E, keep.data(), n, members, outsiders);
    emit_in_rank_order(scores, members, out_ids);
    return DX_OK;
}

extern "C" const char *dx_status_str(dx_status s)
{
    switch (s) {
    case DX_OK: return "DX_OK";
    case DX_ERR_INVALID: return "DX_ERR_INVALID";
    case DX_ERR_BUDGET: return "DX_ERR_BUDGET";
    case DX_ERR_BUSY: return "DX_ERR_BUSY";
    case DX_ERR_NOMEM: return "DX_ERR_NOMEM";
    case DX_ERR_HIP: return "DX_ERR_HIP";
    }
    return "DX_ERR_?";
}

// -------------------------------------------------------------------- context
extern "C" dx_status dx_create(const dx_config *cfg, void *stream, dx_ctx **out)
{
    if (!cfg || !out) return DX_ERR_INVALID;
    *out = nullptr;
    const dx_config &g = *cfg;
    const bool group_ok = g.group == 32 || g.group == 64 || g.group == 128;
    if (g.L <= 0 || g.E <= 0 || g.E > 1024 || g.d <= 0 || g.f <= 0 || g.top_k <= 0 || g.top_k > g.E ||
        g.top_k > 64 || !group_ok || g.d % g.group || g.f % g.group || g.d % 32 || g.f % 32 ||
        g.shared_f < 0 || g.shared_f % 32 || (g.shared_f && g.shared_f % g.group) || g.max_tokens <= 0 ||
        g.alpha_q16 >= 65536u || (g.hi_fmt != DX_FMT_BF16 && g.hi_fmt != DX_FMT_INT4G) ||
        (g.hi_fmt == DX_FMT_INT4G && g.group < 64) || (uint64_t)g.max_tokens * (uint64_t)(g.top_k + 1) > 0x7FFFFFFFull ||
        // (the kernels address inside one expert matrix with 32-bit byte offsets)
        (uint64_t)g.d * (uint64_t)(g.f > g.shared_f ? g.f : g.shared_f) * 2ull > 0xFFFFFFFFull) {
        g_create_err = "dx_create: invalid configuration";
        return DX_ERR_INVALID;
    }
    dx_ctx *c = new (std::nothrow) dx_ctx;
    if (!c) return DX_ERR_NOMEM;
    c->cfg = g;
    c->compute = static_cast<hipStream_t>(stream);
    c->b_hi = dx_expert_bytes(g.d, g.f, g.group, g.hi_fmt);
    c->b_lo = dx_expert_bytes(g.d, g.f, g.group, g.hi_fmt + 1);
    c->b_shared = g.shared_f ? dx_expert_bytes(g.d, g.shared_f, g.group, DX_FMT_BF16) : 0;
    c->fmax = std::max(g.f, g.shared_f);
    c->n_chunks_max = (g.max_tokens + 63) / 64;
    const size_t n_entries = (size_t)g.L * g.E + g.L;
    const size_t n_rows = (size_t)g.max_tokens * (g.top_k + (g.shared_f ? 1 : 0));

    auto fail = [&](hipError_t e, const char *what) {
        g_create_err = std::string("dx_create: ") + what + ": " + hipGetErrorString(e);
        dx_destroy(c);
        return e == hipErrorOutOfMemory ? DX_ERR_NOMEM : DX_ERR_HIP;
    };
    hipError_t e;
    if ((e = hipGetDevice(&c->device)) != hipSuccess) return fail(e, "hipGetDevice");
    if ((e = hipDeviceGetAttribute(&c->n_cu, hipDeviceAttributeMultiprocessorCount, c->device)) != hipSuccess)
        return fail(e, "hipDeviceGetAttribute");
    if (c->n_cu <= 0) c->n_cu = 256;
    if ((e = hipStreamCreateWithFlags(&c->mig, hipStreamNonBlocking)) != hipSuccess) return fail(e, "migration stream");
    for (int i = 0; i < 2; ++i) {
        if ((e = hipStreamCreateWithFlags(&c->aux[i], hipStreamNonBlocking)) != hipSuccess) return fail(e, "side stream");
        if ((e = hipEventCreateWithFlags(&c->join[i], hipEventDisableTiming)) != hipSuccess) return fail(e, "join event");
    }
    if ((e = hipEventCreateWithFlags(&c->fork, hipEventDisableTiming)) != hipSuccess) return fail(e, "fork event");
    if ((e = hipMalloc(&c->d_table, n_entries * sizeof(dx_handle))) != hipSuccess) return fail(e, "handle table");
    if ((e = hipMalloc(&c->d_counters, (size_t)g.L * g.E * 8)) != hipSuccess) return fail(e, "counters");
    if ((e = hipHostMalloc(&c->h_counters, (size_t)g.L * g.E * 8, hipHostMallocDefault)) != hipSuccess)
        return fail(e, "pinned counters");
    if ((e = hipMalloc(&c->d_mask, (size_t)c->n_chunks_max * g.E * 8)) != hipSuccess) return fail(e, "route masks");
    if ((e = hipMalloc(&c->d_chunk_base, (size_t)c->n_chunks_max * g.E * 4)) != hipSuccess) return fail(e, "route bases");
    if ((e = hipMalloc(&c->d_h, n_rows * c->fmax * sizeof(dx_bf16))) != hipSuccess) return fail(e, "H scratch");
    if ((e = hipMalloc(&c->d_o, n_rows * (size_t)g.d * sizeof(float))) != hipSuccess) return fail(e, "O scratch");
    // zero the table and the counters with fill kernels on the compute stream
    if ((e = dxk_fill_u64(reinterpret_cast<unsigned long long *>(c->d_table), n_entries * sizeof(dx_handle) / 8, 0ull,
                          c->compute)) != hipSuccess)
        return fail(e, "table fill");
    if ((e = dxk_fill_u64(c->d_counters, (size_t)g.L * g.E, 0ull, c->compute)) != hipSuccess) return fail(e, "counter fill");
    if ((e = hipStreamSynchronize(c->compute)) != hipSuccess) return fail(e, "sync");
    c->entries.assign(n_entries, dx_entry{});
    c->scores.assign((size_t)g.L * g.E, 0);
    c->hi_count.assign(g.L, 0);
    // per-layer high-precision capacity from the stack budget (shared experts are fixed cost)
    if (g.budget_bytes) {
        const uint64_t fixed = (uint64_t)g.L * c->b_shared;
        const uint64_t per_layer = g.budget_bytes > fixed ? (g.budget_bytes - fixed) / (uint64_t)g.L : 0;
        const int n = dx_budget_capacity(per_layer, g.E, c->b_hi, c->b_lo);
        c->n_hi_cap = n < 0 ? 0 : n;
    } else {
        c->n_hi_cap = g.E;
    }
    *out = c;
    return DX_OK;
}

extern "C" void dx_destroy(dx_ctx *c)
{
    if (!c) return;
    if (c->compute || true) (void)hipStreamSynchronize(c->compute);
    if (c->mig) {
        (void)hipStreamSynchronize(c->mig);
        (void)hipStreamDestroy(c->mig);
    }
    for (int i = 0; i < 2; ++i) {
        if (c->aux[i]) {
            (void)hipStreamSynchronize(c->aux[i]);
            (void)hipStreamDestroy(c->aux[i]);
        }
        if (c->join[i]) (void)hipEventDestroy(c->join[i]);
    }
    if (c->fork) (void)hipEventDestroy(c->fork);
    for (auto &t : c->inflight) (void)hipEventDestroy(t.done);
    for (auto ev : c->event_pool) (void)hipEventDestroy(ev);
    for (auto ev : c->timing_pool) (void)hipEventDestroy(ev);
    for (auto &m : c->marks)
        for (auto ev : m.ev) (void)hipEventDestroy(ev);
    for (dx_block_pool *p : {&c->pool_hi, &c->pool_lo}) {
        for (auto ev : p->reuse_after)
            if (ev) (void)hipEventDestroy(ev);
        if (p->base) (void)hipFree(p->base);
    }
    if (c->staging) (void)hipFree(c->staging);
    if (c->d_table) (void)hipFree(c->d_table);
    if (c->d_counters) (void)hipFree(c->d_counters);
    if (c->h_counters) (void)hipHostFree(c->h_counters);
    if (c->d_mask) (void)hipFree(c->d_mask);
    if (c->d_chunk_base) (void)hipFree(c->d_chunk_base);
    if (c->d_h) (void)hipFree(c->d_h);
    if (c->d_o) (void)hipFree(c->d_o);
    delete c;
}

extern "C" const char *dx_last_error(const dx_ctx *c) { return c ? c->err.c_str() : g_create_err.c_str(); }

// ------------------------------------------------------------------- hot path
extern "C" dx_status dx_route(dx_ctx *c, int layer, const float *logits, int T, int32_t *ids, float *w,
                              int32_t *counts, int32_t *offsets, int32_t *perm)
{
    if (!c) return DX_ERR_INVALID;
    if (!valid_layer(c, layer)) DX_FAIL(c, DX_ERR_INVALID, "dx_route: layer %d out of range", layer);
    if (T < 0 || T > c->cfg.max_tokens) DX_FAIL(c, DX_ERR_INVALID, "dx_route: T=%d outside [0,%d]", T, c->cfg.max_tokens);
    if (!counts || !offsets || (T > 0 && (!logits || !ids || !w || !perm)))
        DX_FAIL(c, DX_ERR_INVALID, "dx_route: null pointer");
    unsigned long long *hot = c->cfg.route_updates_hotness ? c->d_counters + (size_t)layer * c->cfg.E : nullptr;
    DX_HIP(c, dxk_route(logits, T, c->cfg.E, c->cfg.top_k, ids, w, counts, offsets, perm, c->d_mask, c->d_chunk_base,
                        hot, c->compute));
    return DX_OK;
}

namespace {

// validation and kernel arguments shared by dx_moe_forward and dx_route_forward (T > 0)
dx_status forward_args(dx_ctx *c, const char *who, int layer, const dx_handle *table, const void *x, int T,
                       const int32_t *ids, const float *w, const int32_t *offsets, const int32_t *perm, void *y,
                       dx_fwd_args &a)
{
    if (!x || !y || !ids || !w || !offsets || !perm) DX_FAIL(c, DX_ERR_INVALID, "%s: null pointer", who);
    const dx_config &g = c->cfg;
    if (!table) {
        // the context's own table: every expert of the layer must have a published version
        for (int e = 0; e < g.E; ++e)
            if (c->entries[entry_index(c, layer, e)].state == DX_STATE_EMPTY)
                DX_FAIL(c, DX_ERR_INVALID, "%s: expert (%d,%d) has no published version", who, layer, e);
        table = c->d_table + (size_t)layer * g.E;
    }
    a = dx_fwd_args{};
    a.table = table;
    a.shared = nullptr;
    if (g.shared_f) {
        if (c->entries[entry_index(c, layer, g.E)].state == DX_STATE_EMPTY)
            DX_FAIL(c, DX_ERR_INVALID, "%s: shared expert of layer %d not installed", who, layer);
        a.shared = c->d_table + entry_index(c, layer, g.E);
    }
    a.x = static_cast<const dx_bf16 *>(x);
    a.y = static_cast<dx_bf16 *>(y);
    a.ids = ids;
    a.w = w;
    a.offsets = offsets;
    a.perm = perm;
    a.h = c->d_h;
    a.o = c->d_o;
    a.T = T;
    a.E = g.E;
    a.k = g.top_k;
    a.d = g.d;
    a.f = g.f;
    a.group = g.group;
    a.shared_f = g.shared_f;
    a.fmax = c->fmax;
    return DX_OK;
}

// the timing events of a profiled call (from the pool, or new)
dx_status take_marks(dx_ctx *c, dx_marks &m)
{
    m.per_kernel = false;
    for (int i = 0; i < 8; ++i) {
        if (!c->timing_pool.empty()) {
            m.ev[i] = c->timing_pool.back();
            c->timing_pool.pop_back();
        } else {
            hipError_t e = hipEventCreate(&m.ev[i]);
            if (e != hipSuccess) {
                for (int j = 0; j < i; ++j) c->timing_pool.push_back(m.ev[j]);
                DX_FAIL(c, DX_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(e));
            }
        }
    }
    return DX_OK;
}

} // namespace

extern "C" dx_status dx_moe_forward(dx_ctx *c, int layer, const dx_handle *table, const void *x, int T,
                                    const int32_t *ids, const float *w, const int32_t *offsets,
                                    const int32_t *perm, void *y)
{
    if (!c) return DX_ERR_INVALID;
    if (!valid_layer(c, layer)) DX_FAIL(c, DX_ERR_INVALID, "dx_moe_forward: layer %d out of range", layer);
    if (T < 0 || T > c->cfg.max_tokens)
        DX_FAIL(c, DX_ERR_INVALID, "dx_moe_forward: T=%d outside [0,%d]", T, c->cfg.max_tokens);
    if (T == 0) return DX_OK;
    dx_fwd_args a;
    dx_status st = forward_args(c, "dx_moe_forward", layer, table, x, T, ids, w, offsets, perm, y, a);
    if (st != DX_OK) return st;
    const dx_fwd_streams side{{c->aux[0], c->aux[1]}, c->fork, {c->join[0], c->join[1]}};
    if (!c->profiling) {
        DX_HIP(c, dxk_moe_forward(a, c->n_cu, c->compute, &side, nullptr));
        return DX_OK;
    }
    dx_marks m;
    if ((st = take_marks(c, m)) != DX_OK) return st;
    hipError_t e = dxk_moe_forward(a, c->n_cu, c->compute, &side, &m);
    c->marks.push_back(m);
    if (e != hipSuccess) DX_FAIL(c, DX_ERR_HIP, "dx_moe_forward: %s", hipGetErrorString(e));
    return DX_OK;
}

extern "C" dx_status dx_route_forward(dx_ctx *c, int layer, const dx_handle *table, const float *logits, const void *x,
                                      int T, int32_t *ids, float *w, int32_t *counts, int32_t *offsets, int32_t *perm,
                                      void *y)
{
    if (!c) return DX_ERR_INVALID;
    if (!valid_layer(c, layer)) DX_FAIL(c, DX_ERR_INVALID, "dx_route_forward: layer %d out of range", layer);
    if (T < 0 || T > c->cfg.max_tokens)
        DX_FAIL(c, DX_ERR_INVALID, "dx_route_forward: T=%d outside [0,%d]", T, c->cfg.max_tokens);
    if (!counts || !offsets || (T > 0 && (!logits || !ids || !w || !perm)))
        DX_FAIL(c, DX_ERR_INVALID, "dx_route_forward: null pointer");
    bool routed = false;
    if (T > 0) {
        dx_fwd_args a;
        dx_status st = forward_args(c, "dx_route_forward", layer, table, x, T, ids, w, offsets, perm, y, a);
        if (st != DX_OK) return st;
        dx_route_io r{};
        r.logits = logits;
        r.ids = ids;
        r.w = w;
        r.counts = counts;
        r.offsets = offsets;
        r.perm = perm;
        r.hotness = c->cfg.route_updates_hotness ? c->d_counters + (size_t)layer * c->cfg.E : nullptr;
        dx_marks m;
        if (c->profiling && (st = take_marks(c, m)) != DX_OK) return st;
        hipError_t e = dxk_route_forward(a, r, c->n_cu, c->compute, c->profiling ? &m : nullptr, &routed);
        if (c->profiling) {
            if (routed) c->marks.push_back(m);
            else for (auto ev : m.ev) c->timing_pool.push_back(ev);
        }
        if (e != hipSuccess) DX_FAIL(c, DX_ERR_HIP, "dx_route_forward: %s", hipGetErrorString(e));
    }
    if (routed) return DX_OK;
    // shapes the self-routing kernel does not take: the two separate calls
    dx_status st = dx_route(c, layer, logits, T, ids, w, counts, offsets, perm);
    if (st != DX_OK) return st;
    return dx_moe_forward(c, layer, table, x, T, ids, w, offsets, perm, y);
}

extern "C" dx_status dx_router_logits(dx_ctx *c, const void *x, const void *w_router, const float *bias, int T,
                                      float *logits)
{
    if (!c) return DX_ERR_INVALID;
    if (T < 0 || T > c->cfg.max_tokens) DX_FAIL(c, DX_ERR_INVALID, "dx_router_logits: T=%d outside 0..%d", T, c->cfg.max_tokens);
    if (T == 0) return DX_OK;
    if (!x || !w_router || !logits) DX_FAIL(c, DX_ERR_INVALID, "dx_router_logits: null pointer");
    if (((uintptr_t)x & 15) || ((uintptr_t)w_router & 15) || ((uintptr_t)logits & 3) || ((uintptr_t)bias & 3))
        DX_FAIL(c, DX_ERR_INVALID, "dx_router_logits: misaligned pointer");
    DX_HIP(c, dxk_router_gemm(static_cast<const dx_bf16 *>(x), static_cast<const dx_bf16 *>(w_router), bias, T, c->cfg.E,
                              c->cfg.d, logits, c->compute));
    return DX_OK;
}

extern "C" dx_status dx_hotness_update(dx_ctx *c, int layer, const int32_t *counts)
{
    if (!c) return DX_ERR_INVALID;
    if (!valid_layer(c, layer)) DX_FAIL(c, DX_ERR_INVALID, "dx_hotness_update: layer %d out of range", layer);
    if (!counts) DX_FAIL(c, DX_ERR_INVALID, "dx_hotness_update: null counts");
    DX_HIP(c, dxk_hotness_add(c->d_counters + (size_t)layer * c->cfg.E, counts, c->cfg.E, c->compute));
    return DX_OK;
}

extern "C" dx_status dx_get_counters(dx_ctx *c, int64_t *out)
{
    if (!c || !out) return DX_ERR_INVALID;
    const size_t n = (size_t)c->cfg.L * c->cfg.E;
    DX_HIP(c, hipMemcpyAsync(c->h_counters, c->d_counters, n * 8, hipMemcpyDeviceToHost, c->compute));
    DX_HIP(c, hipStreamSynchronize(c->compute));
    std::memcpy(out, c->h_counters, n * 8);
    return DX_OK;
}

extern "C" dx_status dx_window_end(dx_ctx *c, uint64_t *scores_out)
{
    if (!c) return DX_ERR_INVALID;
    const size_t n = (size_t)c->cfg.L * c->cfg.E;
    DX_HIP(c, hipMemcpyAsync(c->h_counters, c->d_counters, n * 8, hipMemcpyDeviceToHost, c->compute));
    DX_HIP(c, dxk_fill_u64(c->d_counters, n, 0ull, c->compute));
    DX_HIP(c, hipStreamSynchronize(c->compute));
    const uint64_t a = c->cfg.alpha_q16;
    for (size_t i = 0; i < n; ++i) {
        const uint64_t cur = (uint64_t)c->h_counters[i] << 16;
        c->scores[i] = (a * c->scores[i] + (65536ull - a) * cur) >> 16;
    }
    if (scores_out) std::memcpy(scores_out, c->scores.data(), n * 8);
    return DX_OK;
}

extern "C" dx_status dx_select_resident(dx_ctx *c, int layer, uint64_t budget_bytes, int32_t *out_ids, int32_t *out_n)
{
    if (!c) return DX_ERR_INVALID;
    if (!out_n) DX_FAIL(c, DX_ERR_INVALID, "dx_select_resident: null out_n");
    *out_n = 0;
    if (!valid_layer(c, layer)) DX_FAIL(c, DX_ERR_INVALID, "dx_select_resident: layer %d out of range", layer);
    if (!out_ids) DX_FAIL(c, DX_ERR_INVALID, "dx_select_resident: null out_ids");
    const int n = dx_budget_capacity(budget_bytes, c->cfg.E, c->b_hi, c->b_lo);
    if (n < 0)
        DX_FAIL(c, DX_ERR_BUDGET, "dx_select_resident: budget %llu B is below the all-int4 layer (%llu B)",
                (unsigned long long)budget_bytes, (unsigned long long)(c->cfg.E * c->b_lo));
    dx_status s = dx_select_topn(c->scores.data() + (size_t)layer * c->cfg.E, c->cfg.E, n, out_ids);
    if (s != DX_OK) DX_FAIL(c, s, "dx_select_resident: selection failed");
    *out_n = n;
    return DX_OK;
}

extern "C" dx_status dx_select_resident_stable(dx_ctx *c, int layer, uint64_t budget_bytes, uint64_t margin_q16,
                                               int rank_slack, int32_t *out_ids, int32_t *out_n)
{
    if (!c) return DX_ERR_INVALID;
    if (!out_n) DX_FAIL(c, DX_ERR_INVALID, "dx_select_resident_stable: null out_n");
    *out_n = 0;
    if (!valid_layer(c, layer)) DX_FAIL(c, DX_ERR_INVALID, "dx_select_resident_stable: layer %d out of range", layer);
    if (!out_ids || rank_slack < 0) DX_FAIL(c, DX_ERR_INVALID, "dx_select_resident_stable: bad argument");
    const int E = c->cfg.E;
    const int n = dx_budget_capacity(budget_bytes, E, c->b_hi, c->b_lo);
    if (n < 0)
        DX_FAIL(c, DX_ERR_BUDGET, "dx_select_resident_stable: budget %llu B is below the all-int4 layer (%llu B)",
                (unsigned long long)budget_bytes, (unsigned long long)(E * c->b_lo));
    std::vector<uint8_t> cur(E);
    for (int e = 0; e < E; ++e) {
        const uint8_t st = c->entries[entry_index(c, layer, e)].state;
        cur[e] = st == DX_STATE_RESIDENT_HI || st == DX_STATE_PROMOTING;
    }
    const uint64_t *S = c->scores.data() + (size_t)layer * E;
    const dx_status s = rank_slack > 0 ? dx_select_rank_slack(S, E, cur.data(), n, rank_slack, out_ids)
                                       : dx_select_hysteresis(S, E, cur.data(), n, margin_q16, out_ids);
    if (s != DX_OK) DX_FAIL(c, s, "dx_select_resident_stable: selection failed");
    *out_n = n;
    return DX_OK;
}

extern "C" dx_status dx_plan_transitions(dx_ctx *c, int layer, const int32_t *target, int n_target, int32_t *promote,
                                         int32_t *n_promote, int32_t *demote, int32_t *n_demote)
{
    if (!c) return DX_ERR_INVALID;
    if (!valid_layer(c, layer) || n_target < 0 || n_target > c->cfg.E || (n_target && !target) || !promote ||
        !n_promote || !demote || !n_demote)
        DX_FAIL(c, DX_ERR_INVALID, "dx_plan_transitions: bad argument");
    const int E = c->cfg.E;
    std::vector<uint8_t> want(E, 0);
    for (int i = 0; i < n_target; ++i) {
        if (target[i] < 0 || target[i] >= E) DX_FAIL(c, DX_ERR_INVALID, "dx_plan_transitions: id %d out of range", target[i]);
        want[target[i]] = 1;
    }
    int np = 0, nd = 0;
    for (int e = 0; e < E; ++e) {
        const uint8_t st = c->entries[entry_index(c, layer, e)].state;
        const bool cur = st == DX_STATE_RESIDENT_HI || st == DX_STATE_PROMOTING;
        if (want[e] && !cur) promote[np++] = e;
        if (cur && !want[e]) demote[nd++] = e;
    }
    *n_promote = np;
    *n_demote = nd;
    return DX_OK;
}

extern "C" dx_status dx_quantize_expert(dx_ctx *c, const void *w, int rows, int K, int group, void *q, void *s,
                                        void *stream)
{
    if (!c) return DX_ERR_INVALID;
    if (rows < 0 || K <= 0 || (group != 32 && group != 64 && group != 128) || K % group)
        DX_FAIL(c, DX_ERR_INVALID, "dx_quantize_expert: rows=%d K=%d group=%d not supported", rows, K, group);
    if (rows == 0) return DX_OK;
    if (!w || !q || !s) DX_FAIL(c, DX_ERR_INVALID, "dx_quantize_expert: null pointer");
    if (((uintptr_t)w & 15) || ((uintptr_t)q & 3) || ((uintptr_t)s & 1))
        DX_FAIL(c, DX_ERR_INVALID, "dx_quantize_expert: misaligned pointer");
    hipStream_t st = stream ? static_cast<hipStream_t>(stream) : c->compute;
    DX_HIP(c, dxk_quantize(static_cast<const dx_bf16 *>(w), rows, K, group, static_cast<uint8_t *>(q),
                           static_cast<dx_bf16 *>(s), st));
    return DX_OK;
}

extern "C" dx_status dx_quantize_expert_int2(dx_ctx *c, const void *w, int rows, int K, int group, void *q, void *s,
                                             void *stream)
{
    if (!c) return DX_ERR_INVALID;
    if (rows < 0 || K <= 0 || (group != 32 && group != 64 && group != 128) || K % group)
        DX_FAIL(c, DX_ERR_INVALID, "dx_quantize_expert_int2: rows=%d K=%d group=%d not supported", rows, K, group);
    if (rows == 0) return DX_OK;
    if (!w || !q || !s) DX_FAIL(c, DX_ERR_INVALID, "dx_quantize_expert_int2: null pointer");
    if (((uintptr_t)w & 15) || ((uintptr_t)q & 1) || ((uintptr_t)s & 1))
        DX_FAIL(c, DX_ERR_INVALID, "dx_quantize_expert_int2: misaligned pointer");
    hipStream_t st = stream ? static_cast<hipStream_t>(stream) : c->compute;
    DX_HIP(c, dxk_quantize2(static_cast<const dx_bf16 *>(w), rows, K, group, static_cast<uint8_t *>(q),
                            static_cast<dx_bf16 *>(s), st));
    return DX_OK;
}

extern "C" dx_status dx_swap_handle(dx_ctx *c, int layer, int expert, const dx_handle *nv, void *producer_event)
{
    if (!c) return DX_ERR_INVALID;
    if (!valid_layer(c, layer) || !valid_expert(c, expert, true) || !nv)
        DX_FAIL(c, DX_ERR_INVALID, "dx_swap_handle: bad (layer, expert) = (%d, %d) or null handle", layer, expert);
    const bool quant = nv->fmt == DX_FMT_INT4G || nv->fmt == DX_FMT_INT2G;
    if (nv->fmt != DX_FMT_BF16 && !quant) DX_FAIL(c, DX_ERR_INVALID, "dx_swap_handle: unknown format %u", nv->fmt);
    if (nv->fmt == DX_FMT_INT2G && c->cfg.group < 64)
        DX_FAIL(c, DX_ERR_INVALID, "dx_swap_handle: the int2 format needs a group of 64 or 128");
    if (expert == c->cfg.E && quant) DX_FAIL(c, DX_ERR_INVALID, "dx_swap_handle: the shared expert is bf16 only");
    if (!nv->w_gate || !nv->w_up || !nv->w_down || (quant && (!nv->s_gate || !nv->s_up || !nv->s_down)))
        DX_FAIL(c, DX_ERR_INVALID, "dx_swap_handle: null weight or scale pointer");
    const uintptr_t all = (uintptr_t)nv->w_gate | (uintptr_t)nv->w_up | (uintptr_t)nv->w_down |
                          (uintptr_t)nv->s_gate | (uintptr_t)nv->s_up | (uintptr_t)nv->s_down;
    if (all & 15) DX_FAIL(c, DX_ERR_INVALID, "dx_swap_handle: pointers must be 16-byte aligned");
    const int idx = entry_index(c, layer, expert);
    dx_entry &en = c->entries[idx];
    if (en.state == DX_STATE_PROMOTING || en.state == DX_STATE_DEMOTING)
        DX_FAIL(c, DX_ERR_BUSY, "dx_swap_handle: expert (%d,%d) is in transition", layer, expert);
    if (producer_event) {
        hipError_t q = hipEventQuery(static_cast<hipEvent_t>(producer_event));
        if (q == hipErrorNotReady) DX_FAIL(c, DX_ERR_BUSY, "dx_swap_handle: the new version is not complete yet");
        if (q != hipSuccess) DX_FAIL(c, DX_ERR_HIP, "hipEventQuery: %s", hipGetErrorString(q));
    }
    if (en.pool >= 0) DX_FAIL(c, DX_ERR_BUSY, "dx_swap_handle: expert (%d,%d) is pool-managed; use the transition calls", layer, expert);
    dx_status s = publish(c, idx, *nv);
    if (s != DX_OK) return s;
    // high tier: the context's hi_fmt (or anything above it); everything below is the low tier
    const bool is_hi = expert == c->cfg.E || (int)nv->fmt <= c->cfg.hi_fmt;
    if (expert < c->cfg.E) {
        if (en.state == DX_STATE_RESIDENT_HI) c->hi_count[layer]--;
        if (is_hi) c->hi_count[layer]++;
    }
    en.state = is_hi ? DX_STATE_RESIDENT_HI : DX_STATE_RESIDENT_LO;
    return DX_OK;
}

// ------------------------------------------------------------ table inspection
extern "C" const dx_handle *dx_handle_table(dx_ctx *c, int layer)
{
    if (!c || !valid_layer(c, layer)) return nullptr;
    return c->d_table + (size_t)layer * c->cfg.E;
}

extern "C" dx_status dx_get_handle(dx_ctx *c, int layer, int expert, dx_handle *out)
{
    if (!c || !out) return DX_ERR_INVALID;
    if (!valid_layer(c, layer) || !valid_expert(c, expert, true)) DX_FAIL(c, DX_ERR_INVALID, "dx_get_handle: out of range");
    *out = c->entries[entry_index(c, layer, expert)].h;
    return DX_OK;
}

extern "C" dx_status dx_get_formats(dx_ctx *c, uint8_t *out)
{
    if (!c || !out) return DX_ERR_INVALID;
    const size_t n = (size_t)c->cfg.L * c->cfg.E;
    for (size_t i = 0; i < n; ++i) out[i] = c->entries[i].state == DX_STATE_EMPTY ? 255 : (uint8_t)c->entries[i].h.fmt;
    return DX_OK;
}

extern "C" dx_status dx_get_states(dx_ctx *c, uint8_t *out)
{
    if (!c || !out) return DX_ERR_INVALID;
    const size_t n = (size_t)c->cfg.L * c->cfg.E;
    for (size_t i = 0; i < n; ++i) out[i] = c->entries[i].state;
    return DX_OK;
}

extern "C" dx_status dx_get_stats(dx_ctx *c, dx_stats *out)
{
    if (!c || !out) return DX_ERR_INVALID;
    c->stats.in_flight = c->inflight.size();
    c->stats.queued = c->update_q.size();
    *out = c->stats;
    return DX_OK;
}

extern "C" dx_status dx_get_pool(dx_ctx *c, int which, void **base, uint64_t *block_bytes, int32_t *n_blocks)
{
    if (!c) return DX_ERR_INVALID;
    if ((which != 0 && which != 1) || !base || !block_bytes || !n_blocks)
        DX_FAIL(c, DX_ERR_INVALID, "dx_get_pool: bad argument");
    const dx_block_pool &p = which == 0 ? c->pool_hi : c->pool_lo;
    *base = p.base;
    *block_bytes = p.block_bytes;
    *n_blocks = p.n_blocks;
    return DX_OK;
}

extern "C" dx_status dx_probe_read(dx_ctx *c, const void *buf, uint64_t bytes)
{
    if (!c) return DX_ERR_INVALID;
    if (!buf || ((uintptr_t)buf & 15) || (bytes & ((1u << 20) - 1)) || bytes >> 20 > 0x7fffffffull)
        DX_FAIL(c, DX_ERR_INVALID, "dx_probe_read: a 16-byte aligned buffer of whole MiB is needed");
    DX_HIP(c, dxk_probe_read(buf, (size_t)bytes, c->n_cu, c->compute));
    return DX_OK;
}

extern "C" dx_status dx_set_profiling(dx_ctx *c, int enable)
{
    if (!c) return DX_ERR_INVALID;
    c->profiling = enable != 0;
    return DX_OK;
}

extern "C" dx_status dx_get_profile(dx_ctx *c, dx_profile *out)
{
    if (!c || !out) return DX_ERR_INVALID;
    *out = dx_profile{};
    DX_HIP(c, hipStreamSynchronize(c->compute));
    for (auto &m : c->marks) {
        // (start, stop) of gate/up, down, combine and of the empty pair
        const int from[4] = {0, m.per_kernel ? 5 : 1, m.per_kernel ? 6 : 2, 7};
        const int to[4] = {1, 2, 3, 4};
        float t[4] = {0.f, 0.f, 0.f, 0.f};
        for (int i = 0; i < 4; ++i) {
            hipError_t e = hipEventElapsedTime(&t[i], m.ev[from[i]], m.ev[to[i]]);
            if (e != hipSuccess) t[i] = 0.f; // a call that recorded nothing (T == 0)
        }
        out->calls++;
        out->gate_up_ms += t[0];
        out->down_ms += t[1];
        out->combine_ms += t[2];
        out->empty_ms += t[3];
        for (auto ev : m.ev) c->timing_pool.push_back(ev);
    }
    c->marks.clear();
    return DX_OK;
}

namespace {

// the six pieces of a pre-packed quantized version, pinned host memory -> a pool block, migration stream
hipError_t copy_packed(dx_ctx *c, const dx_handle &dst, const dx_packed_host &src, int fmt)
{
    const dx_config &g = c->cfg;
    const size_t div = fmt == DX_FMT_INT2G ? 4 : 2;
    const size_t qm = (size_t)g.f * g.d / div, sm = (size_t)g.f * g.d / g.group * 2;
    void *d[6] = {const_cast<void *>(dst.w_gate), const_cast<void *>(dst.w_up), const_cast<void *>(dst.w_down),
                  const_cast<void *>(dst.s_gate), const_cast<void *>(dst.s_up), const_cast<void *>(dst.s_down)};
    hipError_t e = hipSuccess;
    for (int i = 0; i < 6 && e == hipSuccess; ++i)
        e = hipMemcpyAsync(d[i], src.p[i], i < 3 ? qm : sm, hipMemcpyHostToDevice, c->mig);
    return e;
}

} // namespace

extern "C" dx_status dx_register_host_packed(dx_ctx *c, int layer, int expert, int fmt, const void *q_gate, const void *q_up,
                                             const void *q_down, const void *s_gate, const void *s_up, const void *s_down)
{
    if (!c) return DX_ERR_INVALID;
    if (c->cfg.hi_fmt == DX_FMT_BF16)
        DX_FAIL(c, DX_ERR_INVALID, "dx_register_host_packed: only for a context with a quantized precision pair");
    if (!valid_layer(c, layer) || !valid_expert(c, expert, false) || (fmt != c->cfg.hi_fmt && fmt != c->cfg.hi_fmt + 1) ||
        !q_gate || !q_up || !q_down || !s_gate || !s_up || !s_down)
        DX_FAIL(c, DX_ERR_INVALID, "dx_register_host_packed: bad argument");
    auto &reg = c->host_packed[fmt == c->cfg.hi_fmt ? 0 : 1];
    if (reg.empty()) reg.assign((size_t)c->cfg.L * c->cfg.E, dx_packed_host{});
    reg[(size_t)layer * c->cfg.E + expert] = dx_packed_host{{q_gate, q_up, q_down, s_gate, s_up, s_down}};
    return DX_OK;
}

// ------------------------------------------------------ pools and transitions
extern "C" dx_status dx_pools_create(dx_ctx *c, int hi_blocks, int lo_blocks)
{
    if (!c) return DX_ERR_INVALID;
    if (hi_blocks < 0 || lo_blocks < 0) DX_FAIL(c, DX_ERR_INVALID, "dx_pools_create: negative block count");
    if (c->pool_hi.base || c->pool_lo.base || c->staging) DX_FAIL(c, DX_ERR_INVALID, "dx_pools_create: pools already exist");
    const size_t hi_b = round256(std::max(c->b_hi, c->b_shared)), lo_b = round256(c->b_lo);
    // staging holds the bf16 master of one expert (routed or shared) on its way to a quantizer
    const size_t staging_b = round256(std::max<uint64_t>(
        dx_expert_bytes(c->cfg.d, std::max(c->cfg.f, c->cfg.shared_f), c->cfg.group, DX_FMT_BF16), hi_b));
    auto make = [&](dx_block_pool &p, size_t bytes, int n) -> hipError_t {
        p.block_bytes = bytes;
        p.n_blocks = n;
        p.reuse_after.assign(n, nullptr);
        p.free_list.resize(n);
        for (int i = 0; i < n; ++i) p.free_list[i] = n - 1 - i; // block 0 is handed out first
        if (n == 0) return hipSuccess;
        return hipMalloc(reinterpret_cast<void **>(&p.base), bytes * (size_t)n);
    };
    hipError_t e;
    if ((e = make(c->pool_hi, hi_b, hi_blocks)) != hipSuccess ||
        (e = make(c->pool_lo, lo_b, lo_blocks)) != hipSuccess ||
        (e = hipMalloc(reinterpret_cast<void **>(&c->staging), staging_b)) != hipSuccess) {
        for (dx_block_pool *p : {&c->pool_hi, &c->pool_lo}) {
            if (p->base) (void)hipFree(p->base);
            *p = dx_block_pool{};
        }
        if (c->staging) (void)hipFree(c->staging);
        c->staging = nullptr;
        DX_FAIL(c, e == hipErrorOutOfMemory ? DX_ERR_NOMEM : DX_ERR_HIP, "dx_pools_create: %s", hipGetErrorString(e));
    }
    return DX_OK;
}

extern "C" dx_status dx_expert_install(dx_ctx *c, int layer, int expert, int fmt, const void *gate, const void *up,
                                       const void *down, int src_on_device)
{
    if (!c) return DX_ERR_INVALID;
    if (!valid_layer(c, layer) || !valid_expert(c, expert, true) || !gate || !up || !down ||
        (fmt != DX_FMT_BF16 && fmt != DX_FMT_INT4G && fmt != DX_FMT_INT2G))
        DX_FAIL(c, DX_ERR_INVALID, "dx_expert_install: bad argument");
    const bool shared = expert == c->cfg.E;
    if (shared && fmt != DX_FMT_BF16) DX_FAIL(c, DX_ERR_INVALID, "dx_expert_install: the shared expert is bf16 only");
    if (!shared && fmt != c->cfg.hi_fmt && fmt != c->cfg.hi_fmt + 1)
        DX_FAIL(c, DX_ERR_INVALID, "dx_expert_install: format %d is not a tier of this context's precision pair", fmt);
    const bool is_hi = shared || fmt == c->cfg.hi_fmt;
    if (!c->staging) DX_FAIL(c, DX_ERR_INVALID, "dx_expert_install: call dx_pools_create first");
    const int idx = entry_index(c, layer, expert);
    dx_entry &en = c->entries[idx];
    if (en.state != DX_STATE_EMPTY) DX_FAIL(c, DX_ERR_BUSY, "dx_expert_install: expert (%d,%d) already installed", layer, expert);
    const dx_config &g = c->cfg;
    const int f = shared ? g.shared_f : g.f;
    const uint64_t bytes = shared ? c->b_shared : (is_hi ? c->b_hi : c->b_lo);
    const uint64_t cap = g.budget_bytes ? g.budget_bytes + g.transient_bytes : ~0ull;
    if (c->reserved + bytes > cap) {
        c->stats.deferred++;
        DX_FAIL(c, DX_ERR_BUDGET, "dx_expert_install: %llu B reserved + %llu B exceeds the budget", (unsigned long long)c->reserved,
                (unsigned long long)bytes);
    }
    if (!shared && is_hi && g.budget_bytes && c->hi_count[layer] >= c->n_hi_cap) {
        c->stats.deferred++;
        DX_FAIL(c, DX_ERR_BUDGET, "dx_expert_install: layer %d already holds its %d high-precision experts", layer, c->n_hi_cap);
    }
    dx_block_pool &pool = is_hi ? c->pool_hi : c->pool_lo;
    int block;
    dx_status s = pool_take(c, pool, c->compute, &block);
    if (s != DX_OK) return s;
    const size_t mat = (size_t)f * g.d * 2; // bytes of one bf16 matrix
    const hipMemcpyKind kind = src_on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
    dx_handle h = handle_in_block(c, pool.block_ptr(block), fmt, f);
    hipError_t e = hipSuccess;
    if (fmt == DX_FMT_BF16) {
        if (e == hipSuccess) e = hipMemcpyAsync(const_cast<void *>(h.w_gate), gate, mat, kind, c->compute);
        if (e == hipSuccess) e = hipMemcpyAsync(const_cast<void *>(h.w_up), up, mat, kind, c->compute);
        if (e == hipSuccess) e = hipMemcpyAsync(const_cast<void *>(h.w_down), down, mat, kind, c->compute);
    } else {
        const void *src[3] = {gate, up, down};
        void *qd[3] = {const_cast<void *>(h.w_gate), const_cast<void *>(h.w_up), const_cast<void *>(h.w_down)};
        void *sd[3] = {const_cast<void *>(h.s_gate), const_cast<void *>(h.s_up), const_cast<void *>(h.s_down)};
        const int rows[3] = {f, f, g.d}, Ks[3] = {g.d, g.d, f};
        for (int i = 0; i < 3 && e == hipSuccess; ++i) {
            const void *dev_src = src[i];
            if (!src_on_device) {
                dev_src = c->staging + (size_t)i * mat;
                e = hipMemcpyAsync(c->staging + (size_t)i * mat, src[i], mat, hipMemcpyHostToDevice, c->compute);
            }
            if (e == hipSuccess)
                e = (fmt == DX_FMT_INT2G ? dxk_quantize2 : dxk_quantize)(static_cast<const dx_bf16 *>(dev_src), rows[i], Ks[i],
                                                                       g.group, static_cast<uint8_t *>(qd[i]),
                                                                       static_cast<dx_bf16 *>(sd[i]), c->compute);
        }
    }
    if (e == hipSuccess) e = hipStreamSynchronize(c->compute);
    if (e != hipSuccess) {
        pool_give(pool, block, nullptr);
        DX_FAIL(c, DX_ERR_HIP, "dx_expert_install: %s", hipGetErrorString(e));
    }
    s = publish(c, idx, h);
    if (s != DX_OK) {
        pool_give(pool, block, nullptr);
        return s;
    }
    track_reserve(c, bytes);
    en.pool = is_hi ? 0 : 1;
    en.block = block;
    en.state = is_hi ? DX_STATE_RESIDENT_HI : DX_STATE_RESIDENT_LO;
    if (!shared && is_hi) c->hi_count[layer]++;
    return DX_OK;
}

extern "C" dx_status dx_promote_async(dx_ctx *c, int layer, int expert, const void *pg, const void *pu, const void *pd)
{
    if (!c) return DX_ERR_INVALID;
    const bool quant_pair = c->cfg.hi_fmt != DX_FMT_BF16;
    if (!valid_layer(c, layer) || !valid_expert(c, expert, false) || (!quant_pair && (!pg || !pu || !pd)))
        DX_FAIL(c, DX_ERR_INVALID, "dx_promote_async: bad argument");
    const dx_packed_host *packed = nullptr;
    if (quant_pair) { // the pre-packed high-tier version registered for this expert
        if (c->host_packed[0].empty() || !c->host_packed[0][(size_t)layer * c->cfg.E + expert].p[0])
            DX_FAIL(c, DX_ERR_INVALID, "dx_promote_async: no packed high-tier version registered for (%d,%d)", layer, expert);
        packed = &c->host_packed[0][(size_t)layer * c->cfg.E + expert];
    }
    const int idx = entry_index(c, layer, expert);
    dx_entry &en = c->entries[idx];
    if (en.state != DX_STATE_RESIDENT_LO || en.pool != 1)
        DX_FAIL(c, DX_ERR_BUSY, "dx_promote_async: expert (%d,%d) is not a pool-resident int4 expert", layer, expert);
    const dx_config &g = c->cfg;
    // admission: per-layer capacity and the byte budget (try_reserve)
    const uint64_t cap = g.budget_bytes ? g.budget_bytes + g.transient_bytes : ~0ull;
    if ((g.budget_bytes && c->hi_count[layer] >= c->n_hi_cap) || c->reserved + c->b_hi > cap) {
        c->stats.deferred++;
        DX_FAIL(c, DX_ERR_BUDGET, "dx_promote_async: no high-precision capacity for (%d,%d): %d/%d resident, %llu B reserved",
                layer, expert, c->hi_count[layer], c->n_hi_cap, (unsigned long long)c->reserved);
    }
    hipEvent_t done;
    dx_status s = get_event(c, &done);
    if (s != DX_OK) return s;
    int block;
    s = pool_take(c, c->pool_hi, c->mig, &block);
    if (s != DX_OK) {
        c->event_pool.push_back(done);
        if (s == DX_ERR_NOMEM) c->stats.deferred++;
        return s;
    }
    const size_t mat = (size_t)g.f * g.d * 2;
    dx_handle h = handle_in_block(c, c->pool_hi.block_ptr(block), g.hi_fmt, g.f);
    hipError_t e;
    if (quant_pair) {
        e = copy_packed(c, h, *packed, g.hi_fmt);
    } else {
        e = hipMemcpyAsync(const_cast<void *>(h.w_gate), pg, mat, hipMemcpyHostToDevice, c->mig);
        if (e == hipSuccess) e = hipMemcpyAsync(const_cast<void *>(h.w_up), pu, mat, hipMemcpyHostToDevice, c->mig);
        if (e == hipSuccess) e = hipMemcpyAsync(const_cast<void *>(h.w_down), pd, mat, hipMemcpyHostToDevice, c->mig);
    }
    if (e == hipSuccess) e = hipEventRecord(done, c->mig);
    if (e != hipSuccess) {
        (void)hipStreamSynchronize(c->mig);
        pool_give(c->pool_hi, block, nullptr);
        c->event_pool.push_back(done);
        DX_FAIL(c, DX_ERR_HIP, "dx_promote_async: %s", hipGetErrorString(e));
    }
    track_reserve(c, c->b_hi);
    en.state = DX_STATE_PROMOTING;
    en.next_block = block;
    c->hi_count[layer]++;
    c->inflight.push_back({layer, expert, true, done});
    c->stats.peak_in_flight = std::max<uint64_t>(c->stats.peak_in_flight, c->inflight.size());
    c->stats.promotions_issued++;
    c->stats.h2d_bytes += quant_pair ? c->b_hi : 3 * mat;
    return DX_OK;
}

extern "C" dx_status dx_demote_async(dx_ctx *c, int layer, int expert)
{
    if (!c) return DX_ERR_INVALID;
    if (!valid_layer(c, layer) || !valid_expert(c, expert, false)) DX_FAIL(c, DX_ERR_INVALID, "dx_demote_async: bad argument");
    const int idx = entry_index(c, layer, expert);
    dx_entry &en = c->entries[idx];
    if (en.state != DX_STATE_RESIDENT_HI || en.pool != 0)
        DX_FAIL(c, DX_ERR_BUSY, "dx_demote_async: expert (%d,%d) is not a pool-resident high-tier expert", layer, expert);
    const dx_config &g = c->cfg;
    const bool quant_pair = g.hi_fmt != DX_FMT_BF16;
    const dx_packed_host *packed_lo = nullptr;
    if (quant_pair) { // no bf16 version is resident to quantize from: the pre-packed low-tier version is copied in
        if (c->host_packed[1].empty() || !c->host_packed[1][(size_t)layer * g.E + expert].p[0])
            DX_FAIL(c, DX_ERR_INVALID, "dx_demote_async: no packed low-tier version registered for (%d,%d)", layer, expert);
        packed_lo = &c->host_packed[1][(size_t)layer * g.E + expert];
    }
    const uint64_t cap = g.budget_bytes ? g.budget_bytes + g.transient_bytes : ~0ull;
    if (c->reserved + c->b_lo > cap) {
        c->stats.deferred++;
        DX_FAIL(c, DX_ERR_BUDGET, "dx_demote_async: no transient room for the int4 version (%llu B reserved)", (unsigned long long)c->reserved);
    }
    hipEvent_t done;
    dx_status s = get_event(c, &done);
    if (s != DX_OK) return s;
    int block;
    s = pool_take(c, c->pool_lo, c->mig, &block);
    if (s != DX_OK) {
        c->event_pool.push_back(done);
        if (s == DX_ERR_NOMEM) c->stats.deferred++;
        return s;
    }
    dx_handle lo = handle_in_block(c, c->pool_lo.block_ptr(block), g.hi_fmt + 1, g.f);
    const dx_handle &hi = en.h;
    hipError_t e = hipSuccess;
    if (quant_pair) e = copy_packed(c, lo, *packed_lo, g.hi_fmt + 1);
    else e = dxk_quantize(static_cast<const dx_bf16 *>(hi.w_gate), g.f, g.d, g.group,
                          static_cast<uint8_t *>(const_cast<void *>(lo.w_gate)),
                          static_cast<dx_bf16 *>(const_cast<void *>(lo.s_gate)), c->mig);
    if (e == hipSuccess && !quant_pair)
        e = dxk_quantize(static_cast<const dx_bf16 *>(hi.w_up), g.f, g.d, g.group,
                         static_cast<uint8_t *>(const_cast<void *>(lo.w_up)),
                         static_cast<dx_bf16 *>(const_cast<void *>(lo.s_up)), c->mig);
    if (e == hipSuccess && !quant_pair)
        e = dxk_quantize(static_cast<const dx_bf16 *>(hi.w_down), g.d, g.f, g.group,
                         static_cast<uint8_t *>(const_cast<void *>(lo.w_down)),
                         static_cast<dx_bf16 *>(const_cast<void *>(lo.s_down)), c->mig);
    if (e == hipSuccess) e = hipEventRecord(done, c->mig);
    if (e != hipSuccess) {
        (void)hipStreamSynchronize(c->mig);
        pool_give(c->pool_lo, block, nullptr);
        c->event_pool.push_back(done);
        DX_FAIL(c, DX_ERR_HIP, "dx_demote_async: %s", hipGetErrorString(e));
    }
    track_reserve(c, c->b_lo);
    en.state = DX_STATE_DEMOTING;
    en.next_block = block;
    c->inflight.push_back({layer, expert, false, done});
    c->stats.peak_in_flight = std::max<uint64_t>(c->stats.peak_in_flight, c->inflight.size());
    c->stats.demotions_issued++;
    if (quant_pair) {
        c->stats.h2d_bytes += c->b_lo;
    } else {
        c->stats.quantize_read_bytes += c->b_hi;
        c->stats.quantize_write_bytes += c->b_lo;
    }
    return DX_OK;
}

extern "C" dx_status dx_migrate_poll(dx_ctx *c, int wait, int *n_published)
{
    if (!c) return DX_ERR_INVALID;
    int n = 0;
    if (n_published) *n_published = 0;
    while (!c->inflight.empty()) {
        dx_transition t = c->inflight.front();
        hipError_t q = wait ? hipEventSynchronize(t.done) : hipEventQuery(t.done);
        if (q == hipErrorNotReady) break; // publish strictly in issue order
        if (q != hipSuccess) DX_FAIL(c, DX_ERR_HIP, "dx_migrate_poll: %s", hipGetErrorString(q));
        const int idx = entry_index(c, t.layer, t.expert);
        dx_entry &en = c->entries[idx];
        dx_block_pool &new_pool = t.promote ? c->pool_hi : c->pool_lo;
        dx_block_pool &old_pool = t.promote ? c->pool_lo : c->pool_hi;
        const int old_block = en.block;
        dx_handle h = handle_in_block(c, new_pool.block_ptr(en.next_block), t.promote ? c->cfg.hi_fmt : c->cfg.hi_fmt + 1,
                                      c->cfg.f);
        // an event on the compute stream right after the swap: once it has fired, no
        // forward pass can still read the old version, so its block may be rewritten
        hipEvent_t after;
        dx_status s = get_event(c, &after);
        if (s != DX_OK) return s;
        s = publish(c, idx, h);
        if (s != DX_OK) {
            c->event_pool.push_back(after);
            return s;
        }
        // The handle is swapped from here on, so the bookkeeping below must follow whatever happens.  If
        // the event cannot be recorded, wait for the compute stream instead: after that no forward pass
        // reads the old version and its block needs no event to be reused.
        hipError_t e = hipEventRecord(after, c->compute);
        if (e != hipSuccess) {
            (void)hipStreamSynchronize(c->compute);
            c->event_pool.push_back(after);
            after = nullptr;
        }
        pool_give(old_pool, old_block, after);
        track_release(c, t.promote ? c->b_lo : c->b_hi);
        en.block = en.next_block;
        en.next_block = -1;
        en.pool = t.promote ? 0 : 1;
        en.state = t.promote ? DX_STATE_RESIDENT_HI : DX_STATE_RESIDENT_LO;
        if (t.promote) c->stats.promotions_published++;
        else {
            c->stats.demotions_published++;
            c->hi_count[t.layer]--;
        }
        c->event_pool.push_back(t.done);
        c->inflight.pop_front();
        ++n;
    }
    if (n_published) *n_published = n;
    return DX_OK;
}

// ------------------------------------------------ transition queue and worker step
extern "C" dx_status dx_register_host_master(dx_ctx *c, int layer, int expert, const void *pg, const void *pu,
                                             const void *pd)
{
    if (!c) return DX_ERR_INVALID;
    if (!valid_layer(c, layer) || !valid_expert(c, expert, false) || !pg || !pu || !pd)
        DX_FAIL(c, DX_ERR_INVALID, "dx_register_host_master: bad argument");
    if (c->host_master.empty()) c->host_master.assign((size_t)c->cfg.L * c->cfg.E, {nullptr, nullptr, nullptr});
    c->host_master[(size_t)layer * c->cfg.E + expert] = {pg, pu, pd};
    return DX_OK;
}

extern "C" dx_status dx_transitions_limits(dx_ctx *c, int max_inflight)
{
    if (!c) return DX_ERR_INVALID;
    if (max_inflight < 0) DX_FAIL(c, DX_ERR_INVALID, "dx_transitions_limits: negative bound");
    c->max_inflight = max_inflight;
    return DX_OK;
}

extern "C" dx_status dx_transitions_enqueue(dx_ctx *c, int layer, const int32_t *promote, int n_promote,
                                            const int32_t *demote, int n_demote)
{
    if (!c) return DX_ERR_INVALID;
    if (!valid_layer(c, layer) || n_promote < 0 || n_demote < 0 || (n_promote && !promote) || (n_demote && !demote))
        DX_FAIL(c, DX_ERR_INVALID, "dx_transitions_enqueue: bad argument");
    for (int pass = 0; pass < 2; ++pass) {
        const int32_t *ids = pass ? promote : demote;
        const int n = pass ? n_promote : n_demote;
        for (int i = 0; i < n; ++i)
            if (!valid_expert(c, ids[i], false))
                DX_FAIL(c, DX_ERR_INVALID, "dx_transitions_enqueue: expert %d out of range", ids[i]);
    }
    for (int pass = 0; pass < 2; ++pass) {
        const bool is_promote = pass == 1;
        const int32_t *ids = is_promote ? promote : demote;
        const int n = is_promote ? n_promote : n_demote;
        for (int i = 0; i < n; ++i) {
            bool settled = false;
            for (auto it = c->update_q.begin(); it != c->update_q.end(); ++it) {
                if (it->layer != layer || it->expert != ids[i]) continue;
                if (it->promote != is_promote) c->update_q.erase(it); // the newer target wins: both cancel
                settled = true;                                      // (or the same request is already queued)
                break;
            }
            if (!settled) c->update_q.push_back({layer, ids[i], is_promote});
        }
    }
    return DX_OK;
}

extern "C" dx_status dx_transitions_pump(dx_ctx *c, int max_issue, int32_t *n_issued, int32_t *n_published,
                                         int32_t *n_queued)
{
    if (!c) return DX_ERR_INVALID;
    if (n_issued) *n_issued = 0;
    if (n_published) *n_published = 0;
    if (n_queued) *n_queued = (int32_t)c->update_q.size();
    if (max_issue < 0) DX_FAIL(c, DX_ERR_INVALID, "dx_transitions_pump: negative max_issue");
    int published = 0;
    dx_status s = dx_migrate_poll(c, 0, &published);
    if (s != DX_OK) return s;
    if (n_published) *n_published = published;
    const dx_config &g = c->cfg;
    const uint64_t cap = g.budget_bytes ? g.budget_bytes + g.transient_bytes : ~0ull;
    int issued = 0;
    for (auto it = c->update_q.begin(); it != c->update_q.end();) {
        if (issued >= max_issue || (c->max_inflight && (int)c->inflight.size() >= c->max_inflight)) break;
        const dx_request r = *it;
        const uint8_t st = c->entries[entry_index(c, r.layer, r.expert)].state;
        const uint8_t there = r.promote ? DX_STATE_RESIDENT_HI : DX_STATE_RESIDENT_LO;
        const uint8_t going = r.promote ? DX_STATE_PROMOTING : DX_STATE_DEMOTING;
        const uint8_t ready = r.promote ? DX_STATE_RESIDENT_LO : DX_STATE_RESIDENT_HI;
        if (st == there || st == going || st == DX_STATE_EMPTY) { // nothing to do (any more)
            it = c->update_q.erase(it);
            continue;
        }
        if (st != ready) { // in the opposite transition: wait for its publication
            ++it;
            continue;
        }
        // admission, checked here so that a refusal is backpressure, not an error
        bool admit;
        if (r.promote) {
            admit = !(g.budget_bytes && c->hi_count[r.layer] >= c->n_hi_cap) && c->reserved + c->b_hi <= cap &&
                    !c->pool_hi.free_list.empty();
        } else {
            admit = c->reserved + c->b_lo <= cap && !c->pool_lo.free_list.empty();
        }
        if (!admit) {
            c->stats.deferred++;
            ++it;
            continue;
        }
        if (r.promote && g.hi_fmt != DX_FMT_BF16) {
            s = dx_promote_async(c, r.layer, r.expert, nullptr, nullptr, nullptr); // copies the registered packed version
        } else if (r.promote) {
            if (c->host_master.empty() || !c->host_master[(size_t)r.layer * g.E + r.expert][0])
                DX_FAIL(c, DX_ERR_INVALID, "dx_transitions_pump: no host master registered for (%d,%d)", r.layer, r.expert);
            const auto &m = c->host_master[(size_t)r.layer * g.E + r.expert];
            s = dx_promote_async(c, r.layer, r.expert, m[0], m[1], m[2]);
        } else {
            s = dx_demote_async(c, r.layer, r.expert);
        }
        if (s == DX_ERR_BUDGET || s == DX_ERR_NOMEM) { // lost a race with nothing: treat as backpressure
            ++it;
            continue;
        }
        if (s != DX_OK) return s;
        it = c->update_q.erase(it);
        ++issued;
    }
    if (n_issued) *n_issued = issued;
    if (n_queued) *n_queued = (int32_t)c->update_q.size();
    return DX_OK;
}
