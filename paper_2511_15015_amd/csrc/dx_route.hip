// Router top-k, routing weights and the stable permutation of (token, slot)
// pairs into per-expert segments, plus the small table/counter kernels.
//
// Paper: Sec. 3.1 (the worker obtains top-k expert ids from the router and
// indexes the handle table with them); Sec. 3.5 (per-expert selection counts).
//
// Determinism: the order inside an expert segment is by increasing pair
// index p = t*k + j.  Because the k ids of one token are distinct, the rank of
// pair (t, j) inside the segment of expert e equals the number of tokens
// t' < t that selected e.  Tokens are handled in chunks of 64: each chunk
// builds, per expert, a 64-bit mask of the tokens that selected it; ranks are
// population counts of mask prefixes.  No atomics decide any position.
#include "dx_internal.h"
#include "dx_route_core.h"

#include <cfloat>
#include <cstdarg>
#include <mutex>

namespace {

constexpr int kChunk = 64;      // tokens per chunk = bits per mask word
constexpr int kRouteThreads = 1024;
constexpr int kWaves = kRouteThreads / 64;

// exclusive scan of one int per thread across a 1024-thread block
__device__ int block_exclusive_scan(int v, int *lds_wave_tot /*[kWaves]*/, int *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int o = __shfl_up(inc, off, 64);
        if (lane >= off) inc += o;
    }
    if (lane == 63) lds_wave_tot[wave] = inc;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        int t = lds_wave_tot[w];
        if (w < wave) base += t;
        tot += t;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

// One chunk of 64 tokens per block.
// ROWS16 (layers of up to 512 experts): a token per 16-lane row, NV logits per lane of the row (E <= 16*NV), so
// the 16 wavefronts take the chunk's 64 tokens in one pass (the selection code of the decode kernels' routing
// prologue).  Otherwise a token per wavefront, NV consecutive logits per lane (E <= 64*NV), four passes.
template <int NV, bool ROWS16>
__global__ __launch_bounds__(kRouteThreads) void k_route_topk(
    const float *__restrict__ logits, int T, int E, int k, int32_t *__restrict__ ids, float *__restrict__ w,
    int32_t *__restrict__ counts, int32_t *__restrict__ offsets, int32_t *__restrict__ perm,
    unsigned long long *__restrict__ mask_out, unsigned long long *__restrict__ hotness, int fused)
{
    extern __shared__ unsigned long long lds_mask[]; // [E], then int ids [64*k], then wave totals
    int *lds_ids = reinterpret_cast<int *>(lds_mask + E);
    int *lds_tot = lds_ids + kChunk * k;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int chunk = blockIdx.x;
    for (int e = threadIdx.x; e < E; e += kRouteThreads) lds_mask[e] = 0ull;
    // single-chunk launch with the hotness update inside: fetch the counter now, it is added to at the end
    unsigned long long hot_before = 0ull;
    if (fused && hotness && (int)threadIdx.x < E) hot_before = hotness[threadIdx.x];
    __syncthreads();

    if constexpr (ROWS16) {
        static_assert(kChunk == 4 * kWaves, "four tokens per wavefront cover the chunk");
        const int tt = 4 * wave + (lane >> 4), t = chunk * kChunk + tt, c = lane & 15;
        if (chunk * kChunk + 4 * wave < T) { // wave-uniform: some row of this wavefront has a token (T > 0)
            float v[NV];
            dx_route_core::load_logits_rows16<NV>(logits + (size_t)(t < T ? t : T - 1) * E, c, E, v);
            int my_id;
            float my_w;
            dx_route_core::topk_rows16<NV>(v, k, lane, my_id, my_w);
            if (t < T && c < k) {
                ids[(size_t)t * k + c] = my_id;
                w[(size_t)t * k + c] = my_w;
                lds_ids[tt * k + c] = my_id;
                atomicOr(&lds_mask[my_id], 1ull << tt);
            }
        }
    } else
    for (int tt = wave; tt < kChunk; tt += kWaves) {
        const int t = chunk * kChunk + tt;
        if (t >= T) break; // wave-uniform
        const float *row = logits + (size_t)t * E;
        float v[1][NV];
        if constexpr (NV >= 4) dx_route_core::load_logits<NV>(row, lane, E, v[0]);
        else {
#pragma unroll
            for (int s = 0; s < NV; ++s) {
                const int e = NV * lane + s;
                v[0][s] = e < E ? row[e < E ? e : E - 1] : -INFINITY;
            }
        }
        int id1[1];
        float wt1[1];
        dx_route_core::topk_rows<NV, 1>(v, k, lane, id1, wt1);
        const int my_id = id1[0];
        if (lane < k) {
            ids[(size_t)t * k + lane] = my_id;
            w[(size_t)t * k + lane] = wt1[0];
            lds_ids[tt * k + lane] = my_id;
            atomicOr(&lds_mask[my_id], 1ull << tt);
        }
    }
    __syncthreads();

    if (!fused) {
        for (int e = threadIdx.x; e < E; e += kRouteThreads) mask_out[(size_t)chunk * E + e] = lds_mask[e];
        return;
    }
    // single chunk: finish counts, offsets and the permutation here (E <= 1024)
    const int e = threadIdx.x;
    const int c = e < E ? __popcll(lds_mask[e]) : 0;
    int total;
    const int off = block_exclusive_scan(c, lds_tot, &total);
    if (e < E) {
        counts[e] = c;
        offsets[e] = off;
        if (hotness) hotness[e] = hot_before + (unsigned long long)c;
        lds_ids[kChunk * k + kWaves + e] = off; // offsets kept in LDS after the wave totals
    }
    if (e == 0) offsets[E] = total;
    __syncthreads();
    const int *lds_off = lds_ids + kChunk * k + kWaves;
    const int P = T * k;
    for (int p = threadIdx.x; p < P; p += kRouteThreads) {
        const int tt = p / k;
        const int ex_id = lds_ids[p];
        const unsigned long long below = lds_mask[ex_id] & ((1ull << tt) - 1ull);
        perm[lds_off[ex_id] + __popcll(below)] = p;
    }
}

// counts/offsets and per-chunk bases from the chunk masks (one block)
__global__ __launch_bounds__(kRouteThreads) void k_route_scan(
    const unsigned long long *__restrict__ mask, int n_chunks, int E, int32_t *__restrict__ chunk_base,
    int32_t *__restrict__ counts, int32_t *__restrict__ offsets, unsigned long long *__restrict__ hotness)
{
    __shared__ int lds_tot[kWaves];
    const int e = threadIdx.x;
    int run = 0;
    if (e < E) {
        // eight independent mask loads in flight per round
        int c = 0;
        for (; c + 8 <= n_chunks; c += 8) {
            unsigned long long m[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) m[i] = mask[(size_t)(c + i) * E + e];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                chunk_base[(size_t)(c + i) * E + e] = run;
                run += __popcll(m[i]);
            }
        }
        for (; c < n_chunks; ++c) {
            chunk_base[(size_t)c * E + e] = run;
            run += __popcll(mask[(size_t)c * E + e]);
        }
    }
    int total;
    const int off = block_exclusive_scan(run, lds_tot, &total);
    if (e < E) {
        counts[e] = run;
        offsets[e] = off;
        if (hotness) hotness[e] += (unsigned long long)run;
    }
    if (e == 0) offsets[E] = total;
}

__global__ __launch_bounds__(256) void k_route_place(
    const int32_t *__restrict__ ids, int P, int E, int k, const unsigned long long *__restrict__ mask,
    const int32_t *__restrict__ chunk_base, const int32_t *__restrict__ offsets, int32_t *__restrict__ perm)
{
    const int p = blockIdx.x * 256 + threadIdx.x;
    if (p >= P) return;
    const int t = p / k;
    const int c = t / kChunk, bit = t % kChunk;
    const int e = ids[p];
    const unsigned long long below = mask[(size_t)c * E + e] & ((1ull << bit) - 1ull);
    perm[offsets[e] + chunk_base[(size_t)c * E + e] + __popcll(below)] = p;
}

__global__ void k_hotness_add(unsigned long long *__restrict__ counters, const int32_t *__restrict__ counts, int E)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < E) counters[e] += (unsigned long long)counts[e];
}

__global__ void k_fill_u64(unsigned long long *p, size_t n, unsigned long long v)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// Measurement aid: a streaming read as fast as this chip does one (whole lines per load instruction,
// non-temporal hint, as the decode kernels' weight stream).  Block b reads the 1 MiB units b, b + grid, ...;
// 16 bytes per thread and load, eight loads in flight per thread.  What it reads is folded into a value that
// is never equal to the magic number, so the loads cannot be dropped and nothing is written.
__global__ __launch_bounds__(512) void k_probe_read(const char *__restrict__ p, int n_units, unsigned *sink)
{
    typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
    constexpr size_t kUnit = 1u << 20;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (int u = blockIdx.x; u < n_units; u += gridDim.x) {
        const char *base = p + (size_t)u * kUnit + threadIdx.x * 16;
        for (size_t o = 0; o < kUnit; o += (size_t)8 * 512 * 16) {
            u32x4 v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(base + o + (size_t)i * 512 * 16));
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                acc.x ^= v[i].x; acc.y ^= v[i].y; acc.z ^= v[i].z; acc.w ^= v[i].w;
            }
        }
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x5EED1E55u && sink) *sink = 1u;
}

__global__ void k_store_handle(dx_handle *slot, dx_handle h)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) *slot = h;
}

// Router gate: logits = x . W_r^T (+ bias).  One block per 32 tokens x 32 experts; its 4 wavefronts
// take the K-steps of 16 in turn (step s to wavefront s % 4), each multiplying with
// v_mfma_f32_32x32x16_bf16 straight from global memory (lane l: row l % 32, 8 consecutive k from
// 8 * (l / 32)); the four partial tiles meet in LDS and are added in wavefront order.
typedef __attribute__((ext_vector_type(8))) __bf16 rt_bf16x8;
typedef __attribute__((ext_vector_type(16))) float rt_f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t rt_u32x4;

__global__ __launch_bounds__(256) void k_router_gemm(const dx_bf16 *__restrict__ x, const dx_bf16 *__restrict__ w_r,
                                                     const float *__restrict__ bias, int T, int E, int d,
                                                     float *__restrict__ logits)
{
    __shared__ float part[4][32][33];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t0 = blockIdx.y * 32, e0 = blockIdx.x * 32;
    const int r = lane & 31, kq = lane >> 5;
    const int t = min(t0 + r, T - 1), e = min(e0 + r, E - 1); // rows past the end repeat the last one; never stored
    const dx_bf16 *xrow = x + (size_t)t * d + kq * 8;
    const dx_bf16 *wrow = w_r + (size_t)e * d + kq * 8;
    rt_f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    union frag {
        rt_u32x4 u;
        rt_bf16x8 v;
    };
    for (int s = wave; s < d / 16; s += 4) {
        frag a, b;
        a.u = *reinterpret_cast<const rt_u32x4 *>(xrow + s * 16);
        b.u = *reinterpret_cast<const rt_u32x4 *>(wrow + s * 16);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, acc, 0, 0, 0);
    }
    // accumulator element v: token row (v/4)*8 + (lane/32)*4 + v%4, expert column lane%32
#pragma unroll
    for (int v = 0; v < 16; ++v) part[wave][(v >> 2) * 8 + kq * 4 + (v & 3)][r] = acc[v];
    __syncthreads();
    for (int i = threadIdx.x; i < 32 * 32; i += 256) {
        const int tr = i >> 5, ec = i & 31;
        if (t0 + tr >= T || e0 + ec >= E) continue;
        float v = ((part[0][tr][ec] + part[1][tr][ec]) + part[2][tr][ec]) + part[3][tr][ec];
        if (bias) v += bias[e0 + ec];
        logits[(size_t)(t0 + tr) * E + e0 + ec] = v;
    }
}

template <int NV, bool ROWS16>
hipError_t launch_topk(const float *logits, int T, int E, int k, int32_t *ids, float *w, int32_t *counts,
                       int32_t *offsets, int32_t *perm, unsigned long long *mask, unsigned long long *hotness,
                       int n_chunks, hipStream_t s)
{
    const int fused = n_chunks == 1;
    size_t lds = (size_t)E * 8 + (size_t)(kChunk * k + kWaves + E) * 4;
    hipLaunchKernelGGL((k_route_topk<NV, ROWS16>), dim3(n_chunks), dim3(kRouteThreads), lds, s, logits, T, E, k, ids, w,
                       counts, offsets, perm, mask, hotness, fused);
    return hipGetLastError();
}

} // namespace

hipError_t dxk_route(const float *logits, int T, int E, int k, int32_t *ids, float *w, int32_t *counts,
                     int32_t *offsets, int32_t *perm, unsigned long long *mask, int32_t *chunk_base,
                     unsigned long long *hotness, hipStream_t s)
{
    // T == 0 still runs one (empty) chunk so that counts and offsets are written.
    const int n_chunks = T > 0 ? (T + kChunk - 1) / kChunk : 1;
    hipError_t e;
    // (k <= 16: a selected id per lane of the token's row)
    if (k <= 16 && E <= 64) e = launch_topk<4, true>(logits, T, E, k, ids, w, counts, offsets, perm, mask, hotness, n_chunks, s);
    else if (k <= 16 && E <= 128) e = launch_topk<8, true>(logits, T, E, k, ids, w, counts, offsets, perm, mask, hotness, n_chunks, s);
    else if (k <= 16 && E <= 256) e = launch_topk<16, true>(logits, T, E, k, ids, w, counts, offsets, perm, mask, hotness, n_chunks, s);
    else if (k <= 16 && E <= 512) e = launch_topk<32, true>(logits, T, E, k, ids, w, counts, offsets, perm, mask, hotness, n_chunks, s);
    else if (E <= 64) e = launch_topk<1, false>(logits, T, E, k, ids, w, counts, offsets, perm, mask, hotness, n_chunks, s);
    else if (E <= 128) e = launch_topk<2, false>(logits, T, E, k, ids, w, counts, offsets, perm, mask, hotness, n_chunks, s);
    else if (E <= 256) e = launch_topk<4, false>(logits, T, E, k, ids, w, counts, offsets, perm, mask, hotness, n_chunks, s);
    else if (E <= 512) e = launch_topk<8, false>(logits, T, E, k, ids, w, counts, offsets, perm, mask, hotness, n_chunks, s);
    else e = launch_topk<16, false>(logits, T, E, k, ids, w, counts, offsets, perm, mask, hotness, n_chunks, s);
    if (e != hipSuccess || n_chunks == 1) return e;
    hipLaunchKernelGGL(k_route_scan, dim3(1), dim3(kRouteThreads), 0, s, mask, n_chunks, E, chunk_base, counts,
                       offsets, hotness);
    const int P = T * k;
    hipLaunchKernelGGL(k_route_place, dim3((P + 255) / 256), dim3(256), 0, s, ids, P, E, k, mask, chunk_base,
                       offsets, perm);
    return hipGetLastError();
}

hipError_t dxk_router_gemm(const dx_bf16 *x, const dx_bf16 *w_r, const float *bias, int T, int E, int d, float *logits,
                           hipStream_t s)
{
    if (T == 0) return hipSuccess;
    hipLaunchKernelGGL(k_router_gemm, dim3((E + 31) / 32, (T + 31) / 32), dim3(256), 0, s, x, w_r, bias, T, E, d, logits);
    return hipGetLastError();
}

hipError_t dxk_hotness_add(unsigned long long *counters, const int32_t *counts, int E, hipStream_t s)
{
    hipLaunchKernelGGL(k_hotness_add, dim3((E + 255) / 256), dim3(256), 0, s, counters, counts, E);
    return hipGetLastError();
}

hipError_t dxk_fill_u64(unsigned long long *p, size_t n, unsigned long long v, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_fill_u64, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n, v);
    return hipGetLastError();
}

hipError_t dxk_probe_read(const void *buf, size_t bytes, int n_cu, hipStream_t s)
{
    const int n_units = (int)(bytes >> 20);
    if (n_units == 0) return hipSuccess;
    hipLaunchKernelGGL(k_probe_read, dim3(n_cu), dim3(512), 0, s, static_cast<const char *>(buf), n_units,
                       static_cast<unsigned *>(nullptr));
    return hipGetLastError();
}

hipError_t dxk_store_handle(dx_handle *slot, const dx_handle &h, hipStream_t s)
{
    hipLaunchKernelGGL(k_store_handle, dim3(1), dim3(64), 0, s, slot, h);
    return hipGetLastError();
}

// ---- dx_route for callers that cannot allocate ---------------------------------------------------
// The routing scratch (per-chunk token masks and per-chunk segment bases, the two arrays dx_create
// otherwise allocates for a context) lives in a file-scope device array.  Every GPU the library runs
// on holds its own copy at its own address until the process ends; the address is asked for once per
// device, with that device current, and kept.  In host code the array's name is only a stand-in for
// the symbol: kernels get the resolved pointer, never the name.
namespace {

constexpr size_t kStaticEntries = DX_ROUTE_STATIC_MAX_ENTRIES; // (chunks of 64 tokens) x experts
struct route_scratch {
    unsigned long long mask[kStaticEntries];
    int32_t chunk_base[kStaticEntries];
};
static __device__ __align__(256) route_scratch scratch; // 768 KiB per GPU

constexpr int kMaxDevices = 64;
route_scratch *g_scratch_ptr[kMaxDevices]; // per device, null until resolved
std::mutex g_scratch_lock;
thread_local char g_static_err[256] = "";

dx_status static_fail(dx_status code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_static_err, sizeof g_static_err, fmt, ap);
    va_end(ap);
    return code;
}

} // namespace

extern "C" const char *dx_route_static_last_error(void) { return g_static_err; }

extern "C" dx_status dx_route_static(const float *logits, int T, int E, int top_k, int32_t *ids, float *w,
                                     int32_t *counts, int32_t *offsets, int32_t *perm, void *hip_stream)
{
    if (E < 1 || E > 1024) return static_fail(DX_ERR_INVALID, "dx_route_static: E=%d outside [1,1024]", E);
    if (top_k < 1 || top_k > E || top_k > 64)
        return static_fail(DX_ERR_INVALID, "dx_route_static: top_k=%d outside [1,min(E,64)]", top_k);
    if (T < 0) return static_fail(DX_ERR_INVALID, "dx_route_static: T=%d is negative", T);
    const long long n_chunks = T > 0 ? ((long long)T + kChunk - 1) / kChunk : 1;
    if (n_chunks * E > (long long)kStaticEntries)
        return static_fail(DX_ERR_INVALID,
                           "dx_route_static: ceil(T/64)*E = %lld exceeds the static scratch of %zu entries "
                           "(T=%d, E=%d); use dx_route on a context for larger batches",
                           n_chunks * E, kStaticEntries, T, E);
    if (!counts || !offsets || (T > 0 && (!logits || !ids || !w || !perm)))
        return static_fail(DX_ERR_INVALID, "dx_route_static: null pointer");
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return static_fail(DX_ERR_HIP, "dx_route_static: hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return static_fail(DX_ERR_INVALID, "dx_route_static: device %d not supported", dev);
    route_scratch *sp;
    {
        std::lock_guard<std::mutex> hold(g_scratch_lock);
        if (!g_scratch_ptr[dev]) {
            void *p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !p)
                return static_fail(DX_ERR_HIP, "dx_route_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
            g_scratch_ptr[dev] = static_cast<route_scratch *>(p);
        }
        sp = g_scratch_ptr[dev];
    }
    // Nothing in the scratch has to start at zero: every chunk's block writes all E masks of its chunk,
    // and the scan writes every base the placement reads.
    e = dxk_route(logits, T, E, top_k, ids, w, counts, offsets, perm, sp->mask, sp->chunk_base, nullptr,
                  static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return static_fail(DX_ERR_HIP, "dx_route_static: launch: %s", hipGetErrorString(e));
    return DX_OK;
}
