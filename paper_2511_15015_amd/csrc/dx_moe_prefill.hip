// Mixed-precision expert execution for large per-expert token counts
// (prefill): LDS-tiled bf16 MFMA grouped GEMMs.
//
// Paper: Sec. 3.2 (the compute path resolves the handle and runs the kernel of
// the active version).  The paper gives no kernel; this one is built for gfx950.
//
// Regime: experts with more than kSmallSegment tokens.  A block computes a
// 128 x 128 output tile with v_mfma_f32_32x32x16_bf16 (4 wavefronts, each a
// 64 x 64 sub-tile = 2 x 2 MFMA tiles, fp32 accumulators), K in steps of 64
// staged through a double-buffered LDS tile pair (rows padded to 144 bytes:
// conflict-free 128-bit fragment reads).  int4 weights are expanded in
// registers on their way from global memory to LDS (nibble -> fp32 -> times the
// group's scale -> bf16), so the MFMA loop is the same for both formats.
//   gate/up: the tile's 128 columns are 64 gate rows and the 64 up rows of the
//            same indices, and every wavefront owns matching gate/up columns,
//            so SwiGLU happens on the accumulators; H is written once as bf16.
//   down:    plain 128 x 128 tiles of O = H . W_down^T, written as fp32 rows in
//            pair order for the combine kernel.
// Tiles are listed expert-major, column-tile next, row-tile innermost, and the
// list is cut into 8 contiguous ranges, one per XCD (block b works in range
// b % 8), so the row tiles that share a weight tile run on the same L2.
#include "dx_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

#define DX_GLOBAL __attribute__((address_space(1)))
typedef const DX_GLOBAL char *gbytes;
typedef const DX_GLOBAL dx_bf16 *gbf16;
typedef const DX_GLOBAL u32x4 *gvec16;

union frag8 {
    u32x4 u;
    bf16x8 v;
};

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int kRowBytes = BK * 2 + 16; // 144: padded LDS row
constexpr int kTileBytes = BM * kRowBytes;
constexpr int kThreads = 256;
constexpr int kMaxExperts = 1024 + 1;

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ uint32_t float_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// 8 nibbles of `word` times scale -> 8 bf16 in element order
__device__ __forceinline__ u32x4 dequant8(uint32_t word, float scale)
{
    uint32_t p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float lo = (float)((int)(word << (28 - 8 * i)) >> 28) * scale;
        const float hi = (float)((int)(word << (24 - 8 * i)) >> 28) * scale;
        p[i] = float_to_bf16_rne(lo) | (float_to_bf16_rne(hi) << 16);
    }
    return u32x4{p[0], p[1], p[2], p[3]};
}

struct tile_id {
    int e, mt, nt; // expert (E = shared), row tile, column tile
    int seg0, m;
    bool valid;
};

// Every block derives the tile list from `offsets`: experts with more than m_small tokens, each
// ceil(m/128) row tiles x ntn column tiles.  LDS: tile prefix per expert.
__device__ tile_id find_tile(const dx_fwd_args &a, int ntn_routed, int ntn_shared, uint32_t *cum, uint32_t *wave_tot)
{
    const int nE = a.E + (a.shared ? 1 : 0);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int R = (nE + kThreads - 1) / kThreads; // <= 5
    uint32_t mine[5] = {0, 0, 0, 0, 0}, local = 0;
#pragma unroll
    for (int i = 0; i < 5; ++i) {
        const int e = tid * R + i;
        if (i < R && e < nE) {
            const int m = e == a.E ? a.T : a.offsets[e + 1] - a.offsets[e];
            if (m > a.m_small) mine[i] = (uint32_t)((m + BM - 1) / BM) * (e == a.E ? ntn_shared : ntn_routed);
            local += mine[i];
        }
    }
    uint32_t inc = local;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t o = __shfl_up(inc, off, 64);
        if (lane >= off) inc += o;
    }
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    uint32_t base = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
        const uint32_t t = wave_tot[w];
        if (w < wave) base += t;
        total += t;
    }
    uint32_t run = base + inc - local;
#pragma unroll
    for (int i = 0; i < 5; ++i) {
        const int e = tid * R + i;
        if (i < R && e < nE) {
            cum[e] = run;
            run += mine[i];
        }
    }
    if (tid == 0) cum[nE] = total;
    __syncthreads();
    tile_id t;
    t.valid = false;
    t.e = t.mt = t.nt = t.seg0 = t.m = 0;
    // XCD-contiguous ranges of the tile list
    const uint32_t per_xcd = (total + 7) / 8;
    const uint32_t idx = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((blockIdx.x >> 3) >= per_xcd || idx >= total) return t;
    // binary search: the expert whose range contains idx
    int lo = 0, hi = nE; // cum[lo] <= idx < cum[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cum[mid] <= idx) lo = mid;
        else hi = mid;
    }
    // skip experts with empty ranges that share cum[lo]
    t.e = lo;
    const uint32_t local_idx = idx - cum[lo];
    t.m = t.e == a.E ? a.T : a.offsets[t.e + 1] - a.offsets[t.e];
    t.seg0 = t.e == a.E ? a.T * a.k : a.offsets[t.e];
    const int nmt = (t.m + BM - 1) / BM;
    t.nt = local_idx / nmt;
    t.mt = local_idx % nmt;
    t.valid = true;
    return t;
}

// ---- staging: global -> registers -> LDS ----------------------------------------------------
// A tile: 128 rows x 64 bf16 (128 B per row): thread t loads 16-byte pieces (row = p / 8, piece = p % 8)
// for p = t, t + 256, t + 512, t + 768.
struct a_regs {
    u32x4 v[4];
};

__device__ __forceinline__ void load_a(a_regs &r, const gbf16 (&rowp)[4], int k0)
{
    const int piece = threadIdx.x & 7;
#pragma unroll
    for (int i = 0; i < 4; ++i) r.v[i] = *reinterpret_cast<gvec16>(rowp[i] + k0 + piece * 8);
}

__device__ __forceinline__ void store_a(const a_regs &r, char *tile)
{
    const int piece = threadIdx.x & 7;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = (threadIdx.x + i * kThreads) >> 3;
        *reinterpret_cast<u32x4 *>(tile + row * kRowBytes + piece * 16) = r.v[i];
    }
}

// B tile, bf16: same shape as A.  int4: 128 rows x 32 B: thread t takes row t / 2, half t % 2 (32 nibbles).
struct b_regs {
    u32x4 v[4]; // bf16: 4 pieces; int4: v[0] = 32 nibbles
    uint32_t scale;
};

__device__ __forceinline__ void load_b(b_regs &r, bool int4, const gbytes (&rowp)[4], gbytes qrow, gbf16 srow, int k0,
                                       int group)
{
    if (int4) {
        const int half = threadIdx.x & 1;
        r.v[0] = *reinterpret_cast<gvec16>(qrow + ((k0 + half * 32) >> 1));
        r.scale = srow[(k0 + half * 32) / group];
    } else {
        const int piece = threadIdx.x & 7;
#pragma unroll
        for (int i = 0; i < 4; ++i) r.v[i] = *reinterpret_cast<gvec16>(rowp[i] + (size_t)(k0 + piece * 8) * 2);
    }
}

__device__ __forceinline__ void store_b(const b_regs &r, bool int4, char *tile)
{
    if (int4) {
        const int row = threadIdx.x >> 1, half = threadIdx.x & 1;
        const float s = bf16_bits_to_float(r.scale);
        char *dst = tile + row * kRowBytes + half * 64;
        *reinterpret_cast<u32x4 *>(dst) = dequant8(r.v[0].x, s);
        *reinterpret_cast<u32x4 *>(dst + 16) = dequant8(r.v[0].y, s);
        *reinterpret_cast<u32x4 *>(dst + 32) = dequant8(r.v[0].z, s);
        *reinterpret_cast<u32x4 *>(dst + 48) = dequant8(r.v[0].w, s);
    } else {
        const int piece = threadIdx.x & 7;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = (threadIdx.x + i * kThreads) >> 3;
            *reinterpret_cast<u32x4 *>(tile + row * kRowBytes + piece * 16) = r.v[i];
        }
    }
}

// One K-step of 64 on the LDS tiles: wavefront (wm, wn) multiplies rows 64*wm.. of A by the two
// 32-row groups of B starting at brow0 and brow1.
__device__ __forceinline__ void mma_step(const char *ta, const char *tb, int wm, int brow0, int brow1,
                                         f32x16 (&acc)[2][2])
{
    const int lane = threadIdx.x & 63, r = lane & 31, kq = lane >> 5;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
        const int koff = (kk * 16 + kq * 8) * 2;
        frag8 af[2], bf[2];
#pragma unroll
        for (int ms = 0; ms < 2; ++ms)
            af[ms].u = *reinterpret_cast<const u32x4 *>(ta + (wm * 64 + ms * 32 + r) * kRowBytes + koff);
        bf[0].u = *reinterpret_cast<const u32x4 *>(tb + (brow0 + r) * kRowBytes + koff);
        bf[1].u = *reinterpret_cast<const u32x4 *>(tb + (brow1 + r) * kRowBytes + koff);
#pragma unroll
        for (int ms = 0; ms < 2; ++ms)
#pragma unroll
            for (int ns = 0; ns < 2; ++ns)
                acc[ms][ns] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ms].v, bf[ns].v, acc[ms][ns], 0, 0, 0);
    }
}

// accumulator element v of a 32x32 tile: row (v/4)*8 + (lane/32)*4 + v%4, column lane%32
__device__ __forceinline__ int acc_row(int v, int lane) { return (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3); }

template <bool DOWN>
__global__ __launch_bounds__(kThreads) void k_tiled(dx_fwd_args a)
{
    __shared__ __attribute__((aligned(16))) char lds[4 * kTileBytes]; // A0 A1 B0 B1: 72 KB
    __shared__ uint32_t cum[kMaxExperts + 1];
    __shared__ uint32_t wave_tot[kThreads / 64];

    const int ntn_routed = DOWN ? a.d / BN : a.f / (BN / 2);
    const int ntn_shared = DOWN ? a.d / BN : a.shared_f / (BN / 2);
    const tile_id t = find_tile(a, ntn_routed, ntn_shared, cum, wave_tot);
    if (!t.valid) return; // block-uniform

    const bool shared = t.e == a.E;
    const dx_handle hd = shared ? *a.shared : a.table[t.e];
    const bool int4 = hd.fmt == DX_FMT_INT4G;
    const int fe = shared ? a.shared_f : a.f;
    const int K = DOWN ? fe : a.d;
    const size_t wrow_bytes = int4 ? (size_t)K / 2 : (size_t)K * 2;
    const int G = K / a.group;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // ---- source rows of this thread's pieces ----
    gbf16 arow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = (tid + i * kThreads) >> 3;
        int slot = t.mt * BM + row;
        slot = slot < t.m ? slot : t.m - 1;
        if constexpr (DOWN) {
            arow[i] = (gbf16)a.h + (size_t)(t.seg0 + slot) * a.fmax;
        } else {
            const int tok = shared ? slot : a.perm[t.seg0 + slot] / a.k;
            arow[i] = (gbf16)a.x + (size_t)tok * K;
        }
    }
    // B tile row -> weight matrix row.  gate/up: rows 0..63 gate rows 64*nt.., rows 64..127 the up rows.
    auto wrow_of = [&](int brow, gbytes &mat, gbf16 &sc, int &n) {
        if constexpr (DOWN) {
            n = t.nt * BN + brow;
            mat = (gbytes)hd.w_down;
            sc = (gbf16)hd.s_down;
        } else {
            n = t.nt * (BN / 2) + (brow & 63);
            mat = (gbytes)(brow < 64 ? hd.w_gate : hd.w_up);
            sc = (gbf16)(brow < 64 ? hd.s_gate : hd.s_up);
        }
    };
    gbytes brow[4], qrow;
    gbf16 srow;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        gbytes mat;
        gbf16 sc;
        int n;
        wrow_of((tid + i * kThreads) >> 3, mat, sc, n);
        brow[i] = mat + (size_t)n * wrow_bytes;
    }
    {
        gbytes mat;
        gbf16 sc;
        int n;
        wrow_of(tid >> 1, mat, sc, n);
        qrow = mat + (size_t)n * wrow_bytes;
        srow = int4 ? sc + (size_t)n * G : nullptr;
    }

    f32x16 acc[2][2];
#pragma unroll
    for (int ms = 0; ms < 2; ++ms)
#pragma unroll
        for (int ns = 0; ns < 2; ++ns)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ms][ns][v] = 0.f;

    // wavefront's B row groups: gate/up -> 32 gate rows and the matching 32 up rows; down -> 64 rows
    const int brow0 = DOWN ? wn * 64 : wn * 32;
    const int brow1 = DOWN ? wn * 64 + 32 : 64 + wn * 32;

    auto ta = [&](int i) { return lds + i * kTileBytes; };
    auto tb = [&](int i) { return lds + (2 + i) * kTileBytes; };
    a_regs ra;
    b_regs rb;
    const int nk = K / BK;
    load_a(ra, arow, 0);
    load_b(rb, int4, brow, qrow, srow, 0, a.group);
    store_a(ra, ta(0));
    store_b(rb, int4, tb(0));
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) {
            load_a(ra, arow, (kt + 1) * BK);
            load_b(rb, int4, brow, qrow, srow, (kt + 1) * BK, a.group);
        }
        mma_step(ta(cur), tb(cur), wm, brow0, brow1, acc);
        if (kt + 1 < nk) {
            store_a(ra, ta(cur ^ 1));
            store_b(rb, int4, tb(cur ^ 1));
        }
        __syncthreads();
    }

    // ---- epilogue ----
    const int col = lane & 31;
#pragma unroll
    for (int ms = 0; ms < 2; ++ms) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int slot = t.mt * BM + wm * 64 + ms * 32 + acc_row(v, lane);
            if (slot >= t.m) continue;
            if constexpr (DOWN) {
                const size_t orow = shared ? (size_t)(t.seg0 + slot) : (size_t)a.perm[t.seg0 + slot];
                float *dst = a.o + orow * a.d + t.nt * BN + wn * 64 + col;
                dst[0] = acc[ms][0][v];
                dst[32] = acc[ms][1][v];
            } else {
                const float g = acc[ms][0][v], u = acc[ms][1][v];
                const float hv = g / (1.f + expf(-g)) * u;
                a.h[(size_t)(t.seg0 + slot) * a.fmax + t.nt * (BN / 2) + wn * 32 + col] = (dx_bf16)float_to_bf16_rne(hv);
            }
        }
    }
}

} // namespace

// upper bound on the number of tiles: sum over experts of ceil(m/128) <= pairs/128 + experts
hipError_t dxk_moe_forward_tiled(const dx_fwd_args &a, hipStream_t s, hipEvent_t *m_after_gate_up)
{
    const long pairs = (long)a.T * a.k;
    const long row_tiles = pairs / BM + a.E + (a.shared ? (a.T + BM - 1) / BM : 0);
    const int fe = a.shared && a.shared_f > a.f ? a.shared_f : a.f;
    long g1 = row_tiles * (fe / (BN / 2));
    long g2 = row_tiles * (a.d / BN);
    g1 = ((g1 + 7) / 8) * 8;
    g2 = ((g2 + 7) / 8) * 8;
    hipLaunchKernelGGL((k_tiled<false>), dim3((unsigned)g1), dim3(kThreads), 0, s, a);
    if (m_after_gate_up) (void)hipEventRecord(*m_after_gate_up, s);
    hipLaunchKernelGGL((k_tiled<true>), dim3((unsigned)g2), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}
