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
//   down:    plain 128 x 128 tiles of O = H . W_down^T, written as bf16 rows in
//            pair order for the combine kernel.
// Tiles are listed expert-major, column-tile next, row-tile innermost, and the
// list is cut into 8 contiguous ranges, one per XCD (block b works in range
// b % 8), so the row tiles that share a weight tile run on the same L2.
#include "dx_internal.h"

#include <type_traits>

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

// silu(g) * u with the hardware exp2 and reciprocal (their error is far below the bf16 rounding of H)
__device__ __forceinline__ float swiglu_fast(float g, float u)
{
    return g * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g)) * u;
}

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// two fp32 -> two bf16 in one word (the hardware's packed conversion: round to nearest even, the same
// bits as float_to_bf16_rne for finite values)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    const f32x2 v{lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// 8 nibbles of `word` times scale -> 8 bf16 in element order
__device__ __forceinline__ u32x4 dequant8(uint32_t word, float scale)
{
    uint32_t p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        p[i] = pack_bf16((float)((int)(word << (28 - 8 * i)) >> 28) * scale,
                         (float)((int)(word << (24 - 8 * i)) >> 28) * scale);
    return u32x4{p[0], p[1], p[2], p[3]};
}

// 8 two-bit codes (bits 16*half .. of `word`) times scale -> 8 bf16 in element order
__device__ __forceinline__ u32x4 dequant8_crumbs(uint32_t word, int half, float scale)
{
    const uint32_t h = word >> (16 * half);
    uint32_t p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        p[i] = pack_bf16((float)((int)(h << (30 - 4 * i)) >> 30) * scale, (float)((int)(h << (28 - 4 * i)) >> 30) * scale);
    return u32x4{p[0], p[1], p[2], p[3]};
}

struct tile_id {
    int e, mt, nt; // expert (E = shared), row tile, column tile
    int seg0, m;   // first pair slot and number of rows of the part of the segment this kernel owns
    int tok0;      // shared expert: token of row 0 of that part
    bool valid;
};

constexpr int kBigRows = 256; // row granularity of the big-tile kernel

// Rows of expert e that belong to the calling kernel.  Segments up to m_small tokens are not tiled at
// all.  When the big-tile kernel is on (a.m_big), it owns the leading multiple of 256 rows of every
// bf16 expert (and of every int4 expert when a.big_int4) and the 128-row kernel owns the rest.
template <bool BIG>
__device__ __forceinline__ void owned_rows(const dx_fwd_args &a, int e, int &row0, int &rows)
{
    const int m = e == a.E ? a.T : a.offsets[e + 1] - a.offsets[e];
    row0 = rows = 0;
    if (m <= a.m_small) return;
    int lead = 0;
    if (a.m_big && m >= kBigRows) {
        const int fmt = e == a.E ? a.shared->fmt : a.table[e].fmt;
        if (fmt == DX_FMT_BF16 || (fmt == DX_FMT_INT4G && a.big_int4)) lead = m / kBigRows * kBigRows;
    }
    if (BIG) rows = lead;
    else row0 = lead, rows = m - lead;
}

// Every block derives the tile list from `offsets`: per expert ceil(rows/TM) row tiles x ntn column
// tiles, expert-major, column tile next, row tile innermost.  The list is cut into 8 contiguous
// ranges, one per XCD (block b works in range b % 8).  LDS: tile prefix per expert.
template <int THREADS, int TM, bool BIG>
__device__ tile_id find_tile(const dx_fwd_args &a, int ntn_routed, int ntn_shared, uint32_t *cum, uint32_t *wave_tot)
{
    const int nE = a.E + (a.shared ? 1 : 0);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int R = (nE + THREADS - 1) / THREADS; // <= 5
    uint32_t mine[5] = {0, 0, 0, 0, 0}, local = 0;
#pragma unroll
    for (int i = 0; i < 5; ++i) {
        const int e = tid * R + i;
        if (i < R && e < nE) {
            int row0, rows;
            owned_rows<BIG>(a, e, row0, rows);
            mine[i] = (uint32_t)((rows + TM - 1) / TM) * (e == a.E ? ntn_shared : ntn_routed);
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
    for (int w = 0; w < THREADS / 64; ++w) {
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
    t.e = t.mt = t.nt = t.seg0 = t.m = t.tok0 = 0;
    const uint32_t per_xcd = (total + 7) / 8;
    const uint32_t idx = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((blockIdx.x >> 3) >= per_xcd || idx >= total) return t;
    // binary search: the expert whose range contains idx (experts with empty ranges are skipped)
    int lo = 0, hi = nE; // cum[lo] <= idx < cum[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cum[mid] <= idx) lo = mid;
        else hi = mid;
    }
    t.e = lo;
    const uint32_t local_idx = idx - cum[lo];
    int row0, rows;
    owned_rows<BIG>(a, t.e, row0, rows);
    t.m = rows;
    t.tok0 = row0;
    t.seg0 = (t.e == a.E ? a.T * a.k : a.offsets[t.e]) + row0;
    const int nmt = (rows + TM - 1) / TM;
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

// B tile, bf16: same shape as A.  int4: 128 rows x 32 B: thread t takes row t / 2, half t % 2 (32 nibbles);
// int2: 128 rows x 16 B, the same split (32 codes = 8 bytes).  FMT: 0 bf16, 1 int4, 2 int2.
struct b_regs {
    u32x4 v[4]; // bf16: 4 pieces; int4: v[0] = 32 nibbles; int2: v[0].x, v[0].y = 32 codes
    uint32_t scale;
};

typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef const DX_GLOBAL u32x2 *gvec8;

template <int FMT>
__device__ __forceinline__ void load_b(b_regs &r, const gbytes (&rowp)[4], gbytes qrow, gbf16 srow, int k0, int group)
{
    if constexpr (FMT == 2) {
        const int half = threadIdx.x & 1;
        const u32x2 t = *reinterpret_cast<gvec8>(qrow + ((k0 + half * 32) >> 2));
        r.v[0] = u32x4{t.x, t.y, 0u, 0u};
        r.scale = srow[(k0 + half * 32) / group];
    } else if constexpr (FMT == 1) {
        const int half = threadIdx.x & 1;
        r.v[0] = *reinterpret_cast<gvec16>(qrow + ((k0 + half * 32) >> 1));
        r.scale = srow[(k0 + half * 32) / group];
    } else {
        const int piece = threadIdx.x & 7;
#pragma unroll
        for (int i = 0; i < 4; ++i) r.v[i] = *reinterpret_cast<gvec16>(rowp[i] + (size_t)(k0 + piece * 8) * 2);
    }
}

template <int FMT>
__device__ __forceinline__ void store_b(const b_regs &r, char *tile)
{
    if constexpr (FMT == 2) {
        const int row = threadIdx.x >> 1, half = threadIdx.x & 1;
        const float s = bf16_bits_to_float(r.scale);
        char *dst = tile + row * kRowBytes + half * 64;
        *reinterpret_cast<u32x4 *>(dst) = dequant8_crumbs(r.v[0].x, 0, s);
        *reinterpret_cast<u32x4 *>(dst + 16) = dequant8_crumbs(r.v[0].x, 1, s);
        *reinterpret_cast<u32x4 *>(dst + 32) = dequant8_crumbs(r.v[0].y, 0, s);
        *reinterpret_cast<u32x4 *>(dst + 48) = dequant8_crumbs(r.v[0].y, 1, s);
    } else if constexpr (FMT == 1) {
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

// One output tile.  INT4 selects the staging of the weight tile at compile time so that the bf16
// loop carries no trace of the int4 expansion (and the other way round).
template <bool DOWN, int FMT>
__device__ __forceinline__ void tile_main(const dx_fwd_args &a, const tile_id &t, const dx_handle &hd, char *lds)
{
    constexpr bool quant = FMT != 0;
    const bool shared = t.e == a.E;
    const int fe = shared ? a.shared_f : a.f;
    const int K = DOWN ? fe : a.d;
    const size_t wrow_bytes = FMT == 0 ? (size_t)K * 2 : (FMT == 1 ? (size_t)K / 2 : (size_t)K / 4);
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
            const int tok = shared ? t.tok0 + slot : a.perm[t.seg0 + slot] / a.k;
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
        srow = quant ? sc + (size_t)n * G : nullptr;
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
    // Two register stages: while the MFMA loop works on K-step kt from LDS, the tile of kt + 1 is on
    // its way from memory in one register set (it is written to the other LDS buffer at the end of
    // this step) and the loads of kt + 2 are issued into the other set, so every load has two full
    // steps to arrive.  Loads past the end re-read the last tile (never stored).
    a_regs ra[2];
    b_regs rb[2];
    const int nk = K / BK;
    auto k_of = [&](int kt) { return (kt < nk ? kt : nk - 1) * BK; };
    load_a(ra[0], arow, 0);
    load_b<FMT>(rb[0], brow, qrow, srow, 0, a.group);
    load_a(ra[1], arow, k_of(1));
    load_b<FMT>(rb[1], brow, qrow, srow, k_of(1), a.group);
    store_a(ra[0], ta(0));
    store_b<FMT>(rb[0], tb(0));
    __syncthreads();
    auto step = [&](int kt, auto parity) {
        constexpr int P = decltype(parity)::value;
        load_a(ra[P], arow, k_of(kt + 2));
        load_b<FMT>(rb[P], brow, qrow, srow, k_of(kt + 2), a.group);
        mma_step(ta(P), tb(P), wm, brow0, brow1, acc);
        if (kt + 1 < nk) {
            store_a(ra[P ^ 1], ta(P ^ 1));
            store_b<FMT>(rb[P ^ 1], tb(P ^ 1));
        }
        __syncthreads();
    };
    int kt = 0;
    for (; kt + 1 < nk; kt += 2) {
        step(kt, std::integral_constant<int, 0>{});
        step(kt + 1, std::integral_constant<int, 1>{});
    }
    if (kt < nk) step(kt, std::integral_constant<int, 0>{});

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
                dx_bf16 *dst = reinterpret_cast<dx_bf16 *>(a.o) + orow * a.d + t.nt * BN + wn * 64 + col;
                dst[0] = (dx_bf16)float_to_bf16_rne(acc[ms][0][v]);
                dst[32] = (dx_bf16)float_to_bf16_rne(acc[ms][1][v]);
            } else {
                const float g = acc[ms][0][v], u = acc[ms][1][v];
                const float hv = swiglu_fast(g, u);
                a.h[(size_t)(t.seg0 + slot) * a.fmax + t.nt * (BN / 2) + wn * 32 + col] = (dx_bf16)float_to_bf16_rne(hv);
            }
        }
    }
}

template <bool DOWN>
__global__ __launch_bounds__(kThreads) void k_tiled(dx_fwd_args a)
{
    __shared__ __attribute__((aligned(16))) char lds[4 * kTileBytes]; // A0 A1 B0 B1: 72 KB
    __shared__ uint32_t cum[kMaxExperts + 1];
    __shared__ uint32_t wave_tot[kThreads / 64];

    const int ntn_routed = DOWN ? a.d / BN : a.f / (BN / 2);
    const int ntn_shared = DOWN ? a.d / BN : a.shared_f / (BN / 2);
    const tile_id t = find_tile<kThreads, BM, false>(a, ntn_routed, ntn_shared, cum, wave_tot);
    if (!t.valid) return; // block-uniform
    const dx_handle hd = t.e == a.E ? *a.shared : a.table[t.e];
    if (hd.fmt == DX_FMT_INT4G) tile_main<DOWN, 1>(a, t, hd, lds);
    else if (hd.fmt == DX_FMT_INT2G) tile_main<DOWN, 2>(a, t, hd, lds);
    else tile_main<DOWN, 0>(a, t, hd, lds);
}

// ---------------------------------------------------------------------------------------------
// Large segments: 256 x 256 output tiles, 8 wavefronts (2 along rows x 4 along columns, each a
// 128 x 64 sub-tile = 4 x 2 MFMA tiles), K in steps of 64 through a two-stage LDS ring that is
// filled by global_load_lds_dwordx4 (memory to LDS without passing through registers), up to two
// steps ahead of the MFMA loop.  One barrier per step.
//   LDS rows are 128 bytes, one whole line of a token or weight row per step (a load instruction then
//   asks for 8 whole lines; with 64-byte rows and 16 half lines per instruction the same fill runs a
//   quarter slower), unpadded because a wavefront-wide LDS load writes 1 KB contiguously (lane l ->
//   byte 16*l).  The piece stored in slot c of row r is c ^ ((r>>1)&7): the 16 lanes that read one piece
//   index of 16 consecutive rows then hit 16 different bank groups.
//   The loads are inline assembly so that the compiler does not serialise them against the LDS
//   reads; their completion is awaited with explicit vmcnt counts.
// bf16 experts: tokens and weights both arrive that way (8 loads per wavefront per step).
// int4 experts (Q4): the tokens arrive that way; the weights' nibbles and scales take the same kind of
//   load, four bytes per lane, into a small side ring (per slot and wavefront: 4 x 8 rows x 32 bytes of
//   nibbles, 32 rows x one pair of scales), one step before the wavefront that loaded them expands them
//   (nibble -> fp32 -> times the group's scale -> bf16) into the weight half of the stage that has just been
//   freed.  Every wavefront expands only what it loaded itself, so the side ring needs no barrier, only
//   the wavefront's own vmcnt; the expanded rows are published by the step's barrier like the loaded ones
//   (9 loads per wavefront per step).
constexpr int TM = 256, TN = 256, TK = 64;
constexpr int kBigThreads = 512;
constexpr int kRowBytes64 = TK * 2;                      // 128: one line of a row per step
constexpr int kStageBytes = (TM + TN) * kRowBytes64;     // 64 KB: token rows then weight rows
constexpr int kStages = 2;
constexpr int kSideWave = 1280;                          // per wavefront: 4 x 256 bytes of nibbles, 256 of scale pairs
constexpr int kSideStage = (kBigThreads / 64) * kSideWave; // 10 KB
constexpr int kRingBytes = kStages * (kStageBytes + kSideStage);
static_assert(kRingBytes >= TM * (TN * 2 + 16), "the staged output tile reuses the ring");

typedef __attribute__((address_space(3))) char lds_char;

// one wavefront-wide 16-byte-per-lane load: memory (sbase + voff) -> LDS (m0 + 16 * lane)
__device__ __forceinline__ void load_to_lds(uint32_t m0, uint32_t voff, uint64_t sbase)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(m0), "v"(voff), "s"(sbase)
                 : "memory");
}
// the same with 4 bytes per lane: memory (sbase + voff) -> LDS (m0 + 4 * lane)
__device__ __forceinline__ void load_to_lds4(uint32_t m0, uint32_t voff, uint64_t sbase)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(m0), "v"(voff), "s"(sbase)
                 : "memory");
}
// a wave-uniform pointer as a scalar pair (the halves go through unsigned 32-bit values: the builtin
// returns int, which must not be sign-extended into the upper half)
__device__ __forceinline__ uint64_t scalar_ptr(const void *p)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)p);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uintptr_t)p >> 32));
    return (uint64_t)lo | ((uint64_t)hi << 32);
}

template <bool DOWN, bool Q4>
__device__ __forceinline__ void big_tile(const dx_fwd_args &a, const tile_id &t, const dx_handle &hd, char *ring)
{
    const bool shared = t.e == a.E;
    const int fe = shared ? a.shared_f : a.f;
    const int K = DOWN ? fe : a.d;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;

    // ---- loader role: wavefront w fills rows [32w, 32w + 32) of the token part and of the weight part ----
    // A load instruction covers 8 rows x one 128-byte line; lane l writes LDS piece l % 8 of row l / 8 and
    // fetches the memory piece that belongs there: piece p of row r sits in slot p ^ ((r >> 1) & 7).
    // weight-tile row -> matrix row: down: TN consecutive rows; gate/up: 128 gate rows, then the same up rows
    auto wrow = [&](int row) { return DOWN ? t.nt * TN + row : t.nt * (TN / 2) + (row & 127); };
    uint32_t a_off[4], b_off[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = 32 * wave + 8 * i + (lane >> 3);
        const uint32_t piece = (uint32_t)((lane & 7) ^ ((row >> 1) & 7));
        const int slot = t.mt * TM + row; // big tiles are full: slot < t.m
        if constexpr (DOWN) {
            a_off[i] = (uint32_t)(t.seg0 + slot) * (uint32_t)a.fmax * 2u + piece * 16u;
        } else {
            const int tok = shared ? t.tok0 + slot : a.perm[t.seg0 + slot] / a.k;
            a_off[i] = (uint32_t)tok * (uint32_t)K * 2u + piece * 16u;
        }
        // bf16: the lane's 16-byte piece of the row; int4: its four bytes (8 nibbles) of the row's 32 per step
        b_off[i] = Q4 ? (uint32_t)wrow(row) * (uint32_t)(K / 2) + (uint32_t)(lane & 7) * 4u
                      : (uint32_t)wrow(row) * (uint32_t)K * 2u + piece * 16u;
    }
    const uint64_t a_base = (uint64_t)(DOWN ? (const void *)a.h : (const void *)a.x);
    const uint64_t b_base = scalar_ptr(DOWN ? hd.w_down : (wave < 4 ? hd.w_gate : hd.w_up));
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_char *)ring;
    const uint32_t m0_a = lds0 + wave * 32 * kRowBytes64, m0_b = lds0 + TM * kRowBytes64 + wave * 32 * kRowBytes64;
    const int nk = K / TK;
    // int4: scales of the lane's row (lane & 31 of the wavefront's 32 rows), read as the aligned pair that
    // holds the step's groups (the number of groups per row is even there, so a pair never leaves its row;
    // with groups of 32 a step spans exactly the two groups of its pair)
    const int lg = __builtin_ctz((unsigned)a.group);
    const uint32_t s_off = Q4 ? (uint32_t)wrow(32 * wave + (lane & 31)) * (uint32_t)(K >> lg) * 2u : 0u;
    const uint64_t s_base = Q4 ? scalar_ptr(DOWN ? hd.s_down : (wave < 4 ? hd.s_gate : hd.s_up)) : 0;
    const int side_wave = kStages * kStageBytes + wave * kSideWave; // + slot * kSideStage
    auto clamped = [&](int kt) { return kt < nk ? kt : nk - 1; };
    auto issue_tokens = [&](int kt, int stage) {
        const uint64_t kb = (uint64_t)clamped(kt) * kRowBytes64;
        const uint32_t so = (uint32_t)stage * kStageBytes;
#pragma unroll
        for (int i = 0; i < 4; ++i) load_to_lds(m0_a + so + 1024 * i, a_off[i], a_base + kb);
    };
    auto issue_weights = [&](int kt, int stage) { // bf16
        const uint64_t kb = (uint64_t)clamped(kt) * kRowBytes64;
        const uint32_t so = (uint32_t)stage * kStageBytes;
#pragma unroll
        for (int i = 0; i < 4; ++i) load_to_lds(m0_b + so + 1024 * i, b_off[i], b_base + kb);
    };
    auto issue_codes = [&](int kt, int slot) { // int4: nibbles and scale pairs of step kt -> side slot
        const int kc = clamped(kt);
        const uint32_t m0 = lds0 + (uint32_t)(side_wave + slot * kSideStage);
#pragma unroll
        for (int i = 0; i < 4; ++i) load_to_lds4(m0 + 256 * i, b_off[i], b_base + (uint64_t)kc * (TK / 2));
        load_to_lds4(m0 + 1024, s_off, s_base + (uint64_t)((((kc * TK) >> lg) * 2) & ~3));
    };
    // int4: the wavefront's 32 rows of step kt, from side slot `slot` into the weight half of `stage`
    auto expand = [&](int kt, int slot, int stage) {
        const int odd = ((clamped(kt) * TK + 8 * (lane & 7)) >> lg) & 1; // per lane when a group is 32 wide
        const char *side = ring + side_wave + slot * kSideStage;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t codes = *reinterpret_cast<const uint32_t *>(side + 256 * i + 4 * lane);
            const uint32_t pair = *reinterpret_cast<const uint32_t *>(side + 1024 + 4 * (8 * i + (lane >> 3)));
            const float scale = __uint_as_float(odd ? pair & 0xFFFF0000u : pair << 16);
            const int row = 32 * wave + 8 * i + (lane >> 3);
            const int pos = (lane & 7) ^ ((row >> 1) & 7);
            *reinterpret_cast<u32x4 *>(ring + stage * kStageBytes + TM * kRowBytes64 + row * kRowBytes64 + pos * 16) =
                dequant8(codes, scale);
        }
    };

    // ---- MFMA role ----
    const int r = lane & 31, kq = lane >> 5, swz = (r >> 1) & 7;
    const int a_lane = (wm * 128 + r) * kRowBytes64;
    const int b_lane0 = TM * kRowBytes64 + (DOWN ? wn * 64 + r : wn * 32 + r) * kRowBytes64;
    const int b_lane1 = TM * kRowBytes64 + (DOWN ? wn * 64 + 32 + r : 128 + wn * 32 + r) * kRowBytes64;

    f32x16 acc[4][2];
#pragma unroll
    for (int ms = 0; ms < 4; ++ms)
#pragma unroll
        for (int ns = 0; ns < 2; ++ns)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ms][ns][v] = 0.f;

    // Software pipeline.  Each K-step has four quarters (16 k-values each); the fragments of a quarter sit
    // in registers before its MFMAs start.  The barrier comes once the last quarter's fragments have been
    // read, in the shadow of the third quarter's MFMAs: past it every wavefront holds what it needs of
    // stage S, so S is refilled at once with step kt + 2, and the landed stage of step kt + 1 may be read.
    frag8 fa[2][4], fb[2][2];
    auto read_frags = [&](int stage, int quarter, frag8 (&af)[4], frag8 (&bf)[2]) {
        const char *st = ring + stage * kStageBytes;
        const int so = ((2 * quarter + kq) ^ swz) * 16;
#pragma unroll
        for (int ms = 0; ms < 4; ++ms) af[ms].u = *reinterpret_cast<const u32x4 *>(st + a_lane + ms * 32 * kRowBytes64 + so);
        bf[0].u = *reinterpret_cast<const u32x4 *>(st + b_lane0 + so);
        bf[1].u = *reinterpret_cast<const u32x4 *>(st + b_lane1 + so);
    };
    auto mma_quarter = [&](const frag8 (&af)[4], const frag8 (&bf)[2]) {
#pragma unroll
        for (int ms = 0; ms < 4; ++ms)
#pragma unroll
            for (int ns = 0; ns < 2; ++ns)
                acc[ms][ns] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[ns].v, af[ms].v, acc[ms][ns], 0, 0, 0);
    };
    if constexpr (Q4) {
        // The codes of step j are loaded with the tokens of step j - 1 and expanded when step j - 2 frees
        // its stage.  Start: codes 0, 1 and tokens 0, 1; expand 0, 1 as soon as the codes are there; then
        // the codes of step 2.
        issue_codes(0, 0);
        issue_codes(1, 1);
        issue_tokens(0, 0);
        issue_tokens(1, 1);
        asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); // own codes 0, 1
        expand(0, 0, 0);
        expand(1, 1, 1);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // side slot 0 has been read: refill it
        issue_codes(2, 0);
        asm volatile("s_waitcnt vmcnt(9) lgkmcnt(0)" ::: "memory"); // own tokens of step 0; own expansions
    } else {
        issue_tokens(0, 0), issue_weights(0, 0);
        issue_tokens(1, 1), issue_weights(1, 1);
        asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); // own loads of step 0
    }
    __builtin_amdgcn_s_barrier();
    read_frags(0, 0, fa[0], fb[0]);
    auto step = [&](int kt, auto stage_c) {
        constexpr int S = decltype(stage_c)::value;
        // (the scheduling fences keep the LDS reads ahead of the MFMAs they overlap with)
        read_frags(S, 1, fa[1], fb[1]);
        __builtin_amdgcn_sched_barrier(0);
        mma_quarter(fa[0], fb[0]);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(S, 2, fa[0], fb[0]);
        __builtin_amdgcn_sched_barrier(0);
        mma_quarter(fa[1], fb[1]);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(S, 3, fa[1], fb[1]);
        __builtin_amdgcn_sched_barrier(0);
        mma_quarter(fa[0], fb[0]);
        __builtin_amdgcn_sched_barrier(0);
        // own loads of step kt + 1 (int4: and the codes of step kt + 2) have landed; own LDS reads of stage S
        // have returned and own LDS writes are done; after the barrier that holds for every wavefront
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        issue_tokens(kt + 2, S);
        if constexpr (Q4) {
            issue_codes(kt + 3, S ^ 1);
            expand(kt + 2, S, S);
        } else {
            issue_weights(kt + 2, S);
        }
        read_frags(S ^ 1, 0, fa[0], fb[0]);
        __builtin_amdgcn_sched_barrier(0);
        mma_quarter(fa[1], fb[1]);
        __builtin_amdgcn_sched_barrier(0);
    };
    for (int kt = 0; kt < nk; kt += 2) { // nk is even (K a multiple of 128)
        step(kt, std::integral_constant<int, 0>{});
        step(kt + 1, std::integral_constant<int, 1>{});
    }
    // the redundant loads issued past the end still target this block's LDS: drain them
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // ---- epilogue: through LDS, so that the tile leaves as whole rows in 16-byte pieces ----
    // The weights were the first MFMA operand: accumulator element v of a 32 x 32 tile is output column
    // (v/4)*8 + (lane/32)*4 + v%4 of token lane%32, i.e. four consecutive columns per group of four v.
    __builtin_amdgcn_s_barrier(); // every wavefront is done with the ring
    constexpr int OUT_COLS = DOWN ? TN : TN / 2;
    constexpr int OUT_STRIDE = OUT_COLS * 2 + 16; // bytes per staged row
    {
        const int tok_l = lane & 31, nq = (lane >> 5) * 4;
#pragma unroll
        for (int ms = 0; ms < 4; ++ms) {
            char *rowp = ring + (wm * 128 + ms * 32 + tok_l) * OUT_STRIDE;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if constexpr (DOWN) {
#pragma unroll
                    for (int ns = 0; ns < 2; ++ns) {
                        uint2 pk;
                        pk.x = float_to_bf16_rne(acc[ms][ns][4 * q]) | (float_to_bf16_rne(acc[ms][ns][4 * q + 1]) << 16);
                        pk.y = float_to_bf16_rne(acc[ms][ns][4 * q + 2]) | (float_to_bf16_rne(acc[ms][ns][4 * q + 3]) << 16);
                        *reinterpret_cast<uint2 *>(rowp + (wn * 64 + ns * 32 + q * 8 + nq) * 2) = pk;
                    }
                } else {
                    uint32_t hb[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        hb[i] = float_to_bf16_rne(swiglu_fast(acc[ms][0][4 * q + i], acc[ms][1][4 * q + i]));
                    uint2 pk;
                    pk.x = hb[0] | (hb[1] << 16);
                    pk.y = hb[2] | (hb[3] << 16);
                    *reinterpret_cast<uint2 *>(rowp + (wn * 32 + q * 8 + nq) * 2) = pk;
                }
            }
        }
    }
    __syncthreads();
    constexpr int PIECES = OUT_COLS / 8;               // 16-byte pieces per row
    constexpr int ROWS_PER_PASS = kBigThreads / PIECES; // rows written per pass of the block
    const int piece = tid % PIECES;
#pragma unroll 4
    for (int row = tid / PIECES; row < TM; row += ROWS_PER_PASS) {
        const int slot = t.mt * TM + row;
        const u32x4 v = *reinterpret_cast<const u32x4 *>(ring + row * OUT_STRIDE + piece * 16);
        dx_bf16 *dst;
        if constexpr (DOWN) {
            const size_t orow = shared ? (size_t)(t.seg0 + slot) : (size_t)a.perm[t.seg0 + slot];
            dst = reinterpret_cast<dx_bf16 *>(a.o) + orow * a.d + t.nt * TN + piece * 8;
        } else {
            dst = a.h + (size_t)(t.seg0 + slot) * a.fmax + t.nt * (TN / 2) + piece * 8;
        }
        *reinterpret_cast<u32x4 *>(dst) = v;
    }
}

template <bool DOWN>
__global__ __launch_bounds__(kBigThreads) void k_big(dx_fwd_args a)
{
    // the ring (128 KB) and the int4 side ring (20 KB); the staged output tile (256 rows of 512 + 16 bytes) reuses them
    __shared__ __attribute__((aligned(1024))) char ring[kRingBytes];
    __shared__ uint32_t cum[kMaxExperts + 1];
    __shared__ uint32_t wave_tot[kBigThreads / 64];

    const int ntn_routed = DOWN ? a.d / TN : a.f / (TN / 2);
    const int ntn_shared = DOWN ? a.d / TN : a.shared_f / (TN / 2);
    const tile_id t = find_tile<kBigThreads, TM, true>(a, ntn_routed, ntn_shared, cum, wave_tot);
    if (!t.valid) return; // block-uniform
    const dx_handle hd = t.e == a.E ? *a.shared : a.table[t.e];
    if (hd.fmt == DX_FMT_INT4G) big_tile<DOWN, true>(a, t, hd, ring); // block-uniform
    else big_tile<DOWN, false>(a, t, hd, ring);
}

} // namespace

// Grid sizes are upper bounds on the tile counts (sum over experts of ceil(rows/TM) <= pairs/TM + experts);
// surplus blocks find no tile and leave.
hipError_t dxk_moe_forward_tiled(const dx_fwd_args &a, hipStream_t s_big, hipStream_t s_tiled,
                                 hipEvent_t *m_after_gate_up)
{
    const long pairs = (long)a.T * a.k;
    const int fe = a.shared && a.shared_f > a.f ? a.shared_f : a.f;
    auto round8 = [](long g) { return (unsigned)(((g + 7) / 8) * 8); };
    const long row_tiles = pairs / BM + a.E + (a.shared ? (a.T + BM - 1) / BM : 0);
    const long big_tiles = a.m_big ? pairs / TM + (a.shared ? a.T / TM : 0) : 0;
    // the long-running 256-row kernels are queued first
    if (big_tiles) {
        hipLaunchKernelGGL((k_big<false>), dim3(round8(big_tiles * (fe / (TN / 2)))), dim3(kBigThreads), 0, s_big, a);
        if (m_after_gate_up && s_big != s_tiled) (void)hipEventRecord(*m_after_gate_up, s_big);
        hipLaunchKernelGGL((k_big<true>), dim3(round8(big_tiles * (a.d / TN))), dim3(kBigThreads), 0, s_big, a);
    }
    hipLaunchKernelGGL((k_tiled<false>), dim3(round8(row_tiles * (fe / (BN / 2)))), dim3(kThreads), 0, s_tiled, a);
    if (m_after_gate_up && !(big_tiles && s_big != s_tiled)) (void)hipEventRecord(*m_after_gate_up, s_tiled);
    hipLaunchKernelGGL((k_tiled<true>), dim3(round8(row_tiles * (a.d / BN))), dim3(kThreads), 0, s_tiled, a);
    return hipGetLastError();
}
