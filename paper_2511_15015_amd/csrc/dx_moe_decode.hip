// Mixed-precision expert execution for small per-expert token counts
// (decode): SwiGLU gate/up grouped GEMM, down grouped GEMM, weighted combine.
//
// Paper: Sec. 3.2 -- the compute path resolves each expert's stable handle to
// the active version (bf16, or int4 with its quantization parameters) and runs
// the matching kernel.  The paper gives no kernel; this one is built for
// gfx950.
//
// Regime: every activated expert's weights are streamed from HBM exactly once
// and there are at most a few dozen tokens per expert, so the kernels are
// bandwidth-bound.  One wavefront owns a strip of 16 weight rows (two strips:
// gate+up rows of the same index, or two adjacent down strips) over the whole
// K extent and feeds them straight from global memory into the B operand of
// v_mfma_f32_16x16x32_bf16; the (few) token rows are the A operand and come
// from L2.  Lane (r = lane%16, q = lane/16) owns row r and, inside each
// K-chunk of 4*LK elements, the LK consecutive elements starting at q*LK, so a
// strip's row is read in contiguous 4*LK-element pieces (256 B for bf16).  A
// uses the same K ownership, which makes any K order valid for the MFMA.
// int4 weights are expanded to exact small bf16 integers; because a K-chunk
// never crosses a quantization group, the group's scale is applied once to the
// chunk's fp32 partial sums (q*s is never rounded).
#include "dx_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

union frag8 {
    uint4 u;
    bf16x8 v;
};

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ uint32_t float_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// 8 two's-complement nibbles (element t at bits 4t) -> 8 bf16 holding the exact integers
__device__ __forceinline__ bf16x8 nibbles_to_bf16(uint32_t word)
{
    frag8 out;
    uint32_t p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int lo = (int)(word << (28 - 8 * i)) >> 28;
        const int hi = (int)(word << (24 - 8 * i)) >> 28;
        // small integers are exact in bf16: keep the upper 16 bits of the fp32 pattern
        p[i] = (__float_as_uint((float)lo) >> 16) | (__float_as_uint((float)hi) & 0xFFFF0000u);
    }
    out.u = make_uint4(p[0], p[1], p[2], p[3]);
    return out.v;
}

// One pipeline stage: the lane's piece of one K-chunk of NB weight strips and MT token tiles.
template <int NB, int MT, int LK, bool INT4>
struct stage {
    uint4 wb[INT4 ? 1 : NB][INT4 ? 1 : LK / 8]; // bf16 weights
    uint32_t wq[INT4 ? NB : 1][LK / 8];         // int4 weights, 8 nibbles per word
    uint16_t sc[INT4 ? NB : 1];                 // group scales (bf16 bits)
    uint4 a[MT][LK / 8];                        // token rows
};

template <int NB, int MT, int LK, bool INT4>
__device__ __forceinline__ void load_stage(stage<NB, MT, LK, INT4> &st, const char *const (&wrow)[NB],
                                           const dx_bf16 *const (&srow)[NB], const dx_bf16 *const (&arow)[MT],
                                           int c, int q, int chunks_per_group_shift_unused, int group)
{
    constexpr int CHUNK = 4 * LK;
    const int k0 = c * CHUNK + q * LK; // first K element this lane owns in chunk c
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if constexpr (INT4) {
            const char *p = wrow[b] + (k0 >> 1);
            if constexpr (LK == 32) {
                uint4 t = *reinterpret_cast<const uint4 *>(p);
                st.wq[b][0] = t.x; st.wq[b][1] = t.y; st.wq[b][2] = t.z; st.wq[b][3] = t.w;
            } else if constexpr (LK == 16) {
                uint2 t = *reinterpret_cast<const uint2 *>(p);
                st.wq[b][0] = t.x; st.wq[b][1] = t.y;
            } else {
                st.wq[b][0] = *reinterpret_cast<const uint32_t *>(p);
            }
            st.sc[b] = srow[b][(c * CHUNK) / group];
        } else {
            const uint4 *p = reinterpret_cast<const uint4 *>(wrow[b] + (size_t)k0 * 2);
#pragma unroll
            for (int j = 0; j < LK / 8; ++j) st.wb[b][j] = p[j];
        }
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const uint4 *p = reinterpret_cast<const uint4 *>(arow[mt] + k0);
#pragma unroll
        for (int j = 0; j < LK / 8; ++j) st.a[mt][j] = p[j];
    }
    (void)chunks_per_group_shift_unused;
}

template <int NB, int MT, int LK, bool INT4>
__device__ __forceinline__ void compute_stage(const stage<NB, MT, LK, INT4> &st, f32x4 (&acc)[NB][MT])
{
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if constexpr (INT4) {
            f32x4 part[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) part[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < LK / 8; ++j) {
                const bf16x8 wv = nibbles_to_bf16(st.wq[b][j]);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    frag8 a;
                    a.u = st.a[mt][j];
                    part[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, wv, part[mt], 0, 0, 0);
                }
            }
            const float s = bf16_bits_to_float(st.sc[b]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[b][mt] += part[mt] * s;
        } else {
#pragma unroll
            for (int j = 0; j < LK / 8; ++j) {
                frag8 wv;
                wv.u = st.wb[b][j];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    frag8 a;
                    a.u = st.a[mt][j];
                    acc[b][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, wv.v, acc[b][mt], 0, 0, 0);
                }
            }
        }
    }
}

// acc[b][mt] = sum over K of tokens(16 rows of tile mt) x strip b (16 weight rows), for this lane's
// outputs: column n = lane%16 of the strip, token rows 4*(lane/16) .. +3 of the tile.
template <int NB, int MT, int LK, bool INT4>
__device__ __forceinline__ void skinny_gemm(const char *const (&wrow)[NB], const dx_bf16 *const (&srow)[NB],
                                            const dx_bf16 *const (&arow)[MT], int K, int group, int q,
                                            f32x4 (&acc)[NB][MT])
{
    constexpr int CHUNK = 4 * LK;
    const int nc = K / CHUNK;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[b][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    stage<NB, MT, LK, INT4> s0, s1;
    load_stage<NB, MT, LK, INT4>(s0, wrow, srow, arow, 0, q, 0, group);
    for (int c = 0; c < nc; c += 2) {
        if (c + 1 < nc) load_stage<NB, MT, LK, INT4>(s1, wrow, srow, arow, c + 1, q, 0, group);
        compute_stage<NB, MT, LK, INT4>(s0, acc);
        if (c + 1 < nc) {
            if (c + 2 < nc) load_stage<NB, MT, LK, INT4>(s0, wrow, srow, arow, c + 2, q, 0, group);
            compute_stage<NB, MT, LK, INT4>(s1, acc);
        }
    }
}

struct seg_info {
    int seg0;   // first row of the expert's segment in the H/O scratch
    int m;      // tokens in the segment
    bool shared;
};

__device__ __forceinline__ seg_info segment_of(int e, int E, int T, int k, const int32_t *offsets)
{
    seg_info s;
    s.shared = e == E;
    if (s.shared) {
        s.seg0 = T * k;
        s.m = T;
    } else {
        s.seg0 = offsets[e];
        s.m = offsets[e + 1] - s.seg0;
    }
    return s;
}

constexpr int kTilesPerBlock = 4; // independent wavefronts per block

// ---- gate/up + SwiGLU: H[seg row, n] = silu(x . Wg[n]) * (x . Wu[n]) -------------------
template <int LK>
__global__ __launch_bounds__(64 * kTilesPerBlock) void k_gate_up(dx_fwd_args a)
{
    const int e = blockIdx.y;
    const seg_info sg = segment_of(e, a.E, a.T, a.k, a.offsets);
    if (sg.m == 0) return;
    const int fe = sg.shared ? a.shared_f : a.f;
    const int tile = blockIdx.x * kTilesPerBlock + (threadIdx.x >> 6);
    if (tile * 16 >= fe) return;
    const dx_handle hd = sg.shared ? *a.shared : a.table[e];
    const int lane = threadIdx.x & 63, r = lane & 15, q = lane >> 4;
    const int n = tile * 16 + r;
    const int K = a.d;
    const bool int4 = hd.fmt == DX_FMT_INT4G;
    const size_t row_bytes = int4 ? (size_t)K / 2 : (size_t)K * 2;
    const char *wrow[2] = {(const char *)hd.w_gate + (size_t)n * row_bytes, (const char *)hd.w_up + (size_t)n * row_bytes};
    const int G = K / a.group;
    const dx_bf16 *srow[2] = {int4 ? (const dx_bf16 *)hd.s_gate + (size_t)n * G : nullptr,
                              int4 ? (const dx_bf16 *)hd.s_up + (size_t)n * G : nullptr};

    for (int mb = 0; mb < sg.m; mb += 32) {
        const dx_bf16 *arow[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            int slot = mb + 16 * mt + r;
            slot = slot < sg.m ? slot : sg.m - 1;
            const int tok = sg.shared ? slot : a.perm[sg.seg0 + slot] / a.k;
            arow[mt] = a.x + (size_t)tok * K;
        }
        f32x4 acc[2][2];
        const bool two = sg.m - mb > 16;
        if (two) {
            if (int4) skinny_gemm<2, 2, LK, true>(wrow, srow, arow, K, a.group, q, acc);
            else skinny_gemm<2, 2, LK, false>(wrow, srow, arow, K, a.group, q, acc);
        } else {
            const dx_bf16 *arow1[1] = {arow[0]};
            f32x4 acc1[2][1];
            if (int4) skinny_gemm<2, 1, LK, true>(wrow, srow, arow1, K, a.group, q, acc1);
            else skinny_gemm<2, 1, LK, false>(wrow, srow, arow1, K, a.group, q, acc1);
            acc[0][0] = acc1[0][0];
            acc[1][0] = acc1[1][0];
        }
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            if (mt == 1 && !two) break;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int slot = mb + 16 * mt + 4 * q + i;
                if (slot < sg.m) {
                    const float g = acc[0][mt][i], u = acc[1][mt][i];
                    const float hv = g / (1.f + expf(-g)) * u;
                    a.h[(size_t)(sg.seg0 + slot) * a.fmax + n] = (dx_bf16)float_to_bf16_rne(hv);
                }
            }
        }
    }
}

// ---- down: O[out row, n] = H[seg row, :] . Wd[n, :] -------------------------------------
template <int LK>
__global__ __launch_bounds__(64 * kTilesPerBlock) void k_down(dx_fwd_args a)
{
    const int e = blockIdx.y;
    const seg_info sg = segment_of(e, a.E, a.T, a.k, a.offsets);
    if (sg.m == 0) return;
    const int K = sg.shared ? a.shared_f : a.f;
    const int tile = blockIdx.x * kTilesPerBlock + (threadIdx.x >> 6); // 32 output rows per tile
    if (tile * 32 >= a.d) return;
    const dx_handle hd = sg.shared ? *a.shared : a.table[e];
    const int lane = threadIdx.x & 63, r = lane & 15, q = lane >> 4;
    const int n0 = tile * 32 + r;
    const bool int4 = hd.fmt == DX_FMT_INT4G;
    const size_t row_bytes = int4 ? (size_t)K / 2 : (size_t)K * 2;
    const char *wrow[2] = {(const char *)hd.w_down + (size_t)n0 * row_bytes,
                           (const char *)hd.w_down + (size_t)(n0 + 16) * row_bytes};
    const int G = K / a.group;
    const dx_bf16 *srow[2] = {int4 ? (const dx_bf16 *)hd.s_down + (size_t)n0 * G : nullptr,
                              int4 ? (const dx_bf16 *)hd.s_down + (size_t)(n0 + 16) * G : nullptr};

    for (int mb = 0; mb < sg.m; mb += 32) {
        const dx_bf16 *arow[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            int slot = mb + 16 * mt + r;
            slot = slot < sg.m ? slot : sg.m - 1;
            arow[mt] = a.h + (size_t)(sg.seg0 + slot) * a.fmax;
        }
        f32x4 acc[2][2];
        const bool two = sg.m - mb > 16;
        if (two) {
            if (int4) skinny_gemm<2, 2, LK, true>(wrow, srow, arow, K, a.group, q, acc);
            else skinny_gemm<2, 2, LK, false>(wrow, srow, arow, K, a.group, q, acc);
        } else {
            const dx_bf16 *arow1[1] = {arow[0]};
            f32x4 acc1[2][1];
            if (int4) skinny_gemm<2, 1, LK, true>(wrow, srow, arow1, K, a.group, q, acc1);
            else skinny_gemm<2, 1, LK, false>(wrow, srow, arow1, K, a.group, q, acc1);
            acc[0][0] = acc1[0][0];
            acc[1][0] = acc1[1][0];
        }
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            if (mt == 1 && !two) break;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int slot = mb + 16 * mt + 4 * q + i;
                if (slot < sg.m) {
                    const int orow = sg.shared ? sg.seg0 + slot : a.perm[sg.seg0 + slot];
                    a.o[(size_t)orow * a.d + n0] = acc[0][mt][i];
                    a.o[(size_t)orow * a.d + n0 + 16] = acc[1][mt][i];
                }
            }
        }
    }
}

// ---- combine: y[t] = sum_j w[t,j] * O[t*k+j] (+ O[T*k+t] of the shared expert) ----------
__global__ __launch_bounds__(256) void k_combine(dx_fwd_args a)
{
    const int t = blockIdx.y;
    const int c = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (c >= a.d) return;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j = 0; j < a.k; ++j) {
        const float wj = a.w[(size_t)t * a.k + j];
        const float4 o = *reinterpret_cast<const float4 *>(a.o + ((size_t)t * a.k + j) * a.d + c);
        acc.x += wj * o.x; acc.y += wj * o.y; acc.z += wj * o.z; acc.w += wj * o.w;
    }
    if (a.shared) {
        const float4 o = *reinterpret_cast<const float4 *>(a.o + ((size_t)a.T * a.k + t) * a.d + c);
        acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w;
    }
    uint2 out;
    out.x = float_to_bf16_rne(acc.x) | (float_to_bf16_rne(acc.y) << 16);
    out.y = float_to_bf16_rne(acc.z) | (float_to_bf16_rne(acc.w) << 16);
    *reinterpret_cast<uint2 *>(a.y + (size_t)t * a.d + c) = out;
}

template <int LK>
hipError_t launch_all(const dx_fwd_args &a, hipStream_t s)
{
    const int ny = a.E + (a.shared ? 1 : 0);
    const int fe = a.shared && a.shared_f > a.f ? a.shared_f : a.f;
    const dim3 block(64 * kTilesPerBlock);
    const dim3 g1((fe / 16 + kTilesPerBlock - 1) / kTilesPerBlock, ny);
    hipLaunchKernelGGL(k_gate_up<LK>, g1, block, 0, s, a);
    const dim3 g2((a.d / 32 + kTilesPerBlock - 1) / kTilesPerBlock, ny);
    hipLaunchKernelGGL(k_down<LK>, g2, block, 0, s, a);
    const dim3 g3((a.d / 4 + 255) / 256, a.T);
    hipLaunchKernelGGL(k_combine, g3, dim3(256), 0, s, a);
    return hipGetLastError();
}

} // namespace

hipError_t dxk_moe_forward(const dx_fwd_args &a, hipStream_t s)
{
    if (a.T == 0) return hipSuccess;
    // K-chunk = min(group, 128) so that a chunk never crosses a quantization group
    if (a.group >= 128) return launch_all<32>(a, s);
    if (a.group == 64) return launch_all<16>(a, s);
    return launch_all<8>(a, s);
}
