// Mixed-precision expert execution for small per-expert token counts
// (decode): SwiGLU gate/up grouped GEMM, down grouped GEMM, weighted combine.
//
// Paper: Sec. 3.2 -- the compute path resolves each expert's stable handle to
// the active version (bf16, or int4 / int2 with its quantization parameters)
// and runs the matching kernel.  The paper gives no kernel; this one is built for
// gfx950.
//
// Regime: every activated expert's weights are streamed from HBM exactly once
// and there are at most a few dozen tokens per expert, so both GEMM kernels are
// bandwidth-bound.  What decides the achieved bandwidth on this chip is that
// every compute unit streams for the whole duration of the kernel, so:
//   - Persistent grid, one block of 8 wavefronts per compute unit.  The work
//     is the list of (activated expert, 32-token block, strip of 16 weight
//     rows: 16 rows of W_down, or 8 rows of W_gate with the same 8 of W_up),
//     weighed in cost units (units_of, kRunUnits below); block b takes the
//     strips that start in units [b*U/G, (b+1)*U/G).  Every block derives
//     the same partition from `offsets` and the handles' formats in its
//     prologue (a block-wide scan): no atomics, no work queue.
//   - The 8 wavefronts of a block split the K extent of a strip between them
//     (wavefront kw owns CPW consecutive K-chunks of 4*LK elements), so a
//     whole strip is in flight at once and the following ones are prefetched
//     into further register stages while this one is multiplied.  Strips go
//     in pairs (two accumulators, one barrier per pair); when K is short,
//     the block works on several pairs side by side.  Partial sums meet in
//     LDS, are added in a fixed order and finished (SwiGLU, or the store of
//     the down output) by all threads of the block.
//   - The token rows (A operand of v_mfma_f32_16x16x32_bf16) only depend on
//     the expert and the K-chunk, so each wavefront keeps its fragments in
//     registers for all strips of a run: after the first strip, weights are
//     the only global traffic.
//   - Lane (r = lane%16, q = lane/16) owns tile row r.  bf16: step j of a
//     chunk takes elements 32j + 8q .. +7.  int4 / int2: the lane takes the
//     LK consecutive elements at q*LK (one 16-byte / 8-byte piece for LK =
//     32).  Token fragments use the same K ownership, which makes either
//     order valid.  Where the sizes allow it the loads themselves cover whole
//     128-byte lines of 8 rows and a DPP move sorts the pieces into this
//     ownership (see kLines).
//   - Quantized weights are expanded to exact small bf16 integers; a K-chunk
//     never crosses a quantization group, so the group's scale multiplies the
//     chunk's fp32 partial sums once (q*s is never rounded).
// Batches of up to 128 tokens run here alone (segments above 32 tokens in
// blocks of 32); larger ones hand the big segments to the tile kernels.
#include "dx_internal.h"
#include "dx_route_core.h"

#include <hip/hip_ext.h>

#include <cmath>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4; // 16 bytes in registers
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// Pointers that come out of a handle are loaded from memory, so the compiler cannot infer their
// address space and would fall back to FLAT loads (whose wait counters serialise the pipeline).
// Everything the kernels stream is in global memory: say so in the type.
#define DX_GLOBAL __attribute__((address_space(1)))
typedef const DX_GLOBAL char *gbytes;   // weight bytes
typedef const DX_GLOBAL dx_bf16 *gbf16; // bf16 rows (scales, tokens)
typedef const DX_GLOBAL u32x4 *gvec16;
typedef const DX_GLOBAL u32x2 *gvec8;
typedef const DX_GLOBAL uint32_t *gvec4;
typedef const __attribute__((address_space(3))) int *lds_ints; // an int array in LDS

union frag8 {
    u32x4 u;
    bf16x8 v;
};

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ uint32_t float_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// int4 -> bf16 without arithmetic.  XOR with 0x8 turns a two's-complement nibble q into u = q + 8 in
// [0, 15]; OR-ing u into the mantissa of bf16 128.0 (0x4300) gives exactly 128 + u = 136 + q.  One
// shift and one and-or yield two such values, elements t and t+4 of the word, so the 8 elements come
// out in the order (0,4,1,5,2,6,3,7); the token fragment is permuted to match once per run, and the
// bias is removed through  sum_k a_k (136 + q_k) - 136 sum_k a_k.
constexpr float kNibbleBias = 136.f;

// The flip, the mask and the OR are one v_bitop3_b32 per register (x is the shifted word): with two
// constant words p and q the result bit is 0, 1, the bit of x or its complement for (p, q) = (0, 0),
// (0, 1), (1, 0), (1, 1) -- truth table 0x6A over (x, p, q).
__device__ __forceinline__ uint32_t keep_flip_set(uint32_t x, uint32_t p, uint32_t q)
{
    return __builtin_amdgcn_bitop3_b32(x, p, q, 0x6A);
}

__device__ __forceinline__ bf16x8 nibbles_to_biased_bf16(uint32_t word)
{
    constexpr uint32_t p = 0x000F000Fu, q = (0x88888888u & p) | 0x43004300u; // ((x ^ 0x8888...) & p) | 0x4300...
    frag8 out;
    out.u = u32x4{keep_flip_set(word, p, q), keep_flip_set(word >> 4, p, q), keep_flip_set(word >> 8, p, q),
                  keep_flip_set(word >> 12, p, q)};
    return out.v;
}

// int2 (the low tier of the int4 / int2 pair): XOR with binary 10 turns a two's-complement code q in
// [-2, 1] into u = q + 2 in [0, 3]; OR-ed into bf16 128.0 it is 130 + q.  A word holds 16 codes; one
// shift and one and-or yield elements t and t+8, so the first MFMA step of a word takes elements
// (0,8,1,9,2,10,3,11) (shifts 0,2,4,6) and the second (4,12,5,13,6,14,7,15) (shifts 8..14).
constexpr float kCrumbBias = 130.f;

template <int HALF>
__device__ __forceinline__ bf16x8 crumbs_to_biased_bf16(uint32_t word)
{
    constexpr uint32_t p = 0x00030003u, q = (0xAAAAAAAAu & p) | 0x43004300u;
    frag8 out;
    out.u = u32x4{keep_flip_set(word >> (8 * HALF), p, q), keep_flip_set(word >> (8 * HALF + 2), p, q),
                  keep_flip_set(word >> (8 * HALF + 4), p, q), keep_flip_set(word >> (8 * HALF + 6), p, q)};
    return out.v;
}

// the matching order for two consecutive token fragments a = (e0..e7), b = (e8..e15):
// lo = (e0,e8,e1,e9,e2,e10,e3,e11), hi = (e4,e12,e5,e13,e6,e14,e7,e15)
__device__ __forceinline__ void zip_fragments(u32x4 &a, u32x4 &b)
{
    const u32x4 lo = u32x4{(a.x & 0x0000FFFFu) | (b.x << 16), (a.x >> 16) | (b.x & 0xFFFF0000u),
                           (a.y & 0x0000FFFFu) | (b.y << 16), (a.y >> 16) | (b.y & 0xFFFF0000u)};
    const u32x4 hi = u32x4{(a.z & 0x0000FFFFu) | (b.z << 16), (a.z >> 16) | (b.z & 0xFFFF0000u),
                           (a.w & 0x0000FFFFu) | (b.w << 16), (a.w >> 16) | (b.w & 0xFFFF0000u)};
    a = lo;
    b = hi;
}

// the same element order for a token fragment: (e0..e7) -> (e0,e4,e1,e5,e2,e6,e3,e7)
__device__ __forceinline__ u32x4 interleave_halves(u32x4 v)
{
    return u32x4{(v.x & 0x0000FFFFu) | (v.z << 16), (v.x >> 16) | (v.z & 0xFFFF0000u),
                 (v.y & 0x0000FFFFu) | (v.w << 16), (v.y >> 16) | (v.w & 0xFFFF0000u)};
}

constexpr int kWaves = 8;             // wavefronts per block
constexpr int kThreads = 64 * kWaves; // 512
constexpr int kMaxExperts = 1024 + 1; // routed + shared
// Cost units of the partition, from a fit of the blocks' measured times (per-block time stamps of a debug
// build, 30B- and 80B-shaped decode layers, a dozen routing draws each) to
//   time = runs * c_run + sum over the block's strips of c(format, token tiles):
// a bf16 strip for up to 16 tokens is 32 units; the same strip for two token tiles multiplies and finishes
// twice as much (1.25x gate/up, 1.35x down); a quantized strip is a quarter of the bytes or less but
// carries the same per-step work (expansion, barrier, reduction), 0.47x for one tile and 0.8x for two --
// weighed by time, not bytes.  int2 strips (an eighth of the bytes, the same per-step work) are taken a
// little below the int4 ones.
// A run that starts on a new expert pays for the token rows and a cold pipeline (3 to 5 us: two to three
// bf16 gate/up strips, five down strips): every expert's range begins with kRunUnits units that carry no
// strips, so the block that holds an expert boundary gets correspondingly fewer strips.
template <bool DOWN>
constexpr uint32_t kRunUnits = DOWN ? 176 : 84;
template <bool DOWN>
__device__ __forceinline__ uint32_t units_of(uint32_t fmt, int m)
{
    const bool two = m > 16;
    if (fmt == DX_FMT_BF16) return two ? (DOWN ? 43 : 40) : 32;
    const uint32_t q = two ? (DOWN ? 26 : 25) : 15;
    return fmt == DX_FMT_INT4G ? q : q - 3;
}

#ifdef DX_TRACE
// Debug build only: per-block start/end time stamps (100 MHz wall clock).
__device__ unsigned long long g_trace[2][8192][4];
__device__ unsigned long long g_steps[2][4][256];
__device__ unsigned int g_nsteps[2][4];
__device__ unsigned int g_mix[2][8192][8]; // per block: runs, then strips by (format != bf16) * 2 + (second token tile)
#endif

// element offset inside a chunk of MFMA step j for lane quarter q
// FMT: 0 bf16, 1 int4, 2 int2 (the values of dx_fmt)
template <int LK, int FMT>
__device__ __forceinline__ int k_of(int j, int q)
{
    return FMT ? q * LK + 8 * j : 32 * j + 8 * q;
}

// weight registers of one wavefront for one 16-row strip: CPW chunks
template <int LK, int CPW, int FMT>
struct wstage {
    static constexpr int JN = LK / 8;
    static constexpr int NQ = FMT == 1 ? JN : (FMT == 2 ? (JN + 1) / 2 : 1);
    u32x4 w[CPW][FMT ? 1 : JN]; // bf16: JN 16-byte pieces per chunk
    uint32_t wq[CPW][NQ];       // int4: JN words of 8 nibbles; int2: JN/2 words of 16 codes
};

// The cache policy of the weight stream.  With the non-temporal hint a read-only stream of whole 128-byte
// lines is faster on this chip (7.0 against 6.2 TB/s), but only when a load instruction covers whole lines.
// The operand layout of the matrix instruction wants, per instruction, 16 bytes per lane of the lane's own
// row: 64 bytes of each of 16 rows, the other half of every line in the next instruction -- hinted loads of
// that shape measured slower than plain ones (gate/up 46.5 against 44.4 us on the 30B-shaped layer).
// kLines<...> chooses the other shape where the sizes allow it: an instruction covers 128 bytes of each of 8
// rows (lane (r, q) fetches row r % 8 of the strip's lower or upper half, 16-byte piece q + 4 * (r / 8) of
// the line), so half of what a lane receives belongs to the lane 8 places away in its 16-lane row; one DPP
// move per register (row rotation by 8, written to half of the row) puts it there when the stage is used.
// The K order of the operands does not change.
template <typename T>
__device__ __forceinline__ T stream_load(const DX_GLOBAL T *p)
{
    return *p;
}
template <typename T>
__device__ __forceinline__ T line_load(const DX_GLOBAL T *p)
{
    return __builtin_nontemporal_load(p);
}

// bf16: a chunk of 128 elements is two lines per row; int4: two chunks side by side are one line per row
template <int LK, int CPW, int FMT, bool FAST>
constexpr bool kLines = LK == 32 && (FMT == 0 || (FMT == 1 && CPW == 2 && FAST));

// Line-shaped loads of one strip: `row_lo` is row r % 8 of the strip's lower eight rows, `row_hi` row r % 8
// of its upper eight (in a gate/up strip another matrix), `piece` = q + 4 * (r / 8).  Stage register n of
// chunk i then holds load (line n / 2, half n % 2) (bf16) resp. chunk register i holds the load of half i
// (int4) until settle_lines sorts them out.
template <int LK, int CPW, int FMT>
__device__ __forceinline__ void issue_weight_lines(wstage<LK, CPW, FMT> &st, gbytes row_lo, gbytes row_hi, int c0,
                                                   int nc, int piece)
{
    if constexpr (FMT == 0) {
#pragma unroll
        for (int i = 0; i < CPW; ++i) {
            if (c0 + i < nc) { // wavefront-uniform
#pragma unroll
                for (int n = 0; n < 4; ++n)
                    st.w[i][n] = line_load(reinterpret_cast<gvec16>(((n & 1) ? row_hi : row_lo) + (size_t)(c0 + i) * 256 +
                                                                   128 * (n >> 1) + 16 * piece));
            }
        }
    } else {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const u32x4 t = line_load(reinterpret_cast<gvec16>((h ? row_hi : row_lo) + (size_t)c0 * 64 + 16 * piece));
            st.wq[h][0] = t.x; st.wq[h][1] = t.y; st.wq[h][2] = t.z; st.wq[h][3] = t.w;
        }
    }
}

// register pair (a, b) = loads (lower half rows, upper half rows) of the same line: afterwards a holds the
// lane's own row's first piece, b its second (lanes 0..7 of a row keep a and receive b from 8 places up,
// lanes 8..15 keep b and receive a from 8 places down)
__device__ __forceinline__ void settle_pair(uint32_t &a, uint32_t &b)
{
    const int a0 = (int)a, b0 = (int)b;
    a = (uint32_t)__builtin_amdgcn_update_dpp(a0, b0, 0x128 /* row_ror:8 */, 0xF, 0xC, false);
    b = (uint32_t)__builtin_amdgcn_update_dpp(b0, a0, 0x128, 0xF, 0x3, false);
}

template <int LK, int CPW, int FMT>
__device__ __forceinline__ wstage<LK, CPW, FMT> settle_lines(const wstage<LK, CPW, FMT> &in, int c0, int nc)
{
    wstage<LK, CPW, FMT> st = in;
    if constexpr (FMT == 0) {
#pragma unroll
        for (int i = 0; i < CPW; ++i) {
            if (c0 + i < nc) {
#pragma unroll
                for (int l = 0; l < 2; ++l)
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        uint32_t a = st.w[i][2 * l][k], b = st.w[i][2 * l + 1][k];
                        settle_pair(a, b);
                        st.w[i][2 * l][k] = a;
                        st.w[i][2 * l + 1][k] = b;
                    }
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) settle_pair(st.wq[0][k], st.wq[1][k]);
    }
    return st;
}

template <int LK, int CPW, int FMT>
__device__ __forceinline__ void issue_weights(wstage<LK, CPW, FMT> &st, gbytes row, int c0, int nc, int q)
{
    constexpr int CHUNK = 4 * LK, JN = LK / 8;
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
        const int c = c0 + i;
        if (c < nc) { // wavefront-uniform
            if constexpr (FMT == 2) {
                gbytes p = row + ((c * CHUNK + q * LK) >> 2);
                if constexpr (LK == 32) {
                    const u32x2 t = stream_load(reinterpret_cast<gvec8>(p));
                    st.wq[i][0] = t.x; st.wq[i][1] = t.y;
                } else if constexpr (LK == 16) {
                    st.wq[i][0] = stream_load(reinterpret_cast<gvec4>(p));
                } else { // 8 codes = 2 bytes (handles of this format are refused for group 32; kept in bounds)
                    st.wq[i][0] = *reinterpret_cast<const DX_GLOBAL uint16_t *>(p);
                }
            } else if constexpr (FMT == 1) {
                gbytes p = row + ((c * CHUNK + q * LK) >> 1);
                if constexpr (LK == 32) {
                    const u32x4 t = stream_load(reinterpret_cast<gvec16>(p));
                    st.wq[i][0] = t.x; st.wq[i][1] = t.y; st.wq[i][2] = t.z; st.wq[i][3] = t.w;
                } else if constexpr (LK == 16) {
                    const u32x2 t = stream_load(reinterpret_cast<gvec8>(p));
                    st.wq[i][0] = t.x; st.wq[i][1] = t.y;
                } else {
                    st.wq[i][0] = stream_load(reinterpret_cast<gvec4>(p));
                }
            } else {
#pragma unroll
                for (int j = 0; j < JN; ++j)
                    st.w[i][j] = stream_load(reinterpret_cast<gvec16>(row + (size_t)(c * CHUNK + k_of<LK, 0>(j, q)) * 2));
            }
        }
    }
}

template <int LK, int CPW, int FMT, int MT>
__device__ __forceinline__ void load_tokens(u32x4 (&x)[CPW][MT][LK / 8], gbf16 arow0, gbf16 arow1, int c0, int nc,
                                            int q)
{
    constexpr int CHUNK = 4 * LK, JN = LK / 8;
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
        const int c = c0 + i;
        if (c < nc) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int j = 0; j < JN; ++j)
                    x[i][mt][j] = *reinterpret_cast<gvec16>((mt ? arow1 : arow0) + c * CHUNK + k_of<LK, FMT>(j, q));
        }
    }
}

// int4 runs: bring the token fragments into the element order of nibbles_to_biased_bf16 and compute
// bias[i][mt] = 136 * sum over chunk i of the token row (one MFMA against all-ones per step), laid out
// like an accumulator (every column holds the row's sum).
template <int LK, int CPW, int MT, int FMT>
__device__ __forceinline__ void prepare_quant_tokens(u32x4 (&x)[CPW][MT][LK / 8], f32x4 (&bias)[CPW][MT], int c0, int nc)
{
    constexpr int JN = LK / 8;
    frag8 ones;
    ones.u = u32x4{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
        if (c0 + i < nc) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                f32x4 sum = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < JN; ++j) {
                    frag8 a;
                    a.u = x[i][mt][j];
                    sum = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, ones.v, sum, 0, 0, 0);
                    if constexpr (FMT == 1) x[i][mt][j] = interleave_halves(x[i][mt][j]);
                }
                if constexpr (FMT == 2) {
#pragma unroll
                    for (int j = 0; j + 1 < JN; j += 2) zip_fragments(x[i][mt][j], x[i][mt][j + 1]);
                }
                bias[i][mt] = sum * (FMT == 1 ? kNibbleBias : kCrumbBias);
            }
        }
    }
}

template <int LK, int CPW, int FMT, int MT>
__device__ __forceinline__ void multiply(const wstage<LK, CPW, FMT> &st, const u32x4 (&x)[CPW][MT][LK / 8],
                                         const f32x4 (&bias)[CPW][MT], uint32_t scales, int c0, int nc, f32x4 (&acc)[MT])
{
    constexpr int JN = LK / 8;
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
        if (c0 + i < nc) {
            if constexpr (FMT != 0) {
                f32x4 part[MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) part[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < JN; ++j) {
                    bf16x8 wv;
                    if constexpr (FMT == 1) wv = nibbles_to_biased_bf16(st.wq[i][j]);
                    else wv = (j & 1) ? crumbs_to_biased_bf16<1>(st.wq[i][j / 2]) : crumbs_to_biased_bf16<0>(st.wq[i][j / 2]);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        frag8 a;
                        a.u = x[i][mt][j];
                        part[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, wv, part[mt], 0, 0, 0);
                    }
                }
                // (the bf16 scales of the wavefront's chunks, two to a word: chunk 0 in the low half)
                const float scale = __uint_as_float(i == 0 ? scales << 16 : scales & 0xFFFF0000u);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) acc[mt] += (part[mt] - bias[i][mt]) * scale;
            } else {
#pragma unroll
                for (int j = 0; j < JN; ++j) {
                    frag8 wv;
                    wv.u = st.w[i][j];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        frag8 a;
                        a.u = x[i][mt][j];
                        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, wv.v, acc[mt], 0, 0, 0);
                    }
                }
            }
        }
    }
}

// what a block needs to know about the expert it is working on
struct expert_ctx {
    gbytes w0, w1;   // gate/up: the gate and up matrices; down: the down matrix twice
    gbf16 s0, s1;    // their scales (int4)
    uint32_t row_bytes; // of a weight row (a matrix is smaller than 4 GiB)
    int K;           // contraction length
    int G;           // scale groups per row
    int seg0, m;     // segment in the H/O scratch, tokens
    bool shared;
    int fmt;         // dx_fmt of the published version
    lds_ints perm_lds; // the permutation in LDS when the kernel routed itself, else null (a.perm is used)
};

// Strips.  The unit of work is a strip of 16 weight rows against all of K: for the down projection rows
// 16s .. 16s+15 of W_down (16 columns of O); for gate/up the rows 8s .. 8s+7 of W_gate as tile rows 0..7 and
// the same rows of W_up as tile rows 8..15 (8 columns of H: silu(gate) * up pairs column c with column
// c + 8 of the same accumulator).  Strips are worked through in pairs (two accumulators, one barrier and
// one finish per pair); a run of an odd number of strips ends with half a pair.
//
// Add up the partial sums of the pairs that start at strips sb, sb + 2, ... (live_groups of them, side by
// side across the wavefront groups) in a fixed order and finish the strips below h_hi:
// gate/up -> H = silu(gate) * up (bf16); down -> O (fp32 or bf16).  All threads.
// Element (group gg, tile mt, accumulator lane L, component i) is token 4*(L/16)+i, tile column L%16.
// (slot, row of O) of the output elements a thread finishes: idx = threadIdx.x + n * kThreads has the
// same idx % (MT * 256) for every n, so both are fixed for a whole run and the row lookup in the
// permutation happens once, off the critical path of the first finish.
template <bool DOWN, int MT>
__device__ __forceinline__ void finish_target(const dx_fwd_args &a, const expert_ctx &ex, int mb, int &slot, int &orow)
{
    const int rem = threadIdx.x % (MT * 256);
    const int mt = rem / 256, L = rem & 63, i = (rem >> 6) & 3;
    slot = mb * 32 + 16 * mt + 4 * (L >> 4) + i;
    orow = 0;
    if (DOWN && slot < ex.m) orow = ex.shared ? ex.seg0 + slot : a.perm[ex.seg0 + slot];
}

template <bool DOWN, int MT>
__device__ __forceinline__ void finish_batch(const dx_fwd_args &a, const expert_ctx &ex, int slot, int orow, int sb,
                                             int live_groups, int WPS, int h_hi, const float *redf)
{
    if (slot >= ex.m) return;
    for (int idx = threadIdx.x; idx < live_groups * MT * 256; idx += kThreads) {
        const int gg = idx / (MT * 256), rem = idx % (MT * 256);
        const int mt = rem / 256, L = rem & 63, i = (rem >> 6) & 3;
        // down: the thread adds up column L%16 of both strips of the pair; gate/up: column L%16 of the pair's
        // 16 columns of H lies in strip (L%16)/8, its gate sum in tile column L%8 and its up sum 8 columns on
        const int first = DOWN ? 0 : (L >> 3) & 1, second = DOWN ? 1 : first;
        const int l0 = DOWN ? L : (L & 0x37), l1 = DOWN ? L : l0 + 8;
        // the partial sums are read four wavefronts at a time before they are added (in the order of the
        // wavefronts): one LDS round trip per four instead of one each; past WPS a duplicate is read and
        // not added
        float v0 = 0.f, v1 = 0.f;
        for (int w0 = 0; w0 < WPS; w0 += 4) {
            float p0[4], p1[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int ww = w0 + u < WPS ? w0 + u : WPS - 1;
                const float *base = redf + ((gg * WPS + ww) * 4) * 64 * 4 + i;
                p0[u] = base[((first * 2 + mt) * 64 + l0) * 4];
                p1[u] = base[((second * 2 + mt) * 64 + l1) * 4];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (w0 + u < WPS) {
                    v0 += p0[u];
                    v1 += p1[u];
                }
            }
        }
        const int s0 = sb + 2 * gg; // the pair's first strip (below h_hi: the group is live)
        if constexpr (DOWN) {
            const int n = s0 * 16 + (L & 15);
            const bool both = s0 + 1 < h_hi;
            if (a.o_bf16) {
                dx_bf16 *ob = reinterpret_cast<dx_bf16 *>(a.o) + (size_t)orow * a.d + n;
                ob[0] = (dx_bf16)float_to_bf16_rne(v0);
                if (both) ob[16] = (dx_bf16)float_to_bf16_rne(v1);
            } else {
                a.o[(size_t)orow * a.d + n] = v0;
                if (both) a.o[(size_t)orow * a.d + n + 16] = v1;
            }
        } else {
            if (s0 + first < h_hi) {
                const float hv = v0 / (1.f + expf(-v0)) * v1;
                a.h[(size_t)(ex.seg0 + slot) * a.fmax + s0 * 8 + (L & 15)] = (dx_bf16)float_to_bf16_rne(hv);
            }
        }
    }
}

// One run: strips [h_lo, h_hi) of one expert for one block of up to 32 tokens (mb).
// All kThreads threads of the block execute this with identical arguments.
//
// FAST (K is one round of whole chunks: K / (4*LK) = WPS * CPW with WPS <= 8): the steady-state loop
// is straight-line code -- every iteration issues the next strip pair's loads unconditionally (the
// strip index is clamped, so the last iterations of a ragged run fetch a duplicate) -- which lets the
// compiler wait for exactly the loads it is about to use and keep the prefetch in flight.
template <int LK, int CPW, bool DOWN, int FMT, int MT, bool FAST>
__device__ __forceinline__ void run_strips(const dx_fwd_args &a, const expert_ctx &ex, int mb, int h_lo, int h_hi,
                                           f32x4 (*red)[kWaves][4][64], int &pb)
{
    constexpr int CHUNK = 4 * LK;
    // (the wavefront's index through readfirstlane: everything derived from it -- its K-part, its strips, the
    // strips' offsets in the matrices -- is then scalar arithmetic, and the loads take a scalar base plus a
    // per-lane offset that is computed once per run)
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, r = lane & 15, q = lane >> 4;
    const int nc = ex.K / CHUNK;
    // wavefronts per strip pair, strip pairs side by side, K rounds
    const int per = (nc + CPW - 1) / CPW;
    const int WPS = per < kWaves ? per : kWaves;
    const int SPP = kWaves / WPS;
    const int rounds = FAST ? 1 : (per + WPS - 1) / WPS;
    const int g = wave / WPS, kw = wave % WPS;
    const bool idle = g >= SPP;
    const int npairs = (h_hi - h_lo + 1) / 2;
    const int nbatch = (npairs + SPP - 1) / SPP;
    const int nsteps = nbatch * rounds;

    int fin_slot, fin_orow;
    finish_target<DOWN, MT>(a, ex, mb, fin_slot, fin_orow);
    auto finish = [&](int batch) {
        __syncthreads();
        const int sb = h_lo + 2 * batch * SPP;
        const int left = (h_hi - sb + 1) / 2; // pairs from sb on
        const int live_groups = left < SPP ? left : SPP;
        finish_batch<DOWN, MT>(a, ex, fin_slot, fin_orow, sb, live_groups, WPS, h_hi,
                               reinterpret_cast<const float *>(&red[pb][0][0][0]));
        pb ^= 1; // the other half of `red` is free: its readers passed the barrier above
    };

    if (idle) { // wavefronts without a K-part (8 is not a multiple of WPS) only help finishing
        for (int batch = 0; batch < nbatch; ++batch) finish(batch);
        return;
    }

    // FAST: nc counts as "unbounded" so that every chunk predicate folds away
    const int ncp = FAST ? 0x7fffffff : nc;
    u32x4 x[CPW][MT][LK / 8];
    f32x4 bias[CPW][MT];
    gbf16 arow0 = nullptr, arow1 = nullptr; // token rows of this run, looked up after the weight prologue
    auto fetch_tokens = [&](int c0) {
        load_tokens<LK, CPW, FMT, MT>(x, arow0, arow1, c0, ncp, q);
        if constexpr (FMT != 0) prepare_quant_tokens<LK, CPW, MT, FMT>(x, bias, c0, ncp);
    };

    // A step is one strip: step t = (batch * rounds + round) * 2 + b, b = 0 the first strip of the pair,
    // b = 1 the second; the last pair of a run may lack its second strip (no load, no multiply).  NST
    // register stages: the strip of step t + NST - 1 is fetched while step t is multiplied.  A quantized
    // strip is a quarter of the bytes or less, so it gets a deeper pipeline (four stages; with six or eight
    // the runs of a decode batch, a dozen steps each, spend most of their steps outside the steady loop,
    // which measured slower).
    constexpr int NST = FMT ? 4 : 2;
    const int nhalf = 2 * nsteps;
    wstage<LK, CPW, FMT> st[NST];
    const gbytes weight_rows0 = ex.w0, weight_rows1 = ex.w1;
    const uint32_t lane_row8 = (uint32_t)(r & 7) * ex.row_bytes, lane_row16 = (uint32_t)r * ex.row_bytes; // per-lane byte offsets
    // the strip of step t (past the end of the run for the missing half of the last pair and for the pairs of
    // wavefront groups without one in the last batch)
    auto strip_of = [&](int t) { return h_lo + 2 * (((t >> 1) / rounds) * SPP + g) + (t & 1); };
    // row r of a strip's tile in the weight (scale) matrices: row index and which of the two matrices
    auto issue_step = [&](int t, wstage<LK, CPW, FMT> &dst) {
        const int sr = t >> 1;
        int s = strip_of(t);
        s = s < h_hi ? s : h_hi - 1; // ragged tail: fetch a duplicate rather than branch
        const int c0 = ((sr % rounds) * WPS + kw) * CPW;
        const size_t strip_at = (size_t)((DOWN ? 16 : 8) * s) * ex.row_bytes; // scalar
        if constexpr (kLines<LK, CPW, FMT, FAST>) {
            const gbytes p_lo = weight_rows0 + strip_at + lane_row8;
            const gbytes p_hi = DOWN ? weight_rows0 + (strip_at + 8 * ex.row_bytes) + lane_row8 : weight_rows1 + strip_at + lane_row8;
            issue_weight_lines<LK, CPW, FMT>(dst, p_lo, p_hi, c0, ncp, q + 4 * (r >> 3));
        } else {
            const gbytes p = DOWN ? weight_rows0 + strip_at + lane_row16
                                  : (r < 8 ? weight_rows0 + strip_at : weight_rows1 + strip_at) + lane_row8;
            issue_weights<LK, CPW, FMT>(dst, p, c0, ncp, q);
        }
    };
    // Quantized formats: the group scales of the steps [t0, t0 + NST), one per chunk (a chunk never crosses a
    // group).  They travel apart from the weight stages, a whole loop iteration ahead and issued before that
    // iteration's weight loads: the registers they land in are carried around the loop, which costs a copy
    // at the end of every iteration, and the completion counter is in order -- a copy of a load issued
    // last would wait for every load in flight, a copy of the oldest ones waits for nothing.
    static_assert(CPW <= 2, "two chunk scales to a word");
    uint32_t sc_cur[NST], sc_next[NST];
    const gbf16 scale_rows0 = ex.s0, scale_rows1 = ex.s1;
    auto issue_scales = [&](int t0 /* even */, uint32_t (&dst)[NST]) __attribute__((always_inline)) {
        if constexpr (FMT != 0) {
#pragma unroll
            for (int u = 0; u < NST; ++u) {
                const int sr = (t0 >> 1) + (u >> 1); // step t0 + u
                int s = strip_of(t0 + u);
                s = s < h_hi ? s : h_hi - 1;
                const size_t strip_at = (size_t)((DOWN ? 16 : 8) * s) * ex.G; // scalar
                const gbf16 sp = DOWN ? scale_rows0 + strip_at + (uint32_t)(r * ex.G)
                                      : (r < 8 ? scale_rows0 + strip_at : scale_rows1 + strip_at) + (uint32_t)((r & 7) * ex.G);
                const int c0 = ((sr % rounds) * WPS + kw) * CPW;
                if (CPW == 2 && a.group == CHUNK && c0 + 1 < ncp) {
                    // the two chunks' scales are neighbours (c0 is even, a scale row starts 4-byte aligned)
                    dst[u] = *reinterpret_cast<gvec4>(sp + c0);
                } else {
                    uint32_t v = 0;
#pragma unroll
                    for (int i = 0; i < CPW; ++i)
                        if (c0 + i < ncp) v |= (uint32_t)sp[((c0 + i) * CHUNK) / a.group] << (16 * i);
                    dst[u] = v;
                }
            }
        }
    };
    auto rotate_scales = [&]() {
        if constexpr (FMT != 0) {
#pragma unroll
            for (int u = 0; u < NST; ++u) sc_cur[u] = sc_next[u];
        }
    };

    f32x4 acc[2][MT];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[b][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto do_step = [&](int t, const wstage<LK, CPW, FMT> &cur, uint32_t sc,
                       int b /* = t & 1, compile-time at every call */) {
        const int sr = t >> 1;
        const int batch = sr / rounds, rnd = sr % rounds;
        const int c0 = (rnd * WPS + kw) * CPW;
        if (rounds > 1 && b == 0) fetch_tokens(c0);
#ifdef DX_TRACE_STEPS
        if (threadIdx.x == 0 && (blockIdx.x & 63) == 37) {
            const unsigned int n = g_nsteps[DOWN][blockIdx.x >> 6]++;
            if (n < 256) g_steps[DOWN][blockIdx.x >> 6][n] = wall_clock64() | ((unsigned long long)FMT << 60) | ((unsigned long long)(t == 0) << 59);
        }
#endif
        if (strip_of(t) < h_hi) { // wavefront-uniform; a strip past the end was not fetched either, or is a duplicate
            if constexpr (kLines<LK, CPW, FMT, FAST>) multiply<LK, CPW, FMT, MT>(settle_lines<LK, CPW, FMT>(cur, c0, ncp), x, bias, sc, c0, ncp, acc[b]);
            else multiply<LK, CPW, FMT, MT>(cur, x, bias, sc, c0, ncp, acc[b]);
        }
        if (b == 0 || rnd != rounds - 1) return;
        // the strip pairs of this batch are complete: park the partial sums (zeros for a missing second strip)
        const bool live = strip_of(t - 1) < h_hi;
#pragma unroll
        for (int bb = 0; bb < 2; ++bb)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                if (live) red[pb][wave][bb * 2 + mt][lane] = acc[bb][mt];
                acc[bb][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        finish(batch);
    };

    // prologue: the first NST-1 strips (nhalf is even and >= 2) go out before anything that depends on
    // the routing arrays, so that they are in flight while the token rows are looked up
#pragma unroll
    for (int i = 0; i < NST - 1; ++i)
        if (i < nhalf && strip_of(i) < h_hi) issue_step(i, st[i]);
    issue_scales(0, sc_cur);

    // token rows of this run (A operand): row r of tile mt
    {
        gbf16 arow[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            int slot = mb * 32 + 16 * mt + r;
            slot = slot < ex.m ? slot : ex.m - 1;
            if constexpr (DOWN) {
                arow[mt] = (gbf16)a.h + (size_t)(ex.seg0 + slot) * a.fmax;
            } else {
                int tok = slot;
                if (!ex.shared) {
                    const int p = ex.perm_lds ? ex.perm_lds[ex.seg0 + slot] : a.perm[ex.seg0 + slot];
                    tok = p / a.k;
                }
                arow[mt] = (gbf16)a.x + (size_t)tok * ex.K;
            }
        }
        arow0 = arow[0];
        arow1 = arow[1];
    }
    if (rounds == 1) fetch_tokens(kw * CPW);
    int t = 0;
    // steady state: NST strips per iteration, every prefetch unconditional (NST is even, so stage i always
    // holds a strip with b = i & 1)
    for (; t + 2 * NST - 2 < nhalf; t += NST) {
        issue_scales(t + NST, sc_next);
#pragma unroll
        for (int i = 0; i < NST; ++i) {
            issue_step(t + i + NST - 1, st[(i + NST - 1) % NST]);
            do_step(t + i, st[i], sc_cur[i], i & 1);
        }
        rotate_scales();
    }
    // drain: the same, with the prefetch guarded (an unconditional prefetch of duplicates past the end of
    // the run was measured: the next run then starts behind those loads, 72.6 -> 79.1 us per C2 step)
    for (; t < nhalf; t += NST) {
        if (t + NST < nhalf) issue_scales(t + NST, sc_next);
#pragma unroll
        for (int i = 0; i < NST; ++i) {
            if (t + i < nhalf) {
                if (t + i + NST - 1 < nhalf && strip_of(t + i + NST - 1) < h_hi) issue_step(t + i + NST - 1, st[(i + NST - 1) % NST]);
                do_step(t + i, st[i], sc_cur[i], i & 1);
            }
        }
        rotate_scales();
    }
}

// LDS of the partition: per expert its tokens, its segment start and the prefix of the cost units
struct partition_lds {
    uint32_t cum[kMaxExperts + 1];
    int seg_start[kMaxExperts], seg_tokens[kMaxExperts];
    uint32_t wave_tot[kWaves];
    int wave_cnt[kWaves];
    int e_first;
};

// The partition: cost units of every expert, exclusive prefix, this block's unit range [ub0, ub1) and the
// first expert in it.  Experts above m_small tokens belong to the tiled kernels: they count as empty
// here.  All threads; ends with a barrier.
template <bool DOWN>
__device__ __forceinline__ void build_partition(const dx_fwd_args &a, partition_lds &pl, uint32_t &ub0, uint32_t &ub1)
{
    const int nE = a.E + (a.shared ? 1 : 0);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    auto tokens_of = [&](int e) {
        const int m = e == a.E ? a.T : a.offsets[e + 1] - a.offsets[e];
        return m <= a.m_small ? m : 0;
    };
    auto strips_of = [&](int e) { return DOWN ? a.d / 16 : (e == a.E ? a.shared_f : a.f) / 8; };
    auto fmt_of = [&](int e) { return e == a.E ? (uint32_t)DX_FMT_BF16 : a.table[e].fmt; };
    const int R = (nE + kThreads - 1) / kThreads; // experts per thread, consecutive
    uint32_t mine[3] = {0, 0, 0}, local = 0;
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const int e = tid * R + i;
        if (i < R && e < nE) {
            const int m = tokens_of(e);
            pl.seg_tokens[e] = m;
            pl.seg_start[e] = e == a.E ? a.T * a.k : a.offsets[e];
            if (m > 0)
                mine[i] = (uint32_t)((m + 31) / 32) * strips_of(e) * units_of<DOWN>(fmt_of(e), m) + kRunUnits<DOWN>;
            local += mine[i];
        }
    }
    const uint32_t inc = dx_route_core::wave_scan_inclusive(local);
    if (lane == 63) pl.wave_tot[wave] = inc;
    if (tid == 0) pl.e_first = nE;
    __syncthreads();
    uint32_t base = 0, U = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint32_t t = pl.wave_tot[w];
        if (w < wave) base += t;
        U += t;
    }
    uint32_t run = base + inc - local;
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const int e = tid * R + i;
        if (i < R && e < nE) {
            pl.cum[e] = run;
            run += mine[i];
        }
    }
    if (tid == 0) pl.cum[nE] = U;
    // this block's unit range (in double: exact for these sizes, no 64-bit integer division, and every
    // block evaluates the same expression for a boundary it shares)
    const double share = (double)U / (double)gridDim.x;
    ub0 = (uint32_t)(share * (double)blockIdx.x);
    ub1 = blockIdx.x + 1 == gridDim.x ? U : (uint32_t)(share * (double)(blockIdx.x + 1));
    __syncthreads();
    // the expert whose unit range contains ub0 (experts without work have empty ranges)
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const int e = tid * R + i;
        if (i < R && e < nE && pl.cum[e] <= ub0 && ub0 < pl.cum[e + 1]) pl.e_first = e;
    }
    __syncthreads();
}

// This block's share: the strips whose first unit lies in [ub0, ub1), run by run.
template <int LK, int CPW, bool DOWN, bool FAST>
__device__ __forceinline__ void run_share(const dx_fwd_args &a, const partition_lds &pl, uint32_t ub0, uint32_t ub1,
                                          lds_ints perm_lds, f32x4 (*red)[kWaves][4][64])
{
    const int nE = a.E + (a.shared ? 1 : 0);
    int pb = 0;
    if (ub0 >= ub1) return;
    for (int e = pl.e_first; e < nE && pl.cum[e] < ub1; ++e) {
        const uint32_t ue = pl.cum[e + 1] - pl.cum[e];
        if (ue == 0) continue;
        expert_ctx ex;
        ex.shared = e == a.E;
        ex.m = pl.seg_tokens[e];
        ex.seg0 = pl.seg_start[e];
        ex.perm_lds = perm_lds;
        const dx_handle hd = ex.shared ? *a.shared : a.table[e];
        ex.fmt = (int)hd.fmt;
        const int fe = ex.shared ? a.shared_f : a.f;
        ex.K = DOWN ? fe : a.d;
        ex.G = ex.K / a.group;
        ex.row_bytes = ex.fmt == DX_FMT_BF16 ? (uint32_t)ex.K * 2 : (ex.fmt == DX_FMT_INT4G ? (uint32_t)ex.K / 2 : (uint32_t)ex.K / 4);
        ex.w0 = (gbytes)(DOWN ? hd.w_down : hd.w_gate);
        ex.w1 = (gbytes)(DOWN ? hd.w_down : hd.w_up);
        ex.s0 = (gbf16)(DOWN ? hd.s_down : hd.s_gate);
        ex.s1 = (gbf16)(DOWN ? hd.s_down : hd.s_up);
        const int spe = DOWN ? a.d / 16 : fe / 8; // strips per token block of this expert
        const uint32_t wgt = units_of<DOWN>((uint32_t)ex.fmt, ex.m);
        const uint32_t lo = (ub0 > pl.cum[e] ? ub0 : pl.cum[e]) - pl.cum[e];
        const uint32_t hi = (ub1 < pl.cum[e + 1] ? ub1 : pl.cum[e + 1]) - pl.cum[e];
        // strips (flattened over token blocks) whose first unit lies in [lo, hi); strip i starts
        // kRunUnits + i * wgt units into the expert's range
        constexpr uint32_t kRun = kRunUnits<DOWN>;
        const uint32_t lo_p = lo > kRun ? lo - kRun : 0, hi_p = hi > kRun ? hi - kRun : 0;
        int i = (int)((lo_p + wgt - 1) / wgt);
        const int i1 = (int)((hi_p + wgt - 1) / wgt);
        while (i < i1) {
            const int mb = i / spe;
            const int iend = i1 < (mb + 1) * spe ? i1 : (mb + 1) * spe;
            const int s_lo = i - mb * spe, s_hi = iend - mb * spe;
            const bool two = ex.m - mb * 32 > 16;
#ifdef DX_TRACE
            if (threadIdx.x == 0 && blockIdx.x < 8192) {
                g_mix[DOWN][blockIdx.x][0] += 1;
                g_mix[DOWN][blockIdx.x][1 + (ex.fmt != DX_FMT_BF16) * 2 + two] += s_hi - s_lo;
            }
#endif
            if (ex.fmt == DX_FMT_INT4G) {
                if (two) run_strips<LK, CPW, DOWN, 1, 2, FAST>(a, ex, mb, s_lo, s_hi, red, pb);
                else run_strips<LK, CPW, DOWN, 1, 1, FAST>(a, ex, mb, s_lo, s_hi, red, pb);
            } else if (ex.fmt == DX_FMT_INT2G) {
                // (16 codes per word: the library refuses int2 handles when the group is 32, i.e. LK = 8)
                if constexpr (LK >= 16) {
                    if (two) run_strips<LK, CPW, DOWN, 2, 2, FAST>(a, ex, mb, s_lo, s_hi, red, pb);
                    else run_strips<LK, CPW, DOWN, 2, 1, FAST>(a, ex, mb, s_lo, s_hi, red, pb);
                }
            } else {
                if (two) run_strips<LK, CPW, DOWN, 0, 2, FAST>(a, ex, mb, s_lo, s_hi, red, pb);
                else run_strips<LK, CPW, DOWN, 0, 1, FAST>(a, ex, mb, s_lo, s_hi, red, pb);
            }
            i = iend;
        }
    }
}

template <int LK, int CPW, bool DOWN, bool FAST>
__global__ __launch_bounds__(kThreads) void k_stream(dx_fwd_args a)
{
    __shared__ f32x4 red[2][kWaves][4][64]; // 64 KB: partial sums, double buffered
    __shared__ partition_lds pl;
#ifdef DX_TRACE
    const unsigned long long trace_t0 = wall_clock64();
#endif
    uint32_t ub0, ub1;
    build_partition<DOWN>(a, pl, ub0, ub1);
#ifdef DX_TRACE
    const unsigned long long trace_t1 = wall_clock64();
#endif
    run_share<LK, CPW, DOWN, FAST>(a, pl, ub0, ub1, nullptr, red);
#ifdef DX_TRACE
    if (threadIdx.x == 0 && blockIdx.x < 8192) {
        g_trace[DOWN ? 1 : 0][blockIdx.x][0] = trace_t0;
        g_trace[DOWN ? 1 : 0][blockIdx.x][1] = wall_clock64();
        g_trace[DOWN ? 1 : 0][blockIdx.x][2] = ub1 - ub0;
        g_trace[DOWN ? 1 : 0][blockIdx.x][3] = trace_t1;
    }
#endif
}

// Decode batches of at most kRoutedTokens tokens and kRoutedExperts experts: the gate/up kernel routes
// by itself.  Every block repeats the small routing computation (top-k and weights per token, counts,
// offsets and the stable permutation, as dx_route.hip does them) in its prologue and keeps the result in
// LDS, so the forward pass does not wait for a routing kernel and its round trip through memory; block 0
// also writes the routing arrays out for the down and combine kernels and for the caller, and adds the
// counts to the layer's hotness counters.
// NV = logits per lane of a token's 16-lane row (E <= 16 * NV): 8 for up to 128 experts, 32 for up to 512.
// Each thread also owns EPT consecutive experts for the counts, offsets and cost units.
constexpr int kRoutedTokens = DX_ROUTED_MAX_TOKENS, kRoutedExperts = DX_ROUTED_MAX_EXPERTS, kRoutedTopK = DX_ROUTED_MAX_TOPK;

template <int LK, int CPW, int NV>
__global__ __launch_bounds__(kThreads) void k_stream_routed(dx_fwd_args a, dx_route_io r)
{
    constexpr int kE = 16 * NV;                 // experts this instance takes
    constexpr int EPT = kE >= kThreads ? 2 : 1; // experts per thread: E + shared <= kThreads * EPT
    __shared__ f32x4 red[2][kWaves][4][64];
    __shared__ partition_lds pl;
    __shared__ unsigned long long lds_mask[kE];
    __shared__ int lds_perm[kRoutedTokens * kRoutedTopK];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool writer = blockIdx.x == 0;
    const int nE = a.E + (a.shared ? 1 : 0);
    static_assert(kRoutedTokens == 2 * 4 * kWaves && kE <= kRoutedExperts && kRoutedTopK == 16,
                  "two passes of one token per 16-lane row, NV logits per lane, one selected id per lane of the row");
    static_assert(kE + 1 <= kThreads * EPT, "every expert and the shared one have a thread");
#ifdef DX_TRACE
    const unsigned long long trace_t0 = wall_clock64();
    unsigned long long trace_t1 = 0, trace_t2 = 0, trace_t3 = 0;
#endif

    for (int i = tid; i < kE; i += kThreads) lds_mask[i] = 0ull;
    unsigned long long hot_before[EPT];
    uint32_t fmt[EPT]; // of the experts tid * EPT + i
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
        const int e = tid * EPT + i;
        hot_before[i] = 0ull;
        fmt[i] = DX_FMT_BF16;
        if (writer && r.hotness && e < a.E) hot_before[i] = r.hotness[e];
        if (e < a.E) fmt[i] = a.table[e].fmt;
    }
    // ---- top-k and weights: token 32 * pass + 4 * wavefront + row (rows past T repeat the last token); the
    // second pass runs for batches of more than 32 tokens
    const int c = lane & 15, t0 = 4 * wave + (lane >> 4);
    const bool second = a.T > 32; // block-uniform
    int my_id[2] = {0, 0};
    float my_w[2] = {0.f, 0.f};
    {
        float v[2][NV];
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            if (p == 0 || second) {
                const int t = t0 + 32 * p;
                dx_route_core::load_logits_rows16<NV>(r.logits + (size_t)(t < a.T ? t : a.T - 1) * a.E, c, a.E, v[p]);
            }
        }
        __syncthreads(); // the masks are clear
#ifdef DX_TRACE
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        trace_t1 = wall_clock64();
#endif
        if constexpr (NV <= 8) {
            dx_route_core::topk_rows16<NV>(v[0], a.k, lane, my_id[0], my_w[0]);
            if (second) dx_route_core::topk_rows16<NV>(v[1], a.k, lane, my_id[1], my_w[1]);
        } else {
            // wide layers: a threshold first, then the selections over the few entries at or above it; the keys
            // pass through this wavefront's eighth of `red`, which holds nothing yet
            static_assert(sizeof(red) >= sizeof(int) * 64 * NV * kWaves, "NV * 64 words of LDS per wavefront");
            auto scratch = (__attribute__((address_space(3))) int *)&red[0][0][0][0] + wave * 64 * NV;
            dx_route_core::topk_rows16_filtered<NV, 6>(v[0], a.k, lane, my_id[0], my_w[0], scratch);
            if (second) dx_route_core::topk_rows16_filtered<NV, 6>(v[1], a.k, lane, my_id[1], my_w[1], scratch);
        }
#ifdef DX_TRACE
        trace_t2 = wall_clock64();
#endif
    }
    bool have[2]; // this lane holds pair (t, c) of the pass
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int t = t0 + 32 * p;
        have[p] = t < a.T && c < a.k;
        if (have[p]) {
            atomicOr(&lds_mask[my_id[p]], 1ull << t);
            if (writer) {
                r.ids[(size_t)t * a.k + c] = my_id[p];
                r.w[(size_t)t * a.k + c] = my_w[p];
            }
        }
    }
    __syncthreads();
    // ---- counts, offsets (exclusive scan) and the cost units of the partition, EPT consecutive experts per thread
    int cnt[EPT], m[EPT], mine[EPT], cnt_local = 0, mine_local = 0;
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
        const int e = tid * EPT + i;
        cnt[i] = m[i] = mine[i] = 0;
        if (e < a.E) cnt[i] = m[i] = __popcll(lds_mask[e]);
        else if (e == a.E && a.shared) m[i] = a.T;
        if (m[i] > 0)
            mine[i] = ((m[i] + 31) / 32) * ((e == a.E ? a.shared_f : a.f) / 8) * (int)units_of<false>(fmt[i], m[i]) +
                      (int)kRunUnits<false>;
        cnt_local += cnt[i];
        mine_local += mine[i];
    }
    const int inc = dx_route_core::wave_scan_inclusive(mine_local), cinc = dx_route_core::wave_scan_inclusive(cnt_local);
    if (lane == 63) {
        pl.wave_tot[wave] = (uint32_t)inc;
        pl.wave_cnt[wave] = cinc;
    }
    if (tid == 0) pl.e_first = nE;
    __syncthreads();
    uint32_t base = 0, U = 0;
    int cbase = 0, ctot = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint32_t tu = pl.wave_tot[w];
        const int tc = pl.wave_cnt[w];
        if (w < wave) {
            base += tu;
            cbase += tc;
        }
        U += tu;
        ctot += tc;
    }
    // this block's unit range (in double: exact for these sizes, and every block evaluates the same
    // expression for a shared boundary)
    const double share = (double)U / (double)gridDim.x;
    const uint32_t ub0 = (uint32_t)(share * (double)blockIdx.x);
    const uint32_t ub1 = blockIdx.x + 1 == gridDim.x ? U : (uint32_t)(share * (double)(blockIdx.x + 1));
    {
        int off_e = cbase + cinc - cnt_local;
        uint32_t cum_e = base + (uint32_t)(inc - mine_local);
#pragma unroll
        for (int i = 0; i < EPT; ++i) {
            const int e = tid * EPT + i;
            if (e < nE) {
                pl.cum[e] = cum_e;
                pl.seg_tokens[e] = m[i];
                pl.seg_start[e] = e == a.E ? a.T * a.k : off_e;
                if (mine[i] && cum_e <= ub0 && ub0 < cum_e + (uint32_t)mine[i]) pl.e_first = e;
            }
            if (writer && e < a.E) {
                r.counts[e] = cnt[i];
                r.offsets[e] = off_e;
                if (r.hotness) r.hotness[e] = hot_before[i] + (unsigned long long)cnt[i];
            }
            off_e += cnt[i];
            cum_e += (uint32_t)mine[i];
        }
    }
    if (tid == 0) {
        pl.cum[nE] = U;
        if (writer) r.offsets[a.E] = ctot;
    }
    __syncthreads();
    // ---- the permutation: the rank of pair (t, c) inside its segment = tokens below t that chose the expert
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        if (have[p]) {
            const int t = t0 + 32 * p;
            const unsigned long long below = lds_mask[my_id[p]] & ((1ull << t) - 1ull);
            const int at = pl.seg_start[my_id[p]] + __popcll(below);
            lds_perm[at] = t * a.k + c;
            if (writer) r.perm[at] = t * a.k + c;
        }
    }
    __syncthreads();
#ifdef DX_TRACE
    trace_t3 = wall_clock64();
#endif
    run_share<LK, CPW, false, true>(a, pl, ub0, ub1, (lds_ints)lds_perm, red);
#ifdef DX_TRACE
    if (threadIdx.x == 0 && blockIdx.x < 8192) {
        g_trace[0][blockIdx.x][0] = trace_t0;
        g_trace[0][blockIdx.x][1] = wall_clock64();
        g_trace[0][blockIdx.x][2] = trace_t1 - trace_t0 + ((trace_t2 - trace_t1) << 20) + ((trace_t3 - trace_t2) << 40);
        g_trace[0][blockIdx.x][3] = trace_t3;
    }
#endif
}

// ---- combine: y[t] = sum_j w[t,j] * O[t*k+j] (+ O[T*k+t] of the shared expert) ----------
// The rows are fetched eight at a time before they are added (in the order of j), so that a thread has
// its loads in flight together instead of one round trip per row.
__global__ __launch_bounds__(256) void k_combine(dx_fwd_args a)
{
    const int t = blockIdx.y;
    const int c = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (c >= a.d) return;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float4 sh = make_float4(0.f, 0.f, 0.f, 0.f);
    if (a.shared) sh = *reinterpret_cast<const float4 *>(a.o + ((size_t)a.T * a.k + t) * a.d + c);
    for (int j0 = 0; j0 < a.k; j0 += 8) {
        float4 o[8];
        float wj[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int j = j0 + u < a.k ? j0 + u : a.k - 1; // past the end: a duplicate that is not added
            wj[u] = a.w[(size_t)t * a.k + j];
            o[u] = *reinterpret_cast<const float4 *>(a.o + ((size_t)t * a.k + j) * a.d + c);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (j0 + u < a.k) {
                acc.x += wj[u] * o[u].x; acc.y += wj[u] * o[u].y; acc.z += wj[u] * o[u].z; acc.w += wj[u] * o[u].w;
            }
        }
    }
    if (a.shared) {
        acc.x += sh.x; acc.y += sh.y; acc.z += sh.z; acc.w += sh.w;
    }
    uint2 out;
    out.x = float_to_bf16_rne(acc.x) | (float_to_bf16_rne(acc.y) << 16);
    out.y = float_to_bf16_rne(acc.z) | (float_to_bf16_rne(acc.w) << 16);
    *reinterpret_cast<uint2 *>(a.y + (size_t)t * a.d + c) = out;
}

// the same with bf16 O rows: 8 columns per thread
__global__ __launch_bounds__(256) void k_combine_bf16(dx_fwd_args a)
{
    const int t = blockIdx.y;
    const int c = (blockIdx.x * 256 + threadIdx.x) * 8;
    if (c >= a.d) return;
    const dx_bf16 *ob = reinterpret_cast<const dx_bf16 *>(a.o);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    auto add_row = [&](const uint4 &o, float wj) {
        const uint32_t p[4] = {o.x, o.y, o.z, o.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[2 * i] += wj * __uint_as_float(p[i] << 16);
            acc[2 * i + 1] += wj * __uint_as_float(p[i] & 0xFFFF0000u);
        }
    };
    uint4 sh = make_uint4(0u, 0u, 0u, 0u);
    if (a.shared) sh = *reinterpret_cast<const uint4 *>(ob + ((size_t)a.T * a.k + t) * a.d + c);
    for (int j0 = 0; j0 < a.k; j0 += 8) { // eight rows in flight, added in the order of j
        uint4 o[8];
        float wj[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int j = j0 + u < a.k ? j0 + u : a.k - 1;
            wj[u] = a.w[(size_t)t * a.k + j];
            o[u] = *reinterpret_cast<const uint4 *>(ob + ((size_t)t * a.k + j) * a.d + c);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (j0 + u < a.k) add_row(o[u], wj[u]);
    }
    if (a.shared) add_row(sh, 1.f);
    uint4 out;
    out.x = float_to_bf16_rne(acc[0]) | (float_to_bf16_rne(acc[1]) << 16);
    out.y = float_to_bf16_rne(acc[2]) | (float_to_bf16_rne(acc[3]) << 16);
    out.z = float_to_bf16_rne(acc[4]) | (float_to_bf16_rne(acc[5]) << 16);
    out.w = float_to_bf16_rne(acc[6]) | (float_to_bf16_rne(acc[7]) << 16);
    *reinterpret_cast<uint4 *>(a.y + (size_t)t * a.d + c) = out;
}

// Chunks per wavefront for a contraction of nc chunks: the fast path needs nc = WPS * CPW with
// WPS <= 8 wavefronts; prefer the split that leaves the fewest of the 8 wavefronts without a K-part.
struct split_choice {
    int cpw;
    bool fast;
};

split_choice pick_split(int nc_a, int nc_b)
{
    int best = 0, best_busy = -1;
    for (int cpw = 1; cpw <= 2; ++cpw) {
        bool ok = true;
        int busy = kWaves;
        for (int nc : {nc_a, nc_b}) {
            if (nc % cpw || nc / cpw > kWaves) ok = false;
            else {
                const int wps = nc / cpw;
                busy = busy < (kWaves / wps) * wps ? busy : (kWaves / wps) * wps;
            }
        }
        if (ok && busy >= best_busy) { // ties go to the larger cpw: more bytes in flight per wavefront
            best = cpw;
            best_busy = busy;
        }
    }
    if (best) return {best, true};
    return {2, false};
}

// A launch, optionally with events that take the start and stop time stamps of the kernel's own dispatch
// (HIP's extended launch): the duration they give is the kernel's, with no event packets inside it.
template <typename... Args>
void launch(void (*kernel)(Args...), dim3 grid, dim3 block, hipStream_t s, hipEvent_t start, hipEvent_t stop, Args... args)
{
    if (start || stop) hipExtLaunchKernelGGL(kernel, grid, block, 0, s, start, stop, 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, 0, s, args...);
}

template <int LK, bool DOWN>
void launch_stream(const dx_fwd_args &a, split_choice c, dim3 grid, hipStream_t s, hipEvent_t start = nullptr,
                   hipEvent_t stop = nullptr)
{
    const dim3 block(kThreads);
    if (c.fast) {
        if (c.cpw == 2) launch(k_stream<LK, 2, DOWN, true>, grid, block, s, start, stop, a);
        else launch(k_stream<LK, 1, DOWN, true>, grid, block, s, start, stop, a);
    } else {
        launch(k_stream<LK, 2, DOWN, false>, grid, block, s, start, stop, a);
    }
}

// Up to this many tokens per call the streaming kernels alone are faster than the three-chain prefill
// pass (measured on the 30B-shaped layer: 140 us against 171 us at T = 128, equal at T = 256).
constexpr int kStreamOnlyTokens = 128;

// r: null, or the routing inputs and outputs of a call that asks the gate/up kernel to route; *routed
// then tells whether it did (if not, nothing has been launched).
template <int LK>
hipError_t launch_all(const dx_fwd_args &a_in, int n_cu, hipStream_t s, const dx_fwd_streams *side, dx_marks *mk,
                      const dx_route_io *r, bool *routed)
{
    constexpr int CHUNK = 4 * LK;
    dx_fwd_args a = a_in;
    // Few tokens per call (decode): the streaming kernels take every expert.  Otherwise experts above
    // 32 tokens go to the tiled MFMA kernels (when the shapes fit their tiles).
    const bool tiles_fit = a.d % 128 == 0 && a.f % 64 == 0 && (!a.shared || a.shared_f % 64 == 0);
    const bool mixed = a.T > kStreamOnlyTokens && tiles_fit;
    a.m_small = mixed ? 32 : 0x7fffffff;
    // the 256 x 256 kernel addresses rows with 32-bit byte offsets from the matrix base
    const uint64_t span_x = (uint64_t)a.T * a.d * 2, span_h = (uint64_t)a.T * (a.k + 1) * a.fmax * 2;
    const bool big_fit = a.d % 256 == 0 && a.f % 128 == 0 && (!a.shared || a.shared_f % 128 == 0) &&
                         span_x < (1ull << 32) && span_h < (1ull << 32) && (uint64_t)a.d * a.fmax * 2 < (1ull << 32);
    a.m_big = mixed && big_fit ? 256 : 0;
    // its int4 path reads a row's scales as aligned pairs: an even number of groups along both contractions
    a.big_int4 = a.m_big && (a.d / a.group) % 2 == 0 && (a.f / a.group) % 2 == 0;
    a.o_bf16 = mixed; // d % 128 == 0 there, so rows split into 8-column pieces
    const split_choice gu = pick_split(a.d / CHUNK, a.d / CHUNK);
    const split_choice dn = pick_split(a.f / CHUNK, (a.shared ? a.shared_f : a.f) / CHUNK);
    if (r) {
        *routed = !mixed && gu.fast && a.T >= 1 && a.T <= kRoutedTokens && a.E <= kRoutedExperts && a.k <= kRoutedTopK;
        if (!*routed) return hipSuccess;
    }
    hipEvent_t *marks = mk ? mk->ev : nullptr;
    hipEvent_t combine_start = nullptr, combine_stop = nullptr;
    if (mk) mk->per_kernel = !mixed;
    if (!mixed) {
        // profiled: every kernel's own start and stop stamps
        const dim3 grid(n_cu);
        hipEvent_t ev[8] = {};
        if (marks)
            for (int i = 0; i < 8; ++i) ev[i] = marks[i];
        if (r && a.E <= 128) {
            if (gu.cpw == 2) launch(k_stream_routed<LK, 2, 8>, grid, dim3(kThreads), s, ev[0], ev[1], a, *r);
            else launch(k_stream_routed<LK, 1, 8>, grid, dim3(kThreads), s, ev[0], ev[1], a, *r);
        } else if (r) {
            if (gu.cpw == 2) launch(k_stream_routed<LK, 2, 32>, grid, dim3(kThreads), s, ev[0], ev[1], a, *r);
            else launch(k_stream_routed<LK, 1, 32>, grid, dim3(kThreads), s, ev[0], ev[1], a, *r);
        } else {
            launch_stream<LK, false>(a, gu, grid, s, ev[0], ev[1]);
        }
        launch_stream<LK, true>(a, dn, grid, s, ev[5], ev[2]);
        combine_start = ev[6];
        combine_stop = ev[3];
    } else if (!side) {
        const dim3 grid(n_cu);
        launch_stream<LK, false>(a, gu, grid, s);
        launch_stream<LK, true>(a, dn, grid, s);
        if (marks) (void)hipEventRecord(marks[0], s);
        const hipError_t e = dxk_moe_forward_tiled(a, s, s, marks ? &marks[1] : nullptr);
        if (e != hipSuccess) return e;
        if (marks) (void)hipEventRecord(marks[2], s);
    } else {
        // Three chains on three streams.  The streamed experts are bound by memory, the tiles by the
        // matrix cores, and the tail of each tiled grid leaves compute units idle: run together they
        // fill each other's gaps.  Once the tiles carry most of the work the streaming grid shrinks to
        // a quarter of the chip, so that the 256-row tile kernel (whose LDS footprint does not share a
        // compute unit with it) keeps the rest; measured better from a mean segment of 256 tokens up.
        hipError_t e;
        if ((e = hipEventRecord(side->fork, s)) != hipSuccess) return e;
        for (int i = 0; i < 2; ++i)
            if ((e = hipStreamWaitEvent(side->aux[i], side->fork, 0)) != hipSuccess) return e;
        if (marks) (void)hipEventRecord(marks[0], s);
        hipStream_t s_tiled = a.m_big ? side->aux[1] : s;
        if ((e = dxk_moe_forward_tiled(a, s, s_tiled, marks ? &marks[1] : nullptr)) != hipSuccess) return e;
        if (marks) (void)hipEventRecord(marks[2], s);
        const bool tiles_dominate = (long)a.T * a.k >= 256L * a.E; // mean segment of 256 tokens or more
        const dim3 grid(tiles_dominate && n_cu >= 8 ? n_cu / 4 : n_cu);
        launch_stream<LK, false>(a, gu, grid, side->aux[0]);
        launch_stream<LK, true>(a, dn, grid, side->aux[0]);
        for (int i = 0; i < 2; ++i) {
            if ((e = hipEventRecord(side->join[i], side->aux[i])) != hipSuccess) return e;
            if ((e = hipStreamWaitEvent(s, side->join[i], 0)) != hipSuccess) return e;
        }
    }
    if (a.o_bf16) {
        launch(k_combine_bf16, dim3((a.d / 8 + 255) / 256, a.T), dim3(256), s, combine_start, combine_stop, a);
    } else {
        launch(k_combine, dim3((a.d / 4 + 255) / 256, a.T), dim3(256), s, combine_start, combine_stop, a);
    }
    if (marks) {
        if (!combine_stop) (void)hipEventRecord(marks[3], s);
        (void)hipEventRecord(marks[7], s); // two records back to back: the cost of an event pair itself
        (void)hipEventRecord(marks[4], s);
    }
    return hipGetLastError();
}

} // namespace

#ifdef DX_TRACE
extern "C" int dx_debug_read_trace(void *dst, size_t bytes)
{
    return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(g_trace), bytes, 0, hipMemcpyDeviceToHost);
}
extern "C" int dx_debug_read_mix(void *dst) // reads and clears
{
    int rc = (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(g_mix), sizeof(unsigned int) * 2 * 8192 * 8, 0, hipMemcpyDeviceToHost);
    void *p = nullptr;
    rc |= (int)hipGetSymbolAddress(&p, HIP_SYMBOL(g_mix));
    if (p) rc |= (int)hipMemset(p, 0, sizeof(unsigned int) * 2 * 8192 * 8);
    return rc;
}
extern "C" int dx_debug_read_steps(void *dst, void *counts)
{
    unsigned int zero[2][4] = {};
    int rc = (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(g_steps), sizeof(unsigned long long) * 2 * 4 * 256, 0, hipMemcpyDeviceToHost);
    rc |= (int)hipMemcpyFromSymbol(counts, HIP_SYMBOL(g_nsteps), sizeof zero, 0, hipMemcpyDeviceToHost);
    rc |= (int)hipMemcpyToSymbol(HIP_SYMBOL(g_nsteps), zero, sizeof zero, 0, hipMemcpyHostToDevice);
    return rc;
}
#endif

hipError_t dxk_moe_forward(const dx_fwd_args &a, int n_cu, hipStream_t s, const dx_fwd_streams *side, dx_marks *marks)
{
    if (a.T == 0) return hipSuccess;
    // K-chunk = min(group, 128) so that a chunk never crosses a quantization group
    if (a.group >= 128) return launch_all<32>(a, n_cu, s, side, marks, nullptr, nullptr);
    if (a.group == 64) return launch_all<16>(a, n_cu, s, side, marks, nullptr, nullptr);
    return launch_all<8>(a, n_cu, s, side, marks, nullptr, nullptr);
}

hipError_t dxk_route_forward(const dx_fwd_args &a, const dx_route_io &r, int n_cu, hipStream_t s, dx_marks *marks,
                             bool *routed)
{
    *routed = false;
    if (a.T == 0) return hipSuccess;
    if (a.group >= 128) return launch_all<32>(a, n_cu, s, nullptr, marks, &r, routed);
    if (a.group == 64) return launch_all<16>(a, n_cu, s, nullptr, marks, &r, routed);
    return launch_all<8>(a, n_cu, s, nullptr, marks, &r, routed);
}
