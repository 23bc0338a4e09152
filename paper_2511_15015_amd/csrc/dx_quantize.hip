// Demotion quantizer: bf16 [rows,K] -> symmetric group-wise int4 + bf16 scales.
//
// The paper prepares the low-precision version offline (Sec. 4,
// Implementation) and names no quantizer; the format here is: groups of
// `group` consecutive elements along K, scale = bf16_rne(absmax / 7) computed
// in fp32, q = clamp(rint(w / scale), -8, 7) with an IEEE fp32 divide and
// round-half-to-even, two's-complement nibbles, element 2i in the low nibble.
//
// Every thread handles UNR vectors of 8 consecutive bf16 (128-bit non-temporal loads, all issued before any
// is used) and writes one 32-bit (16-bit) word of codes per vector; a group's absmax is a DPP reduction
// over its group/8 neighbouring lanes.  At HBM speed the kernel has a budget of roughly a hundred vector
// instructions per 16 input bytes, and a correctly rounded fp32 divide per element alone takes more than
// that, so the codes come from an exact shortcut instead (see quantize_vector): the divide stays only in
// the scale, once per vector, and in a fall-back for scales outside the shortcut's range.  Built without
// fast-math.
#include "dx_internal.h"

namespace {

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ uint32_t float_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u); // finite inputs only
    return u >> 16;
}

template <int CTRL>
__device__ __forceinline__ float dpp_max(float x)
{
    return fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x), CTRL, 0xF, 0xF, false)));
}

// Codes of one vector of 8 bf16 values against the group scale s (a bf16 value), packed BITS bits each,
// element 0 lowest.  The rule is q = rint(w / s) with an IEEE fp32 divide and round-half-to-even.
// Shortcut: w and s carry 8 significant bits each and |w / s| < 8, so the exact quotient is either exactly
// half-way between two integers or at least 2^-11 away from any half-way point; the correctly rounded
// fp32 quotient (error 2^-24 relative) and w * rcp(s) (error below 2^-22 relative) therefore round to
// the same integer as the exact quotient unless it is an exact tie.  t = fma(w, rcp(s), 1.5 * 2^23) rounds
// to that integer in one step, the integer sits in the low bits of t's bit pattern (two's complement), and
// the residual e = w - q * s is exact in fp32: |e| == s / 2 marks the ties, which go to the even neighbour.
// BITS = 2 (the low tier of the int4 / int2 pair) uses the same rule with q in [-2, 1].
template <int BITS>
__device__ __forceinline__ uint32_t quantize_vector(const float (&v)[8], float s)
{
    constexpr float kMagic = 12582912.f; // 1.5 * 2^23: ulp 1, room for negative integers below it
    constexpr float kQMax = BITS == 4 ? 7.f : 1.f, kQMin = BITS == 4 ? -8.f : -2.f;
    constexpr uint32_t kMask = (1u << BITS) - 1u;
    uint32_t packed = 0;
    const bool fast = s >= 0x1p-100f && s <= 0x1p100f; // rcp(s) and the products below stay normal numbers
    const float inv = __builtin_amdgcn_rcpf(s), half = 0.5f * s;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float t = fmaf(v[j], inv, kMagic);
        const float qf = t - kMagic;
        const float e = fmaf(-qf, s, v[j]);
        uint32_t bits = __float_as_uint(t);
        const bool tie = fabsf(e) == half;
        if (__ballot(tie) != 0ull) { // rare: some lane of the wavefront sits on an exact tie
            if (tie && (bits & 1u)) bits += e > 0.f ? 1u : 0xFFFFFFFFu;
        }
        packed = __builtin_amdgcn_alignbit(bits, packed, BITS); // the new code enters at the top
    }
    if (BITS == 2) packed >>= 16;
    if (__ballot(!fast) != 0ull) { // a scale of zero or outside the shortcut's range: the rule as written
        if (!fast) {
            packed = 0;
            if (s != 0.f) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    float r = rintf(v[j] / s);
                    r = fminf(fmaxf(r, kQMin), kQMax);
                    packed |= ((uint32_t)(int)r & kMask) << (BITS * j);
                }
            }
        }
    }
    return packed;
}

// BITS = 4: scale = bf16_rne(absmax / 7), q = clamp(rint(w / scale), -8, 7), element 2i in the low nibble of
// byte i.  BITS = 2: scale = bf16_rne(absmax / 1), q = clamp(rint(w / scale), -2, 1), element 4i in the two
// low bits of byte i; a thread's 8 codes are one 16-bit store.  (|w / scale| <= 7 (1 + 2^-8) resp. 1, so
// the clamp never acts on finite inputs; the fall-back keeps it.)
template <int LANES, int BITS, int UNR> // lanes per group = group / 8
__global__ __launch_bounds__(256) void k_quantize(const uint4 *__restrict__ w, size_t n_vec, void *__restrict__ q,
                                                  dx_bf16 *__restrict__ sc)
{
    constexpr float kQMax = BITS == 4 ? 7.f : 1.f;
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
    const size_t first = (size_t)blockIdx.x * (UNR * 256) + threadIdx.x;
    u32x4 raw[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        const size_t i = first + (size_t)u * 256;
        raw[u] = u32x4{0u, 0u, 0u, 0u};
        if (i < n_vec) raw[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(w) + i);
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        const size_t i = first + (size_t)u * 256;
        float v[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v[2 * j] = bf16_bits_to_float(raw[u][j] & 0xFFFFu);
            v[2 * j + 1] = __uint_as_float(raw[u][j] & 0xFFFF0000u);
        }
        float amax = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf(v[j]));
        // the group's lanes are neighbours inside one 16-lane row (a tile starts on a multiple of 256 vectors)
        amax = dpp_max<0xB1>(amax);                        // quad_perm [1,0,3,2]
        amax = dpp_max<0x4E>(amax);                        // quad_perm [2,3,0,1]
        if constexpr (LANES >= 8) amax = dpp_max<0x141>(amax);  // row_half_mirror
        if constexpr (LANES >= 16) amax = dpp_max<0x140>(amax); // row_mirror
        const uint32_t sbits = float_to_bf16_rne(amax / kQMax);
        const uint32_t packed = quantize_vector<BITS>(v, bf16_bits_to_float(sbits));
        if (i < n_vec) {
            if constexpr (BITS == 4) __builtin_nontemporal_store(packed, static_cast<uint32_t *>(q) + i);
            else __builtin_nontemporal_store((uint16_t)packed, static_cast<uint16_t *>(q) + i);
            if ((i % LANES) == 0) sc[i / LANES] = (dx_bf16)sbits;
        }
    }
}

template <int BITS>
hipError_t launch_quantize(const dx_bf16 *w, int rows, int K, int group, uint8_t *q, dx_bf16 *sc, hipStream_t s)
{
    constexpr int UNR = 4;
    const size_t n_vec = (size_t)rows * K / 8;
    if (n_vec == 0) return hipSuccess;
    const dim3 grid((unsigned)((n_vec + UNR * 256 - 1) / (UNR * 256))), block(256);
    const uint4 *wv = reinterpret_cast<const uint4 *>(w);
    switch (group / 8) {
    case 4: hipLaunchKernelGGL((k_quantize<4, BITS, UNR>), grid, block, 0, s, wv, n_vec, q, sc); break;
    case 8: hipLaunchKernelGGL((k_quantize<8, BITS, UNR>), grid, block, 0, s, wv, n_vec, q, sc); break;
    case 16: hipLaunchKernelGGL((k_quantize<16, BITS, UNR>), grid, block, 0, s, wv, n_vec, q, sc); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

} // namespace

hipError_t dxk_quantize(const dx_bf16 *w, int rows, int K, int group, uint8_t *q, dx_bf16 *sc, hipStream_t s)
{
    return launch_quantize<4>(w, rows, K, group, q, sc, s);
}

hipError_t dxk_quantize2(const dx_bf16 *w, int rows, int K, int group, uint8_t *q, dx_bf16 *sc, hipStream_t s)
{
    return launch_quantize<2>(w, rows, K, group, q, sc, s);
}
