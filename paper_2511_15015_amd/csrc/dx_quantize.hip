// Demotion quantizer: bf16 [rows,K] -> symmetric group-wise int4 + bf16 scales.
//
// The paper prepares the low-precision version offline (Sec. 4,
// Implementation) and names no quantizer; the format here is: groups of
// `group` consecutive elements along K, scale = bf16_rne(absmax / 7) computed
// in fp32, q = clamp(rint(w / scale), -8, 7) with an IEEE fp32 divide and
// round-half-to-even, two's-complement nibbles, element 2i in the low nibble.
//
// HBM-bound: every thread reads 8 consecutive bf16 (one 128-bit load) and
// writes one 32-bit word of nibbles; the group's absmax is a shuffle
// reduction over the group/8 neighbouring lanes.  Built without fast-math so
// that the divide stays correctly rounded.
#include "dx_internal.h"

namespace {

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ uint32_t float_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u); // finite inputs only
    return u >> 16;
}

// BITS = 4: the format above.  BITS = 2: the same rule with its constants moved to two bits (the low
// tier of the int4 / int2 precision pair): scale = bf16_rne(absmax / 1), q = clamp(rint(w / scale), -2, 1),
// element 4i in the two low bits of byte i; a thread's 8 codes are one 16-bit store.
template <int LANES, int BITS> // lanes per group = group / 8
__global__ __launch_bounds__(256) void k_quantize(const uint4 *__restrict__ w, size_t n_vec, int vec_per_group_row,
                                                  void *__restrict__ q, dx_bf16 *__restrict__ sc)
{
    constexpr float kQMax = BITS == 4 ? 7.f : 1.f, kQMin = BITS == 4 ? -8.f : -2.f;
    constexpr uint32_t kMask = (1u << BITS) - 1u;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const bool live = i < n_vec;
    uint4 raw = make_uint4(0, 0, 0, 0);
    if (live) raw = w[i];
    float v[8];
    v[0] = bf16_bits_to_float(raw.x & 0xFFFFu);
    v[1] = bf16_bits_to_float(raw.x >> 16);
    v[2] = bf16_bits_to_float(raw.y & 0xFFFFu);
    v[3] = bf16_bits_to_float(raw.y >> 16);
    v[4] = bf16_bits_to_float(raw.z & 0xFFFFu);
    v[5] = bf16_bits_to_float(raw.z >> 16);
    v[6] = bf16_bits_to_float(raw.w & 0xFFFFu);
    v[7] = bf16_bits_to_float(raw.w >> 16);
    float amax = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf(v[j]));
#pragma unroll
    for (int off = 1; off < LANES; off <<= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
    const uint32_t sbits = float_to_bf16_rne(amax / kQMax);
    const float s = bf16_bits_to_float(sbits);
    uint32_t packed = 0;
    if (s != 0.f) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float r = rintf(v[j] / s);
            r = fminf(fmaxf(r, kQMin), kQMax);
            packed |= ((uint32_t)(int)r & kMask) << (BITS * j);
        }
    }
    if (live) {
        if constexpr (BITS == 4) static_cast<uint32_t *>(q)[i] = packed;
        else static_cast<uint16_t *>(q)[i] = (uint16_t)packed;
        if ((i % LANES) == 0) sc[i / LANES] = (dx_bf16)sbits;
    }
    (void)vec_per_group_row;
}

template <int BITS>
hipError_t launch_quantize(const dx_bf16 *w, int rows, int K, int group, uint8_t *q, dx_bf16 *sc, hipStream_t s)
{
    const size_t n_vec = (size_t)rows * K / 8;
    if (n_vec == 0) return hipSuccess;
    const dim3 grid((unsigned)((n_vec + 255) / 256)), block(256);
    const uint4 *wv = reinterpret_cast<const uint4 *>(w);
    switch (group / 8) {
    case 4: hipLaunchKernelGGL((k_quantize<4, BITS>), grid, block, 0, s, wv, n_vec, 0, q, sc); break;
    case 8: hipLaunchKernelGGL((k_quantize<8, BITS>), grid, block, 0, s, wv, n_vec, 0, q, sc); break;
    case 16: hipLaunchKernelGGL((k_quantize<16, BITS>), grid, block, 0, s, wv, n_vec, 0, q, sc); break;
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
