// Device code of the router's top-k, shared by the route kernel and by the decode kernel that routes in
// its own prologue: both must pick the same ids and compute the same weights, bit for bit.
//
// Paper: Sec. 2.1 / 3.1 (the router scores the experts per token and the top-k of them run).
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

namespace dx_route_core {

// Wave-wide max / sum in six DPP steps (no LDS round trips).  Lane 63 ends up with the reduction over
// all 64 lanes and is read back as a scalar.
template <int CTRL, int ROW_MASK, bool BOUND>
__device__ __forceinline__ float dpp_move(float old, float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(x), CTRL, ROW_MASK, 0xF, BOUND));
}

__device__ __forceinline__ float wave_max(float x)
{
    x = fmaxf(x, dpp_move<0xB1, 0xF, false>(x, x));  // quad_perm [1,0,3,2]
    x = fmaxf(x, dpp_move<0x4E, 0xF, false>(x, x));  // quad_perm [2,3,0,1]
    x = fmaxf(x, dpp_move<0x141, 0xF, false>(x, x)); // row_half_mirror
    x = fmaxf(x, dpp_move<0x140, 0xF, false>(x, x)); // row_mirror: every 16-lane row is uniform now
    x = fmaxf(x, dpp_move<0x142, 0xA, false>(x, x)); // row_bcast:15 into rows 1 and 3
    x = fmaxf(x, dpp_move<0x143, 0xC, false>(x, x)); // row_bcast:31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

__device__ __forceinline__ float wave_sum(float x)
{
    // inclusive scan inside each row by shifts (lanes shifted in from outside the row contribute 0) ...
    x += dpp_move<0x111, 0xF, true>(0.f, x); // row_shr:1
    x += dpp_move<0x112, 0xF, true>(0.f, x); // row_shr:2
    x += dpp_move<0x114, 0xF, true>(0.f, x); // row_shr:4
    x += dpp_move<0x118, 0xF, true>(0.f, x); // row_shr:8 -> lane 15 of every row holds the row's sum
    // ... then the row sums travel to lane 63
    x += dpp_move<0x142, 0xA, false>(0.f, x); // row_bcast:15 into rows 1 and 3
    x += dpp_move<0x143, 0xC, false>(0.f, x); // row_bcast:31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

// Top-k ids and routing weights of NT token rows by one wavefront.  v[i][s] is the logit of expert
// NV*lane + s of row i (-inf past the last expert); it is consumed.  On return lane j < k holds the
// j-th id of row i (descending logit, ties to the lower index) in id[i] and its weight, the softmax over
// the k selected logits, in wt[i].
// One selection: every lane finds its own largest entry (the lowest slot among equals), the wave maximum
// of those is the winner's logit, the lowest lane that holds it is the winner (experts ascend with the
// lane and the slot, so this is the lowest index), and that lane retires the entry.
template <int NV, int NT>
__device__ __forceinline__ void topk_rows(float (&v)[NT][NV], int k, int lane, int (&id)[NT], float (&wt)[NT])
{
    float lg[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        id[i] = 0;
        lg[i] = -INFINITY;
    }
    for (int j = 0; j < k; ++j) {
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            float best = v[i][0];
            int slot = 0;
#pragma unroll
            for (int s = 1; s < NV; ++s)
                if (v[i][s] > best) {
                    best = v[i][s];
                    slot = s;
                }
            const float top = wave_max(best);
            const unsigned long long holders = __ballot(best == top); // never empty: top is some lane's best
            const int win = __builtin_ctzll(holders);
            const int wslot = __builtin_amdgcn_readlane(slot, win);
#pragma unroll
            for (int s = 0; s < NV; ++s)
                if (lane == win && s == wslot) v[i][s] = -INFINITY;
            if (lane == j) {
                id[i] = NV * win + wslot;
                lg[i] = top;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        const float top0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(lg[i]), 0));
        const float ex = lane < k ? expf(lg[i] - top0) : 0.f;
        const float sum = wave_sum(ex);
        wt[i] = ex / sum;
    }
}

// Inclusive prefix sum over the 64 lanes in six DPP steps (the scan inside wave_sum, for integers).
__device__ __forceinline__ int wave_scan_inclusive(int x)
{
    x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xF, 0xF, true); // row_shr:1 (zero from outside the row)
    x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xF, 0xF, true); // row_shr:2
    x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xF, 0xF, true); // row_shr:4
    x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xF, 0xF, true); // row_shr:8
    x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xA, 0xF, false); // row_bcast:15 into rows 1 and 3
    x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xC, 0xF, false); // row_bcast:31 into rows 2 and 3
    return x;
}

__device__ __forceinline__ uint32_t wave_scan_inclusive(uint32_t x) // the same, modulo 2^32
{
    auto shifted = [](uint32_t v, auto ctrl, auto row_mask, auto bound) {
        return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, decltype(ctrl)::value, decltype(row_mask)::value, 0xF,
                                                     decltype(bound)::value);
    };
    using std::integral_constant;
    x += shifted(x, integral_constant<int, 0x111>{}, integral_constant<int, 0xF>{}, integral_constant<bool, true>{});
    x += shifted(x, integral_constant<int, 0x112>{}, integral_constant<int, 0xF>{}, integral_constant<bool, true>{});
    x += shifted(x, integral_constant<int, 0x114>{}, integral_constant<int, 0xF>{}, integral_constant<bool, true>{});
    x += shifted(x, integral_constant<int, 0x118>{}, integral_constant<int, 0xF>{}, integral_constant<bool, true>{});
    x += shifted(x, integral_constant<int, 0x142>{}, integral_constant<int, 0xA>{}, integral_constant<bool, false>{});
    x += shifted(x, integral_constant<int, 0x143>{}, integral_constant<int, 0xC>{}, integral_constant<bool, false>{});
    return x;
}

// Four token rows per wavefront, one per 16-lane row, so that one instruction stream serves all four:
// lane c of a row owns the experts NV*c .. NV*c+NV-1 of its token (E <= 16*NV), v[s] is the logit of expert
// NV*c+s (-inf past the last expert) and is consumed.  Same results as topk_rows: on return lane c < k of
// a row holds the c-th id of its token and its weight (k <= 16).  The weights add up in the order of
// wave_sum (a 16-lane row scan), so they are the same bits.
template <int NV>
__device__ __forceinline__ void topk_rows16(float (&v)[NV], int k, int lane, int &id, float &wt)
{
    const int c = lane & 15;
    // Order-preserving integer keys (x + 0 turns -0 into +0, so equal logits have equal keys): integer
    // max / compare, no NaN handling in the way.  A taken entry gets the lowest key, below -inf's.
    int key[NV];
#pragma unroll
    for (int s = 0; s < NV; ++s) {
        const int b = __float_as_int(v[s] + 0.f);
        key[s] = b ^ ((b >> 31) & 0x7fffffff);
    }
    constexpr int kTaken = (int)0x80000000;
    id = 0;
    int lgk = kTaken;
    for (int j = 0; j < k; ++j) {
        int top = key[0];
#pragma unroll
        for (int s = 1; s < NV; ++s) top = max(top, key[s]);
        top = max(top, __builtin_amdgcn_mov_dpp(top, 0xB1, 0xF, 0xF, false));  // quad_perm [1,0,3,2]
        top = max(top, __builtin_amdgcn_mov_dpp(top, 0x4E, 0xF, 0xF, false));  // quad_perm [2,3,0,1]
        top = max(top, __builtin_amdgcn_mov_dpp(top, 0x141, 0xF, 0xF, false)); // row_half_mirror
        top = max(top, __builtin_amdgcn_mov_dpp(top, 0x140, 0xF, 0xF, false)); // row_mirror: uniform over the row
        // the lowest expert index that holds it: lowest own candidate, then the minimum over the row
        int cand = 0x7fffffff;
#pragma unroll
        for (int s = NV - 1; s >= 0; --s)
            if (key[s] == top) cand = NV * c + s;
        cand = min(cand, __builtin_amdgcn_mov_dpp(cand, 0xB1, 0xF, 0xF, false));
        cand = min(cand, __builtin_amdgcn_mov_dpp(cand, 0x4E, 0xF, 0xF, false));
        cand = min(cand, __builtin_amdgcn_mov_dpp(cand, 0x141, 0xF, 0xF, false));
        cand = min(cand, __builtin_amdgcn_mov_dpp(cand, 0x140, 0xF, 0xF, false));
#pragma unroll
        for (int s = 0; s < NV; ++s)
            if (cand == NV * c + s) key[s] = kTaken;
        if (c == j) {
            id = cand;
            lgk = top;
        }
    }
    const float lg = __int_as_float(lgk ^ ((lgk >> 31) & 0x7fffffff)); // back to the logit
    const float top0 = __shfl(lg, lane & 48, 64);
    const float ex = c < k ? expf(lg - top0) : 0.f;
    float x = ex;
    x += dpp_move<0x111, 0xF, true>(0.f, x); // row_shr:1
    x += dpp_move<0x112, 0xF, true>(0.f, x); // row_shr:2
    x += dpp_move<0x114, 0xF, true>(0.f, x); // row_shr:4
    x += dpp_move<0x118, 0xF, true>(0.f, x); // row_shr:8 -> lane 15 of the row holds its sum
    const float sum = __shfl(x, lane | 15, 64);
    wt = ex / sum;
}

// The NV consecutive logits row[NV*c .. NV*c+NV-1] of one lane (-inf past the last expert E), every load
// unconditional: 16-byte loads when the row is a whole number of them and starts on a 16-byte boundary
// (E % 4 == 0 and an aligned array: then every token's row does), else single loads on clamped indices -- never one round trip per logit.
template <int NV>
__device__ __forceinline__ void load_logits(const float *row, int c, int E, float (&v)[NV])
{
    float raw[NV];
    if ((E & 3) == 0 && (reinterpret_cast<uintptr_t>(row) & 15) == 0) {
#pragma unroll
        for (int s = 0; s < NV; s += 4) {
            const int e0 = NV * c + s < E ? NV * c + s : E - 4;
            const float4 t = *reinterpret_cast<const float4 *>(row + e0);
            raw[s] = t.x; raw[s + 1] = t.y; raw[s + 2] = t.z; raw[s + 3] = t.w;
        }
    } else {
#pragma unroll
        for (int s = 0; s < NV; ++s) raw[s] = row[NV * c + s < E ? NV * c + s : E - 1];
    }
#pragma unroll
    for (int s = 0; s < NV; ++s) v[s] = NV * c + s < E ? raw[s] : -INFINITY;
}

} // namespace dx_route_core
