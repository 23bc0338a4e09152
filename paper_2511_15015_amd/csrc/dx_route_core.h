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

// ---- four token rows per wavefront, one per 16-lane row, so that one instruction stream serves all four ----

__device__ __forceinline__ int row_max(int x) // maximum over the 16-lane row, in every lane of it
{
    x = max(x, __builtin_amdgcn_mov_dpp(x, 0xB1, 0xF, 0xF, false));  // quad_perm [1,0,3,2]
    x = max(x, __builtin_amdgcn_mov_dpp(x, 0x4E, 0xF, 0xF, false));  // quad_perm [2,3,0,1]
    x = max(x, __builtin_amdgcn_mov_dpp(x, 0x141, 0xF, 0xF, false)); // row_half_mirror
    x = max(x, __builtin_amdgcn_mov_dpp(x, 0x140, 0xF, 0xF, false)); // row_mirror
    return x;
}

__device__ __forceinline__ int row_min(int x)
{
    x = min(x, __builtin_amdgcn_mov_dpp(x, 0xB1, 0xF, 0xF, false));
    x = min(x, __builtin_amdgcn_mov_dpp(x, 0x4E, 0xF, 0xF, false));
    x = min(x, __builtin_amdgcn_mov_dpp(x, 0x141, 0xF, 0xF, false));
    x = min(x, __builtin_amdgcn_mov_dpp(x, 0x140, 0xF, 0xF, false));
    return x;
}

constexpr int kTakenKey = (int)0x80000000; // below every logit's key, -inf's included

// Order-preserving integer key of a logit (x + 0 turns -0 into +0, so equal logits have equal keys): integer
// max / compare, no NaN handling in the way.
__device__ __forceinline__ int key_of(float x)
{
    const int b = __float_as_int(x + 0.f);
    return b ^ ((b >> 31) & 0x7fffffff);
}

// k selections over the row's entries: lane c holds N of them, key[s] with expert index ix[s], the indices
// ascending in s (unused places: kTakenKey with an index above every expert's).  Each selection takes the
// largest key of the row and, among equals, the lowest expert index; lane j < k of the row ends up with
// the j-th selection's index in id and its key in lgk.  key is consumed.
template <int N>
__device__ __forceinline__ void select_rows16(int (&key)[N], const int (&ix)[N], int k, int c, int &id, int &lgk)
{
    id = 0;
    lgk = kTakenKey;
    for (int j = 0; j < k; ++j) {
        int top = key[0];
#pragma unroll
        for (int s = 1; s < N; ++s) top = max(top, key[s]);
        top = row_max(top);
        // the lowest expert index that holds it: lowest own candidate, then the minimum over the row
        int cand = 0x7fffffff;
#pragma unroll
        for (int s = N - 1; s >= 0; --s)
            if (key[s] == top) cand = ix[s];
        cand = row_min(cand);
#pragma unroll
        for (int s = 0; s < N; ++s)
            if (ix[s] == cand) key[s] = kTakenKey;
        if (c == j) {
            id = cand;
            lgk = top;
        }
    }
}

// The routing weight of the row's lane c < k from the selected keys: the softmax over the k selected logits.
// The terms add up in the order of wave_sum (a 16-lane row scan), so the weights are the same bits.
__device__ __forceinline__ float weight_rows16(int lgk, int k, int lane)
{
    const int c = lane & 15;
    const float lg = __int_as_float(lgk ^ ((lgk >> 31) & 0x7fffffff)); // back to the logit
    const float top0 = __shfl(lg, lane & 48, 64);
    const float ex = c < k ? expf(lg - top0) : 0.f;
    float x = ex;
    x += dpp_move<0x111, 0xF, true>(0.f, x); // row_shr:1
    x += dpp_move<0x112, 0xF, true>(0.f, x); // row_shr:2
    x += dpp_move<0x114, 0xF, true>(0.f, x); // row_shr:4
    x += dpp_move<0x118, 0xF, true>(0.f, x); // row_shr:8 -> lane 15 of the row holds its sum
    const float sum = __shfl(x, lane | 15, 64);
    return ex / sum;
}

// Which experts lane c of a row owns (E <= 16*NV): slot s is expert 64 * (s / 4) + 4 * c + s % 4, ascending
// in s.  Four consecutive slots are four consecutive logits, and the row's 16 lanes together read 256
// consecutive bytes of the token's logits per 16-byte load (consecutive ownership, NV logits per lane,
// would touch 16 different lines per load instruction and come back to each of them NV / 4 times).
__device__ __forceinline__ int rows16_expert(int c, int s) { return 64 * (s >> 2) + 4 * c + (s & 3); }

// v[s] = the logit of expert rows16_expert(c, s) of the token whose logits start at `row` (-inf past the last
// expert E), every load unconditional: 16-byte loads when the row is a whole number of them and starts on a
// 16-byte boundary (E % 4 == 0 and an aligned array: then every token's row does), else single loads on
// clamped indices.
template <int NV>
__device__ __forceinline__ void load_logits_rows16(const float *row, int c, int E, float (&v)[NV])
{
    static_assert(NV % 4 == 0, "whole groups of four slots");
    float raw[NV];
    if ((E & 3) == 0 && (reinterpret_cast<uintptr_t>(row) & 15) == 0) {
#pragma unroll
        for (int s = 0; s < NV; s += 4) {
            const int e = rows16_expert(c, s), e0 = e < E ? e : E - 4;
            const float4 t = *reinterpret_cast<const float4 *>(row + e0);
            raw[s] = t.x; raw[s + 1] = t.y; raw[s + 2] = t.z; raw[s + 3] = t.w;
        }
    } else {
#pragma unroll
        for (int s = 0; s < NV; ++s) {
            const int e = rows16_expert(c, s);
            raw[s] = row[e < E ? e : E - 1];
        }
    }
#pragma unroll
    for (int s = 0; s < NV; ++s) v[s] = rows16_expert(c, s) < E ? raw[s] : -INFINITY;
}

// v[s] is the logit of expert rows16_expert(c, s) of the row's token (-inf past the last expert).  Same
// results as topk_rows: on return lane c < k of a row holds the c-th id of its token and its weight (k <= 16).
template <int NV>
__device__ __forceinline__ void topk_rows16(const float (&v)[NV], int k, int lane, int &id, float &wt)
{
    const int c = lane & 15;
    int key[NV], ix[NV];
#pragma unroll
    for (int s = 0; s < NV; ++s) {
        key[s] = key_of(v[s]);
        ix[s] = rows16_expert(c, s);
    }
    int lgk;
    select_rows16<NV>(key, ix, k, c, id, lgk);
    wt = weight_rows16(lgk, k, lane);
}

// The same for many logits per lane (wide layers), where k selections over NV entries each are most of a
// decode kernel's prologue.  A threshold first: the k-th of the row's lane maxima taken one value at a time
// (all lanes that hold the value retire together, so ties only lower it) has at least k entries at or above
// it, hence every selected entry is among those -- a dozen or two per row instead of 16*NV.  Each lane keeps
// up to C of them (its keys go through `scratch`, NV*64 words of LDS of this wavefront alone, to be fetched
// by a position that differs from lane to lane) and the selections run over C entries.  When some lane of
// the wavefront has more than C entries at or above the threshold (heavy ties, a token whose favourites are
// neighbours), the wavefront selects over all NV as above: the results are the same either way.
template <int NV, int C>
__device__ __forceinline__ void topk_rows16_filtered(const float (&v)[NV], int k, int lane, int &id, float &wt,
                                                     __attribute__((address_space(3))) int *scratch)
{
    static_assert(NV <= 32, "the entries at or above the threshold are a 32-bit mask");
    const int c = lane & 15;
    int key[NV];
#pragma unroll
    for (int s = 0; s < NV; ++s) key[s] = key_of(v[s]);
    int best = key[0];
#pragma unroll
    for (int s = 1; s < NV; ++s) best = max(best, key[s]);
    int tau = kTakenKey;
    for (int j = 0; j < k; ++j) {
        tau = row_max(best);
        if (best == tau) best = kTakenKey;
    }
    uint32_t above = 0;
#pragma unroll
    for (int s = 0; s < NV; ++s) above |= (key[s] >= tau ? 1u : 0u) << s;
    int lgk;
    if (__ballot(__popc(above) > C) != 0ull) { // wavefront-uniform
        int ix[NV];
#pragma unroll
        for (int s = 0; s < NV; ++s) ix[s] = rows16_expert(c, s);
        select_rows16<NV>(key, ix, k, c, id, lgk);
    } else {
#pragma unroll
        for (int s = 0; s < NV; ++s) scratch[s * 64 + lane] = key[s];
        int ck[C], ci[C];
#pragma unroll
        for (int j = 0; j < C; ++j) {
            const bool have = above != 0u;
            const int slot = have ? __builtin_ctz(above) : 0;
            above &= above - 1u;
            const int got = scratch[slot * 64 + lane];
            ck[j] = have ? got : kTakenKey;
            ci[j] = have ? rows16_expert(c, slot) : 0x7fffffff;
        }
        select_rows16<C>(ck, ci, k, c, id, lgk);
    }
    wt = weight_rows16(lgk, k, lane);
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
