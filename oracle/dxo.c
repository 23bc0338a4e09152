/*
 * dxo.c -- CPU oracle for the mixed-precision MoE layer of DynaExq
 * (arXiv 2511.15015, "Dynamic Expert Quantization for Scalable
 * Mixture-of-Experts Inference").
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously correct
 * statement of what the layer computes, used by the tests, by the smoke check
 * and by the benchmark's CPU-baseline leg.  The product path never calls it,
 * and it shares no code, header, table or helper with the HIP kernels.
 *
 * What the paper fixes and what it leaves open:
 *   - Sec. 3.1 (Overview): the worker obtains top-k expert ids from the
 *     router, indexes a handle table, and runs the expert version the handle
 *     points to (high precision or low precision).
 *   - Sec. 3.5 (Online Scheduling Policy): per-(layer, expert) counters c,
 *     score S <- alpha*S + (1-alpha)*c at the end of an interval, counters
 *     reset, H = TopN(S, n_hi), promote = H \ H_cur, demote = H_cur \ H.
 *   - Sec. 3.3 (GPU Memory Management): the resident footprint may never
 *     exceed the budget; capacities n_hi come from budget initialisation.
 *   The paper names no router formula, no quantizer and no data layout; the
 *   readings used here are:
 *     top-k      k largest logits, ties to the lower index, ids in order of
 *                descending logit;
 *     weights    softmax over the k selected logits;
 *     int4       symmetric, groups of `group` consecutive elements along K,
 *                scale = bf16_rne(absmax / 7) computed in fp32,
 *                q = clamp(rint(w / scale), -8, 7) with fp32 IEEE divide and
 *                round-half-to-even, two's-complement nibbles, element 2i in
 *                the low nibble of byte i;
 *     expert     o = W_down (silu(W_gate x) * (W_up x)), silu(z) = z/(1+e^-z);
 *     layer      y[t] = sum_j w[t,j] * o_{ids[t,j]}(x[t]) (+ shared expert);
 *     budget     a layer with n bf16 experts costs n*b_hi + (E-n)*b_lo bytes.
 *
 * Arithmetic: stored weights are widened/dequantised to fp32 exactly
 * (q*scale has at most 12 significant bits), every sum runs sequentially in
 * fp64 over increasing index, nothing is rounded in between.  Decisions that
 * produce integers from floating point (the quantizer) are taken in fp32, the
 * precision the storage format defines.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define DXO_FMT_BF16 0
#define DXO_FMT_INT4 1
#define DXO_FMT_INT2 2

/* one stored expert version, host pointers */
typedef struct {
    const void *w_gate, *w_up, *w_down;   /* bf16 [f,d],[f,d],[d,f]  or packed u8 [f,d/2],[f,d/2],[d,f/2] (int4),
                                             [f,d/4],[f,d/4],[d,f/4] (int2) */
    const void *s_gate, *s_up, *s_down;   /* bf16 scales [rows, K/group] (int4 and int2) */
    int32_t fmt;
    int32_t pad;
} dxo_expert;

/* ------------------------------------------------------------------ bf16 */
static float bf16_widen(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static uint16_t bf16_round(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u)      /* NaN stays NaN */
        return (uint16_t)((u >> 16) | 0x40u);
    uint32_t keep_lsb = (u >> 16) & 1u;
    u += 0x7FFFu + keep_lsb;                   /* round to nearest, ties to even */
    return (uint16_t)(u >> 16);
}

int dxo_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------- router: the logits   */
/* The router of the MoE layer (Sec. 2.1 / 3.1: a learned linear gate scores
 * every expert for every token): logits[t,e] = sum_c x[t,c] * W_r[e,c]
 * (+ bias[e]), bf16 inputs, every sum in fp64, one rounding to fp32 at the
 * end.  bias may be NULL. */
int dxo_router_logits(const uint16_t *x, const uint16_t *w_r, const float *bias, int T, int E, int d,
                      float *logits)
{
    if (T < 0 || E <= 0 || d <= 0) return 1;
    for (int t = 0; t < T; ++t)
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c)
                acc += (double)bf16_widen(x[(size_t)t * d + c]) * (double)bf16_widen(w_r[(size_t)e * d + c]);
            if (bias) acc += (double)bias[e];
            logits[(size_t)t * E + e] = (float)acc;
        }
    return 0;
}

/* ------------------------------------------------------- router: top-k  */
/* Sec. 3.1: "the router [gives] top-k expert IDs".  ids[t,0..k) are the k
 * largest logits of token t, largest first, equal logits to the lower index.
 * w[t,j] is the softmax over those k logits (fp64). */
int dxo_topk(const float *logits, int T, int E, int k, int32_t *ids, double *w)
{
    if (T < 0 || E <= 0 || k <= 0 || k > E) return 1;
    char *taken = (char *)malloc((size_t)E);
    if (!taken) return 4;
    for (int t = 0; t < T; ++t) {
        const float *row = logits + (size_t)t * E;
        memset(taken, 0, (size_t)E);
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || row[e] > row[best]) best = e;   /* strict >: first index wins ties */
            }
            taken[best] = 1;
            ids[(size_t)t * k + j] = best;
        }
        double top = (double)row[ids[(size_t)t * k]];
        double z = 0.0;
        for (int j = 0; j < k; ++j) {
            double ex = exp((double)row[ids[(size_t)t * k + j]] - top);
            w[(size_t)t * k + j] = ex;
            z += ex;
        }
        for (int j = 0; j < k; ++j) w[(size_t)t * k + j] /= z;
    }
    free(taken);
    return 0;
}

/* ------------------------------------- permutation into expert segments */
/* counts[e] = number of (token, slot) pairs routed to e; offsets = exclusive
 * prefix sum with offsets[E] = T*k; perm lists the pair indices p = t*k + j
 * grouped by expert, increasing p inside each segment (a stable counting
 * sort of the ids). */
int dxo_permute(const int32_t *ids, int T, int E, int k,
                int32_t *counts, int32_t *offsets, int32_t *perm)
{
    int P = T * k;
    for (int e = 0; e < E; ++e) counts[e] = 0;
    for (int p = 0; p < P; ++p) {
        if (ids[p] < 0 || ids[p] >= E) return 1;
        counts[ids[p]] += 1;
    }
    offsets[0] = 0;
    for (int e = 0; e < E; ++e) offsets[e + 1] = offsets[e] + counts[e];
    int32_t *cursor = (int32_t *)malloc(sizeof(int32_t) * (size_t)E);
    if (!cursor) return 4;
    for (int e = 0; e < E; ++e) cursor[e] = offsets[e];
    for (int p = 0; p < P; ++p) perm[cursor[ids[p]]++] = p;
    free(cursor);
    return 0;
}

/* --------------------------------------------------------- int4 quantizer */
/* One matrix [rows, K] of bf16 -> packed nibbles [rows, K/2] + bf16 scales
 * [rows, K/group].  Decisions in fp32 (see the header comment). */
int dxo_quantize(const uint16_t *w, int rows, int K, int group, uint8_t *q, uint16_t *s)
{
    if (rows < 0 || K <= 0 || group <= 0 || (K % group) || (group & 1)) return 1;
    int G = K / group;
    for (int r = 0; r < rows; ++r) {
        for (int g = 0; g < G; ++g) {
            const uint16_t *src = w + (size_t)r * K + (size_t)g * group;
            float amax = 0.0f;
            for (int i = 0; i < group; ++i) {
                float a = fabsf(bf16_widen(src[i]));
                if (a > amax) amax = a;
            }
            uint16_t sb = bf16_round(amax / 7.0f);
            float sc = bf16_widen(sb);
            s[(size_t)r * G + g] = sb;
            for (int i = 0; i < group; i += 2) {
                int code[2];
                for (int h = 0; h < 2; ++h) {
                    int v = 0;
                    if (sc != 0.0f) {
                        float x = rintf(bf16_widen(src[i + h]) / sc);   /* default rounding mode: half to even */
                        if (x < -8.0f) x = -8.0f;
                        if (x > 7.0f) x = 7.0f;
                        v = (int)x;
                    }
                    code[h] = v & 0xF;
                }
                q[(size_t)r * (K / 2) + ((size_t)g * group + i) / 2] = (uint8_t)(code[0] | (code[1] << 4));
            }
        }
    }
    return 0;
}

/* The second precision pair of Sec. 4 (int4 as the high tier, int2 as the low
 * one): the same symmetric group quantizer at 2 bits.  The paper names no
 * format; this is the int4 rule with its constants moved to 2 bits:
 * scale = bf16_rne(absmax / q_max) with q_max = 2^(b-1) - 1 = 1, code =
 * clamp(rint(w / scale), -2, 1), two's complement, element i in bits
 * 2*(i%4).. of byte i/4.  [rows, K] bf16 -> [rows, K/4] bytes + scales. */
int dxo_quantize2(const uint16_t *w, int rows, int K, int group, uint8_t *q, uint16_t *s)
{
    if (rows < 0 || K <= 0 || group <= 0 || (K % group) || (group & 3)) return 1;
    int G = K / group;
    for (int r = 0; r < rows; ++r) {
        for (int g = 0; g < G; ++g) {
            const uint16_t *src = w + (size_t)r * K + (size_t)g * group;
            float amax = 0.0f;
            for (int i = 0; i < group; ++i) {
                float a = fabsf(bf16_widen(src[i]));
                if (a > amax) amax = a;
            }
            uint16_t sb = bf16_round(amax / 1.0f);
            float sc = bf16_widen(sb);
            s[(size_t)r * G + g] = sb;
            for (int i = 0; i < group; i += 4) {
                unsigned byte = 0;
                for (int h = 0; h < 4; ++h) {
                    int v = 0;
                    if (sc != 0.0f) {
                        float x = rintf(bf16_widen(src[i + h]) / sc);
                        if (x < -2.0f) x = -2.0f;
                        if (x > 1.0f) x = 1.0f;
                        v = (int)x;
                    }
                    byte |= (unsigned)(v & 0x3) << (2 * h);
                }
                q[(size_t)r * (K / 4) + ((size_t)g * group + i) / 4] = (uint8_t)byte;
            }
        }
    }
    return 0;
}

/* signed value of the 2-bit code `idx` of a packed row */
static int crumb_at(const uint8_t *row, int idx)
{
    int v = (row[idx >> 2] >> (2 * (idx & 3))) & 0x3;
    return v >= 2 ? v - 4 : v;
}

/* signed value of nibble `idx` of a packed row */
static int nibble_at(const uint8_t *row, int idx)
{
    int b = row[idx >> 1];
    int v = (idx & 1) ? (b >> 4) : (b & 0xF);
    return v >= 8 ? v - 16 : v;
}

/* stored weight (row, col) of one matrix widened to fp32 -- exact */
static float weight_at(const void *wptr, const void *sptr, int fmt, int K, int group, int row, int col)
{
    if (fmt == DXO_FMT_BF16)
        return bf16_widen(((const uint16_t *)wptr)[(size_t)row * K + col]);
    const uint8_t *qrow = (const uint8_t *)wptr + (size_t)row * (K / 2);
    uint16_t sb = ((const uint16_t *)sptr)[(size_t)row * (K / group) + col / group];
    return (float)nibble_at(qrow, col) * bf16_widen(sb);
}

/* the same for a matrix stored as 2-bit codes */
static float weight_at_int2(const void *wptr, const void *sptr, int K, int group, int row, int col)
{
    const uint8_t *crow = (const uint8_t *)wptr + (size_t)row * (K / 4);
    uint16_t sb = ((const uint16_t *)sptr)[(size_t)row * (K / group) + col / group];
    return (float)crumb_at(crow, col) * bf16_widen(sb);
}

/* packed int2 + scales -> fp32 matrix [rows, K] */
int dxo_dequantize2(const uint8_t *q, const uint16_t *s, int rows, int K, int group, float *out)
{
    if (rows < 0 || K <= 0 || group <= 0 || (K % group) || (K & 3)) return 1;
    for (int r = 0; r < rows; ++r)
        for (int c = 0; c < K; ++c)
            out[(size_t)r * K + c] = weight_at_int2(q, s, K, group, r, c);
    return 0;
}

/* packed int4 + scales -> fp32 matrix [rows, K] */
int dxo_dequantize(const uint8_t *q, const uint16_t *s, int rows, int K, int group, float *out)
{
    if (rows < 0 || K <= 0 || group <= 0 || (K % group) || (K & 1)) return 1;
    for (int r = 0; r < rows; ++r)
        for (int c = 0; c < K; ++c)
            out[(size_t)r * K + c] = weight_at(q, s, DXO_FMT_INT4, K, group, r, c);
    return 0;
}

/* ------------------------------------------------------------ one expert */
/* o = W_down ( silu(W_gate x) * (W_up x) ) on the stored (dequantised)
 * weights, all sums in fp64.  hbuf has room for f doubles. */
/* the same expert on int2-stored matrices */
static void expert_apply_int2(const dxo_expert *ex, int d, int f, int group,
                              const float *x, double *hbuf, double *o)
{
    for (int n = 0; n < f; ++n) {
        double g = 0.0, u = 0.0;
        for (int c = 0; c < d; ++c) {
            g += (double)weight_at_int2(ex->w_gate, ex->s_gate, d, group, n, c) * (double)x[c];
            u += (double)weight_at_int2(ex->w_up, ex->s_up, d, group, n, c) * (double)x[c];
        }
        double silu = g / (1.0 + exp(-g));
        hbuf[n] = silu * u;
    }
    for (int n = 0; n < d; ++n) {
        double acc = 0.0;
        for (int c = 0; c < f; ++c)
            acc += (double)weight_at_int2(ex->w_down, ex->s_down, f, group, n, c) * hbuf[c];
        o[n] = acc;
    }
}

static void expert_apply(const dxo_expert *ex, int d, int f, int group,
                         const float *x, double *hbuf, double *o)
{
    if (ex->fmt == DXO_FMT_INT2) {
        expert_apply_int2(ex, d, f, group, x, hbuf, o);
        return;
    }
    for (int n = 0; n < f; ++n) {
        double g = 0.0, u = 0.0;
        for (int c = 0; c < d; ++c) {
            g += (double)weight_at(ex->w_gate, ex->s_gate, ex->fmt, d, group, n, c) * (double)x[c];
            u += (double)weight_at(ex->w_up, ex->s_up, ex->fmt, d, group, n, c) * (double)x[c];
        }
        double silu = g / (1.0 + exp(-g));
        hbuf[n] = silu * u;
    }
    for (int n = 0; n < d; ++n) {
        double acc = 0.0;
        for (int c = 0; c < f; ++c)
            acc += (double)weight_at(ex->w_down, ex->s_down, ex->fmt, f, group, n, c) * hbuf[c];
        o[n] = acc;
    }
}

/* ------------------------------------------------------------- the layer */
/* y[t] = sum_{j<k} w[t,j] * expert_{ids[t,j]}(x[t])  (+ shared(x[t]) with
 * weight 1 when `shared` is given, intermediate size shared_f).
 * Only the tokens listed in `tokens` (n_tokens of them; NULL = all T) are
 * computed; row i of y_out belongs to tokens[i] (or token i). */
int dxo_moe_forward(const dxo_expert *experts, int E, int d, int f, int group,
                    const uint16_t *x_bf16, int T, int k,
                    const int32_t *ids, const double *w,
                    const dxo_expert *shared, int shared_f,
                    const int32_t *tokens, int n_tokens, double *y_out)
{
    if (E <= 0 || d <= 0 || f <= 0 || T < 0 || k <= 0) return 1;
    int n = tokens ? n_tokens : T;
    int status = 0;
    int fmax = f > shared_f ? f : shared_f;
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n; ++i) {
        int t = tokens ? tokens[i] : i;
        float *x = (float *)malloc(sizeof(float) * (size_t)d);
        double *h = (double *)malloc(sizeof(double) * (size_t)fmax);
        double *o = (double *)malloc(sizeof(double) * (size_t)d);
        double *y = y_out + (size_t)i * d;
        if (!x || !h || !o || t < 0 || t >= T) {
#pragma omp atomic write
            status = 1;
        } else {
            for (int c = 0; c < d; ++c) x[c] = bf16_widen(x_bf16[(size_t)t * d + c]);
            for (int c = 0; c < d; ++c) y[c] = 0.0;
            for (int j = 0; j < k; ++j) {
                int e = ids[(size_t)t * k + j];
                if (e < 0 || e >= E) {
#pragma omp atomic write
                    status = 1;
                    continue;
                }
                expert_apply(&experts[e], d, f, group, x, h, o);
                double wj = w[(size_t)t * k + j];
                for (int c = 0; c < d; ++c) y[c] += wj * o[c];
            }
            if (shared) {
                expert_apply(shared, d, shared_f, group, x, h, o);
                for (int c = 0; c < d; ++c) y[c] += o[c];
            }
        }
        free(x); free(h); free(o);
    }
    return status;
}

/* ---------------------------------------------------- hotness and policy */
/* Sec. 3.5, "Hotness Estimation": c[e] accumulates how often the router
 * selected expert e in the current interval. */
void dxo_hotness_update(int64_t *c, const int32_t *counts, int E)
{
    for (int e = 0; e < E; ++e) c[e] += counts[e];
}

/* End of an interval: S <- alpha*S + (1-alpha)*c, then c <- 0 (the EMA
 * equation of Sec. 3.5).  To keep the score an exact, reproducible integer,
 * alpha = alpha_q16 / 65536 and S is held in units of 2^-16 counts:
 *   S <- floor( (alpha_q16 * S + (65536 - alpha_q16) * (c * 65536)) / 65536 ).
 * alpha_q16 = 0 gives S = c * 65536, i.e. plain windowed counts. */
int dxo_window_end(uint64_t *S, int64_t *c, int E, uint32_t alpha_q16)
{
    if (alpha_q16 >= 65536u) return 1;
    for (int e = 0; e < E; ++e) {
        uint64_t cur = (uint64_t)c[e] << 16;
        S[e] = ((uint64_t)alpha_q16 * S[e] + (uint64_t)(65536u - alpha_q16) * cur) >> 16;
        c[e] = 0;
    }
    return 0;
}

/* bytes of one expert's three matrices in each format */
uint64_t dxo_expert_bytes(int d, int f, int group, int fmt)
{
    uint64_t params = 3ull * (uint64_t)d * (uint64_t)f;
    if (fmt == DXO_FMT_BF16) return 2ull * params;
    if (fmt == DXO_FMT_INT2) return params / 4ull + 2ull * (params / (uint64_t)group);
    return params / 2ull + 2ull * (params / (uint64_t)group);
}

/* Budget initialisation (Sec. 3.1 / 3.3): the largest n with
 * n*b_hi + (E-n)*b_lo <= budget, clamped to [0, E]; -1 when even the all-low
 * layer does not fit. */
int dxo_budget_capacity(uint64_t budget, int E, uint64_t b_hi, uint64_t b_lo)
{
    if (b_hi <= b_lo || E <= 0) return -1;
    int n = -1;
    for (int c = 0; c <= E; ++c)
        if ((uint64_t)c * b_hi + (uint64_t)(E - c) * b_lo <= budget) n = c;
    return n;
}

/* H = TopN(S, n): the n experts with the largest score, equal scores to the
 * lower index; out_ids in rank order (Sec. 3.5, "Budget-feasible Selection"). */
int dxo_select_topn(const uint64_t *S, int E, int n, int32_t *out_ids)
{
    if (n < 0 || n > E) return 1;
    char *taken = (char *)calloc((size_t)E, 1);
    if (!taken) return 4;
    for (int r = 0; r < n; ++r) {
        int best = -1;
        for (int e = 0; e < E; ++e) {
            if (taken[e]) continue;
            if (best < 0 || S[e] > S[best]) best = e;
        }
        taken[best] = 1;
        out_ids[r] = best;
    }
    free(taken);
    return 0;
}

/* rank order of Sec. 3.5's TopN: a ranks above b when its score is larger,
 * equal scores to the lower index */
static int ranks_above(const uint64_t *S, int a, int b)
{
    return S[a] != S[b] ? S[a] > S[b] : a < b;
}

/* lowest-ranked member (in = 1) or highest-ranked outsider (in = 0) of the
 * set flagged by `member`; -1 when there is none */
static int extreme_of(const uint64_t *S, const uint8_t *member, int E, int in)
{
    int pick = -1;
    for (int e = 0; e < E; ++e) {
        if ((member[e] != 0) != in) continue;
        if (pick < 0) pick = e;
        else if (in ? ranks_above(S, pick, e) : ranks_above(S, e, pick)) pick = e;
    }
    return pick;
}

static void members_in_rank_order(const uint64_t *S, const uint8_t *member, int E, int32_t *out_ids)
{
    int n = 0;
    for (int e = 0; e < E; ++e)
        if (member[e]) out_ids[n++] = e;
    for (int i = 1; i < n; ++i)
        for (int j = i; j > 0 && ranks_above(S, out_ids[j], out_ids[j - 1]); --j) {
            int32_t t = out_ids[j]; out_ids[j] = out_ids[j - 1]; out_ids[j - 1] = t;
        }
}

/* Hysteresis with an additive margin (Sec. 3.5, "Hysteresis for Stability").
 * Start from the current set H_cur (flags `cur`).  An outsider replaces the
 * lowest-ranked member only if its score exceeds that member's by more than
 * `margin`; the member it replaces is, by the same inequality, below the
 * highest-ranked outsider by more than the margin.  Repeat until the best
 * outsider no longer beats the worst member.  The capacity n is kept: a set
 * above n first loses its lowest-ranked members, a set below n takes the
 * highest-ranked outsiders into its empty slots (no member to displace, so
 * no margin applies).  margin = 0 gives exactly TopN(S, n).  out_ids in rank
 * order.  Returns 0, or 1 for a bad argument. */
int dxo_select_hysteresis(const uint64_t *S, int E, const uint8_t *cur, int n, uint64_t margin,
                          int32_t *out_ids)
{
    if (E <= 0 || n < 0 || n > E) return 1;
    uint8_t *member = (uint8_t *)malloc((size_t)E);
    if (!member) return 4;
    int size = 0;
    for (int e = 0; e < E; ++e) size += (member[e] = cur[e] != 0);
    while (size > n) { member[extreme_of(S, member, E, 1)] = 0; --size; }
    while (size < n) { member[extreme_of(S, member, E, 0)] = 1; ++size; }
    for (;;) {
        const int lo = extreme_of(S, member, E, 1), out = extreme_of(S, member, E, 0);
        if (lo < 0 || out < 0) break;
        const int beats = margin ? (S[out] > S[lo] && S[out] - S[lo] > margin) : ranks_above(S, out, lo);
        if (!beats) break;
        member[lo] = 0;
        member[out] = 1;
    }
    members_in_rank_order(S, member, E, out_ids);
    free(member);
    return 0;
}

/* Hysteresis as a rank slack (same paragraph): a member keeps its place as
 * long as it ranks inside the wider candidate set, the top n + slack; the
 * places of the members that fell out of it (and empty places) go to the
 * highest-ranked outsiders.  slack = 0 gives exactly TopN(S, n). */
int dxo_select_rank_slack(const uint64_t *S, int E, const uint8_t *cur, int n, int slack, int32_t *out_ids)
{
    if (E <= 0 || n < 0 || n > E || slack < 0) return 1;
    uint8_t *member = (uint8_t *)malloc((size_t)E);
    if (!member) return 4;
    int size = 0;
    for (int e = 0; e < E; ++e) {
        int rank = 0; /* experts that rank above e */
        for (int o = 0; o < E; ++o) rank += o != e && ranks_above(S, o, e);
        member[e] = cur[e] != 0 && rank < n + slack;
        size += member[e];
    }
    while (size > n) { member[extreme_of(S, member, E, 1)] = 0; --size; }
    while (size < n) { member[extreme_of(S, member, E, 0)] = 1; ++size; }
    members_in_rank_order(S, member, E, out_ids);
    free(member);
    return 0;
}

/* promote = H \ H_cur, demote = H_cur \ H, each in increasing expert id
 * (Sec. 3.5).  is_hi_cur / is_hi_new are 0/1 flags of length E. */
void dxo_transition_sets(const uint8_t *is_hi_cur, const uint8_t *is_hi_new, int E,
                         int32_t *promote, int32_t *n_promote,
                         int32_t *demote, int32_t *n_demote)
{
    int np = 0, nd = 0;
    for (int e = 0; e < E; ++e) {
        if (is_hi_new[e] && !is_hi_cur[e]) promote[np++] = e;
        if (is_hi_cur[e] && !is_hi_new[e]) demote[nd++] = e;
    }
    *n_promote = np;
    *n_demote = nd;
}
