"""Element-wise error bound of the HIP path's layer output against the fp64 oracle.

The HIP path computes every product of bf16 values exactly and accumulates in fp32; what separates
its result from the fp64 oracle's are its bf16 roundings: H = silu(g) * u is stored as bf16 (relative
error at most 2^-9 per element), y is stored as bf16 (2^-9 of |y|), and batches above 128 tokens also
store the expert outputs O as bf16 (2^-9 of |o|).  Propagating the first through the down projection
and the combine gives, for token t and column c,

    |y_hip - y_ref| <= 2^-9 * ( |y_ref| + A[t,c] ) (+ 2^-9 * A[t,c] with bf16 O),
    A[t,c] = sum_j w[t,j] * sum_n |W_down[e_j][c,n]| * |h_j[n]|   (>= sum_j w[t,j] |o_j[c]|),

the worst case in which every rounding error has the same sign.  The test tolerance is that bound with
head-room for the fp32 accumulation and the hardware exp/divide of the SwiGLU (factor 1.25 on A) and
for the second-order terms (2^-8 instead of 2^-9 on |y_ref|).  A typical error is far smaller (the
rounding errors are independent), so the relative-L2 gate stays the tight one; this bound is what
catches a single wrong element, which a norm hides.  A is computed here in numpy from the weights as
the oracle dequantises them."""
import numpy as np

from paper_2511_15015_amd.workloads import bf16_bits_to_f32


def dense_matrices(dxo, ev, group):
    """(W_gate [f,d], W_up [f,d], W_down [d,f]) of one oracle-side expert version as fp32 (exact)."""
    a = ev.arrays
    if ev.fmt == dxo.FMT_BF16:
        return tuple(bf16_bits_to_f32(m) for m in a[:3])
    deq = dxo.dequantize if ev.fmt == dxo.FMT_INT4 else dxo.dequantize2
    return tuple(deq(a[i], a[3 + i], group) for i in range(3))


def elementwise_tolerance(dxo, versions, group, x_bits, ids, w, y_ref, shared=None, tokens=None, o_rounded=False):
    x = bf16_bits_to_f32(x_bits)
    T = x.shape[0]
    tokens = np.arange(T) if tokens is None else np.asarray(tokens)
    A = np.zeros_like(y_ref)

    def add(ev, rows, weights):
        """rows: indices into `tokens`; adds weights[i] * |W_down| |h(x[tokens[rows[i]]])| to A[rows[i]].
        fp32 matrix products: the bound needs no more."""
        wg, wu, wd = dense_matrices(dxo, ev, group)
        xe = x[tokens[rows]]
        g = (xe @ wg.T).astype(np.float64)
        u = (xe @ wu.T).astype(np.float64)
        h = np.abs(g / (1.0 + np.exp(-g)) * u).astype(np.float32)
        A[rows] += np.asarray(weights, np.float64)[:, None] * (h @ np.abs(wd).T).astype(np.float64)

    sel = ids[tokens]                                   # [n, k]
    for e in np.unique(sel):
        rows, js = np.nonzero(sel == e)
        add(versions[int(e)], rows, w[tokens[rows], js])
    if shared is not None:
        add(shared, np.arange(len(tokens)), np.ones(len(tokens)))
    return 2.0 ** -8 * np.abs(y_ref) + (2.25 if o_rounded else 1.25) * 2.0 ** -9 * A


def assert_elementwise(dxo, y_gpu_bits, y_ref, versions, group, x_bits, ids, w, shared=None, tokens=None, T_call=None):
    """y_gpu_bits / y_ref: the rows of `tokens` (all rows when None).  T_call: tokens of the forward call
    (above 128 the HIP path stores O as bf16)."""
    T_call = x_bits.shape[0] if T_call is None else T_call
    tol = elementwise_tolerance(dxo, versions, group, x_bits, ids, w, y_ref, shared=shared, tokens=tokens,
                                o_rounded=T_call > 128)
    y = bf16_bits_to_f32(y_gpu_bits).astype(np.float64)
    assert np.isfinite(y).all()
    excess = np.abs(y - y_ref) - tol
    worst = np.unravel_index(np.argmax(excess), excess.shape)
    assert excess[worst] <= 0.0, (f"element {worst}: |{y[worst]} - {y_ref[worst]}| = {abs(y[worst] - y_ref[worst]):.3e} "
                                  f"> bound {tol[worst]:.3e}")
    return float(np.max(np.abs(y - y_ref) / tol))     # the largest used fraction of the bound
