"""Where the parity tolerances come from: the rounding behaviour of fp32 dot products, in numpy.

Nothing here is the method's arithmetic.  The GPU kernels accumulate every dot product in fp32
(the precision the mask decision is taken in).  Two consequences are derived and pinned here:

* A sum of n products evaluated in fp32 carries an absolute error of c * eps32 * S, S = sum_i |w_i x_i|,
  whatever the order (c grows with the depth of the longest addition chain: at most n, d/256 + 6 for the
  kernels' 64 strided lanes plus a butterfly; about 0.1 in practice).  Relative to the result that is
  eps32 * kappa with kappa = S / |sum_i w_i x_i|.  One neuron whose up-projection dot nearly cancels
  therefore cannot be within 1e-5 of the fp64 value; with thousands of neurons the badly conditioned
  ones are a vanishing part of y.  `decode_condition` gives the per-row condition number of y that the
  few-neuron parity cases add to the bar.
* The pre-activation error bounds how close to tau an activation can be decided: `BAND_ABS`.
"""
import numpy as np

EPS32 = 2.0 ** -24          # unit round-off of fp32


def f32_dot_lanes(w, x, vec=4, lanes=64):
    """fp32 dot product in the kernels' summation shape: lane l owns elements vec*(c*lanes + l) .. +vec of
    every chunk c, adds its products one after the other with fused multiply-adds, then the lanes are
    folded by a pairwise tree.  Inputs are taken as float32; returns a Python float (the fp32 value)."""
    w = np.asarray(w, np.float32).astype(np.float64)
    x = np.asarray(x, np.float32).astype(np.float64)
    n = w.size
    step = vec * lanes
    acc = np.zeros(lanes, np.float32)
    for c0 in range(0, n, step):
        for e in range(vec):
            idx = c0 + np.arange(lanes) * vec + e
            ok = idx < n
            idx = np.minimum(idx, n - 1)
            prod = np.where(ok, w[idx] * x[idx], 0.0)                  # exact in fp64 (24 x 24 bits)
            acc = (acc.astype(np.float64) + prod).astype(np.float32)  # one rounding per fused multiply-add
    v = acc
    while v.size > 1:
        v = (v[0::2] + v[1::2]).astype(np.float32)
    return float(v[0])


def dot_condition(w, x):
    """(sum, S = sum |w_i x_i|) in fp64 for every row of w [F][d] against every row of x [B][d]: [B][F] each."""
    w = np.asarray(w, np.float64)
    x = np.atleast_2d(np.asarray(x, np.float64))
    return x @ w.T, np.abs(x) @ np.abs(w).T


def _sigma_and_slope(g, sigma):
    if sigma == "relu":
        return np.maximum(g, 0.0), (g > 0).astype(np.float64)
    if sigma == "silu":
        s = 1.0 / (1.0 + np.exp(-g))
        return g * s, s + g * s * (1.0 - s)
    if sigma == "gelu_tanh":
        k = np.sqrt(2.0 / np.pi)
        u = k * (g + 0.044715 * g ** 3)
        t = np.tanh(u)
        return 0.5 * g * (1.0 + t), 0.5 * (1.0 + t) + 0.5 * g * (1.0 - t * t) * k * (1.0 + 3 * 0.044715 * g * g)
    raise ValueError(sigma)


def decode_condition(w_gate, w_up, w_down, x, mask, sigma="silu", b_in=None):
    """Per-row condition number kappa_b of the decode output with respect to the rounding of its dot
    products: the first-order bound
        |y_b - y_ref,b|_2 <= c eps32 * sum_{j kept} |W_down[j,:]|_2 (|a_j| S^u_j + |sigma'(g_j) u_j| S^g_j)
    divided by |y_ref,b|_2 (w_up = None: the non-gated family, h = a).  Returns (kappa [B], y_ref [B][d])."""
    x = np.atleast_2d(np.asarray(x, np.float64))
    mask = np.atleast_2d(np.asarray(mask, bool))
    g, sg = dot_condition(w_gate, x)
    if b_in is not None:
        g = g + np.asarray(b_in, np.float64)[None, :]
        sg = sg + np.abs(np.asarray(b_in, np.float64))[None, :]
    a, slope = _sigma_and_slope(g, sigma)
    if w_up is None:
        h = a
        err_h = np.abs(slope) * sg
    else:
        u, su = dot_condition(w_up, x)
        h = a * u
        err_h = np.abs(a) * su + np.abs(slope * u) * sg
    wd = np.asarray(w_down, np.float64)
    y = (h * mask) @ wd
    bound = (err_h * mask) @ np.linalg.norm(wd, axis=1)
    return bound / np.maximum(np.linalg.norm(y, axis=1), 1e-300), y
