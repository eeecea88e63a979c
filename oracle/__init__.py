"""fp64 CPU oracle for the CLADA sparse-FFN decode path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrappers over ``clada_oracle.c`` (plain C, fp64, written from the
paper's definitions).  Nothing here is used by the product path; only tests,
the smoke check and the benchmark's ``cpu_baseline`` leg import this package.
It shares no code with the HIP library and never imports it.

All array inputs are numpy arrays holding the exact stored values as float32
(bf16 values widen to float32 exactly); all results are float64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "clada_oracle.c")
_LIB = os.path.join(_HERE, "libclada_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC",
               "-shared", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.clada_oracle_quantile_rank.restype = C.c_int64
        _lib.clada_oracle_quantile_rank.argtypes = [C.c_int64, C.c_float]
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(C.POINTER(C.c_float))


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(C.POINTER(C.c_double))


def _out(shape, dtype=np.float64):
    a = np.empty(shape, dtype=dtype)
    ct = {np.float64: C.c_double, np.uint8: C.c_uint8, np.int32: C.c_int32}[dtype]
    return a, a.ctypes.data_as(C.POINTER(ct))


def num_threads() -> int:
    return int(_load().clada_oracle_num_threads())


SIGMAS = {"silu": 0, "gelu_tanh": 1}


def _set_sigma(sigma):
    """Select sigma of the gated FFN for the next call: "silu" (LLaMA / Mistral) or "gelu_tanh" (Gemma)."""
    rc = _load().clada_oracle_set_sigma(SIGMAS[sigma])
    assert rc == 0, rc


def _weights(w_gate, w_up, w_down):
    wg, pg = _f32(w_gate)
    wu, pu = _f32(w_up)
    wd, pd = _f32(w_down)
    F, d = wg.shape
    assert wu.shape == (F, d) and wd.shape == (F, d), "weights must be neuron-major [d_ff][d]"
    return (wg, wu, wd), (pg, pu, pd), d, F


def prefix_stats(w_gate, w_up, w_down, x, want_y=True, want_pool=True, sigma="silu"):
    """Dense FFN over the prefix x [T][d] and the per-neuron aggregates."""
    keep, (pg, pu, pd), d, F = _weights(w_gate, w_up, w_down)
    xx, px = _f32(x)
    T = xx.shape[0]
    assert xx.shape == (T, d)
    y, py = _out((T, d)) if want_y else (None, None)
    pool, pp = _out((T, F)) if want_pool else (None, None)
    outs = [_out((F,)) for _ in range(5)]
    _set_sigma(sigma)
    rc = _load().clada_oracle_prefix_stats(pg, pu, pd, d, F, px, T, py,
                                           *[o[1] for o in outs], pp)
    assert rc == 0, rc
    names = ["sum_abs_act", "sum_sq_act", "max_abs_act", "sum_sq_h", "A"]
    res = {n: o[0] for n, o in zip(names, outs)}
    res["y"] = y
    res["abs_act_pool"] = pool
    return res


def quantile_rank(n: int, q) -> int:
    return int(_load().clada_oracle_quantile_rank(int(n), np.float32(q)))


def calibrate(pool, q) -> float:
    """Nearest-rank q-quantile of the pooled magnitudes (base-threshold stand-in)."""
    p, pp = _f64(np.ravel(pool))
    tau = C.c_double()
    rc = _load().clada_oracle_calibrate(pp, C.c_int64(p.size), C.c_float(float(np.float32(q))),
                                        C.byref(tau))
    assert rc == 0, rc
    return tau.value


def signals(logits, token_ids):
    """(surprisal [B], entropy [B]) in nats from logits [B][V]."""
    z, pz = _f32(np.atleast_2d(logits))
    B, V = z.shape
    tok = np.ascontiguousarray(np.ravel(token_ids), dtype=np.int32)
    assert tok.size == B
    s, ps = _out((B,))
    h, ph = _out((B,))
    rc = _load().clada_oracle_signals(pz, B, V, tok.ctypes.data_as(C.POINTER(C.c_int32)), ps, ph)
    assert rc == 0, rc
    return s, h


def threshold(tau_base, lam, gam, surprisal, entropy, tau_s, tau_H):
    """tau_final [L][B] from per-layer base thresholds and per-token signals."""
    tb, ptb = _f64(np.ravel(tau_base))
    la, pla = _f64(np.ravel(lam))
    ga, pga = _f64(np.ravel(gam))
    s, ps = _f64(np.ravel(surprisal))
    h, ph = _f64(np.ravel(entropy))
    L, B = tb.size, s.size
    assert la.size == L and ga.size == L and h.size == B
    out, po = _out((L, B))
    rc = _load().clada_oracle_threshold(ptb, pla, pga, L, ps, ph, B, C.c_double(tau_s),
                                        C.c_double(tau_H), po)
    assert rc == 0, rc
    return out


def gate_act(w_gate, x, sigma="silu"):
    wg, pg = _f32(w_gate)
    xx, px = _f32(np.atleast_2d(x))
    F, d = wg.shape
    B = xx.shape[0]
    act, pa = _out((B, F))
    _set_sigma(sigma)
    rc = _load().clada_oracle_gate_act(pg, d, F, px, B, pa)
    assert rc == 0, rc
    return act


def sparse_decode(w_gate, w_up, w_down, x, tau, sigma="silu"):
    """One layer's thresholded sparse FFN for x [B][d], tau [B]."""
    keep, (pg, pu, pd), d, F = _weights(w_gate, w_up, w_down)
    xx, px = _f32(np.atleast_2d(x))
    B = xx.shape[0]
    assert xx.shape == (B, d)
    t, pt = _f64(np.ravel(tau))
    assert t.size == B
    y, py = _out((B, d))
    act, pa = _out((B, F))
    mask, pm = _out((B, F), np.uint8)
    idx, pi = _out((F,), np.int32)
    na, pn = _out((1 + B,), np.int32)
    _set_sigma(sigma)
    rc = _load().clada_oracle_sparse_decode(pg, pu, pd, d, F, px, B, pt, py, pa, pm, pi, pn)
    assert rc == 0, rc
    return {"y": y, "act": act, "mask": mask.astype(bool), "active_idx": idx[: na[0]].copy(),
            "n_active": na}


def decode_given_mask(w_gate, w_up, w_down, x, mask, sigma="silu"):
    keep, (pg, pu, pd), d, F = _weights(w_gate, w_up, w_down)
    xx, px = _f32(np.atleast_2d(x))
    B = xx.shape[0]
    m = np.ascontiguousarray(np.atleast_2d(mask), dtype=np.uint8)
    assert m.shape == (B, F)
    y, py = _out((B, d))
    _set_sigma(sigma)
    rc = _load().clada_oracle_decode_given_mask(pg, pu, pd, d, F, px, B,
                                                m.ctypes.data_as(C.POINTER(C.c_uint8)), py)
    assert rc == 0, rc
    return y


def dense_decode(w_gate, w_up, w_down, x, sigma="silu"):
    keep, (pg, pu, pd), d, F = _weights(w_gate, w_up, w_down)
    xx, px = _f32(np.atleast_2d(x))
    B = xx.shape[0]
    y, py = _out((B, d))
    _set_sigma(sigma)
    rc = _load().clada_oracle_dense_decode(pg, pu, pd, d, F, px, B, py)
    assert rc == 0, rc
    return y


def cett(w_gate, w_up, w_down, x, eps, sigma="silu"):
    """Per-token CETT of the validation tokens x [T][d] at cut threshold eps, and its mean."""
    keep, (pg, pu, pd), d, F = _weights(w_gate, w_up, w_down)
    xx, px = _f32(x)
    T = xx.shape[0]
    assert xx.shape == (T, d)
    out, po = _out((T,))
    mean = C.c_double()
    _set_sigma(sigma)
    rc = _load().clada_oracle_cett(pg, pu, pd, d, F, px, T, C.c_double(float(eps)), po, C.byref(mean))
    assert rc == 0, rc
    return out, mean.value


def cett_search(w_gate, w_up, w_down, x, bound=0.2, sigma="silu"):
    """(tau_base, mean CETT at tau_base, rc): the largest eps whose mean CETT over x [T][d] is <= bound.
    rc 0 = attained at a pooled magnitude, 3 = unbounded (tau = inf), 4 = nothing feasible."""
    keep, (pg, pu, pd), d, F = _weights(w_gate, w_up, w_down)
    xx, px = _f32(x)
    T = xx.shape[0]
    assert xx.shape == (T, d)
    tau, mean = C.c_double(), C.c_double()
    _set_sigma(sigma)
    rc = _load().clada_oracle_cett_search(pg, pu, pd, d, F, px, T, C.c_double(float(bound)),
                                          C.byref(tau), C.byref(mean))
    assert rc in (0, 3, 4), rc
    return tau.value, mean.value, rc


def static_mask_threshold(A, tau):
    """(mask bool [F], ascending idx) of the neurons with A_j >= tau."""
    a, pa = _f64(np.ravel(A))
    F = a.size
    mask, pm = _out((F,), np.uint8)
    idx, pi = _out((F,), np.int32)
    n = C.c_int32()
    rc = _load().clada_oracle_static_mask_threshold(pa, F, C.c_double(float(tau)), pm, pi, C.byref(n))
    assert rc == 0, rc
    return mask.astype(bool), idx[: n.value].copy()


def static_mask_topk(score, k):
    """(mask bool [F], ascending idx) of the k largest scores (ties to the lower index, NaN last)."""
    a, pa = _f64(np.ravel(score))
    F = a.size
    mask, pm = _out((F,), np.uint8)
    idx, pi = _out((F,), np.int32)
    n = C.c_int32()
    rc = _load().clada_oracle_static_mask_topk(pa, F, int(k), pm, pi, C.byref(n))
    assert rc == 0, rc
    return mask.astype(bool), idx[: n.value].copy()


def relu_decode(w_in, b_in, w_out, b_out, x, tau=None, mask=None):
    """Non-gated ReLU FFN (OPT family): a = relu(W_in x + b_in), y = sum_kept a W_out[j,:] + b_out.
    tau [B] -> keep iff a >= tau; mask [B][F] -> as given; neither -> dense.  Returns a dict like
    sparse_decode."""
    wi, pi = _f32(w_in)
    wo, po = _f32(w_out)
    F, d = wi.shape
    assert wo.shape == (F, d)
    xx, px = _f32(np.atleast_2d(x))
    B = xx.shape[0]
    bi = bo = None
    pbi = pbo = None
    if b_in is not None:
        bi, pbi = _f32(b_in)
        assert bi.shape == (F,)
    if b_out is not None:
        bo, pbo = _f32(b_out)
        assert bo.shape == (d,)
    pt = pm = None
    if tau is not None:
        t, pt = _f64(np.broadcast_to(np.asarray(tau, np.float64), (B,)))
    elif mask is not None:
        mm = np.ascontiguousarray(np.atleast_2d(mask), dtype=np.uint8)
        assert mm.shape == (B, F)
        pm = mm.ctypes.data_as(C.POINTER(C.c_uint8))
    y, py = _out((B, d))
    act, pa = _out((B, F))
    mo, pmo = _out((B, F), np.uint8)
    idx, pidx = _out((F,), np.int32)
    na, pna = _out((1 + B,), np.int32)
    rc = _load().clada_oracle_relu_decode(pi, pbi, po, pbo, d, F, px, B, pt, pm, py, pa, pmo, pidx, pna)
    assert rc == 0, rc
    return {"y": y, "act": act, "mask": mo.astype(bool), "active_idx": idx[: na[0]].copy(), "n_active": na}


def relu_prefix_stats(w_in, b_in, w_out, b_out, x, want_y=True, want_pool=True):
    """Prefill aggregates of the non-gated ReLU FFN over the prefix x [T][d] (dict like prefix_stats)."""
    wi, pi = _f32(w_in)
    wo, po = _f32(w_out)
    F, d = wi.shape
    xx, px = _f32(x)
    T = xx.shape[0]
    pbi = pbo = None
    if b_in is not None:
        bi, pbi = _f32(b_in)
    if b_out is not None:
        bo, pbo = _f32(b_out)
    y, py = _out((T, d)) if want_y else (None, None)
    pool, pp = _out((T, F)) if want_pool else (None, None)
    names = ("sum_abs_act", "sum_sq_act", "max_abs_act", "sum_sq_h", "A")
    outs = [_out((F,)) for _ in names]
    rc = _load().clada_oracle_relu_prefix_stats(pi, pbi, po, pbo, d, F, px, T, py, *[o[1] for o in outs], pp)
    assert rc == 0, rc
    res = {n: o[0] for n, o in zip(names, outs)}
    res["y"] = y
    res["abs_act_pool"] = pool
    return res


def _relu_args(w_in, b_in, w_out, b_out, x):
    wi, pi = _f32(w_in)
    wo, po = _f32(w_out)
    F, d = wi.shape
    assert wo.shape == (F, d)
    xx, px = _f32(x)
    T = xx.shape[0]
    assert xx.shape == (T, d)
    keep = [wi, wo, xx]
    pbi = pbo = None
    if b_in is not None:
        bi, pbi = _f32(b_in)
        keep.append(bi)
    if b_out is not None:
        bo, pbo = _f32(b_out)
        keep.append(bo)
    return keep, (pi, pbi, po, pbo, d, F, px, T)


def relu_cett(w_in, b_in, w_out, b_out, x, eps):
    """Per-token CETT of the non-gated ReLU FFN over x [T][d] at cut threshold eps, and its mean."""
    keep, args = _relu_args(w_in, b_in, w_out, b_out, x)
    out, po = _out((args[-1],))
    mean = C.c_double()
    rc = _load().clada_oracle_relu_cett(*args, C.c_double(float(eps)), po, C.byref(mean))
    assert rc == 0, rc
    return out, mean.value


def relu_cett_search(w_in, b_in, w_out, b_out, x, bound=0.2):
    """(tau_base, mean CETT at tau_base, rc) for the ReLU FFN; rc as in cett_search."""
    keep, args = _relu_args(w_in, b_in, w_out, b_out, x)
    tau, mean = C.c_double(), C.c_double()
    rc = _load().clada_oracle_relu_cett_search(*args, C.c_double(float(bound)), C.byref(tau), C.byref(mean))
    assert rc in (0, 3, 4), rc
    return tau.value, mean.value, rc
