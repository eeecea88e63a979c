"""GPU parity: the non-gated ReLU FFN family (OPT shapes) through the decode calls."""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import BAND, DEV, band_width, TOL_Y, assert_close_y, to_dev, to_np, unpack_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def clada():
    import paper_2502_19078_amd as m
    m.load_library()
    return m


def _layer(clada, cfg, w, biases=True):
    from paper_2502_19078_amd import binding
    w_in, b_in, w_out, b_out = w
    return clada.Layer(to_dev(w_in, cfg.dtype), None, to_dev(w_out, cfg.dtype), kind=binding.RELU,
                       b_in=torch.from_numpy(b_in).to(DEV) if biases else None,
                       b_out=torch.from_numpy(b_out).to(DEV) if biases else None)


CASES = [
    ("o350", 1024, 4096, 1),     # OPT-350M shape: 2 KiB rows, batch-1 kernel
    ("o27", 2560, 10240, 1),     # OPT-2.7B shape: 5 KiB rows, batch-1 kernel with balancing
    ("o27", 2560, 1000, 1),      # ragged neuron count, fewer neurons than the balanced kernel wants
    ("o27", 2560, 640, 4),       # batch > 1, bf16: matrix-core path (five waves), per-token thresholds
    ("o350", 1024, 4096, 8),     # OPT-350M shape at batch 8: matrix-core path, gate tiles only
    ("o27", 2560, 3000, 16),     # a full 16-token pass, ragged neuron count
    ("o27", 2560, 900, 17),      # two passes (9 + 8)
    ("c1", 96, 200, 3),          # fp32, odd row length: generic kernel
    ("o27", 4096, 1024, 1),      # 8 KiB rows (OPT-6.7B width)
    ("o27", 5120, 768, 1),       # 10 KiB rows (OPT-13B width)
]


@pytest.mark.parametrize("cfg_name,d,F,B", CASES)
@pytest.mark.parametrize("biases,b1", [(True, 1), (False, 1), (True, 3)])
def test_relu_sparse_and_dense_parity(clada, cfg_name, d, F, B, biases, b1):
    cfg = synth.CONFIGS[cfg_name]
    w = synth.relu_layer(cfg, 2, 3, d=d, d_ff=F)
    x = synth.decode_hidden(cfg, 2, 3, 0, B=B, d=d)
    wb = w if biases else (w[0], None, w[2], None)
    ctx = clada.Context(0, clada.workspace_bytes(d, F, B, 0, 0))
    ctx.set_option("decode.b1", b1)                      # 3: the balanced batch-1 kernel wherever it can run
    layer = _layer(clada, cfg, w, biases)
    xd = to_dev(x, cfg.dtype)
    act = oracle.relu_decode(*wb, x)["act"]
    for q in (0.0, 0.7, 0.9):
        tau = np.quantile(act, q, axis=1).astype(np.float32)
        if q == 0.7:
            tau = np.maximum(tau, np.float32(1e-6))               # above the exact zeros
        y, idx, cnt, bits = clada.sparse_ffn_decode(ctx, layer, xd, torch.from_numpy(tau).to(DEV), want_lists=True)
        torch.cuda.synchronize()
        ref = oracle.relu_decode(*wb, x, tau=tau.astype(np.float64))
        mask_gpu = unpack_bits(bits, F)
        diff = mask_gpu != ref["mask"]
        band = np.abs(ref["act"] - tau[:, None]) <= band_width(tau)[:, None]
        assert not (diff & ~band).any(), f"q={q}: mask differs outside the band"
        ref_y = oracle.relu_decode(*wb, x, mask=mask_gpu)["y"]
        assert_close_y(to_np(y), ref_y, TOL_Y[cfg.dtype], f"relu sparse q={q}")
        union = np.flatnonzero(mask_gpu.any(0))
        c = cnt.cpu().numpy()
        assert c[0] == union.size and np.array_equal(idx.cpu().numpy()[: c[0]], union)
        assert np.array_equal(c[1:], mask_gpu.sum(1))
    yd = clada.dense_ffn_decode(ctx, layer, xd)
    torch.cuda.synchronize()
    assert_close_y(to_np(yd), oracle.relu_decode(*wb, x)["y"], TOL_Y[cfg.dtype], "relu dense twin")
    # tau = +inf keeps nothing: the output is the output bias
    y_inf = clada.sparse_ffn_decode(ctx, layer, xd, torch.full((B,), float("inf"), device=DEV))
    want = np.broadcast_to(w[3] if biases else np.zeros(d, np.float32), (B, d))
    assert_close_y(to_np(y_inf), want.astype(np.float64), TOL_Y[cfg.dtype] if biases else 0.0, "tau=inf")


def test_relu_tau_zero_equals_dense_and_small_tau_drops_only_zeros(clada):
    cfg = synth.CONFIGS["o27"]
    d, F = 2560, 10240
    w = synth.relu_layer(cfg, 0, 0)
    x = synth.decode_hidden(cfg, 0, 0, 0, B=1)
    ctx = clada.Context(0, clada.workspace_bytes(d, F, 1, 0, 0))
    layer = _layer(clada, cfg, w)
    xd = to_dev(x, cfg.dtype)
    y0, _, c0, _ = clada.sparse_ffn_decode(ctx, layer, xd, torch.zeros(1, device=DEV), want_lists=True)
    y0 = y0.clone()
    yt, _, ct, _ = clada.sparse_ffn_decode(ctx, layer, xd, torch.full((1,), 1e-30, device=DEV), want_lists=True)
    yd = clada.dense_ffn_decode(ctx, layer, xd)
    torch.cuda.synchronize()
    assert int(c0[0]) == F                                   # a >= 0 always: tau = 0 keeps every neuron
    assert 0.3 * F < int(ct[0]) < 0.7 * F                    # the exact zeros of the ReLU are gone
    # dropping exact zeros changes nothing but the summation order
    assert_close_y(to_np(yt), to_np(y0), 2e-2, "zeros dropped")
    assert_close_y(to_np(y0), to_np(yd), 2e-2, "tau=0 vs dense twin")


@pytest.mark.parametrize("d,F,B", [(2560, 900, 2),      # matrix-core path over the list
                                   (2560, 3000, 1),     # streaming list kernel, 5 KiB rows
                                   (1024, 4096, 1),     # streaming list kernel, 2 KiB rows (OPT-350M shape)
                                   (1000, 700, 1)])     # generic list kernel
def test_relu_static_list_decode(clada, d, F, B):
    cfg = synth.CONFIGS["o27"]
    w = synth.relu_layer(cfg, 1, 1, d=d, d_ff=F)
    x = synth.decode_hidden(cfg, 1, 1, 0, B=B, d=d)
    ctx = clada.Context(0, clada.workspace_bytes(d, F, B, 0, 0))
    layer = _layer(clada, cfg, w)
    keep = np.random.default_rng(3).random(F) < 0.4
    idx = torch.zeros(F, dtype=torch.int32, device=DEV)
    ii = np.flatnonzero(keep).astype(np.int32)
    idx[: ii.size] = torch.from_numpy(ii).to(DEV)
    n = torch.tensor([ii.size], dtype=torch.int32, device=DEV)
    y = clada.static_ffn_decode(ctx, layer, to_dev(x, cfg.dtype), idx, n)
    torch.cuda.synchronize()
    ref = oracle.relu_decode(*w, x, mask=np.broadcast_to(keep, (B, F)))["y"]
    assert_close_y(to_np(y), ref, TOL_Y[cfg.dtype], "relu list decode")


@pytest.mark.parametrize("cfg_name,d,F,T,tile", [("o27", 2560, 700, 300, 1), ("o27", 2560, 700, 300, 2),
                                                 ("o350", 1024, 4096, 512, 0), ("c1", 96, 200, 130, 0)])
def test_relu_prefix_stats_parity_and_calibration(clada, cfg_name, d, F, T, tile):
    cfg = synth.CONFIGS[cfg_name]
    w = synth.relu_layer(cfg, 5, 2, d=d, d_ff=F)
    X = synth.prefix_hidden(cfg, 5, 2, T=T, d=d)
    ctx = clada.Context(0, clada.workspace_bytes(d, F, 0, T, 0))
    ctx.set_option("prefix.tile", tile)
    layer = _layer(clada, cfg, w)
    st = clada.prefix_stats(ctx, layer, to_dev(X, cfg.dtype))
    torch.cuda.synchronize()
    ref = oracle.relu_prefix_stats(*w, X)
    np.testing.assert_allclose(to_np(st.abs_act_pool), ref["abs_act_pool"], rtol=1e-4, atol=2e-6)
    for name in ("sum_abs_act", "sum_sq_act", "max_abs_act", "sum_sq_h", "A"):
        np.testing.assert_allclose(to_np(getattr(st, name)), ref[name], rtol=3e-5, atol=1e-6, err_msg=name)
    assert_close_y(to_np(st.y), ref["y"], TOL_Y[cfg.dtype], "relu prefill y")
    tau = clada.threshold_calibrate(ctx, st.abs_act_pool, cfg.q if cfg_name != "c1" else 0.7)
    torch.cuda.synchronize()
    assert float(tau.item()) == oracle.calibrate(to_np(st.abs_act_pool), cfg.q if cfg_name != "c1" else 0.7)
    assert float(tau.item()) > 0.0                      # above the ReLU's own zeros


# as in test_gpu_cett.py; for bf16 the denominator additionally goes through the stored (bf16) output
TOL_CETT = {"f32": 2e-5, "bf16": 3 * 2.0 ** -9}


@pytest.mark.parametrize("cfg_name,d,F,T,tile", [("o27", 2560, 700, 300, 1), ("o27", 2560, 1024, 257, 2),
                                                 ("o350", 1024, 4096, 512, 0), ("c1", 96, 200, 130, 0), ("c1", 8, 5, 1, 0)])
def test_relu_cett_eval_and_search_parity(clada, cfg_name, d, F, T, tile):
    """CETT of the non-gated family: n_j = a_j W_out[j,:], the output bias in the denominator only.  The cut
    set is read off the device's own activation pool (band-validated) and the oracle evaluated on it."""
    cfg = synth.CONFIGS[cfg_name]
    dt = cfg.dtype
    w = synth.relu_layer(cfg, 6, 3, d=d, d_ff=F)
    if dt == "bf16":
        w = (synth.store(w[0], dt), w[1], synth.store(w[2], dt), w[3])
    X = synth.prefix_hidden(cfg, 6, 3, T=T, d=d)
    ctx = clada.Context(0, clada.workspace_bytes(d, F, 0, T, 0))
    ctx.set_option("prefix.tile", tile)
    layer = _layer(clada, cfg, w)
    Xd = to_dev(X, dt)
    a_ref = oracle.relu_prefix_stats(*w, X, want_y=False)["abs_act_pool"]
    pool_gpu = clada.prefix_stats(ctx, layer, Xd, want_y=False).abs_act_pool.cpu().numpy()
    dense = oracle.relu_decode(*w, X)["y"]
    nd = np.linalg.norm(dense, axis=1)
    pos = np.sort(a_ref[a_ref > 0])
    for qq in (0.0, 0.3, 0.8):
        eps = float(np.float32(pos[int(qq * (len(pos) - 1))] * 1.00037 + 1e-9))
        got, mean = clada.cett_eval(ctx, layer, Xd, eps)
        torch.cuda.synchronize()
        cut_gpu = pool_gpu < np.float32(eps)
        flips = cut_gpu != (a_ref < eps)
        assert not (flips & (np.abs(a_ref - eps) > band_width(eps))).any(), "cut sets differ outside the band"
        kept = oracle.relu_decode(*w, X, mask=~cut_gpu)["y"]                    # keeps the rest, adds b_out
        ref = np.where(nd > 0, np.linalg.norm(dense - kept, axis=1) / np.where(nd > 0, nd, 1.0), 0.0)
        np.testing.assert_allclose(to_np(got), ref, rtol=TOL_CETT[dt], atol=1e-6, err_msg=f"q={qq}")
        assert float(mean.item()) == pytest.approx(ref.mean(), rel=TOL_CETT[dt], abs=1e-6)
        if not flips.any():
            np.testing.assert_allclose(to_np(got), oracle.relu_cett(*w, X, eps)[0], rtol=TOL_CETT[dt], atol=1e-6)
    got, mean = clada.cett_eval(ctx, layer, Xd, 0.0)
    assert torch.all(got == 0) and float(mean.item()) == 0.0
    # search: feasible just below, infeasible just above (both by the oracle), near the oracle's maximum
    for bound in (0.2, 0.05):
        tau_d, mean_d = clada.threshold_search_cett(ctx, layer, Xd, bound)
        torch.cuda.synchronize()
        tau, mean = float(tau_d.item()), float(mean_d.item())
        tol = TOL_CETT[dt] if dt == "bf16" else 1e-4
        tau_ref, _, rc = oracle.relu_cett_search(*w, X, bound)
        m_below = oracle.relu_cett(*w, X, tau * (1 - 1e-5))[1]
        assert m_below <= bound * (1 + tol) + 1e-6
        assert mean == pytest.approx(m_below, rel=tol, abs=1e-6) and mean <= bound
        if rc == 3:     # even cutting every neuron stays within the bound (the bias carries the output): no maximum
            assert tau > a_ref.max()
            continue
        m_above = oracle.relu_cett(*w, X, tau * (1 + 1e-5))[1]
        assert m_above >= bound * (1 - tol) - 1e-6
        if rc == 0 and T * F >= 20000:
            assert tau == pytest.approx(tau_ref, rel=2e-3 if dt == "bf16" else 1e-4)
