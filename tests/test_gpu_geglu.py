"""GPU parity: the GELU-gated FFN family (Gemma shape; sigma = tanh-form GELU) through every call that
takes a layer.  Same kernels as the SiLU-gated family, so the cases go for one of each code path."""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import BAND, DEV, band_width, TOL_Y, assert_close_y, to_dev, to_np, unpack_bits

pytestmark = pytest.mark.gpu
SIG = "gelu_tanh"
TOL_CETT = {"f32": 2e-5, "bf16": 2 * 2.0 ** -9}      # as in test_gpu_cett.py


@pytest.fixture(scope="module")
def clada():
    import paper_2502_19078_amd as m
    m.load_library()
    return m


def _layer(clada, cfg, w):
    from paper_2502_19078_amd import binding
    return clada.Layer(*[to_dev(a, cfg.dtype) for a in w], kind=binding.GEGLU)


CASES = [
    ("g2b", 2048, 16384, 1, 1),  # Gemma-2B layer: 4 KiB rows, 64 neurons per workgroup, batch-1 kernel
    ("g2b", 2048, 1500, 1, 3),   # balanced batch-1 kernel forced, ragged neuron count
    ("g2b", 2048, 700, 1, 0),    # generic kernels
    ("g2b", 2048, 3000, 8, 1),   # matrix-core batched path
    ("g2b", 2048, 640, 20, 1),   # more than 16 tokens: two passes of the batched path
    ("c1", 96, 200, 3, 1),       # fp32, odd row length: generic kernel
    ("c2", 4096, 1024, 1, 1),    # 8 KiB rows
]


@pytest.mark.parametrize("cfg_name,d,F,B,b1", CASES)
def test_geglu_sparse_and_dense_parity(clada, cfg_name, d, F, B, b1):
    cfg = synth.CONFIGS[cfg_name]
    w = synth.layer_weights(cfg, 4, 2, d=d, d_ff=F)
    x = synth.decode_hidden(cfg, 4, 2, 0, B=B, d=d)
    ctx = clada.Context(0, clada.workspace_bytes(d, F, B, 0, 0))
    ctx.set_option("decode.b1", b1)
    layer = _layer(clada, cfg, w)
    xd = to_dev(x, cfg.dtype)
    act = np.abs(oracle.gate_act(w[0], x, sigma=SIG))
    for q in (0.0, 0.45, 0.8):
        tau = (np.quantile(act, q, axis=1) * np.resize([1.0, 1.12, 1.8, 1.92], B)).astype(np.float32) if q else np.zeros(B, np.float32)
        y, idx, cnt, bits = clada.sparse_ffn_decode(ctx, layer, xd, torch.from_numpy(tau).to(DEV), want_lists=True)
        torch.cuda.synchronize()
        ref = oracle.sparse_decode(*w, x, tau.astype(np.float64), sigma=SIG)
        mask_gpu = unpack_bits(bits, F)
        diff = mask_gpu != ref["mask"]
        band = np.abs(np.abs(ref["act"]) - tau[:, None]) <= band_width(tau)[:, None]
        assert not (diff & ~band).any(), f"q={q}: mask differs outside the band"
        ref_y = oracle.decode_given_mask(*w, x, mask_gpu, sigma=SIG)
        assert_close_y(to_np(y), ref_y, TOL_Y[cfg.dtype], f"geglu sparse q={q}")
        union = np.flatnonzero(mask_gpu.any(0))
        c = cnt.cpu().numpy()
        assert c[0] == union.size and np.array_equal(idx.cpu().numpy()[: c[0]], union)
        assert np.array_equal(c[1:], mask_gpu.sum(1))
        if q == 0.0:
            assert c[0] == F
    yd = clada.dense_ffn_decode(ctx, layer, xd)
    torch.cuda.synchronize()
    dense = oracle.dense_decode(*w, x, sigma=SIG)
    assert_close_y(to_np(yd), dense, TOL_Y[cfg.dtype], "geglu dense twin")
    # it is not the SiLU layer
    assert np.linalg.norm(dense - oracle.dense_decode(*w, x)) > 0.05 * np.linalg.norm(dense)
    y_inf = clada.sparse_ffn_decode(ctx, layer, xd, torch.full((B,), float("inf"), device=DEV))
    torch.cuda.synchronize()
    assert not to_np(y_inf).any()


@pytest.mark.parametrize("cfg_name,d,F,T,tile", [("g2b", 2048, 700, 300, 1), ("g2b", 2048, 512, 300, 2),
                                                 ("c1", 96, 200, 130, 0)])
def test_geglu_prefix_stats_calibration_and_cett(clada, cfg_name, d, F, T, tile):
    cfg = synth.CONFIGS[cfg_name]
    w = synth.layer_weights(cfg, 5, 1, d=d, d_ff=F)
    X = synth.prefix_hidden(cfg, 5, 1, T=T, d=d)
    ctx = clada.Context(0, clada.workspace_bytes(d, F, 0, T, 0))
    ctx.set_option("prefix.tile", tile)
    layer = _layer(clada, cfg, w)
    Xd = to_dev(X, cfg.dtype)
    st = clada.prefix_stats(ctx, layer, Xd)
    torch.cuda.synchronize()
    ref = oracle.prefix_stats(*w, X, sigma=SIG)
    np.testing.assert_allclose(to_np(st.abs_act_pool), ref["abs_act_pool"], rtol=1e-4, atol=1e-6)
    for name in ("sum_abs_act", "sum_sq_act", "max_abs_act", "sum_sq_h", "A"):
        np.testing.assert_allclose(to_np(getattr(st, name)), ref[name], rtol=2e-5, atol=1e-7, err_msg=name)
    assert_close_y(to_np(st.y), ref["y"], TOL_Y[cfg.dtype], "geglu prefill y")
    tau = clada.threshold_calibrate(ctx, st.abs_act_pool, 0.45)
    torch.cuda.synchronize()
    assert float(tau.item()) == oracle.calibrate(to_np(st.abs_act_pool), 0.45)
    # CETT of a probe between two pooled magnitudes: the cut set is the same on both sides
    pool = np.sort(ref["abs_act_pool"].ravel())
    k = int(0.5 * pool.size)
    while pool[k + 1] - pool[k] < 1e-4 * pool[k]:
        k += 1
    eps = float(np.float32(0.5 * (pool[k] + pool[k + 1])))
    got, mean = clada.cett_eval(ctx, layer, Xd, eps)
    torch.cuda.synchronize()
    per, m = oracle.cett(*w, X, eps, sigma=SIG)
    if np.array_equal(to_np(st.abs_act_pool) < np.float32(eps), ref["abs_act_pool"] < eps):
        np.testing.assert_allclose(to_np(got), per, rtol=TOL_CETT[cfg.dtype], atol=1e-6)
        assert float(mean.item()) == pytest.approx(m, rel=TOL_CETT[cfg.dtype])
    tau_d, mean_d = clada.threshold_search_cett(ctx, layer, Xd, 0.2)
    torch.cuda.synchronize()
    t = float(tau_d.item())
    assert oracle.cett(*w, X, t * (1 - 1e-5), sigma=SIG)[1] <= 0.2 * (1 + TOL_CETT[cfg.dtype])
    assert oracle.cett(*w, X, t * 1.002, sigma=SIG)[1] > 0.2 * (1 - TOL_CETT[cfg.dtype])


def test_geglu_static_list_decode(clada):
    cfg = synth.CONFIGS["g2b"]
    for d, F, B in ((2048, 3000, 1), (2048, 900, 3)):
        w = synth.layer_weights(cfg, 1, 1, d=d, d_ff=F)
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
        ref = oracle.decode_given_mask(*w, x, np.broadcast_to(keep, (B, F)), sigma=SIG)
        assert_close_y(to_np(y), ref, TOL_Y[cfg.dtype], "geglu list decode")
