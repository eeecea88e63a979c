"""GPU parity: clada_cett_eval and clada_threshold_search_cett (section 3.2.2) against the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import BAND, DEV, band_width, to_dev, to_np

pytestmark = pytest.mark.gpu

# Per-token CETT: fp32 layers differ from fp64 by accumulation rounding only; bf16 layers round h
# to bf16 (at most 2^-9 relative per neuron) before both projections, so numerator and denominator
# norms each move by at most 2^-9 relative when the terms do not cancel: 2 * 2^-9 on the ratio
# (reached with a few dozen cut neurons; with thousands the independent roundings average out).
TOL_CETT = {"f32": 2e-5, "bf16": 2 * 2.0 ** -9}
# Search properties judged by the oracle just below / above tau: a few neurons inside that gap may
# fall on either side of the fp64 comparison, each moving one token's CETT by ~1e-3 relative.
TOL_SEARCH = {"f32": 1e-4, "bf16": 2 * 2.0 ** -9}
# tau_base: the device search stops at a boundary of its own feasible set; rounding moves the mean
# by <= TOL_CETT * bound, i.e. a handful of neighbouring pooled magnitudes.
TOL_TAU = {"f32": 1e-4, "bf16": 2e-3}


@pytest.fixture(scope="module")
def clada():
    import paper_2502_19078_amd as m
    m.load_library()
    return m


def _setup(clada, cfg_name, d, F, T, seed=0, layer_id=2, tile=0):
    cfg = synth.CONFIGS[cfg_name]
    w = synth.layer_weights(cfg, seed, layer_id, d=d, d_ff=F)
    X = synth.prefix_hidden(cfg, seed, layer_id, T=T, d=d)
    ctx = clada.Context(0, clada.workspace_bytes(d, F, 0, T, 0))
    ctx.set_option("prefix.tile", tile)
    layer = clada.Layer(*[to_dev(a, cfg.dtype) for a in w])
    return cfg, w, X, ctx, layer, to_dev(X, cfg.dtype)


def _cett_given_cut(w, X, cut):
    """Oracle CETT for a given cut set (bool [T][F]): ||sum of the cut contributions|| / ||dense output||,
    from the oracle's decode functions."""
    y_cut = oracle.decode_given_mask(*w, X, cut)
    dense = oracle.dense_decode(*w, X)
    nd = np.linalg.norm(dense, axis=1)
    return np.where(nd > 0, np.linalg.norm(y_cut, axis=1) / np.where(nd > 0, nd, 1.0), 0.0)


# last entry: option prefix.tile (0 = the library's choice, 2 = the 256-row tiles of both prefill GEMMs)
CASES = [
    ("c1", 512, 1376, 64, 0),    # config 1 as written (fp32)
    ("c1", 96, 200, 130, 0),     # ragged in every dimension
    ("c1", 8, 5, 1, 0),          # one token
    ("c2", 1024, 1000, 300, 0),  # bf16, ragged tiles
    ("c2", 72, 129, 257, 0),
    ("c2", 512, 416, 300, 2),    # 256 x 256 down-projection tiles: 13 k-tiles of 32, d_ff not a multiple of 64
    ("c2", 256, 64, 257, 2),     # two k-tiles; the second token tile holds one token
    ("c2", 256, 768, 257, 0),    # down projection split three ways along d_ff, row norms from the combining pass
]


@pytest.mark.parametrize("cfg_name,d,F,T,tile", CASES)
def test_cett_eval_parity(clada, cfg_name, d, F, T, tile):
    """The device's cut set is read off the device's own |a| pool (the same kernel feeds the masking
    pass), validated against the oracle's inside the band around eps, and the oracle is evaluated on
    that set: a neuron within rounding of eps may fall on either side, everything else is fixed."""
    cfg, w, X, ctx, layer, Xd = _setup(clada, cfg_name, d, F, T, tile=tile)
    a_ref = oracle.prefix_stats(*w, X, want_y=False)["abs_act_pool"]
    pool_ref = np.sort(a_ref.ravel())
    pool_gpu = clada.prefix_stats(ctx, layer, Xd, want_y=False).abs_act_pool.cpu().numpy()
    tol = TOL_CETT[cfg.dtype]
    for q in (0.0, 0.2, 0.45, 0.8):
        eps = float(np.float32(pool_ref[int(q * (len(pool_ref) - 1))] * 1.00037 + 1e-9))
        got, mean = clada.cett_eval(ctx, layer, Xd, eps)
        torch.cuda.synchronize()
        cut_gpu = pool_gpu < np.float32(eps)
        cut_ref = a_ref < eps
        flips = cut_gpu != cut_ref
        # the band of the decode masks (relative to eps, with the absolute floor for a tiny eps: q = 0 gives
        # eps ~ 1e-7, where the fp32 accumulation error of the pre-activation is what decides)
        assert not (flips & (np.abs(a_ref - eps) > band_width(eps))).any(), "cut sets differ outside the band"
        ref = _cett_given_cut(w, X, cut_gpu)
        np.testing.assert_allclose(to_np(got), ref, rtol=tol, atol=1e-6, err_msg=f"q={q}")
        assert float(mean.item()) == pytest.approx(ref.mean(), rel=tol, abs=1e-6)
        if not flips.any():
            np.testing.assert_allclose(to_np(got), oracle.cett(*w, X, eps)[0], rtol=tol, atol=1e-6)
    # limits: eps = 0 cuts nothing, eps = +inf cuts everything
    got, mean = clada.cett_eval(ctx, layer, Xd, 0.0)
    assert torch.all(got == 0) and float(mean.item()) == 0.0
    got, mean = clada.cett_eval(ctx, layer, Xd, float("inf"))
    np.testing.assert_allclose(to_np(got), 1.0, rtol=1e-6)


@pytest.mark.parametrize("cfg_name,d,F,T,tile", CASES)
@pytest.mark.parametrize("bound", [0.2, 0.05])
def test_cett_search_parity(clada, cfg_name, d, F, T, tile, bound):
    cfg, w, X, ctx, layer, Xd = _setup(clada, cfg_name, d, F, T, tile=tile)
    tau_d, mean_d = clada.threshold_search_cett(ctx, layer, Xd, bound)
    torch.cuda.synchronize()
    tau, mean = float(tau_d.item()), float(mean_d.item())
    tol = TOL_SEARCH[cfg.dtype]
    # What is unique: the result is feasible and sits at a boundary of the feasible set, both judged
    # by the oracle.  tau is one of the device's own magnitudes, so the oracle is asked just below it
    # (that neuron surely kept) and just above it (surely cut).
    m_below = oracle.cett(*w, X, tau * (1 - 1e-5))[1]
    m_above = oracle.cett(*w, X, tau * (1 + 1e-5))[1]
    assert m_below <= bound * (1 + tol) + 1e-6
    assert m_above >= bound * (1 - tol) - 1e-6
    assert mean == pytest.approx(m_below, rel=tol, abs=1e-6) and mean <= bound
    # and it agrees with the exact maximum where single-neuron wiggles are small against the bound
    tau_ref, mean_ref, rc = oracle.cett_search(*w, X, bound)
    assert rc == 0
    if T * F >= 20000:
        assert tau == pytest.approx(tau_ref, rel=TOL_TAU[cfg.dtype])


def test_cett_search_bound_zero_returns_smallest_magnitude(clada):
    """Nothing may be lost: the largest eps that cuts nothing is the smallest pooled magnitude."""
    cfg, w, X, ctx, layer, Xd = _setup(clada, "c1", 64, 96, 20)
    st = clada.prefix_stats(ctx, layer, Xd, want_y=False)
    pmin = float(st.abs_act_pool.min().item())
    tau, mean = clada.threshold_search_cett(ctx, layer, Xd, 0.0)
    assert float(tau.item()) == pmin and float(mean.item()) == 0.0


def test_cett_search_fewer_probes_stay_feasible_and_below(clada):
    cfg, w, X, ctx, layer, Xd = _setup(clada, "c2", 256, 384, 96)
    full = float(clada.threshold_search_cett(ctx, layer, Xd, 0.2, 31)[0].item())
    prev = 0.0
    for n in (4, 8, 12, 20):
        tau_d, mean_d = clada.threshold_search_cett(ctx, layer, Xd, 0.2, n)
        tau = float(tau_d.item())
        assert prev <= tau <= full and float(mean_d.item()) <= 0.2
        prev = tau
    # run to run the whole search is bit-reproducible
    again = float(clada.threshold_search_cett(ctx, layer, Xd, 0.2, 31)[0].item())
    assert again == full


def test_cett_argument_errors(clada):
    from paper_2502_19078_amd.binding import CladaError
    cfg, w, X, ctx, layer, Xd = _setup(clada, "c1", 64, 96, 20)
    for bad in (1.0, -0.1, float("nan")):
        with pytest.raises(CladaError):
            clada.threshold_search_cett(ctx, layer, Xd, bad)
    for n in (0, 32):
        with pytest.raises(CladaError):
            clada.threshold_search_cett(ctx, layer, Xd, 0.2, n)
    with pytest.raises(CladaError):
        clada.cett_eval(ctx, layer, Xd, float("nan"))
    small = clada.Context(0, 4096)
    with pytest.raises(CladaError):
        clada.threshold_search_cett(small, layer, Xd, 0.2)


def test_cett_search_full_size_7b_layer(clada):
    """Config 2's layer shape and prefix length as the validation set: the result is checked with two
    oracle evaluations (feasible at tau, over the bound just above it)."""
    cfg = synth.CONFIGS["c2"]
    d, F, T = cfg.d, cfg.d_ff, 128
    cfg, w, X, ctx, layer, Xd = _setup(clada, "c2", d, F, T, layer_id=5)
    tau_d, mean_d = clada.threshold_search_cett(ctx, layer, Xd, 0.2)
    torch.cuda.synchronize()
    tau, mean = float(tau_d.item()), float(mean_d.item())
    m_at = oracle.cett(*w, X, tau * (1 - 1e-5))[1]
    m_above = oracle.cett(*w, X, tau * 1.002)[1]
    assert m_at <= 0.2 * (1 + TOL_CETT["bf16"]) and m_above > 0.2 * (1 - TOL_CETT["bf16"])
    assert mean == pytest.approx(m_at, rel=TOL_CETT["bf16"])
    assert 0.19 < m_at <= 0.2002


def test_cett_search_graph_replay_matches_eager(clada):
    """The bracket lives on the device and every probe reads it there: the whole search can be
    captured once and replayed; each replay must give the eager bits."""
    cfg, w, X, ctx, layer, Xd = _setup(clada, "c2", 512, 640, 200)
    tau_e, mean_e = clada.threshold_search_cett(ctx, layer, Xd, 0.2)
    torch.cuda.synchronize()
    tau_e, mean_e = tau_e.clone(), mean_e.clone()
    out = torch.zeros(1, dtype=torch.float32, device=DEV)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        clada.threshold_search_cett(ctx, layer, Xd, 0.2, out=out)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        clada.threshold_search_cett(ctx, layer, Xd, 0.2, out=out)
    for _ in range(3):
        out.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, tau_e)
        again = clada.threshold_search_cett(ctx, layer, Xd, 0.2)[0]      # eager call between replays
        torch.cuda.synchronize()
        assert torch.equal(again, tau_e)
