"""GPU parity: clada_prefix_stats (MFMA prefill + fused aggregates) and the calibration chain."""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import DEV, TOL_Y, assert_close_y, to_dev, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def clada():
    import paper_2502_19078_amd as m
    m.load_library()
    return m


def _rel(a, b):
    return np.linalg.norm(np.asarray(a, np.float64) - b) / max(np.linalg.norm(b), 1e-300)


@pytest.mark.parametrize("cfg_name,d,F,T", [
    ("c1", 512, 1376, 64),       # config 1 as written (fp32 MFMA)
    ("c1", 96, 200, 130),        # ragged in every dimension, K not a multiple of the 32-wide k-tile
    ("c1", 8, 5, 1),             # degenerate: one token, one k-chunk
    ("c2", 1024, 1000, 300),     # bf16 MFMA, ragged tiles
    ("c2", 4096, 384, 512),      # bf16, real K and prefix length of config 2, three neuron tiles
    ("c2", 72, 129, 257),
    ("c2", 64, 200, 300),        # two 32-deep k-tiles: shorter than the 256-token kernel's pipeline
    ("c2", 128, 100, 257),       # four k-tiles: exactly the four LDS stages, no steady-state iteration
    ("c2", 192, 129, 513),       # six k-tiles; the last 256-token tile holds one token
    ("c2", 320, 64, 129),        # ten k-tiles; second half of the only 256-token tile holds one token
    ("c2", 512, 700, 1024),      # 8 token tiles: the blocked tile order, 6 neuron tiles padded to 8
    ("c2", 256, 384, 2000),      # 16 token tiles (last one ragged), 3 neuron tiles
    ("c2", 64, 40, 1),           # bf16, one token: every row of a tile repeats it
    ("c2", 512, 32, 300),        # a single 32-deep k-tile in the 256 x 256 down projection
    ("c2", 768, 96, 520),        # three column tiles, three k-tiles
    ("c2", 512, 1024, 300),      # few tiles, long d_ff: the down projection splits d_ff four ways
    ("c2", 256, 800, 130),       # split three ways, 25 k-tiles (uneven parts)
])
@pytest.mark.parametrize("tile", [1, 2])
def test_prefix_stats_parity(clada, cfg_name, d, F, T, tile):
    """tile = workgroup tile of the bf16 gate/up GEMM (128 or 256 tokens); fp32 layers have one kernel."""
    cfg = synth.CONFIGS[cfg_name]
    if tile == 2 and cfg.dtype != "bf16":
        pytest.skip("the 256-token tile is a bf16 kernel")
    w = synth.layer_weights(cfg, 0, 1, d=d, d_ff=F)
    X = synth.prefix_hidden(cfg, 0, 1, T=T, d=d)
    ctx = clada.Context(0, clada.workspace_bytes(d, F, 0, T, 0))
    ctx.set_option("prefix.tile", tile)
    layer = clada.Layer(*[to_dev(a, cfg.dtype) for a in w])
    st = clada.prefix_stats(ctx, layer, to_dev(X, cfg.dtype))
    torch.cuda.synchronize()
    ref = oracle.prefix_stats(*w, X)
    tol = 1e-5
    # statistics come from fp32 accumulators of exact products in both dtypes
    assert _rel(to_np(st.abs_act_pool), ref["abs_act_pool"]) < tol
    np.testing.assert_allclose(to_np(st.abs_act_pool), ref["abs_act_pool"], rtol=1e-4, atol=1e-6)
    for name in ("sum_abs_act", "sum_sq_act", "max_abs_act", "sum_sq_h", "A"):
        got = to_np(getattr(st, name))
        np.testing.assert_allclose(got, ref[name], rtol=2e-5, atol=1e-7, err_msg=name)
    assert_close_y(to_np(st.y), ref["y"], TOL_Y[cfg.dtype], "prefill y")
    # A_j for T=1 reduces to |h_j| * ||W_down[j]||
    # calibration chain: the GPU quantile of the GPU pool is an exact order statistic of that pool
    tau = clada.threshold_calibrate(ctx, st.abs_act_pool, cfg.q)
    torch.cuda.synchronize()
    assert float(tau.item()) == oracle.calibrate(to_np(st.abs_act_pool), cfg.q)
    assert float(tau.item()) == pytest.approx(oracle.calibrate(ref["abs_act_pool"], cfg.q), rel=1e-4)


def test_prefix_stats_without_optional_outputs(clada):
    cfg = synth.CONFIGS["c2"]
    d, F, T = 256, 300, 100
    w = synth.layer_weights(cfg, 1, 0, d=d, d_ff=F)
    X = synth.prefix_hidden(cfg, 1, 0, T=T, d=d)
    ctx = clada.Context(0, clada.workspace_bytes(d, F, 0, T, 0))
    layer = clada.Layer(*[to_dev(a, cfg.dtype) for a in w])
    st = clada.prefix_stats(ctx, layer, to_dev(X, cfg.dtype), want_y=False, want_pool=False)
    torch.cuda.synchronize()
    ref = oracle.prefix_stats(*w, X, want_y=False)
    assert st.y is None and st.abs_act_pool is None
    np.testing.assert_allclose(to_np(st.A), ref["A"], rtol=2e-5, atol=1e-7)


def test_calibrated_threshold_gives_target_decode_sparsity(clada):
    """Prefill -> calibrate -> decode on fresh tokens: measured sparsity is near the target."""
    cfg = synth.CONFIGS["c2"]
    d, F, T = 1024, 2752, 512
    w = synth.layer_weights(cfg, 2, 0, d=d, d_ff=F)
    X = synth.prefix_hidden(cfg, 2, 0, T=T, d=d)
    ctx = clada.Context(0, clada.workspace_bytes(d, F, 8, T, 0))
    layer = clada.Layer(*[to_dev(a, cfg.dtype) for a in w])
    st = clada.prefix_stats(ctx, layer, to_dev(X, cfg.dtype), want_y=False)
    tau = clada.threshold_calibrate(ctx, st.abs_act_pool, cfg.q)
    x = synth.decode_hidden(cfg, 2, 0, 0, B=8, d=d)
    y, idx, cnt, bits = clada.sparse_ffn_decode(ctx, layer, to_dev(x, cfg.dtype), tau.expand(8).contiguous(),
                                                want_lists=True)
    torch.cuda.synchronize()
    rho = 1.0 - cnt[1:].float().mean().item() / F
    assert abs(rho - cfg.q) < 0.03


@pytest.mark.parametrize("cfg_name,layer_id", [("c4", 3), ("c2", 7)])
def test_prefix_stats_full_size_layers_sampled(clada, cfg_name, layer_id):
    """One full-size layer with the configuration's own prefix length (LLaMA-3-8B shape with 4096
    tokens, LLaMA2-7B shape with 512), in the launch the benchmark times.  The oracle is too slow
    for the whole prefill, so it checks what it can compute piece by piece: per-neuron aggregates
    and pool columns of sampled neurons (each neuron's statistics depend on its own three weight
    rows only), and the output rows of sampled tokens (the prefill output of a token is its dense
    decode)."""
    cfg = synth.CONFIGS[cfg_name]
    d, F, T = cfg.d, cfg.d_ff, cfg.T
    w = synth.layer_weights(cfg, 0, layer_id)
    X = synth.prefix_hidden(cfg, 0, layer_id)
    assert X.shape == (T, d)
    ctx = clada.Context(0, clada.workspace_bytes(d, F, 0, T, 0))
    layer = clada.Layer(*[to_dev(a, cfg.dtype) for a in w])
    st = clada.prefix_stats(ctx, layer, to_dev(X, cfg.dtype))
    torch.cuda.synchronize()
    rng = np.random.default_rng(11)
    # neurons at tile borders of both kernels' tilings plus random ones
    S = np.unique(np.concatenate([[0, 31, 32, 63, 64, 127, 128, F - 129, F - 128, F - 1],
                                  rng.integers(0, F, 54)])).astype(np.int64)
    ref = oracle.prefix_stats(w[0][S], w[1][S], w[2][S], X, want_y=False)
    pool = to_np(st.abs_act_pool[:, torch.from_numpy(S).to(DEV)])
    np.testing.assert_allclose(pool, ref["abs_act_pool"], rtol=1e-4, atol=1e-6)
    for name in ("sum_abs_act", "sum_sq_act", "max_abs_act", "sum_sq_h", "A"):
        np.testing.assert_allclose(to_np(getattr(st, name))[S], ref[name], rtol=2e-5, atol=1e-7, err_msg=name)
    toks = np.unique(np.concatenate([[0, 127, 128, 255, 256, T - 1], rng.integers(0, T, 4)]))
    y = to_np(st.y)
    for t in toks:
        assert_close_y(y[t:t + 1], oracle.dense_decode(*w, X[t:t + 1]), TOL_Y[cfg.dtype], f"prefill y, token {t}")
