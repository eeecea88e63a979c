"""GPU parity: prefix-static masks (threshold on A_j, hard top-k) and the list decode."""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import BAND, DEV, TOL_Y, assert_close_y, to_dev, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def clada():
    import paper_2502_19078_amd as m
    m.load_library()
    return m


def _ctx(clada, d, F, B, T=0):
    return clada.Context(0, clada.workspace_bytes(d, F, B, T, 0))


@pytest.mark.parametrize("F", [1, 5, 64, 1000, 1376, 11008, 262144])
def test_mask_threshold_bit_exact(clada, F):
    rng = np.random.default_rng(F)
    A = np.abs(rng.standard_normal(F)).astype(np.float32)
    if F >= 64:
        A[7] = np.nan
        A[11] = A[12] = A[13]                         # equal magnitudes
    ctx = _ctx(clada, 64, min(F, 4096), 1)
    Ad = torch.from_numpy(A).to(DEV)
    for tau in (0.0, float(np.median(A[np.isfinite(A)])), float(A[min(12, F - 1)]) if F >= 64 else 0.5, 9.0, float("inf")):
        idx, n = clada.static_mask_threshold(ctx, Ad, torch.tensor([tau], dtype=torch.float32, device=DEV))
        torch.cuda.synchronize()
        want = oracle.static_mask_threshold(A, np.float32(tau))[1]
        assert int(n.item()) == want.size
        assert np.array_equal(idx.cpu().numpy()[: want.size], want)


@pytest.mark.parametrize("F", [1, 5, 64, 1000, 1376, 11008, 262144])
def test_mask_topk_bit_exact(clada, F):
    rng = np.random.default_rng(F + 1)
    s = np.round(rng.standard_normal(F), 2).astype(np.float32)      # many ties, both signs
    if F >= 64:
        s[3] = np.nan
        s[20] = 0.0
        s[21] = -0.0
        s[40] = np.inf
        s[41] = -np.inf
    ctx = _ctx(clada, 64, min(F, 4096), 1)
    sd = torch.from_numpy(s).to(DEV)
    for k in sorted({0, min(1, F), min(2, F), F // 3, F // 2, max(F - 2, 0), F}):
        idx, n = clada.static_mask_topk(ctx, sd, k)
        torch.cuda.synchronize()
        want = oracle.static_mask_topk(s, k)[1]
        assert int(n.item()) == k == want.size
        assert np.array_equal(idx.cpu().numpy()[:k], want), f"F={F} k={k}"


CASES = [
    ("c1", 512, 1376, 1),
    ("c1", 96, 200, 3),
    ("c1", 8, 5, 1),
    ("c2", 1024, 1000, 1),
    ("c2", 4096, 640, 1),        # config 2's row length, whole-KiB rows
    ("c2", 72, 129, 4),
    ("c5", 5120, 512, 2),        # batch > 1, bf16: matrix-core path over the list
    ("c2", 4096, 3000, 8),       #   8 KiB rows, 8 tokens
    ("c2", 1024, 20000, 16),     #   wide layer: several rounds per workgroup, 16 tokens
    ("c2", 2048, 700, 17),       #   two passes (9 + 8)
    ("c5", 5120, 700, 1),        # 10 KiB rows: the unpipelined variant of the list kernel
    ("c2", 2560, 900, 1),        # 5 KiB rows
    ("c1", 512, 4100, 1),        # fp32, 2 KiB rows, 16 entries per workgroup and a ragged tail
]


@pytest.mark.parametrize("cfg_name,d,F,B", CASES)
def test_list_decode_parity(clada, cfg_name, d, F, B):
    cfg = synth.CONFIGS[cfg_name]
    w = synth.layer_weights(cfg, 3, 1, d=d, d_ff=F)
    x = synth.decode_hidden(cfg, 3, 1, 0, B=B, d=d)
    ctx = _ctx(clada, d, F, B)
    layer = clada.Layer(*[to_dev(a, cfg.dtype) for a in w])
    xd = to_dev(x, cfg.dtype)
    rng = np.random.default_rng(d + F)
    for frac in (0.0, 0.1, 0.55, 1.0):
        keep = rng.random(F) < frac
        if frac == 1.0:
            keep[:] = True
        idx_np = np.flatnonzero(keep).astype(np.int32)
        idx = torch.zeros(F, dtype=torch.int32, device=DEV)
        idx[: idx_np.size] = torch.from_numpy(idx_np).to(DEV)
        n = torch.tensor([idx_np.size], dtype=torch.int32, device=DEV)
        y = clada.static_ffn_decode(ctx, layer, xd, idx, n)
        y2 = clada.static_ffn_decode(ctx, layer, xd, idx, n)
        torch.cuda.synchronize()
        assert torch.equal(y, y2), "not bit-reproducible"
        ref = oracle.decode_given_mask(*w, x, np.broadcast_to(keep, (B, F)))
        assert_close_y(to_np(y), ref, TOL_Y[cfg.dtype], f"list decode frac={frac}")
    # the full list is the dense twin
    yd = clada.dense_ffn_decode(ctx, layer, xd)
    assert_close_y(to_np(y), to_np(yd).astype(np.float64), 4 * TOL_Y[cfg.dtype] if cfg.dtype == "bf16" else 1e-5,
                   "full list vs dense twin")


@pytest.mark.parametrize("mode", ["threshold", "topk"])
def test_prefix_static_chain(clada, mode):
    """Prefill magnitudes -> mask -> list decode, each link against the oracle.  The device's A_j are
    fp32; a neuron whose fp64 A_j lies within the band around tau may fall on either side."""
    cfg = synth.CONFIGS["c2"]
    d, F, T = 1024, 1500, 96
    w = synth.layer_weights(cfg, 4, 0, d=d, d_ff=F)
    X = synth.prefix_hidden(cfg, 4, 0, T=T, d=d)
    x = synth.decode_hidden(cfg, 4, 0, 0, B=1, d=d)
    ctx = _ctx(clada, d, F, 1, T)
    layer = clada.Layer(*[to_dev(a, cfg.dtype) for a in w])
    st = clada.prefix_stats(ctx, layer, to_dev(X, cfg.dtype), want_y=False, want_pool=False)
    A_gpu = st.A.cpu().numpy()
    A_ref = oracle.prefix_stats(*w, X, want_y=False, want_pool=False)["A"]
    np.testing.assert_allclose(A_gpu, A_ref, rtol=2e-5)
    if mode == "threshold":
        tau = np.float32(np.quantile(A_ref, 0.45))
        idx, n = clada.static_mask_threshold(ctx, st.A, torch.tensor([tau], dtype=torch.float32, device=DEV))
        keep_ref = oracle.static_mask_threshold(A_ref, tau)[0]
        exact = oracle.static_mask_threshold(A_gpu, tau)[1]
    else:
        k = int(0.55 * F)
        idx, n = clada.static_mask_topk(ctx, st.A, k)
        keep_ref = oracle.static_mask_topk(A_ref, k)[0]
        exact = oracle.static_mask_topk(A_gpu, k)[1]
        tau = np.sort(A_ref)[F - k]
    torch.cuda.synchronize()
    cnt = int(n.item())
    got = idx.cpu().numpy()[:cnt]
    assert np.array_equal(got, exact)                       # integer work on identical inputs: bit-exact
    keep_gpu = np.zeros(F, bool)
    keep_gpu[got] = True
    flips = keep_gpu != keep_ref
    assert not (flips & (np.abs(A_ref - tau) > BAND * tau)).any()
    y = clada.static_ffn_decode(ctx, layer, to_dev(x, cfg.dtype), idx, n)
    torch.cuda.synchronize()
    ref = oracle.decode_given_mask(*w, x, keep_gpu[None, :])
    assert_close_y(to_np(y), ref, TOL_Y[cfg.dtype], "chain output")
    assert 0.3 * F < cnt < 0.8 * F


@pytest.mark.parametrize("cfg_name", ["c2", "c4", "c5"])
def test_list_decode_full_size_layers(clada, cfg_name):
    """Full layer shapes at batch 1, list = hard top-k at the configuration's target sparsity."""
    cfg = synth.CONFIGS[cfg_name]
    d, F = cfg.d, cfg.d_ff
    w = synth.layer_weights(cfg, 0, 7)
    x = synth.decode_hidden(cfg, 0, 7, 0, B=1)
    ctx = _ctx(clada, d, F, 1)
    layer = clada.Layer(*[to_dev(a, cfg.dtype) for a in w])
    xd = to_dev(x, cfg.dtype)
    score = np.abs(np.random.default_rng(5).standard_normal(F)).astype(np.float32)
    k = int(round((1 - 0.45) * F))
    idx, n = clada.static_mask_topk(ctx, torch.from_numpy(score).to(DEV), k)
    y = clada.static_ffn_decode(ctx, layer, xd, idx, n)
    ctx.set_option("decode.b1", 0)                       # the generic list kernels on the same list
    y_gen = clada.static_ffn_decode(ctx, layer, xd, idx, n)
    torch.cuda.synchronize()
    keep = oracle.static_mask_topk(score, k)[0]
    assert np.array_equal(np.flatnonzero(keep), idx.cpu().numpy()[:k])
    ref = oracle.decode_given_mask(*w, x, keep[None, :])
    assert_close_y(to_np(y), ref, TOL_Y[cfg.dtype], "list kernel")
    assert_close_y(to_np(y_gen), ref, TOL_Y[cfg.dtype], "generic list kernel")


def test_list_decode_accepts_the_dynamic_calls_lists(clada):
    """active_idx / n_active of clada_sparse_ffn_decode feed the list decode: same neurons, same output
    up to summation order."""
    cfg = synth.CONFIGS["c2"]
    d, F = 4096, 1024
    w = synth.layer_weights(cfg, 6, 0, d=d, d_ff=F)
    x = synth.decode_hidden(cfg, 6, 0, 0, B=1, d=d)
    ctx = _ctx(clada, d, F, 1)
    layer = clada.Layer(*[to_dev(a, cfg.dtype) for a in w])
    xd = to_dev(x, cfg.dtype)
    tau = torch.tensor([0.25], dtype=torch.float32, device=DEV)
    y_dyn, idx, cnt, _ = clada.sparse_ffn_decode(ctx, layer, xd, tau, want_lists=True)
    y_dyn = y_dyn.clone()
    y_list = clada.static_ffn_decode(ctx, layer, xd, idx, cnt)
    torch.cuda.synchronize()
    assert_close_y(to_np(y_list), to_np(y_dyn), 2e-2, "list vs dynamic")


def test_static_argument_errors(clada):
    from paper_2502_19078_amd.binding import CladaError
    ctx = _ctx(clada, 64, 96, 1)
    s = torch.zeros(96, dtype=torch.float32, device=DEV)
    with pytest.raises(CladaError):
        clada.static_mask_topk(ctx, s, 97)
    with pytest.raises(CladaError):
        clada.static_mask_topk(ctx, s, -1)


def test_static_chain_graph_replay_matches_eager(clada):
    """Mask builder + list decode captured together; the list and its count stay on the device."""
    cfg = synth.CONFIGS["c2"]
    d, F = 4096, 2048
    w = synth.layer_weights(cfg, 8, 0, d=d, d_ff=F)
    x = synth.decode_hidden(cfg, 8, 0, 0, B=1, d=d)
    ctx = _ctx(clada, d, F, 1)
    layer = clada.Layer(*[to_dev(a, cfg.dtype) for a in w])
    xd = to_dev(x, cfg.dtype)
    score = torch.rand(F, device=DEV)
    tau = torch.tensor([0.4], dtype=torch.float32, device=DEV)
    idx, n = clada.static_mask_threshold(ctx, score, tau)
    y_e = clada.static_ffn_decode(ctx, layer, xd, idx, n).clone()
    torch.cuda.synchronize()
    lib, h = ctx._lib, ctx._h
    import ctypes as C
    cl = layer.c_struct()
    idx_g = torch.zeros(F, dtype=torch.int32, device=DEV)
    n_g = torch.zeros(1, dtype=torch.int32, device=DEV)
    y_g = torch.empty_like(y_e)
    side = torch.cuda.Stream()

    def body():
        sp = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        ctx.check(lib.clada_static_mask_threshold(h, score.data_ptr(), F, tau.data_ptr(), idx_g.data_ptr(),
                                                  n_g.data_ptr(), sp))
        ctx.check(lib.clada_static_ffn_decode(h, C.byref(cl), xd.data_ptr(), 1, idx_g.data_ptr(), n_g.data_ptr(),
                                              y_g.data_ptr(), sp))

    with torch.cuda.stream(side):
        body()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        body()
    for _ in range(3):
        y_g.zero_()
        n_g.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert int(n_g.item()) == int(n.item()) and torch.equal(y_g, y_e)
        y2 = clada.static_ffn_decode(ctx, layer, xd, idx, n)
        torch.cuda.synchronize()
        assert torch.equal(y2, y_e)


@pytest.mark.parametrize("F", [1, 31, 32, 33, 1000, 11008, 262144])
def test_mask_pack_unpack_bit_exact(clada, F):
    """Packed storage: the words are numpy's little-endian bit packing of the mask, the round trip is
    the identity, and the dynamic call's own mask_bits unpack to its own list."""
    rng = np.random.default_rng(F + 7)
    keep = rng.random(F) < 0.55
    ctx = _ctx(clada, 64, min(F, 4096), 1)
    ii = np.flatnonzero(keep).astype(np.int32)
    idx = torch.full((F,), -1, dtype=torch.int32, device=DEV)
    idx[: ii.size] = torch.from_numpy(ii).to(DEV)
    n = torch.tensor([ii.size], dtype=torch.int32, device=DEV)
    bits = clada.mask_pack(ctx, idx, n, F)
    torch.cuda.synchronize()
    words = (F + 31) // 32
    want = np.packbits(np.pad(keep, (0, words * 32 - F)), bitorder="little").view(np.uint32)
    assert np.array_equal(bits.cpu().numpy().view(np.uint32), want)
    idx2, n2 = clada.mask_unpack(ctx, bits, F)
    torch.cuda.synchronize()
    assert int(n2.item()) == ii.size and np.array_equal(idx2.cpu().numpy()[: ii.size], ii)
    # garbage above d_ff in the last word is ignored
    if F % 32:
        bits[-1] |= torch.tensor(-1 << (F % 32), dtype=torch.int32, device=DEV)
        idx3, n3 = clada.mask_unpack(ctx, bits, F)
        assert int(n3.item()) == ii.size and np.array_equal(idx3.cpu().numpy()[: ii.size], ii)


def test_dynamic_mask_bits_unpack_to_the_dynamic_list(clada):
    cfg = synth.CONFIGS["c2"]
    d, F = 1024, 3000
    w = synth.layer_weights(cfg, 2, 0, d=d, d_ff=F)
    x = synth.decode_hidden(cfg, 2, 0, 0, B=1, d=d)
    ctx = _ctx(clada, d, F, 1)
    layer = clada.Layer(*[to_dev(a, cfg.dtype) for a in w])
    y, idx, cnt, bits = clada.sparse_ffn_decode(ctx, layer, to_dev(x, cfg.dtype),
                                                torch.tensor([0.25], dtype=torch.float32, device=DEV), want_lists=True)
    idx2, n2 = clada.mask_unpack(ctx, bits[0].contiguous(), F)
    torch.cuda.synchronize()
    k = int(cnt[0].item())
    assert int(n2.item()) == k and torch.equal(idx2[:k], idx[:k])
