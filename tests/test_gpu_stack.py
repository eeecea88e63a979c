"""GPU parity: the whole-stack calls against the per-layer calls, bit for bit, and against the fp64 oracle.
Modes of the call (option decode.stack): 3 = lanes, the default (the layers go round two or three streams);
2 = chained launches (every layer's kernel also sums the previous layer's partial outputs); 1 = one
persistent launch for the L layers; 0 = the per-layer calls."""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import DEV, TOL_Y, assert_close_y, check_mask_band, to_dev, to_np, unpack_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def clada():
    import paper_2502_19078_amd as m
    m.load_library()
    return m


def _stack(clada, cfg_name, d, F, L, seed, relu=False, geglu=False):
    from paper_2502_19078_amd import binding
    cfg = synth.CONFIGS[cfg_name]
    ws, layers = [], []
    for l in range(L):
        if relu:
            w = synth.relu_layer(cfg, seed, l, d=d, d_ff=F)
            layers.append(clada.Layer(to_dev(w[0], cfg.dtype), None, to_dev(w[2], cfg.dtype), kind=binding.RELU,
                                      b_in=torch.from_numpy(w[1]).to(DEV), b_out=torch.from_numpy(w[3]).to(DEV)))
        else:
            w = synth.layer_weights(cfg, seed, l, d=d, d_ff=F)
            layers.append(clada.Layer(*[to_dev(a, cfg.dtype) for a in w], kind=binding.GEGLU if geglu else binding.SWIGLU))
        ws.append(w)
    x = np.concatenate([synth.decode_hidden(cfg, seed, l, 0, B=1, d=d) for l in range(L)])       # [L][d]
    return cfg, ws, layers, x


# cfg, d, F, L, q, options: shapes with a persistent instance (4, 8 and 10 KiB rows; balanced and not; odd
# and even L; F not a multiple of the workgroup count), and shapes that run as per-layer calls inside the call
CASES = [
    ("c2", 4096, 11008, 5, 0.45, {}),                 # 7B layer shape: balanced persistent kernel
    ("c2", 4096, 11008, 2, 0.45, {"decode.b1": 2}),   # the same without balancing
    ("c2", 4096, 2700, 7, 0.60, {"decode.b1": 3}),    # balancing forced on a short layer, ragged neuron count
    ("c2", 4096, 2700, 3, 0.30, {}),                  # short layer: no balancing by default
    ("c5", 5120, 13824, 3, 0.50, {}),                 # 13B layer shape (10 KiB rows)
    ("c2", 2048, 16384, 4, 0.45, {}),                 # 4 KiB rows, 64 neurons per workgroup: unbalanced
    ("c2", 1024, 1000, 3, 0.45, {}),                  # no persistent instance: per-layer calls inside
    ("c1", 512, 1376, 2, 0.40, {}),                   # fp32: per-layer calls inside
]


# shapes only the chained launches have instances for: fp32 rows of 8 KiB, 12 KiB rows worked off in rounds
# (more than 64 neurons per workgroup), 2 KiB rows, a single layer (nothing to chain)
CHAINED_ONLY = [
    ("c1", 2048, 1500, 3, 0.40, {}),
    ("c2", 6144, 16500, 2, 0.45, {}),
    ("c2", 1024, 3000, 4, 0.45, {}),
    ("c2", 4096, 11008, 1, 0.45, {}),
]


@pytest.mark.parametrize("mode,cfg_name,d,F,L,q,opts", [(1, *c) for c in CASES] + [(m, *c) for m in (2, 3) for c in CASES + CHAINED_ONLY])
def test_stack_call_is_the_per_layer_calls_bit_for_bit(clada, mode, cfg_name, d, F, L, q, opts):
    cfg, ws, layers, x = _stack(clada, cfg_name, d, F, L, seed=21)
    ctx = clada.Context(0, clada.workspace_bytes(d, F, 1, 0, 0))
    ctx.set_option("decode.stack", mode)
    for k, v in opts.items():
        ctx.set_option(k, v)
    tau = np.array([np.quantile(np.abs(oracle.gate_act(ws[l][0], x[l:l + 1])), q) for l in range(L)], np.float32)
    tau[L - 1] *= 1.92                                  # thresholds differ per layer
    xd, td = to_dev(x, cfg.dtype), torch.from_numpy(tau).to(DEV)
    y_ref, cnt_ref = [], []
    if mode >= 3:                                       # the two-lane modes run the unbalanced instances: those are their bits
        ctx.set_option("decode.b1", 2)
    for l in range(L):
        yl, _, cl, _ = clada.sparse_ffn_decode(ctx, layers[l], xd[l:l + 1].contiguous(), td[l:l + 1].contiguous(), want_lists=True)
        y_ref.append(yl[0].clone())
        cnt_ref.append(cl.clone())
    for rep in range(3):                                # repeated launches: counters and parities carry over
        if mode >= 2 and rep < 2:                       # (a chained call that is asked for counts runs the per-layer calls)
            y = clada.sparse_ffn_stack_decode(ctx, layers, xd, td)
            cnt = None
        else:
            y, cnt = clada.sparse_ffn_stack_decode(ctx, layers, xd, td, want_counts=True)
        torch.cuda.synchronize()
        for l in range(L):
            assert torch.equal(y[l], y_ref[l]), f"rep {rep} layer {l}: bits differ from the per-layer call"
            assert cnt is None or torch.equal(cnt[l], cnt_ref[l]), f"rep {rep} layer {l}: kept count"
    assert not ctx.device_fault()
    # dense twin
    yd = clada.dense_ffn_stack_decode(ctx, layers, xd)
    for l in range(L):
        assert torch.equal(yd[l], clada.dense_ffn_decode(ctx, layers[l], xd[l:l + 1].contiguous())[0])
    # per-layer calls still work on the same context afterwards
    assert torch.equal(clada.sparse_ffn_decode(ctx, layers[0], xd[:1].contiguous(), td[:1].contiguous())[0], y_ref[0])
    # and the oracle, on two layers
    for l in (0, L - 1):
        ref = oracle.sparse_decode(*ws[l], x[l:l + 1], tau[l:l + 1].astype(np.float64))
        assert abs(int(cnt[l, 0]) - int(ref["n_active"][0])) <= 3
        if int(cnt[l, 0]) == int(ref["n_active"][0]):
            assert_close_y(to_np(y[l:l + 1]), ref["y"], TOL_Y[cfg.dtype], f"layer {l} vs oracle")


@pytest.mark.parametrize("mode", [1, 2, 3])
def test_stack_call_other_families_and_long_stacks(clada, mode):
    # non-gated ReLU family at the OPT-2.7B width (5 KiB rows, biases)
    cfg, ws, layers, x = _stack(clada, "o27", 2560, 10240, 3, seed=22, relu=True)
    ctx = clada.Context(0, clada.workspace_bytes(2560, 10240, 1, 0, 0))
    ctx.set_option("decode.stack", mode)
    xd = to_dev(x, cfg.dtype)
    td = torch.full((3,), 0.05, dtype=torch.float32, device=DEV)
    y = clada.sparse_ffn_stack_decode(ctx, layers, xd, td)
    for l in range(3):
        assert torch.equal(y[l], clada.sparse_ffn_decode(ctx, layers[l], xd[l:l + 1].contiguous(), td[l:l + 1].contiguous())[0])
    ref = oracle.relu_decode(*ws[1], x[1:2], tau=np.array([0.05]))
    assert_close_y(to_np(y[1:2]), ref["y"], TOL_Y[cfg.dtype], "relu stack vs oracle")
    # GELU-gated family, and more layers than one launch takes (the same small layers listed 25 times each)
    cfg, ws, layers, x = _stack(clada, "c2", 4096, 512, 2, seed=23, geglu=True)
    long_layers = layers * 25
    xd = to_dev(np.tile(x, (25, 1)), cfg.dtype)
    td = torch.full((50,), 0.1, dtype=torch.float32, device=DEV)
    ctx = clada.Context(0, clada.workspace_bytes(4096, 512, 1, 0, 0))
    ctx.set_option("decode.stack", mode)
    y = clada.sparse_ffn_stack_decode(ctx, long_layers, xd, td)
    y0 = clada.sparse_ffn_decode(ctx, layers[0], xd[:1].contiguous(), td[:1].contiguous())[0]
    y1 = clada.sparse_ffn_decode(ctx, layers[1], xd[1:2].contiguous(), td[:1].contiguous())[0]
    torch.cuda.synchronize()
    for l in range(50):
        assert torch.equal(y[l], y0 if l % 2 == 0 else y1), f"layer {l}"
    assert not ctx.device_fault()


def test_stack_call_rejects_mixed_layers_and_bad_arguments(clada):
    from paper_2502_19078_amd.binding import CladaError
    cfg, ws, layers, x = _stack(clada, "c2", 1024, 300, 2, seed=24)
    other = clada.Layer(*[to_dev(a, cfg.dtype) for a in synth.layer_weights(cfg, 24, 5, d=1024, d_ff=301)])
    ctx = clada.Context(0, clada.workspace_bytes(1024, 301, 1, 0, 0))
    xd, td = to_dev(x, cfg.dtype), torch.zeros(2, device=DEV)
    with pytest.raises(CladaError):
        clada.sparse_ffn_stack_decode(ctx, [layers[0], other], xd, td)
    with pytest.raises(CladaError):
        ctx.check(ctx._lib.clada_sparse_ffn_stack_decode(ctx._h, None, 2, xd.data_ptr(), 1, td.data_ptr(), xd.data_ptr(), None, None))


@pytest.mark.parametrize("mode", [1, 2])      # (the lanes run kernels that wait for nobody)
def test_bounded_waits_of_the_stack_kernel_give_up_cleanly(clada, mode):
    """Spin limit forced to zero from the host: every workgroup still runs to its end, the outputs are NaN
    and the context reports the fault."""
    cfg, ws, layers, x = _stack(clada, "c2", 4096, 11008, 3, seed=25)
    ctx = clada.Context(0, clada.workspace_bytes(4096, 11008, 1, 0, 0))
    ctx.set_option("decode.b1", 3)
    ctx.set_option("decode.stack", mode)
    xd, td = to_dev(x, cfg.dtype), torch.full((3,), 0.25, dtype=torch.float32, device=DEV)
    good = clada.sparse_ffn_stack_decode(ctx, layers, xd, td).clone()
    assert not ctx.device_fault() and torch.isfinite(good.float()).all()
    ctx.set_option("decode.spin_limit", 0)
    bad = clada.sparse_ffn_stack_decode(ctx, layers, xd, td)
    torch.cuda.synchronize()
    assert ctx.device_fault() and torch.isnan(bad.float()).any()
    if mode == 2:                                       # every layer of a chain, the last one's own reduction included
        assert torch.isnan(bad.float()).all()


def test_stack_call_modes_agree_and_replay_from_a_graph(clada):
    """The modes give the same bits; captured calls (lanes: a fork and a join inside the capture; chained
    launches) replay correctly on changed inputs."""
    cfg, ws, layers, x = _stack(clada, "c2", 4096, 11008, 4, seed=26)
    ctx = clada.Context(0, clada.workspace_bytes(4096, 11008, 1, 0, 0))
    ctx.set_option("decode.b1", 2)                      # no balancing: every mode then adds in the same order
    xd, td = to_dev(x, cfg.dtype), torch.full((4,), 0.25, dtype=torch.float32, device=DEV)
    y2, cnt = clada.sparse_ffn_stack_decode(ctx, layers, xd, td, want_counts=True)
    y2 = clada.sparse_ffn_stack_decode(ctx, layers, xd, td).clone()          # default: lanes
    for mode in (0, 1, 2):
        ctx.set_option("decode.stack", mode)
        assert torch.equal(clada.sparse_ffn_stack_decode(ctx, layers, xd, td), y2), f"mode {mode}"
    ctx.set_option("decode.stack", 3)
    ctx2 = ctx                                          # (unbalanced per-layer calls: the reference bits below)
    for l in range(4):
        yl, _, cl, _ = clada.sparse_ffn_decode(ctx, layers[l], xd[l:l + 1].contiguous(), td[l:l + 1].contiguous(), want_lists=True)
        assert torch.equal(y2[l], yl[0]) and torch.equal(cnt[l], cl)
    # graph: static input and output buffers, replays with other inputs and thresholds in between eager work;
    # lanes, and chained launches of the balanced kernel (whose call counter the chain advances itself)
    for mode, b1 in ((3, 1), (2, 1), (2, 2)):
        ctx = clada.Context(0, clada.workspace_bytes(4096, 11008, 1, 0, 0))
        ctx.set_option("decode.stack", mode)
        ctx.set_option("decode.b1", b1)
        xs, ts = xd.clone(), td.clone()
        ys = torch.empty_like(xs)
        stream = torch.cuda.Stream()
        stream.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(stream):
            clada.sparse_ffn_stack_decode(ctx, layers, xs, ts, y=ys)            # warm-up on the capture stream
            stream.synchronize()
            clada.graph_begin(ctx)
            clada.sparse_ffn_stack_decode(ctx, layers, xs, ts, y=ys)
            g = clada.graph_end(ctx)
            for rep in range(4):
                xs.copy_(torch.roll(xd, rep, dims=0))
                ts.fill_(0.2 + 0.05 * rep)
                g.launch()
                stream.synchronize()
                got = ys.clone()
                want = clada.sparse_ffn_stack_decode(ctx, layers, xs, ts)        # eager, between the replays
                stream.synchronize()
                assert torch.equal(got, want), f"mode {mode} replay {rep}"
                if b1 == 2 or mode == 3:
                    assert torch.equal(got[0], clada.sparse_ffn_decode(ctx2, layers[0], xs[:1].contiguous(), ts[:1].contiguous())[0])
        del g
    assert not ctx.device_fault()


def _batch_stack(clada, cfg_name, d, F, L, B, seed, shared_frac=0.5):
    cfg = synth.CONFIGS[cfg_name]
    ws = [synth.layer_weights(cfg, seed, l, d=d, d_ff=F) for l in range(L)]
    layers = [clada.Layer(*[to_dev(a, cfg.dtype) for a in w]) for w in ws]
    x = np.stack([synth.decode_hidden(cfg, seed, l, 0, B=B, d=d, shared_frac=shared_frac) for l in range(L)])   # [L][B][d]
    return cfg, ws, layers, x


# cfg, d, F, L, B: three lanes on the matrix-core path (one and two passes of tokens per layer, 4 and 10 KiB
# rows, fewer units than lanes), and batches that path does not take (fp32; a width it has no instance for)
BATCH_CASES = [
    ("c3", 4096, 3000, 5, 8),
    ("c5", 5120, 2100, 4, 16),
    ("c3", 4096, 1500, 3, 20),
    ("c3", 4096, 1024, 2, 64),
    ("c3", 2048, 2048, 3, 33),
    ("c3", 2048, 1024, 1, 4),
    ("c1", 512, 700, 3, 4),
    ("c3", 1536, 900, 3, 3),
]


@pytest.mark.parametrize("cfg_name,d,F,L,B", BATCH_CASES)
def test_batched_stack_call_is_the_per_layer_calls_bit_for_bit(clada, cfg_name, d, F, L, B):
    cfg, ws, layers, x = _batch_stack(clada, cfg_name, d, F, L, B, seed=31)
    ctx = clada.Context(0, clada.workspace_bytes(d, F, B, 0, 0))
    tau = np.stack([np.quantile(np.abs(oracle.gate_act(ws[l][0], x[l])), 0.45, axis=1) for l in range(L)]).astype(np.float32)
    xd, td = to_dev(x, cfg.dtype), torch.from_numpy(tau).to(DEV)
    y_ref, cnt_ref, yd_ref = [], [], []
    for l in range(L):
        yl, _, cl, _ = clada.sparse_ffn_decode(ctx, layers[l], xd[l], td[l], want_lists=True)
        y_ref.append(yl.clone())
        cnt_ref.append(cl.clone())
        yd_ref.append(clada.dense_ffn_decode(ctx, layers[l], xd[l]).clone())
    for rep in range(3):
        if rep < 2:
            y, cnt = clada.sparse_ffn_stack_decode(ctx, layers, xd, td), None
        else:
            y, cnt = clada.sparse_ffn_stack_decode(ctx, layers, xd, td, want_counts=True)
        torch.cuda.synchronize()
        for l in range(L):
            assert torch.equal(y[l], y_ref[l]), f"rep {rep} layer {l}: bits differ from the per-layer call"
            assert cnt is None or torch.equal(cnt[l], cnt_ref[l])
    yd = clada.dense_ffn_stack_decode(ctx, layers, xd)
    for l in range(L):
        assert torch.equal(yd[l], yd_ref[l])
    # the oracle, on the last layer: masks inside the band, y on the device's own masks
    l = L - 1
    ref = oracle.sparse_decode(*ws[l], x[l], tau[l].astype(np.float64))
    _, _, _, bits = clada.sparse_ffn_decode(ctx, layers[l], xd[l], td[l], want_lists=True)
    mask = unpack_bits(bits, F)
    check_mask_band(mask, ref["act"], tau[l], "batched stack")
    want = oracle.decode_given_mask(*ws[l], x[l], mask)
    assert_close_y(to_np(y[l]), want, TOL_Y[cfg.dtype], f"layer {l} vs oracle on the device's masks")


def test_batched_stack_call_replays_from_a_graph(clada):
    cfg, ws, layers, x = _batch_stack(clada, "c3", 4096, 2048, 6, 8, seed=32)
    ctx = clada.Context(0, clada.workspace_bytes(4096, 2048, 8, 0, 0))
    xd = to_dev(x, cfg.dtype)
    td = torch.full((6, 8), 0.2, dtype=torch.float32, device=DEV)
    xs, ts, ys = xd.clone(), td.clone(), torch.empty_like(xd)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        clada.sparse_ffn_stack_decode(ctx, layers, xs, ts, y=ys)
        stream.synchronize()
        clada.graph_begin(ctx)
        clada.sparse_ffn_stack_decode(ctx, layers, xs, ts, y=ys)
        g = clada.graph_end(ctx)
        for rep in range(4):
            xs.copy_(torch.roll(xd, rep, dims=0))
            ts.fill_(0.15 + 0.05 * rep)
            g.launch()
            stream.synchronize()
            got = ys.clone()
            for l in (0, 5):
                assert torch.equal(got[l], clada.sparse_ffn_decode(ctx, layers[l], xs[l], ts[l])), f"replay {rep} layer {l}"
            stream.synchronize()
    assert not ctx.device_fault()


def test_stack_call_inside_a_torch_graph(clada):
    """A capture that the library does not own (torch.cuda.graph on a side stream): the lanes join it through
    their fork and join events; replays on changed inputs give the eager bits."""
    cfg, ws, layers, x = _stack(clada, "c2", 4096, 11008, 6, seed=27)
    ctx = clada.Context(0, clada.workspace_bytes(4096, 11008, 1, 0, 0))
    xd = to_dev(x, cfg.dtype)
    xs, ts, ys = xd.clone(), torch.full((6,), 0.25, dtype=torch.float32, device=DEV), torch.empty_like(xd)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        clada.sparse_ffn_stack_decode(ctx, layers, xs, ts, y=ys)            # first call: creates the lane streams
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        clada.sparse_ffn_stack_decode(ctx, layers, xs, ts, y=ys)
    for rep in range(3):
        xs.copy_(torch.roll(xd, rep + 1, dims=0))
        ts.fill_(0.15 + 0.1 * rep)
        ys.zero_()
        g.replay()
        torch.cuda.synchronize()
        got = ys.clone()
        want = clada.sparse_ffn_stack_decode(ctx, layers, xs, ts)
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"replay {rep}"
    assert not ctx.device_fault()
