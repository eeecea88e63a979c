"""GPU: one decode step (signals, thresholds, a sparse FFN per layer) captured with the library's own
graph helpers and replayed.  Replays are interleaved with eager work and must reproduce the eager bits,
also after the inputs were refreshed in place."""
import ctypes as C

import numpy as np
import pytest
import torch

import synth
from gpu_util import DEV, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def clada():
    import paper_2502_19078_amd as m
    m.load_library()
    return m


@pytest.mark.parametrize("cfg_name,d,F,B,L", [("c2", 4096, 2752, 1, 3), ("c3", 4096, 1024, 8, 2), ("c1", 96, 200, 3, 2)])
def test_captured_step_replays_bit_exactly(clada, cfg_name, d, F, B, L):
    from paper_2502_19078_amd import binding
    from paper_2502_19078_amd.binding import CladaError
    cfg = synth.CONFIGS[cfg_name]
    V = 4000
    lib = clada.load_library()
    ctx = clada.Context(0, clada.workspace_bytes(d, F, B, 0, V))
    layers = [clada.Layer(*[to_dev(a, cfg.dtype) for a in synth.layer_weights(cfg, 3, l, d=d, d_ff=F)]) for l in range(L)]
    cl = [l.c_struct() for l in layers]
    rng = np.random.default_rng(5)
    steps = 3
    x_all = torch.stack([torch.stack([to_dev(synth.decode_hidden(cfg, 3, l, s, B=B, d=d), cfg.dtype) for l in range(L)])
                         for s in range(steps)])                                    # [step][layer][B][d]
    z_all = torch.from_numpy(rng.standard_normal((steps, B, V)).astype(np.float32) * 2).to(DEV)
    tok_all = torch.from_numpy(rng.integers(0, V, (steps, B)).astype(np.int32)).to(DEV)
    x, z, tok = x_all[0].clone(), z_all[0].clone(), tok_all[0].clone()
    sur, ent = torch.empty(B, device=DEV), torch.empty(B, device=DEV)
    tau_base = torch.full((L,), 0.12, device=DEV)
    lam, gam = torch.full((L,), 0.8, device=DEV), torch.full((L,), 0.12, device=DEV)
    tau_final = torch.empty(L, B, device=DEV)
    y = torch.empty_like(x)
    tau_s, tau_h = float(np.log(V) + 0.5), float(np.log(V) - 0.8)

    def step(sp):
        ctx.check(lib.clada_cognitive_signals(ctx._h, z.data_ptr(), binding.F32, B, V, tok.data_ptr(), sur.data_ptr(),
                                              ent.data_ptr(), sp))
        ctx.check(lib.clada_threshold(ctx._h, tau_base.data_ptr(), lam.data_ptr(), gam.data_ptr(), L, sur.data_ptr(),
                                      ent.data_ptr(), B, tau_s, tau_h, tau_final.data_ptr(), sp))
        for l in range(L):
            ctx.check(lib.clada_sparse_ffn_decode(ctx._h, C.byref(cl[l]), x[l].data_ptr(), B, tau_final[l].data_ptr(),
                                                  y[l].data_ptr(), None, None, None, sp))

    side = torch.cuda.Stream()
    sp = C.c_void_p(side.cuda_stream)
    # eager reference for every step (also the warm-up the capture needs)
    want = []
    with torch.cuda.stream(side):
        for s in range(steps):
            x.copy_(x_all[s]); z.copy_(z_all[s]); tok.copy_(tok_all[s])
            step(sp)
            side.synchronize()
            want.append((y.clone(), tau_final.clone(), sur.clone()))
        assert not torch.equal(want[0][0], want[1][0])
        with pytest.raises(CladaError):                     # the default stream cannot be captured
            ctx.check(lib.clada_graph_begin(ctx._h, None))
        x.copy_(x_all[0]); z.copy_(z_all[0]); tok.copy_(tok_all[0])
        side.synchronize()
        clada.graph_begin(ctx)
        with pytest.raises(CladaError):                     # one capture at a time
            clada.graph_begin(ctx)
        step(sp)
        g = clada.graph_end(ctx)
        with pytest.raises(CladaError):
            clada.graph_end(ctx)
        for rep in range(2):
            for s in range(steps):
                x.copy_(x_all[s]); z.copy_(z_all[s]); tok.copy_(tok_all[s])
                y.zero_(); tau_final.zero_()
                g.launch()
                side.synchronize()
                assert torch.equal(y, want[s][0]) and torch.equal(tau_final, want[s][1]) and torch.equal(sur, want[s][2])
                # eager calls of the same context between replays
                y2 = clada.dense_ffn_decode(ctx, layers[0], x[0])
                side.synchronize()
                assert torch.isfinite(y2.float()).all()
        del g
