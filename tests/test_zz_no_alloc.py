"""GPU test of clada_cognitive_signals_static, the entry point for callers that cannot allocate: its scratch
is a fixed array in the library's device code.  Called through the C ABI; compared with clada_cognitive_signals
(the existing entry point, scratch in a context's workspace) bit for bit and with the oracle within the
signals' tolerance, on two calls in a row, the second on a smaller input."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import DEV, TOL_SIGNAL

pytestmark = pytest.mark.gpu


def _call(lib, fn, h, z, tok):
    B, V = z.shape
    s = torch.full((B,), -7.0, dtype=torch.float32, device=DEV)
    e = torch.full((B,), -7.0, dtype=torch.float32, device=DEV)
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = fn(h, C.c_void_p(z.data_ptr()), 0, B, V, C.c_void_p(tok.data_ptr()), C.c_void_p(s.data_ptr()),
            C.c_void_p(e.data_ptr()), st)
    assert rc == 0, lib.clada_last_error(h)
    torch.cuda.synchronize()
    return s.cpu().numpy(), e.cpu().numpy()


def test_static_scratch_entry_point_matches_workspace_entry_point():
    import paper_2502_19078_amd as clada
    lib = clada.load_library()
    with_ws = clada.Context(0, clada.workspace_bytes(0, 0, 16, 0, 400000))
    h0 = C.c_void_p()
    assert lib.clada_create(C.byref(h0), 0, 0) == 0                 # no workspace: this context allocates nothing
    try:
        # calls in a row on the shared array, most with fewer rows or a shorter vocabulary than the one before
        for cfg_name, B, V in (("c4", 4, 400000), ("c4", 2, 300001), ("c4", 16, 128256), ("c2", 3, 32000), ("c1", 1, 1000),
                               ("c4", 5, 128256), ("c4", 1, 262145)):
            cfg = synth.CONFIGS[cfg_name]
            z, _ = synth.logits(cfg, 9, 0, B=B, V=V)
            tok = synth.draw_tokens(cfg, 9, 0, z)
            zd = torch.from_numpy(z).to(DEV)
            td = torch.from_numpy(np.asarray(tok, np.int32)).to(DEV)
            s1, e1 = _call(lib, lib.clada_cognitive_signals_static, h0, zd, td)
            s2, e2 = _call(lib, lib.clada_cognitive_signals, with_ws._h, zd, td)
            assert np.array_equal(s1.view(np.int32), s2.view(np.int32)), (cfg_name, B, V)
            assert np.array_equal(e1.view(np.int32), e2.view(np.int32)), (cfg_name, B, V)
            s_ref, e_ref = oracle.signals(z, tok)
            np.testing.assert_allclose(s1, s_ref, atol=TOL_SIGNAL, rtol=0)
            np.testing.assert_allclose(e1, e_ref, atol=TOL_SIGNAL, rtol=0)
        # beyond the array's capacity: a clear error, nothing launched
        big = torch.zeros(1, (1 << 20) + 1, dtype=torch.float32, device=DEV)
        s = torch.zeros(1, dtype=torch.float32, device=DEV)
        rc = lib.clada_cognitive_signals_static(h0, C.c_void_p(big.data_ptr()), 0, 1, big.shape[1],
                                                C.c_void_p(torch.zeros(1, dtype=torch.int32, device=DEV).data_ptr()),
                                                C.c_void_p(s.data_ptr()), C.c_void_p(s.data_ptr()), None)
        assert rc == 2 and b"static scratch" in lib.clada_last_error(h0)
    finally:
        lib.clada_destroy(h0)
