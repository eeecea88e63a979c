"""GPU parity, bit for bit: stored masks (clada_mask_pack / _unpack, clada_mask_sparse_encode / _decode)
against oracle/mask_codec.py."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import DEV, to_dev
from oracle import mask_codec as mc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def clada():
    import paper_2502_19078_amd as m
    m.load_library()
    return m


@pytest.fixture(scope="module")
def ctx(clada):
    return clada.Context(0, clada.workspace_bytes(64, 4096, 1, 0, 0))


def _dev_words(words):
    return torch.from_numpy(np.array(words, np.uint32).view(np.int32)).to(DEV)


def _host_words(t):
    return [int(v) for v in t.cpu().numpy().view(np.uint32)]


def _roundtrip(clada, ctx, m, ref_m, d_ff, what):
    words = mc.pack(np.flatnonzero(m), d_ff)
    ref = None if ref_m is None else mc.pack(np.flatnonzero(ref_m), d_ff)
    want_stream, want_n = mc.sparse_encode(words, ref, d_ff)
    wd, rd = _dev_words(words), None if ref is None else _dev_words(ref)
    stream, n = clada.mask_sparse_encode(ctx, wd, rd, d_ff)
    torch.cuda.synchronize()
    nb, npos = (int(v) for v in n.cpu())
    assert (nb, npos) == (len(want_stream), want_n), what
    assert bytes(stream[:nb].cpu().numpy()) == want_stream, what
    assert stream.numel() == mc.sparse_max_bytes(d_ff) or d_ff < 1
    back = clada.mask_sparse_decode(ctx, stream, n, rd, d_ff)
    torch.cuda.synchronize()
    assert _host_words(back) == words == mc.sparse_decode(want_stream, ref, d_ff), what
    return nb


def test_hand_worked_example(clada, ctx):
    kept = [0, 1, 5, 31, 32, 63, 64, 200, 299]
    refk = [0, 1, 5, 31, 33, 63, 64, 299]
    m = np.zeros(300, bool); m[kept] = True
    r = np.zeros(300, bool); r[refk] = True
    assert _roundtrip(clada, ctx, m, None, 300, "plain") == 10
    assert _roundtrip(clada, ctx, m, r, 300, "against the reference") == 4


@pytest.mark.parametrize("d_ff,density,flip", [(1, 1.0, 1.0), (1, 0.0, 0.0), (31, 0.5, 0.3), (32, 0.5, 0.3), (33, 1.0, 1.0),
                                               (300, 0.5, 0.02), (11008, 0.55, 0.01), (14336, 0.45, 0.0),
                                               (13824, 0.5, 0.5), (40000, 0.0, 0.0), (40000, 0.001, 0.0005),
                                               (262144, 0.3, 0.0002), (262144, 1.0, 0.0), (262144, 0.5, 0.5)])
def test_sparse_form_bit_exact_against_oracle(clada, ctx, d_ff, density, flip):
    r = np.random.default_rng(d_ff * 7 + int(1000 * density))
    ref_m = r.random(d_ff) < density
    m = ref_m ^ (r.random(d_ff) < flip)
    _roundtrip(clada, ctx, m, ref_m, d_ff, "against a reference")
    _roundtrip(clada, ctx, m, None, d_ff, "plain")
    if d_ff > 20000:                                    # gaps of three bytes
        far = np.zeros(d_ff, bool)
        far[[3, 3 + 16384 + 1, d_ff - 1]] = True
        _roundtrip(clada, ctx, far, None, d_ff, "wide gaps")


def test_consecutive_decode_masks_cost_about_a_byte_per_changed_neuron(clada):
    """Masks of the 7B layer shape for tokens that share most of their hidden state: the second is coded
    against the first; stream, count and the decoded mask are the oracle's, and the stream is far below
    d_ff / 8 bytes."""
    cfg = synth.CONFIGS["c2"]
    d, F = 1024, 11008
    w = synth.layer_weights(cfg, 3, 0, d=d, d_ff=F)
    layer = clada.Layer(*[to_dev(a, cfg.dtype) for a in w])
    ctx = clada.Context(0, clada.workspace_bytes(d, F, 1, 0, 0))
    x = synth.decode_hidden(cfg, 3, 0, 0, B=2, d=d, shared_frac=0.9999)
    tau = torch.tensor([0.25], dtype=torch.float32, device=DEV)
    bits = []
    for b in range(2):
        _, _, _, mb = clada.sparse_ffn_decode(ctx, layer, to_dev(x[b:b + 1], cfg.dtype), tau, want_lists=True)
        bits.append(mb[0].contiguous())
    stream, n = clada.mask_sparse_encode(ctx, bits[1], bits[0], F)
    torch.cuda.synchronize()
    nb, npos = (int(v) for v in n.cpu())
    want_stream, want_n = mc.sparse_encode(_host_words(bits[1]), _host_words(bits[0]), F)
    assert (nb, npos) == (len(want_stream), want_n) and bytes(stream[:nb].cpu().numpy()) == want_stream
    assert 0 < npos < F // 20 and nb < F // 8 // 2           # the bit mask takes F / 8 bytes
    back = clada.mask_sparse_decode(ctx, stream, n, bits[0], F, out=bits[0].clone())
    assert torch.equal(back, bits[1])
    inplace = bits[0].clone()                            # decoding into the reference's own array
    clada.mask_sparse_decode(ctx, stream, n, inplace, F, out=inplace)
    assert torch.equal(inplace, bits[1])


def test_capacity_and_damaged_streams(clada, ctx):
    d_ff = 5000
    m = np.zeros(d_ff, bool); m[::7] = True
    wd = _dev_words(mc.pack(np.flatnonzero(m), d_ff))
    want_stream, want_n = mc.sparse_encode(mc.pack(np.flatnonzero(m), d_ff), None, d_ff)
    stream, n = clada.mask_sparse_encode(ctx, wd, None, d_ff, capacity=len(want_stream))
    assert [int(v) for v in n.cpu()] == [len(want_stream), want_n]            # exactly fits
    stream, n = clada.mask_sparse_encode(ctx, wd, None, d_ff, capacity=len(want_stream) - 1)
    assert [int(v) for v in n.cpu()] == [-1, want_n]                          # does not fit
    stream, n = clada.mask_sparse_encode(ctx, wd, None, d_ff, capacity=0)
    assert [int(v) for v in n.cpu()] == [-1, want_n]
    # damaged streams: positions past d_ff, a number cut off at the end, a count beyond the capacity
    bad = torch.tensor([5, 0xff, 0xff, 0x7f, 3, 0x80], dtype=torch.uint8, device=DEV)   # 5 | 2^21-1 (past d_ff) | 3 | cut
    out = clada.mask_sparse_decode(ctx, bad, torch.tensor([1000], dtype=torch.int32, device=DEV), None, d_ff)
    torch.cuda.synchronize()
    assert mc.unpack(_host_words(out), d_ff) == [5]
    out = clada.mask_sparse_decode(ctx, bad, torch.tensor([-4], dtype=torch.int32, device=DEV), None, d_ff)
    assert mc.unpack(_host_words(out), d_ff) == []


@pytest.mark.parametrize("F", [1, 33, 1376, 11008, 262144])
def test_bit_mask_pack_unpack_against_oracle(clada, ctx, F):
    r = np.random.default_rng(F)
    keep = np.flatnonzero(r.random(F) < 0.55).astype(np.int32)
    idx = torch.full((F,), -1, dtype=torch.int32, device=DEV)
    idx[: keep.size] = torch.from_numpy(keep).to(DEV)
    n = torch.tensor([keep.size], dtype=torch.int32, device=DEV)
    bits = clada.mask_pack(ctx, idx, n, F)
    torch.cuda.synchronize()
    assert _host_words(bits) == mc.pack(keep, F)
    idx2, n2 = clada.mask_unpack(ctx, bits, F)
    assert idx2[: int(n2)].cpu().tolist() == mc.unpack(_host_words(bits), F) == keep.tolist()


@pytest.mark.parametrize("d_ff,n,mode", [(300, 5, "shared"), (11008, 16, "shared"), (11008, 16, "chain"), (14336, 7, "none"),
                                         (262144, 3, "chain"), (33, 64, "shared")])
def test_batch_calls_are_the_single_calls_mask_by_mask(clada, ctx, d_ff, n, mode):
    """n masks in one launch: one shared reference (a layer's prefix-static mask), one reference each (the
    previous token's mask) or none.  Streams, counts and decoded masks are the oracle's, mask by mask; a
    capacity that some streams do not fit marks exactly those."""
    r = np.random.default_rng(d_ff + n)
    base = r.random(d_ff) < 0.5
    masks = [base ^ (r.random(d_ff) < 0.002 * (m + 1)) for m in range(n)]
    words = [mc.pack(np.flatnonzero(m), d_ff) for m in masks]
    if mode == "shared":
        refs = [mc.pack(np.flatnonzero(base), d_ff)] * n
        rd = _dev_words(refs[0])
    elif mode == "chain":
        refs = [mc.pack(np.flatnonzero(base), d_ff)] + words[:-1]
        rd = torch.stack([_dev_words(w) for w in refs])
    else:
        refs, rd = [None] * n, None
    wd = torch.stack([_dev_words(w) for w in words])
    streams, n_out = clada.mask_sparse_encode_batch(ctx, wd, rd, d_ff)
    back = clada.mask_sparse_decode_batch(ctx, streams, n_out, rd, d_ff)
    torch.cuda.synchronize()
    want = [mc.sparse_encode(words[m], refs[m], d_ff) for m in range(n)]
    for m in range(n):
        nb, npos = (int(v) for v in n_out[m].cpu())
        assert (nb, npos) == (len(want[m][0]), want[m][1]), m
        assert bytes(streams[m, :nb].cpu().numpy()) == want[m][0], m
        assert _host_words(back[m]) == words[m], m
    # a capacity between the shortest and the longest stream
    lens = sorted(len(w[0]) for w in want)
    if lens[0] < lens[-1]:
        cap = (lens[0] + lens[-1]) // 2
        streams2, n2 = clada.mask_sparse_encode_batch(ctx, wd, rd, d_ff, capacity=cap)
        torch.cuda.synchronize()
        for m in range(n):
            nb = int(n2[m, 0])
            assert nb == (len(want[m][0]) if len(want[m][0]) <= cap else -1), m
            assert int(n2[m, 1]) == want[m][1]
            if nb >= 0:
                assert bytes(streams2[m, :nb].cpu().numpy()) == want[m][0]
