"""Shared helpers of the GPU parity tests (marshalling and the comparison rules)."""
import numpy as np
import torch

import synth

DEV = "cuda:0"

# Tolerances of the parity bar: relative error of FFN outputs per dtype, absolute error of
# surprisal/entropy, relative half-width of the band around tau inside which a neuron's
# keep decision may differ from the oracle's.
TOL_Y = {"f32": 1e-5, "bf16": 2e-2}
TOL_SIGNAL = 1e-4
BAND = 1e-3
# Absolute floor of the band.  The kernels accumulate the gate pre-activation in fp32 (the precision the
# mask decision is taken in); over d = 2048..5120 terms of size ~1/sqrt(d) its rounding error reaches
# ~4e-6, and |sigma'| <= 1.13, so an activation within ~5e-6 of the threshold cannot be decided by any
# fp32 evaluation.  It only matters for thresholds below 1e-2 (the q = 0 cases: tau = the smallest
# magnitude of the row, 1e-4 .. 1e-16); at the paper's operating points (tau ~ 0.25) BAND * tau is 25x wider.
BAND_ABS = 1e-5


def band_width(tau):
    """Half-width of the zone around tau in which the mask bit may fall on either side."""
    return np.maximum(BAND * np.asarray(tau, np.float64), BAND_ABS)


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    """Stored values (float32 array) -> device tensor of the storage dtype, bit-exact."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        bits = synth.bf16_bits(a).view(np.int16)
        return torch.from_numpy(bits).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(a).to(DEV)


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def assert_close_y(y, y_ref, tol, what=""):
    """|y - ref|_2 <= tol |ref|_2 and every element within tol (|ref_i| + rms(ref))."""
    y = np.asarray(y, np.float64)
    y_ref = np.asarray(y_ref, np.float64)
    assert y.shape == y_ref.shape, (y.shape, y_ref.shape)
    for b in range(y.shape[0]) if y.ndim == 2 else [slice(None)]:
        r, g = y_ref[b], y[b]
        nr = np.linalg.norm(r)
        if nr == 0.0:
            assert np.all(g == 0.0), f"{what}: expected exact zeros"
            continue
        rel = np.linalg.norm(g - r) / nr
        assert rel <= tol, f"{what} row {b}: relative L2 error {rel:.3e} > {tol}"
        rms = nr / np.sqrt(r.size)
        worst = np.max(np.abs(g - r) / (np.abs(r) + rms))
        assert worst <= tol, f"{what} row {b}: elementwise error {worst:.3e} > {tol}"


def unpack_bits(bits: torch.Tensor, F: int) -> np.ndarray:
    """mask_bits [B][ceil(F/32)] int32 -> bool [B][F]."""
    w = bits.cpu().numpy().view(np.uint32)
    j = np.arange(F)
    return ((w[:, j // 32] >> (j % 32).astype(np.uint32)) & 1).astype(bool)


def check_mask_band(mask_gpu, act_ref, tau, what=""):
    """Masks must agree except where |a_ref| lies within BAND*tau of tau; returns #flips."""
    mask_ref = np.abs(act_ref) >= tau[:, None]
    diff = mask_gpu != mask_ref
    allowed = np.abs(np.abs(act_ref) - tau[:, None]) <= band_width(tau)[:, None]
    bad = diff & ~allowed
    assert not bad.any(), f"{what}: {bad.sum()} mask bits differ outside the +-{BAND} band around tau"
    return int(diff.sum())
