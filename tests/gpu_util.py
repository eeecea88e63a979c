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
# Absolute floor of the band, for thresholds below TAU_SMALL only.  The kernels accumulate the gate
# pre-activation in fp32 (the precision the mask decision is taken in).  Its rounding error over d = 5120
# products of N(0,1) hidden states with N(0,1/d) or N(0,0.02^2) weights stays below 5e-6 (pinned on the CPU
# by tests/test_tolerances.py with an fp32 emulation of the kernels' summation shape) and |sigma'| <= 1.13,
# so no fp32 evaluation can decide an activation closer than ~6e-6 to the threshold: the floor is 1e-5.
# From tau = 1e-2 up the relative band is at least as wide and the floor is not applied at all (at the
# method's operating points, tau ~ 0.25, the band is 25x the floor); below it (the tests' q = 0 cases, tau =
# the smallest magnitude of a row, 1e-4 .. 1e-16) the relative band alone would ask fp32 for fp64 decisions.
BAND_ABS = 1e-5
TAU_SMALL = 1e-2
# Prefill statistics against the fp64 oracle: an activation carries the pre-activation's rounding error
# (above) times |sigma'|, which grows with the magnitudes themselves (a ReLU passes them on undamped), so
# the pool's absolute tolerance is 2e-6 per unit of the largest magnitude; sums over T tokens of such
# values agree to a few 1e-5 relative.
POOL_RTOL, POOL_ATOL_PER_UNIT = 1e-4, 2e-6
AGG_RTOL, AGG_ATOL = 3e-5, 1e-6


def band_width(tau):
    """Half-width of the zone around tau in which the mask bit may fall on either side: BAND * tau, and
    where tau < TAU_SMALL at least BAND_ABS."""
    tau = np.asarray(tau, np.float64)
    return np.where(tau < TAU_SMALL, np.maximum(BAND * tau, BAND_ABS), BAND * tau)


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    """Stored values (float32 array) -> device tensor of the storage dtype, bit-exact."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        bits = synth.bf16_bits(a).view(np.int16)
        return torch.from_numpy(bits).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(a).to(DEV)


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def assert_close_y(y, y_ref, tol, what="", extra=None):
    """|y - ref|_2 <= tol |ref|_2 and every element within tol (|ref_i| + rms(ref)).  extra [B]: per-row
    addition to tol (the few-neuron cases add eps32 * kappa_b, see tolerances.decode_condition)."""
    y = np.asarray(y, np.float64)
    y_ref = np.asarray(y_ref, np.float64)
    assert y.shape == y_ref.shape, (y.shape, y_ref.shape)
    tol0 = tol
    for b in range(y.shape[0]) if y.ndim == 2 else [slice(None)]:
        tol = tol0 + (float(extra[b]) if extra is not None else 0.0)
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
    """Masks must agree except where |a_ref| lies within the band around tau; returns #flips.  Flips that
    only the absolute floor admits (tau < TAU_SMALL) are reported on stdout so the relaxation stays visible."""
    tau = np.asarray(tau, np.float64)
    mask_ref = np.abs(act_ref) >= tau[:, None]
    diff = mask_gpu != mask_ref
    dist = np.abs(np.abs(act_ref) - tau[:, None])
    allowed = dist <= band_width(tau)[:, None]
    bad = diff & ~allowed
    assert not bad.any(), f"{what}: {bad.sum()} mask bits differ outside the +-{BAND} band around tau"
    floor_only = diff & (dist > BAND * tau[:, None])
    if floor_only.any():
        print(f"[band] {what}: {int(floor_only.sum())} of {int(diff.sum())} flips lie in the absolute floor "
              f"(tau < {TAU_SMALL}: {np.unique(tau[floor_only.any(1)])[:4]})")
    return int(diff.sum())
