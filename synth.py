"""Seeded synthetic inputs for the CLADA sparse-FFN path.

This module only *draws data*: weights, hidden states, logits and token ids
with the shapes and value distributions of the benchmark configurations.  It
holds none of the method's arithmetic and is the only module that both the CPU
oracle's tests and the GPU tests/benchmark use.  Every tensor comes from its own
numpy PCG64 stream keyed by (seed, config, tensor kind, layer, step), so any
layer or step can be regenerated alone and in any order.

Values are returned as float32 arrays that already hold the *stored* values: for
a bf16 configuration they are rounded to bf16 (round-to-nearest-even) first, so
the oracle (which widens them to fp64) and the GPU (which gets the same bits as
bfloat16) see identical numbers.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

# tensor-kind tags for the stream keys
_W_GATE, _W_UP, _W_DOWN, _PREFIX, _HIDDEN, _LOGITS, _TOKENS, _PERM, _BIAS = range(9)


@dataclass(frozen=True)
class Config:
    """One benchmark configuration (shapes follow LLaMA/Mistral FFN blocks)."""
    cid: int
    name: str
    L: int
    d: int
    d_ff: int
    dtype: str          # "f32" | "bf16"
    w_std: float        # standard deviation of the weight entries
    B: int              # decode batch
    T: int              # prefix length
    V: int              # vocabulary size of the logits
    q: float            # target sparsity (quantile of prefix |SiLU(gate)|)
    logits: str         # "spike" | "zipf"
    steps: int          # decode steps the configuration names


CONFIGS = {
    # single fp32 layer, weights N(0, 1/d); logits N(0, var 2) + one +6 spike
    "c1": Config(1, "toy-f32", 1, 512, 1376, "f32", 512 ** -0.5, 1, 64, 1000, 0.40, "spike", 16),
    # LLaMA2-7B FFN shape, bf16, weights N(0, std 0.02)
    "c2": Config(2, "llama2-7b", 32, 4096, 11008, "bf16", 0.02, 1, 512, 32000, 0.45, "zipf", 64),
    # Mistral-7B FFN shape, decode batch 8
    "c3": Config(3, "mistral-7b", 32, 4096, 14336, "bf16", 0.02, 8, 2048, 32000, 0.45, "zipf", 16),
    # LLaMA-3-8B FFN shape, large vocabulary
    "c4": Config(4, "llama3-8b", 32, 4096, 14336, "bf16", 0.02, 1, 4096, 128256, 0.45, "zipf", 256),
    # LLaMA2-13B FFN shape, decode batch 16
    "c5": Config(5, "llama2-13b", 40, 5120, 13824, "bf16", 0.02, 16, 2048, 32000, 0.45, "zipf", 16),
    # non-gated ReLU FFN shapes of the OPT models the paper also evaluates (not in the benchmark
    # list; the target sparsity sits above the 50 % of exact zeros a ReLU produces by itself)
    "o27": Config(6, "opt-2.7b", 32, 2560, 10240, "bf16", 0.02, 1, 512, 50272, 0.70, "zipf", 64),
    "o350": Config(7, "opt-350m", 24, 1024, 4096, "bf16", 0.02, 1, 512, 50272, 0.70, "zipf", 64),
    # GELU-gated FFN shape of the Gemma-2B model the paper also evaluates (not in the benchmark list)
    "g2b": Config(8, "gemma-2b", 18, 2048, 16384, "bf16", 0.02, 1, 512, 256000, 0.45, "zipf", 64),
}


def _rng(seed, cid, kind, a=0, b=0):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, cid, kind, a, b])))


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_widen(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> the same values as float32 (exact)."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def store(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 samples to the storage dtype; result is float32 holding stored values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return bf16_widen(bf16_bits(a)) if dtype == "bf16" else a


def _normal(rng, shape, std, dtype):
    a = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return store(a, dtype)


def layer_weights(cfg: Config, seed: int, layer: int, d: int | None = None, d_ff: int | None = None):
    """(w_gate, w_up, w_down), each [d_ff][d] neuron-major, stored values as float32."""
    d = d or cfg.d
    F = d_ff or cfg.d_ff
    return tuple(_normal(_rng(seed, cfg.cid, k, layer), (F, d), cfg.w_std, cfg.dtype)
                 for k in (_W_GATE, _W_UP, _W_DOWN))


def relu_layer(cfg: Config, seed: int, layer: int, d: int | None = None, d_ff: int | None = None):
    """(w_in, b_in, w_out, b_out) of a non-gated ReLU FFN: weights [d_ff][d] neuron-major in the
    storage dtype, biases fp32 ~ N(0, w_std)."""
    d = d or cfg.d
    F = d_ff or cfg.d_ff
    w_in = _normal(_rng(seed, cfg.cid, _W_GATE, layer), (F, d), cfg.w_std, cfg.dtype)
    w_out = _normal(_rng(seed, cfg.cid, _W_DOWN, layer), (F, d), cfg.w_std, cfg.dtype)
    rb = _rng(seed, cfg.cid, _BIAS, layer)
    b_in = (rb.standard_normal(F, dtype=np.float32) * np.float32(cfg.w_std)).astype(np.float32)
    b_out = (rb.standard_normal(d, dtype=np.float32) * np.float32(cfg.w_std)).astype(np.float32)
    return w_in, b_in, w_out, b_out


def prefix_hidden(cfg: Config, seed: int, layer: int, T: int | None = None, d: int | None = None):
    """Prefix hidden states [T][d] ~ N(0,1) for one layer."""
    return _normal(_rng(seed, cfg.cid, _PREFIX, layer), (T or cfg.T, d or cfg.d), 1.0, cfg.dtype)


def decode_hidden(cfg: Config, seed: int, layer: int, step: int, B: int | None = None,
                  d: int | None = None, shared_frac: float = 0.0):
    """Decode hidden states [B][d] ~ N(0,1) for one (layer, step).

    shared_frac = c in [0,1] mixes a component common to the batch:
    x_b = sqrt(c) x_shared + sqrt(1-c) x_b'  (c = 0 is the configuration as written).
    """
    B = B or cfg.B
    d = d or cfg.d
    rng = _rng(seed, cfg.cid, _HIDDEN, layer, step)
    own = rng.standard_normal((B, d), dtype=np.float32)
    if shared_frac > 0.0:
        shared = rng.standard_normal((1, d), dtype=np.float32)
        own = np.float32(np.sqrt(shared_frac)) * shared + np.float32(np.sqrt(1.0 - shared_frac)) * own
    return store(own, cfg.dtype)


def logits(cfg: Config, seed: int, step: int, B: int | None = None, V: int | None = None,
           temperature: float = 1.0):
    """Logits [B][V], float32.

    "spike": N(0, variance 2) noise plus +6 at one seeded index per row.
    "zipf":  -1.1 * log(rank) under a seeded permutation of the vocabulary plus
             N(0,1) noise, divided by ``temperature`` (small = peaked, large = flat).
    Returns (logits, spike_index_or_None).
    """
    B = B or cfg.B
    V = V or cfg.V
    rng = _rng(seed, cfg.cid, _LOGITS, step)
    if cfg.logits == "spike":
        z = rng.standard_normal((B, V), dtype=np.float32) * np.float32(np.sqrt(2.0))
        spike = rng.integers(0, V, size=B)
        z[np.arange(B), spike] += np.float32(6.0)
        return np.ascontiguousarray(z / np.float32(temperature)), spike.astype(np.int32)
    perm = _rng(seed, cfg.cid, _PERM).permutation(V)
    prior = (-1.1 * np.log(np.arange(1, V + 1, dtype=np.float64)))[perm].astype(np.float32)
    z = prior[None, :] + rng.standard_normal((B, V), dtype=np.float32)
    return np.ascontiguousarray(z / np.float32(temperature)), None


def draw_tokens(cfg: Config, seed: int, step: int, z: np.ndarray) -> np.ndarray:
    """One token id per row drawn from the distribution the logits define.

    Uses the Gumbel-max construction (argmax of z + Gumbel noise), which samples
    from the categorical distribution with these logits without normalising it.
    """
    rng = _rng(seed, cfg.cid, _TOKENS, step)
    g = rng.gumbel(size=z.shape)
    return np.argmax(z.astype(np.float64) + g, axis=-1).astype(np.int32)
