"""ctypes binding of libclada (argument marshalling only; no arithmetic here).

Function names mirror the C ABI in ``include/clada.h``.  Tensors are torch CUDA
tensors; kernels are enqueued on torch's current stream of the tensor's device.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libclada.so")
_lib = None

F32, BF16 = 0, 1
_STATUS = ["CLADA_OK", "CLADA_ERR_NULL", "CLADA_ERR_SHAPE", "CLADA_ERR_DTYPE", "CLADA_ERR_ALIGN",
           "CLADA_ERR_WORKSPACE", "CLADA_ERR_VALUE", "CLADA_ERR_HIP"]


class CladaError(RuntimeError):
    def __init__(self, status: int, text: str):
        self.status = status
        name = _STATUS[status] if 0 <= status < len(_STATUS) else f"status {status}"
        super().__init__(f"{name}: {text}")


SWIGLU, RELU, GEGLU = 0, 1, 2      # clada_ffn_kind


class _CLayer(C.Structure):
    _fields_ = [("w_gate", C.c_void_p), ("w_up", C.c_void_p), ("w_down", C.c_void_p),
                ("d", C.c_int32), ("d_ff", C.c_int32), ("dtype", C.c_int), ("kind", C.c_int),
                ("b_in", C.c_void_p), ("b_out", C.c_void_p)]


class _CPrefixOut(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("sum_abs_act", "sum_sq_act", "max_abs_act", "sum_sq_h", "A", "abs_act_pool")]


def lib_path() -> str:
    return _LIB_PATH


def load_library() -> C.CDLL:
    """Load libclada.so; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with "
                           f"`python -m paper_2502_19078_amd.build` (hipcc, gfx950)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, f32 = C.c_void_p, C.c_int32, C.c_float
    lib.clada_create.argtypes = [C.POINTER(vp), C.c_int, C.c_size_t]
    lib.clada_destroy.argtypes = [vp]
    lib.clada_destroy.restype = None
    lib.clada_status_str.argtypes = [C.c_int]
    lib.clada_status_str.restype = C.c_char_p
    lib.clada_last_error.argtypes = [vp]
    lib.clada_last_error.restype = C.c_char_p
    lib.clada_set_option.argtypes = [vp, C.c_char_p, i32]
    lib.clada_workspace_bytes.argtypes = [i32] * 5
    lib.clada_workspace_bytes.restype = C.c_size_t
    lib.clada_prefix_stats.argtypes = [vp, C.POINTER(_CLayer), vp, i32, vp, C.POINTER(_CPrefixOut), vp]
    lib.clada_threshold_calibrate.argtypes = [vp, vp, C.c_int64, f32, vp, vp]
    lib.clada_cognitive_signals.argtypes = [vp, vp, C.c_int, i32, i32, vp, vp, vp, vp]
    lib.clada_threshold.argtypes = [vp, vp, vp, vp, i32, vp, vp, i32, f32, f32, vp, vp]
    lib.clada_cognitive_signals_static.argtypes = [vp, vp, C.c_int, i32, i32, vp, vp, vp, vp]
    lib.clada_cognitive_signals_static.restype = C.c_int
    lib.clada_signals_threshold.argtypes = [vp, vp, C.c_int, i32, i32, vp, vp, vp, vp, i32, f32, f32, vp, vp, vp, vp]
    lib.clada_sparse_ffn_decode.argtypes = [vp, C.POINTER(_CLayer), vp, i32, vp, vp, vp, vp, vp, vp]
    lib.clada_dense_ffn_decode.argtypes = [vp, C.POINTER(_CLayer), vp, i32, vp, vp]
    lib.clada_sparse_ffn_stack_decode.argtypes = [vp, C.POINTER(_CLayer), i32, vp, i32, vp, vp, vp, vp]
    lib.clada_sparse_ffn_stack_decode.restype = C.c_int
    lib.clada_dense_ffn_stack_decode.argtypes = [vp, C.POINTER(_CLayer), i32, vp, i32, vp, vp]
    lib.clada_dense_ffn_stack_decode.restype = C.c_int
    lib.clada_diag_stream_read.argtypes = [vp, vp, C.c_size_t, i32, vp]
    lib.clada_diag_copy.argtypes = [vp, vp, vp, C.c_size_t, vp]
    lib.clada_threshold_search_cett.argtypes = [vp, C.POINTER(_CLayer), vp, i32, C.c_float, i32, vp, vp, vp]
    lib.clada_cett_eval.argtypes = [vp, C.POINTER(_CLayer), vp, i32, C.c_float, vp, vp, vp]
    lib.clada_static_mask_threshold.argtypes = [vp, vp, i32, vp, vp, vp, vp]
    lib.clada_static_mask_topk.argtypes = [vp, vp, i32, i32, vp, vp, vp]
    lib.clada_static_ffn_decode.argtypes = [vp, C.POINTER(_CLayer), vp, i32, vp, vp, vp, vp]
    lib.clada_mask_pack.argtypes = [vp, vp, vp, i32, vp, vp]
    lib.clada_mask_unpack.argtypes = [vp, vp, i32, vp, vp, vp]
    lib.clada_mask_sparse_max_bytes.argtypes = [i32]
    lib.clada_mask_sparse_max_bytes.restype = C.c_size_t
    lib.clada_mask_sparse_encode.argtypes = [vp, vp, vp, i32, vp, i32, vp, vp]
    lib.clada_mask_sparse_encode.restype = C.c_int
    lib.clada_mask_sparse_decode.argtypes = [vp, vp, vp, i32, vp, i32, vp, vp]
    lib.clada_mask_sparse_decode.restype = C.c_int
    lib.clada_mask_sparse_encode_batch.argtypes = [vp, vp, vp, C.c_int64, i32, i32, vp, i32, vp, vp]
    lib.clada_mask_sparse_encode_batch.restype = C.c_int
    lib.clada_mask_sparse_decode_batch.argtypes = [vp, vp, vp, C.c_int64, i32, vp, C.c_int64, i32, i32, vp, vp]
    lib.clada_mask_sparse_decode_batch.restype = C.c_int
    lib.clada_device_fault.argtypes = [vp, C.POINTER(C.c_int32)]
    lib.clada_graph_begin.argtypes = [vp, vp]
    lib.clada_graph_end.argtypes = [vp, vp, C.POINTER(vp)]
    lib.clada_graph_launch.argtypes = [vp, vp, vp]
    lib.clada_graph_destroy.argtypes = [vp]
    lib.clada_graph_destroy.restype = None
    lib.clada_diag_kernel_times.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_float)]
    for name in ("clada_diag_stream_read", "clada_diag_copy", "clada_diag_kernel_times", "clada_device_fault",
                 "clada_threshold_search_cett", "clada_cett_eval", "clada_static_mask_threshold",
                 "clada_static_mask_topk", "clada_static_ffn_decode", "clada_mask_pack", "clada_mask_unpack", "clada_create", "clada_set_option", "clada_prefix_stats", "clada_threshold_calibrate",
                 "clada_cognitive_signals", "clada_threshold", "clada_signals_threshold", "clada_sparse_ffn_decode",
                 "clada_dense_ffn_decode"):
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def workspace_bytes(d: int, d_ff: int, B: int, T: int, V: int) -> int:
    return int(load_library().clada_workspace_bytes(d, d_ff, B, T, V))


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(t: torch.Tensor):
    return C.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


class Context:
    """Owns a libclada context (its device workspace)."""

    def __init__(self, device: int = 0, workspace_bytes: int = 0):
        self._lib = load_library()
        h = C.c_void_p()
        st = self._lib.clada_create(C.byref(h), int(device), int(workspace_bytes))
        if st != 0:
            raise CladaError(st, self._lib.clada_last_error(None).decode())
        self._h = h
        self.device = device

    def close(self):
        if getattr(self, "_h", None):
            self._lib.clada_destroy(self._h)
            self._h = None

    __del__ = close

    def check(self, st: int):
        if st != 0:
            raise CladaError(st, self._lib.clada_last_error(self._h).decode())

    def device_fault(self) -> bool:
        """True once a balanced decode kernel of this context has given up its bounded wait."""
        f = C.c_int32()
        self.check(self._lib.clada_device_fault(self._h, C.byref(f)))
        return f.value != 0

    def set_option(self, name: str, value: int):
        self.check(self._lib.clada_set_option(self._h, name.encode(), int(value)))


@dataclass
class Layer:
    """Neuron-major weights of one FFN layer, each [d_ff][d] on the GPU.  kind = SWIGLU or GEGLU (gated, sigma = SiLU or tanh-form GELU:
    w_gate, w_up, w_down) or RELU (non-gated, OPT family: w_gate = W_in, w_up = None, w_down = W_out
    neuron-major, optional fp32 biases b_in [d_ff], b_out [d])."""
    w_gate: torch.Tensor
    w_up: torch.Tensor | None
    w_down: torch.Tensor
    kind: int = 0
    b_in: torch.Tensor | None = None
    b_out: torch.Tensor | None = None

    def c_struct(self) -> _CLayer:
        F, d = self.w_gate.shape
        ws = (self.w_gate, self.w_down) if self.kind == RELU else (self.w_gate, self.w_up, self.w_down)
        for w in ws:
            assert w.is_cuda and w.is_contiguous() and tuple(w.shape) == (F, d) and w.dtype == self.w_gate.dtype
        for b, n in ((self.b_in, F), (self.b_out, d)):
            assert b is None or (b.is_cuda and b.is_contiguous() and b.dtype == torch.float32 and b.numel() == n)
        return _CLayer(self.w_gate.data_ptr(), None if self.w_up is None else self.w_up.data_ptr(),
                       self.w_down.data_ptr(), d, F, _dtype_code(self.w_gate), self.kind,
                       None if self.b_in is None else self.b_in.data_ptr(),
                       None if self.b_out is None else self.b_out.data_ptr())


@dataclass
class PrefixStats:
    sum_abs_act: torch.Tensor
    sum_sq_act: torch.Tensor
    max_abs_act: torch.Tensor
    sum_sq_h: torch.Tensor
    A: torch.Tensor
    abs_act_pool: torch.Tensor | None
    y: torch.Tensor | None


def prefix_stats(ctx: Context, layer: Layer, x: torch.Tensor, want_y: bool = True,
                 want_pool: bool = True) -> PrefixStats:
    cl = layer.c_struct()
    T = x.shape[0]
    assert x.is_cuda and x.is_contiguous() and x.shape == (T, cl.d) and x.dtype == layer.w_gate.dtype
    f = lambda *s: torch.empty(*s, dtype=torch.float32, device=x.device)
    stats = [f(cl.d_ff) for _ in range(5)]
    pool = f(T, cl.d_ff) if want_pool else None
    y = torch.empty_like(x) if want_y else None
    out = _CPrefixOut(*[s.data_ptr() for s in stats], pool.data_ptr() if want_pool else None)
    ctx.check(ctx._lib.clada_prefix_stats(ctx._h, C.byref(cl), _ptr(x), T, _ptr(y), C.byref(out), _stream(x)))
    return PrefixStats(*stats, pool, y)


def threshold_calibrate(ctx: Context, abs_act_pool: torch.Tensor, target_sparsity: float,
                        out: torch.Tensor | None = None) -> torch.Tensor:
    p = abs_act_pool
    assert p.is_cuda and p.is_contiguous() and p.dtype == torch.float32
    if out is None:
        out = torch.empty(1, dtype=torch.float32, device=p.device)
    ctx.check(ctx._lib.clada_threshold_calibrate(ctx._h, _ptr(p), p.numel(), float(target_sparsity),
                                                 _ptr(out), _stream(p)))
    return out


def threshold_search_cett(ctx: Context, layer: Layer, x_val: torch.Tensor, bound: float = 0.2,
                          n_probes: int = 31, out: torch.Tensor | None = None):
    """(tau_base [1], mean CETT at tau_base [1]) of the error-bounded base-threshold search."""
    cl = layer.c_struct()
    T = x_val.shape[0]
    assert x_val.is_cuda and x_val.is_contiguous() and x_val.shape == (T, cl.d) and x_val.dtype == layer.w_gate.dtype
    if out is None:
        out = torch.empty(1, dtype=torch.float32, device=x_val.device)
    mean = torch.empty(1, dtype=torch.float32, device=x_val.device)
    ctx.check(ctx._lib.clada_threshold_search_cett(ctx._h, C.byref(cl), _ptr(x_val), T, float(bound), int(n_probes),
                                                   _ptr(out), _ptr(mean), _stream(x_val)))
    return out, mean


def cett_eval(ctx: Context, layer: Layer, x_val: torch.Tensor, eps: float):
    """(per-token CETT [T], mean [1]) at cut threshold eps."""
    cl = layer.c_struct()
    T = x_val.shape[0]
    assert x_val.is_cuda and x_val.is_contiguous() and x_val.shape == (T, cl.d) and x_val.dtype == layer.w_gate.dtype
    c = torch.empty(T, dtype=torch.float32, device=x_val.device)
    mean = torch.empty(1, dtype=torch.float32, device=x_val.device)
    ctx.check(ctx._lib.clada_cett_eval(ctx._h, C.byref(cl), _ptr(x_val), T, float(eps), _ptr(c), _ptr(mean),
                                       _stream(x_val)))
    return c, mean


def cognitive_signals(ctx: Context, logits: torch.Tensor, token_ids: torch.Tensor):
    B, V = logits.shape
    assert logits.is_cuda and logits.is_contiguous()
    assert token_ids.is_cuda and token_ids.dtype == torch.int32 and token_ids.numel() == B
    s = torch.empty(B, dtype=torch.float32, device=logits.device)
    h = torch.empty(B, dtype=torch.float32, device=logits.device)
    ctx.check(ctx._lib.clada_cognitive_signals(ctx._h, _ptr(logits), _dtype_code(logits), B, V,
                                               _ptr(token_ids), _ptr(s), _ptr(h), _stream(logits)))
    return s, h


def cognitive_signals_static(ctx: Context, logits: torch.Tensor, token_ids: torch.Tensor,
                             out: tuple[torch.Tensor, torch.Tensor] | None = None):
    """clada_cognitive_signals_static: scratch inside the library, nothing allocated by the call when `out`
    = (surprisal, entropy) is given."""
    B, V = logits.shape
    assert logits.is_cuda and logits.is_contiguous()
    assert token_ids.is_cuda and token_ids.dtype == torch.int32 and token_ids.numel() == B
    if out is None:
        out = (torch.empty(B, dtype=torch.float32, device=logits.device),
               torch.empty(B, dtype=torch.float32, device=logits.device))
    s, h = out
    ctx.check(ctx._lib.clada_cognitive_signals_static(ctx._h, _ptr(logits), _dtype_code(logits), B, V,
                                                      _ptr(token_ids), _ptr(s), _ptr(h), _stream(logits)))
    return s, h


def threshold(ctx: Context, tau_base, lam, gam, surprisal, entropy, tau_s: float, tau_H: float,
              out: torch.Tensor | None = None) -> torch.Tensor:
    L, B = tau_base.numel(), surprisal.numel()
    for t in (tau_base, lam, gam, surprisal, entropy):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
    assert lam.numel() == L and gam.numel() == L and entropy.numel() == B
    if out is None:
        out = torch.empty(L, B, dtype=torch.float32, device=tau_base.device)
    ctx.check(ctx._lib.clada_threshold(ctx._h, _ptr(tau_base), _ptr(lam), _ptr(gam), L, _ptr(surprisal),
                                       _ptr(entropy), B, float(tau_s), float(tau_H), _ptr(out),
                                       _stream(tau_base)))
    return out


def signals_threshold(ctx: Context, logits: torch.Tensor, token_ids: torch.Tensor, tau_base, lam, gam,
                      tau_s: float, tau_H: float, out: torch.Tensor | None = None):
    """(surprisal [B], entropy [B], tau_final [L][B]) from one launch."""
    B, V = logits.shape
    L = tau_base.numel()
    assert logits.is_cuda and logits.is_contiguous()
    assert token_ids.is_cuda and token_ids.dtype == torch.int32 and token_ids.numel() == B
    for t in (tau_base, lam, gam):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == L
    s = torch.empty(B, dtype=torch.float32, device=logits.device)
    h = torch.empty(B, dtype=torch.float32, device=logits.device)
    if out is None:
        out = torch.empty(L, B, dtype=torch.float32, device=logits.device)
    ctx.check(ctx._lib.clada_signals_threshold(ctx._h, _ptr(logits), _dtype_code(logits), B, V, _ptr(token_ids),
                                               _ptr(tau_base), _ptr(lam), _ptr(gam), L, float(tau_s), float(tau_H),
                                               _ptr(s), _ptr(h), _ptr(out), _stream(logits)))
    return s, h, out


def sparse_ffn_decode(ctx: Context, layer: Layer, x: torch.Tensor, tau_final: torch.Tensor,
                      y: torch.Tensor | None = None, want_lists: bool = False):
    """Returns y, or (y, active_idx, n_active, mask_bits) when want_lists."""
    cl = layer.c_struct()
    B = x.shape[0]
    assert x.is_cuda and x.is_contiguous() and x.shape == (B, cl.d) and x.dtype == layer.w_gate.dtype
    assert tau_final.is_cuda and tau_final.dtype == torch.float32 and tau_final.numel() == B
    assert tau_final.is_contiguous()
    if y is None:
        y = torch.empty_like(x)
    idx = cnt = bits = None
    if want_lists:
        idx = torch.full((cl.d_ff,), -1, dtype=torch.int32, device=x.device)
        cnt = torch.empty(1 + B, dtype=torch.int32, device=x.device)
        bits = torch.empty(B, (cl.d_ff + 31) // 32, dtype=torch.int32, device=x.device)
    ctx.check(ctx._lib.clada_sparse_ffn_decode(ctx._h, C.byref(cl), _ptr(x), B, _ptr(tau_final), _ptr(y),
                                               _ptr(idx), _ptr(cnt), _ptr(bits), _stream(x)))
    return (y, idx, cnt, bits) if want_lists else y


def dense_ffn_decode(ctx: Context, layer: Layer, x: torch.Tensor, y: torch.Tensor | None = None):
    cl = layer.c_struct()
    B = x.shape[0]
    assert x.is_cuda and x.is_contiguous() and x.shape == (B, cl.d) and x.dtype == layer.w_gate.dtype
    if y is None:
        y = torch.empty_like(x)
    ctx.check(ctx._lib.clada_dense_ffn_decode(ctx._h, C.byref(cl), _ptr(x), B, _ptr(y), _stream(x)))
    return y


def layer_array(layers):
    """Host array of clada_layer structs for the whole-stack calls (keep it alive while calls use it)."""
    return (_CLayer * len(layers))(*[l.c_struct() for l in layers])


def _stack_batch(layers, x):
    L = len(layers)
    assert x.is_cuda and x.is_contiguous() and x.shape[0] == L and x.dim() in (2, 3) and x.dtype == layers[0].w_gate.dtype
    return L, (1 if x.dim() == 2 else x.shape[1])


def sparse_ffn_stack_decode(ctx: Context, layers, x: torch.Tensor, tau_final: torch.Tensor,
                            y: torch.Tensor | None = None, want_counts: bool = False, c_layers=None):
    """x [L][d] or [L][B][d], tau_final [L] or [L][B] -> y like x (and n_active [L][1+B] int32 with
    want_counts): the L layers of a stack in one call."""
    L, B = _stack_batch(layers, x)
    arr = c_layers if c_layers is not None else layer_array(layers)
    assert tau_final.is_cuda and tau_final.dtype == torch.float32 and tau_final.numel() == L * B and tau_final.is_contiguous()
    if y is None:
        y = torch.empty_like(x)
    cnt = torch.empty(L, 1 + B, dtype=torch.int32, device=x.device) if want_counts else None
    ctx.check(ctx._lib.clada_sparse_ffn_stack_decode(ctx._h, arr, L, _ptr(x), B, _ptr(tau_final), _ptr(y), _ptr(cnt), _stream(x)))
    return (y, cnt) if want_counts else y


def dense_ffn_stack_decode(ctx: Context, layers, x: torch.Tensor, y: torch.Tensor | None = None, c_layers=None):
    L, B = _stack_batch(layers, x)
    arr = c_layers if c_layers is not None else layer_array(layers)
    if y is None:
        y = torch.empty_like(x)
    ctx.check(ctx._lib.clada_dense_ffn_stack_decode(ctx._h, arr, L, _ptr(x), B, _ptr(y), _stream(x)))
    return y


def static_mask_threshold(ctx: Context, A: torch.Tensor, tau_final: torch.Tensor):
    """(active_idx [F] int32, n_active [1] int32): ascending neurons with A_j >= tau_final[0]."""
    assert A.is_cuda and A.dtype == torch.float32 and A.is_contiguous()
    assert tau_final.is_cuda and tau_final.dtype == torch.float32 and tau_final.numel() >= 1
    idx = torch.empty(A.numel(), dtype=torch.int32, device=A.device)
    n = torch.empty(1, dtype=torch.int32, device=A.device)
    ctx.check(ctx._lib.clada_static_mask_threshold(ctx._h, _ptr(A), A.numel(), _ptr(tau_final), _ptr(idx), _ptr(n),
                                                   _stream(A)))
    return idx, n


def static_mask_topk(ctx: Context, score: torch.Tensor, k: int):
    """(active_idx [F] int32, n_active [1] int32): ascending indices of the k largest scores."""
    assert score.is_cuda and score.dtype == torch.float32 and score.is_contiguous()
    idx = torch.empty(score.numel(), dtype=torch.int32, device=score.device)
    n = torch.empty(1, dtype=torch.int32, device=score.device)
    ctx.check(ctx._lib.clada_static_mask_topk(ctx._h, _ptr(score), score.numel(), int(k), _ptr(idx), _ptr(n),
                                              _stream(score)))
    return idx, n


def mask_pack(ctx: Context, active_idx: torch.Tensor, n_active: torch.Tensor, d_ff: int) -> torch.Tensor:
    """Ascending list -> packed bit mask [ceil(d_ff/32)] int32."""
    assert active_idx.is_cuda and active_idx.dtype == torch.int32 and n_active.dtype == torch.int32
    bits = torch.empty((d_ff + 31) // 32, dtype=torch.int32, device=active_idx.device)
    ctx.check(ctx._lib.clada_mask_pack(ctx._h, _ptr(active_idx), _ptr(n_active), int(d_ff), _ptr(bits),
                                       _stream(active_idx)))
    return bits


def mask_unpack(ctx: Context, mask_bits: torch.Tensor, d_ff: int):
    """Packed bit mask -> (active_idx [d_ff] int32, n_active [1] int32)."""
    assert mask_bits.is_cuda and mask_bits.dtype == torch.int32 and mask_bits.numel() >= (d_ff + 31) // 32
    idx = torch.empty(d_ff, dtype=torch.int32, device=mask_bits.device)
    n = torch.empty(1, dtype=torch.int32, device=mask_bits.device)
    ctx.check(ctx._lib.clada_mask_unpack(ctx._h, _ptr(mask_bits), int(d_ff), _ptr(idx), _ptr(n), _stream(mask_bits)))
    return idx, n


def mask_sparse_encode(ctx: Context, mask_bits: torch.Tensor, ref_bits: torch.Tensor | None, d_ff: int,
                       capacity: int | None = None):
    """Bit mask (against a reference mask or None) -> (stream uint8 [capacity], n int32 [2] = bytes or -1, positions)."""
    words = (d_ff + 31) // 32
    assert mask_bits.is_cuda and mask_bits.dtype == torch.int32 and mask_bits.numel() >= words and mask_bits.is_contiguous()
    assert ref_bits is None or (ref_bits.is_cuda and ref_bits.dtype == torch.int32 and ref_bits.numel() >= words
                                and ref_bits.is_contiguous())
    if capacity is None:
        capacity = int(ctx._lib.clada_mask_sparse_max_bytes(int(d_ff)))
    stream = torch.empty(max(capacity, 1), dtype=torch.uint8, device=mask_bits.device)
    n = torch.empty(2, dtype=torch.int32, device=mask_bits.device)
    ctx.check(ctx._lib.clada_mask_sparse_encode(ctx._h, _ptr(mask_bits), _ptr(ref_bits), int(d_ff), _ptr(stream),
                                                int(capacity), _ptr(n), _stream(mask_bits)))
    return stream, n


def mask_sparse_decode(ctx: Context, stream: torch.Tensor, n_bytes: torch.Tensor, ref_bits: torch.Tensor | None,
                       d_ff: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """Stream (+ the reference it was coded against) -> bit mask [ceil(d_ff/32)] int32."""
    assert stream.is_cuda and stream.dtype == torch.uint8 and stream.is_contiguous()
    assert n_bytes.is_cuda and n_bytes.dtype == torch.int32 and n_bytes.numel() >= 1
    if out is None:
        out = torch.empty((d_ff + 31) // 32, dtype=torch.int32, device=stream.device)
    ctx.check(ctx._lib.clada_mask_sparse_decode(ctx._h, _ptr(stream), _ptr(n_bytes), int(stream.numel()), _ptr(ref_bits),
                                                int(d_ff), _ptr(out), _stream(stream)))
    return out


def _ref_stride(ref_bits, n, words):
    if ref_bits is None or ref_bits.dim() == 1:
        return 0
    assert ref_bits.shape == (n, words)
    return words


def mask_sparse_encode_batch(ctx: Context, mask_bits: torch.Tensor, ref_bits: torch.Tensor | None, d_ff: int,
                             capacity: int | None = None):
    """mask_bits [n][words] against ref_bits ([words] shared, [n][words] one each, or None)
    -> (streams uint8 [n][capacity], n_out int32 [n][2])."""
    words = (d_ff + 31) // 32
    assert mask_bits.is_cuda and mask_bits.dtype == torch.int32 and mask_bits.dim() == 2 and mask_bits.shape[1] == words
    assert mask_bits.is_contiguous() and (ref_bits is None or (ref_bits.is_cuda and ref_bits.dtype == torch.int32
                                                               and ref_bits.is_contiguous()))
    n = mask_bits.shape[0]
    if capacity is None:
        capacity = int(ctx._lib.clada_mask_sparse_max_bytes(int(d_ff)))
    streams = torch.empty(n, max(capacity, 1), dtype=torch.uint8, device=mask_bits.device)
    n_out = torch.empty(n, 2, dtype=torch.int32, device=mask_bits.device)
    ctx.check(ctx._lib.clada_mask_sparse_encode_batch(ctx._h, _ptr(mask_bits), _ptr(ref_bits), _ref_stride(ref_bits, n, words),
                                                      int(d_ff), n, _ptr(streams), int(streams.shape[1]), _ptr(n_out),
                                                      _stream(mask_bits)))
    return streams, n_out


def mask_sparse_decode_batch(ctx: Context, streams: torch.Tensor, n_out: torch.Tensor, ref_bits: torch.Tensor | None,
                             d_ff: int) -> torch.Tensor:
    """Streams [n][capacity] with the encoder's n_out [n][2] -> bit masks [n][words] int32."""
    words = (d_ff + 31) // 32
    assert streams.is_cuda and streams.dtype == torch.uint8 and streams.dim() == 2 and streams.is_contiguous()
    n = streams.shape[0]
    assert n_out.is_cuda and n_out.dtype == torch.int32 and n_out.shape == (n, 2) and n_out.is_contiguous()
    out = torch.empty(n, words, dtype=torch.int32, device=streams.device)
    ctx.check(ctx._lib.clada_mask_sparse_decode_batch(ctx._h, _ptr(streams), _ptr(n_out), 2, int(streams.shape[1]),
                                                      _ptr(ref_bits), _ref_stride(ref_bits, n, words), int(d_ff), n,
                                                      _ptr(out), _stream(streams)))
    return out


def static_ffn_decode(ctx: Context, layer: Layer, x: torch.Tensor, active_idx: torch.Tensor,
                      n_active: torch.Tensor, y: torch.Tensor | None = None) -> torch.Tensor:
    cl = layer.c_struct()
    B = x.shape[0]
    assert x.is_cuda and x.is_contiguous() and x.shape == (B, cl.d) and x.dtype == layer.w_gate.dtype
    assert active_idx.is_cuda and active_idx.dtype == torch.int32 and active_idx.is_contiguous()
    assert n_active.is_cuda and n_active.dtype == torch.int32 and n_active.numel() >= 1
    if y is None:
        y = torch.empty_like(x)
    ctx.check(ctx._lib.clada_static_ffn_decode(ctx._h, C.byref(cl), _ptr(x), B, _ptr(active_idx), _ptr(n_active),
                                               _ptr(y), _stream(x)))
    return y


def diag_stream_read(ctx: Context, src: torch.Tensor, blocks_per_cu: int = 1):
    ctx.check(ctx._lib.clada_diag_stream_read(ctx._h, _ptr(src), src.numel() * src.element_size(),
                                              blocks_per_cu, _stream(src)))


class Graph:
    """One captured decode step (clada_graph_*).  The calls issued on torch's current stream between
    graph_begin and graph_end are recorded; launch() replays them on the current stream."""

    def __init__(self, ctx: Context, handle):
        self._ctx, self._g = ctx, handle

    def launch(self):
        st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        self._ctx.check(self._ctx._lib.clada_graph_launch(self._ctx._h, self._g, st))

    def __del__(self):
        if getattr(self, "_g", None):
            self._ctx._lib.clada_graph_destroy(self._g)
            self._g = None


def graph_begin(ctx: Context):
    ctx.check(ctx._lib.clada_graph_begin(ctx._h, C.c_void_p(torch.cuda.current_stream().cuda_stream)))


def graph_end(ctx: Context) -> Graph:
    g = C.c_void_p()
    ctx.check(ctx._lib.clada_graph_end(ctx._h, C.c_void_p(torch.cuda.current_stream().cuda_stream), C.byref(g)))
    return Graph(ctx, g)


def diag_copy(ctx: Context, src: torch.Tensor, dst: torch.Tensor):
    assert src.numel() * src.element_size() == dst.numel() * dst.element_size()
    ctx.check(ctx._lib.clada_diag_copy(ctx._h, _ptr(src), _ptr(dst), src.numel() * src.element_size(),
                                       _stream(src)))


def diag_kernel_times(ctx: Context):
    """(main_us, finalize_us) of the context's last decode call; needs option diag.kernel_events = 1."""
    a, b = C.c_float(), C.c_float()
    ctx.check(ctx._lib.clada_diag_kernel_times(ctx._h, C.byref(a), C.byref(b)))
    return a.value, b.value
