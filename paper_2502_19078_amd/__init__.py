"""MI355X-native implementation of CLADA's decode-time hot path (arXiv 2502.19078):
the thresholded sparse SwiGLU FFN and the calls that feed it.

Every step runs in hand-written HIP kernels inside ``libclada.so`` (C ABI declared
in ``include/clada.h``); this package is only the ctypes binding.  PyTorch is used
for device memory and streams.  There is no CPU fallback: calls raise if the
library is not built.
"""
from .binding import (Context, Layer, PrefixStats, CladaError, cognitive_signals,  # noqa: F401
                      dense_ffn_decode, lib_path, load_library, prefix_stats,
                      sparse_ffn_decode, threshold, threshold_calibrate, signals_threshold,
                      threshold_search_cett, cett_eval, static_mask_threshold,
                      static_mask_topk, static_ffn_decode, mask_pack, mask_unpack,
                      mask_sparse_encode, mask_sparse_decode, mask_sparse_encode_batch,
                      mask_sparse_decode_batch, sparse_ffn_stack_decode,
                      dense_ffn_stack_decode, layer_array,
                      workspace_bytes, Graph, graph_begin, graph_end)
