"""MaxScore routing hot path on one MI355X: thin Python binding over libmaxscore.so.

Every step runs in the HIP kernels of the shared library; this package only marshals arguments
(torch supplies device memory and the current stream).  Importing works without a GPU; calling
any compute function without the built library or without a GPU raises.
"""
from .binding import (MaxScoreError, Stats, lib_path, load_library, exported_symbols, workspace_bytes,
                      router_logits, router_softtopk, softtopk, scores_op, assign_i32, assign_caps_i32, assign_kvec_i32, assign_top1_residual_i32, assign_top1_sinkhorn, assign_iter_i32, gates, aux_loss, gates_backward, dispatch, dispatch_static, dispatch_tokens, combine,
                      route_scores, route_logits, route_xw, set_kernel_timing, copy_bytes, status_string)

__all__ = ["MaxScoreError", "Stats", "lib_path", "load_library", "exported_symbols", "workspace_bytes",
           "router_logits", "router_softtopk", "softtopk", "scores_op", "assign_i32", "assign_caps_i32", "assign_kvec_i32", "assign_top1_residual_i32", "assign_top1_sinkhorn", "assign_iter_i32", "gates", "aux_loss", "gates_backward", "dispatch", "dispatch_static", "dispatch_tokens", "combine",
           "route_scores", "route_logits", "route_xw",
           "set_kernel_timing", "copy_bytes", "status_string"]
