"""MI355X-native quantized linear layers (Q-Palette inference hot path).

Thin Python binding over the C-ABI library declared in include/qp.h: the
functions here have the same names as the C entry points and only marshal
arguments (torch tensors -> device pointers, the current HIP stream).  Every
step of the path runs in the library's HIP kernels; there is no CPU fallback —
if the library cannot be loaded, importing `binding` users fail loudly.
"""
from .binding import *  # noqa: F401,F403  (the option constants QP_OPT_*, QP_KERNEL_*, QP_DEQUANT_*)
from .binding import (QP_SQ, QP_VQ, QP_TCQ, QP_TCQH, QP_TCQHH, QP_LAYOUT_CANONICAL, QP_LAYOUT_NATIVE, QpError, Weight,
                      load_library, qp_dequant, qp_hadamard, qp_linear, qp_linear_workspace_bytes,
                      qp_encode, qp_encode_workspace_bytes, qp_kmeans, qp_kmeans_workspace_bytes, qp_msq_solve, qp_row_normalize, qp_native_bytes, qp_repack, qp_rotate_linear, qp_rotate_linear_workspace_bytes, qp_rotate_linear_launches,
                      qp_status_string, qp_validate, qp_version, qp_set_option, qp_get_option, qp_reset_options,
                      qp_rotate_linear_static, qp_rotate_linear_static_max_bytes,
                      qp_bench_stream_read, qp_bench_empty_launch, Block, qp_block_workspace_bytes, qp_block_enqueue,
                      qp_block_create, qp_block_run, qp_block_destroy)

__all__ = ["QP_SQ", "QP_VQ", "QP_TCQ", "QP_TCQH", "QP_TCQHH", "QP_LAYOUT_CANONICAL", "QP_LAYOUT_NATIVE", "QpError", "Weight",
           "load_library", "qp_dequant", "qp_hadamard", "qp_linear", "qp_linear_workspace_bytes",
           "qp_encode", "qp_encode_workspace_bytes", "qp_kmeans", "qp_kmeans_workspace_bytes", "qp_msq_solve", "qp_row_normalize", "qp_native_bytes", "qp_repack", "qp_rotate_linear", "qp_rotate_linear_workspace_bytes", "qp_rotate_linear_launches",
           "qp_status_string", "qp_validate", "qp_version", "qp_set_option", "qp_get_option", "qp_reset_options",
           "qp_rotate_linear_static", "qp_rotate_linear_static_max_bytes",
           "qp_bench_stream_read", "qp_bench_empty_launch", "Block", "qp_block_workspace_bytes", "qp_block_enqueue",
           "qp_block_create", "qp_block_run", "qp_block_destroy"]
