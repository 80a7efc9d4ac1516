// Host-side launcher prototypes (one per kernel family).  Each returns QP_OK or
// QP_ERR_DEVICE / QP_ERR_UNSUPPORTED; arguments were validated by the caller.
#pragma once
#include <hip/hip_runtime.h>

#include "qp_dev.h"

qp_status qp_launch_dequant(const QpW &w, int scheme, int cb, void *out, hipStream_t st);
// native layout only: one 16 x 1024 block per wavefront, the fused kernel's decoders
qp_status qp_launch_dequant_blocks(const QpW &w, int scheme, int cb, void *out, hipStream_t st);
qp_status qp_launch_linear_rowwave(const QpW &w, int scheme, int cb, const void *x, int B, int64_t ldx,
                                   void *y, int64_t ldy, hipStream_t st);
// the row kernel with the rotation inside (batch 1, x and y contiguous rows); the predicate says where it exists
bool qp_rowwave_rotates(int scheme, int cb, int N, int rot_block);
qp_status qp_launch_linear_rowwave_rot(const QpW &w, int scheme, int cb, const void *x, const int8_t *signs,
                                       int rot_block, void *y, hipStream_t st);
bool qp_linear_rotates_blocks(int scheme, int M, int N, int rot_block);
qp_status qp_launch_linear_mfma(const QpW &w, int scheme, int cb, const void *x, int B, int64_t ldx, void *y,
                                int64_t ldy, int x_packed, const int8_t *signs, int rot_block, hipStream_t st);
// pack_bp: 0 writes xr row-major; a power of two >= B writes the fragment order that
// qp_launch_linear_mfma reads with x_packed (pack_bp * n halves of room, n rounded up to a multiple of 1024)
qp_status qp_launch_hadamard(const void *x, const int8_t *signs, int B, int n, int block, int64_t ldx,
                             void *xr, int64_t ldxr, int pack_bp, hipStream_t st);
qp_status qp_launch_pack_x(const void *x, int B, int n, int64_t ldx, void *xp, int pack_bp, hipStream_t st);
// encoders (canonical output); workspace only for the trellis schemes
qp_status qp_launch_encode(int scheme, int cb, int tlut_bits, int M, int N, const uint16_t *lut, const void *W, int64_t ldw,
                           void *codes, int64_t row_stride, void *workspace, size_t workspace_bytes, float *tile_err,
                           hipStream_t st);
qp_status qp_launch_row_normalize(void *W, int64_t ldw, int M, int N, void *scales, hipStream_t st);
size_t qp_encode_min_workspace(int scheme, int cb);   // bytes one workgroup needs; 0 for SQ / VQ
qp_status qp_launch_repack(const QpW &src, int span_bytes, void *dst, hipStream_t st);
// half-TCQ: spans of 16 cb bytes in the first N/2 columns, 16 (cb + 1) in the rest
qp_status qp_launch_repack_half(const QpW &src, int cb, void *dst, hipStream_t st);

// Lloyd's algorithm (code book construction); workspace of qp_kmeans_workspace(k, d) bytes
size_t qp_kmeans_workspace(int k, int d);
qp_status qp_launch_kmeans(const float *x, int64_t n, int d, float *centres, int k, int max_iter, float tol,
                           void *workspace, int32_t *assign_out, uint16_t *centres_f16, double *stats_out,
                           hipStream_t st);

// current value of a tuning option (qp_option); defined beside qp_set_option
int32_t qp_opt(int option);

static inline qp_status qp_check_launch() {
    return hipGetLastError() == hipSuccess ? QP_OK : QP_ERR_DEVICE;
}
