/*
 * qp.h — C ABI of the MI355X (gfx950) quantized-linear library.
 *
 * The library computes the inference hot path of Q-Palette: a linear layer whose
 * weight matrix W^ is never stored but decoded on the fly from packed
 * fractional-bit codes, applied to activations that were rotated by a randomized
 * Hadamard transform:
 *
 *        y[b, j] = s[j] * sum_i xr[b, i] * W^[j, i]          (Section 3.3)
 *
 * with W^ given by one of the quantizer families of the paper (Section 3.2, Appendix C):
 *   QP_SQ   non-uniform scalar quantizer:  W^[j,i]           = LUT[code]          (App. C.1 "Dequantization")
 *   QP_VQ   2-D vector quantizer:          (W^[j,2m],W^[j,2m+1]) = LUT[code]      (App. C.2 "Dequantization")
 *   QP_TCQ  bitshift trellis, tail-biting: W^[j,tT+i]        = LUT[r_t[ik : ik+L]] (App. C.3.1 "Dequantization")
 *   QP_TCQH the paper's own trellis: V = 2 weights per step of s bits (s/2 bits per weight),
 *           (W^[j,tT+2i], W^[j,tT+2i+1]) = LUT[r_t[is : is+16]], with the 2^16 x 2 LUT *computed* from a
 *           small table tlut[2^tb][2]: h = x(x+1), entry (h >> (15-tb)) mod 2^tb, component 0 negated
 *           when bit 15 of h is set (App. C.3.1 "Codebook construction")
 *   QP_TCQHH half-TCQ (Section 3.2, App. C.3.2): QP_TCQH with s bits per step on the first N/2 input
 *           channels and s + 1 on the remaining N/2 (s/2 + 1/4 bits per weight), both halves decoded
 *           with the one small table that belongs to s + 1
 *
 * Notation: M = out_features = rows of W^, N = in_features = columns, B = batch.
 *
 * CANONICAL LAYOUT (QP_LAYOUT_CANONICAL).  Row j of W^ is one bitstream of
 * N/vec codes of code_bits bits, starting at codes + j*row_stride.  Stream bit p
 * is bit (p mod 8) of byte floor(p/8); a code that starts at stream bit q has the
 * value sum_t bit(q+t) 2^t.  For QP_TCQ a row is N/tile consecutive tiles of
 * code_bits*tile bits; inside a tile weight i is LUT[window], the window being
 * the window_bits stream bits from i*code_bits on, taken modulo the tile's length.
 *
 * For QP_TCQHH a row is the N/512 tiles of the first half (16 s bytes each) followed by the N/512
 * tiles of the second half (16 (s + 1) bytes each).
 *
 * NATIVE LAYOUT (QP_LAYOUT_NATIVE), produced by qp_repack; needs M % 16 == 0 and
 * N % 256 == 0.  The matrix is cut into blocks of 16 rows x 1024 columns (ceil(N / 1024) per
 * block row; where N is not a multiple of 1024 - 11008, 13824 - the spans of the last column
 * block that lie beyond N hold zero bytes and the kernels multiply what those decode to - finite
 * table entries, which is all a table may hold - with zeros), stored
 * block-row-major (all column blocks of rows 0..15, then rows 16..31, ...).  Within
 * a block, "lane" l = 16*g + i (g = 0..3, i = 0..15) owns row i, columns
 * 256*g .. 256*g+255 of the block: the same 32*bpw bytes that the canonical stream
 * holds for that span (bpw = code_bits/vec).  Those bytes are cut into P = 2*bpw
 * pieces of 16 bytes; piece p of lane l sits at byte (p*64 + l)*16 of the block, so
 * one 128-bit load per lane of a 64-wide wavefront reads 1 KiB contiguously.
 * row_stride is ignored for this layout.  It is the layout the kernels are fastest on; layers
 * of these shapes run the same matrix-core kernel from the canonical layout too, some
 * 25 % slower, anything else a layout-agnostic kernel.  QP_TCQHH (needs N % 2048 == 0): the column blocks of the
 * second half have one piece more than those of the first; a block row is the N/2048 blocks of the
 * first half followed by the N/2048 blocks of the second.
 *
 * All pointers named "device" are device (HBM) pointers owned by the caller; the
 * library allocates no device memory.  Its only mutable state is the table of process-wide
 * tuning options behind qp_set_option (kernel choices for tests and measurements; the defaults
 * are the measured best choices and nothing reads the process environment) and the fixed
 * scratch array of qp_rotate_linear_static.  Every entry
 * point validates its arguments on the host first and returns a QP_ERR_* code
 * without touching the device when they are bad; it then only enqueues kernels on
 * the given hipStream_t (passed as void*; NULL is the default stream) and returns
 * without synchronising.  A failed launch returns QP_ERR_DEVICE.  Nothing throws.
 */
#ifndef QP_H
#define QP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QP_OK = 0,
    QP_ERR_NULL = 1,        /* a required pointer is NULL                                  */
    QP_ERR_SHAPE = 2,       /* M, N, B, n, block, ld* out of range or not divisible        */
    QP_ERR_UNSUPPORTED = 3, /* (scheme, code_bits, vec, window_bits, tile) not in the set  */
    QP_ERR_ALIGN = 4,       /* pointer or stride not aligned as documented                 */
    QP_ERR_LAYOUT = 5,      /* layout value unknown, or shape not representable in it      */
    QP_ERR_DEVICE = 6,      /* HIP reported a launch error                                 */
    QP_ERR_WORKSPACE = 7,   /* workspace smaller than qp_linear_workspace_bytes()          */
    QP_ERR_MEMORY = 8       /* host memory exhausted (qp_msq_solve*: tables too large)     */
} qp_status;

typedef enum { QP_SQ = 0, QP_VQ = 1, QP_TCQ = 2, QP_TCQH = 3, QP_TCQHH = 4 } qp_scheme;
typedef enum { QP_LAYOUT_CANONICAL = 0, QP_LAYOUT_NATIVE = 1 } qp_layout;

#define QP_MAX_BATCH 16
#define QP_MAX_LDX (1 << 26)   /* largest row stride of the activations, in elements */

/* One quantized layer.  Supported set:
 *   QP_SQ : vec 1, code_bits 4                       (16-entry fp16 LUT)
 *   QP_VQ : vec 2, code_bits 5 or 7                  (2.5 / 3.5 bits per weight; LUT fp16 [2^code_bits][2])
 *   QP_TCQ: vec 1, window_bits 16, tile 256, code_bits 2, 3 or 4  (LUT fp16 [65536])
 *   QP_TCQH: vec 2, window_bits 16, tile 256, code_bits s = 3..10 (1.5 .. 5 bits per weight),
 *            tlut_bits 9 for s <= 8, 10 for s = 9, 11 for s = 10, the table sizes of App. C.3.1
 *            (lut = the small table, fp16 [2^tlut_bits][2])
 *   QP_TCQHH: vec 2, window_bits 16, tile 256, code_bits s = 3..9 (1.75 .. 4.75 bits per weight),
 *            N % 512 == 0, tlut_bits that of s + 1 (9 for s <= 7, 10 for s = 8, 11 for s = 9)
 * Fused layers (QKV, gate+up; Section 4.2) are one qp_weight with M the sum of the
 * members' out_features. */
typedef struct {
    int32_t scheme;      /* qp_scheme                                                          */
    int32_t M, N;        /* rows (output channels), columns (input channels)                   */
    int32_t code_bits;   /* SQ: bits per weight; VQ: bits per vec-vector; TCQ: bits shifted per step */
    int32_t vec;         /* V                                                                  */
    int32_t window_bits; /* TCQ: L; otherwise 0                                                */
    int32_t tile;        /* TCQ: T, weights per tail-biting tile; otherwise 0                  */
    int32_t layout;      /* qp_layout                                                          */
    int64_t row_stride;  /* canonical: bytes between rows of codes, multiple of 16, >= row bytes */
    const void *codes;   /* device, 16-byte aligned                                            */
    const void *lut;     /* device, fp16, 4-byte aligned: SQ 2^code_bits; VQ 2^code_bits*vec; TCQ 2^L*vec; TCQH, TCQHH 2^tlut_bits*vec */
    const void *scales;  /* device, fp16 [M], 2-byte aligned: per-output-channel factor s      */
    int32_t tlut_bits;   /* QP_TCQH, QP_TCQHH: log2 of the small table's entries; otherwise 0  */
    int32_t reserved;    /* 0                                                                  */
} qp_weight;

/* Fused dequantize-and-multiply (Section 3.3 "Kernel implementation"; the fused
 * kernels of Appendix D).  x: device fp16 [B, ldx] (already rotated; this call does
 * not rotate), 16-byte aligned with ldx % 8 == 0, N <= ldx <= QP_MAX_LDX.  y: device fp16
 * [B, ldy], ldy >= M; written for all b < B, j < M, rounded to nearest even from
 * the fp32 value s[j]*acc.  1 <= B <= QP_MAX_BATCH.  Accumulation is fp32; the
 * summation order is unspecified.  workspace: optional device scratch, 256-byte aligned, of
 * at least qp_linear_workspace_bytes(w, B) bytes (0 for most layers and batch sizes): given
 * one, large layers at batch > 4 first copy the activations into the order in which their
 * kernel reads them (one more small launch, the layer itself up to twice as fast at batch
 * 9 - 16).  NULL, too small or misaligned: the activations are read where they are.  Same
 * result, bit for bit, either way; the workspace's contents on exit are unspecified. */
qp_status qp_linear(const qp_weight *w, const void *x, int32_t B, int64_t ldx, void *y, int64_t ldy,
                    void *workspace, size_t workspace_bytes, void *hip_stream);

/* Dequantize only (the dequantization-only kernels of Appendix D): writes the
 * unscaled W^ as fp16 [M, N] row-major, ld = N, to W_out (device, 16-byte aligned).
 * Every element is a bit copy of a LUT entry. */
qp_status qp_dequant(const qp_weight *w, void *W_out, void *hip_stream);

/* Online rotation of activations, X -> X R (Section 3.3 "Reducing rotation
 * overhead"): for each row b < B and each contiguous block of `block` entries,
 *     xr_block = H_block (signs .* x)_block / sqrt(block)
 * with H the Sylvester Hadamard matrix in natural order.  x: device fp16 [B, ldx];
 * signs: device int8 in {-1,+1} [n]; xr: device fp16 [B, ldxr], may alias x
 * exactly (same pointer and ld) but must not overlap it otherwise.  n % block == 0,
 * block a power of two in 2..16384, 1 <= B, B*(n/block) <= 2^31-1.  fp32 butterflies, one rounding to
 * fp16 at the end. */
qp_status qp_hadamard(const void *x, const int8_t *signs, int32_t B, int32_t n, int32_t block,
                      int64_t ldx, void *xr, int64_t ldxr, void *hip_stream);

/* Rotation and fused layer in one call (Section 3.3: with QKV and gate+up fused into one
 * layer each, every online rotation feeds exactly one linear layer).  Same result, bit for
 * bit, as qp_hadamard(x, signs, B, N, block, ...) followed by qp_linear on its output.
 * Two kernels are enqueued, with the rotated activations (fp16) passing through the workspace
 * in whatever order the layer's kernel reads them best (for the native layout: the order of
 * its matrix-core operand fragments, so that its activation loads stay contiguous at every
 * batch size) - or one kernel, at batch 1, where the layer's kernel can rotate the activations
 * itself while its first weights are on the way (the workspace is then not touched): block == N
 * a power of two between 1024 and 8192, or blocks of 1024 in a layer of at most 4096 x 16384 -
 * not the V = 1 trellis; tiny and ragged layers (those the row kernel takes) with N a multiple
 * of 1024 up to 8192 likewise, the V = 1 trellis with blocks of 1024 only.
 * qp_rotate_linear_launches tells which.
 * x: device fp16 [B, ldx], unrotated, 16-byte aligned, ldx % 8 == 0, N <= ldx <= QP_MAX_LDX;
 * signs: device int8 [N], 16-byte aligned.  workspace: device, 256-byte aligned, at least
 * qp_rotate_linear_workspace_bytes(w, B) bytes; contents on entry and exit are unspecified. */
qp_status qp_rotate_linear(const qp_weight *w, const void *x, const int8_t *signs, int32_t block, int32_t B,
                           int64_t ldx, void *y, int64_t ldy, void *workspace, size_t workspace_bytes,
                           void *hip_stream);
size_t qp_rotate_linear_workspace_bytes(const qp_weight *w, int32_t B);
/* How many kernels qp_rotate_linear launches for this layer, batch and block with the options in
 * force: 1 when the layer's kernel rotates the activations itself, else 2 (0 for a NULL descriptor). */
int32_t qp_rotate_linear_launches(const qp_weight *w, int32_t B, int32_t block);

/* A decoder block's rotations and fused layers as one unit (Section 4.2: layers that share an input
 * are what fusion groups; Appendix E.2 measures a block end to end): n items, each one qp_rotate_linear
 * call's arguments, run in order on one stream with no host work between them.  Consecutive items
 * with the same (x, signs, block, B, ldx) and the same N share one rotation where that is cheaper
 * than rotating inside each layer's kernel: q, k, v read one rotated copy, gate and up another.
 * Every y is the same, bit for bit, as the qp_rotate_linear call of its item.
 *   qp_block_enqueue   validates every item, then launches everything (two workspaces' worth of
 *                      room: qp_block_workspace_bytes; device, 256-byte aligned).
 *   qp_block_create    the same sequence captured once into a HIP graph that the library owns;
 *                      qp_block_run replays it with one graph launch, qp_block_destroy frees it.
 *                      The graph holds the pointers of the items and of the workspace as they were
 *                      at creation (the buffers' contents may change between runs, their addresses
 *                      and shapes may not) and the tuning options in force then.  Creation allocates
 *                      host and driver objects (not device memory through this library) and must not
 *                      itself run under stream capture; runs that overlap in time share the workspace
 *                      and race.
 * Errors: those of qp_rotate_linear for the first offending item (nothing is launched then);
 * QP_ERR_SHAPE for n < 1 or n > 4096; QP_ERR_DEVICE when capture or instantiation fails. */
typedef struct qp_block_item {
    const qp_weight *w;
    const void *x;          /* device fp16 [B, ldx], unrotated */
    const int8_t *signs;    /* device int8 [N] */
    int32_t block;
    int32_t B;
    int64_t ldx;
    void *y;                /* device fp16 [B, ldy] */
    int64_t ldy;
} qp_block_item;
typedef struct qp_block qp_block;
size_t qp_block_workspace_bytes(const qp_block_item *items, int32_t n);
qp_status qp_block_enqueue(const qp_block_item *items, int32_t n, void *workspace, size_t workspace_bytes,
                           void *hip_stream);
qp_status qp_block_create(const qp_block_item *items, int32_t n, void *workspace, size_t workspace_bytes,
                          qp_block **out);
qp_status qp_block_run(const qp_block *blk, void *hip_stream);
qp_status qp_block_destroy(qp_block *blk);

/* qp_rotate_linear for callers that cannot allocate device memory or hand in a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * without the workspace, same kernels, same result bit for bit; the rotated activations pass
 * through a fixed array of qp_rotate_linear_static_max_bytes() = 1 MiB of device memory that
 * belongs to the library (one per GPU, held until the process ends).  Nothing is allocated or
 * freed, here or in any routine this calls.  Layers with qp_rotate_linear_workspace_bytes(w, B)
 * above that size (N > 32768 at batch 16) are refused with QP_ERR_WORKSPACE; QP_ERR_DEVICE if the
 * array's address cannot be obtained on the current device.  All calls on one GPU share the
 * array: calls that overlap in time on one GPU (two streams, two threads) race on it and must be
 * serialised by the caller; calls that follow each other on one stream are safe. */
qp_status qp_rotate_linear_static(const qp_weight *w, const void *x, const int8_t *signs, int32_t block,
                                  int32_t B, int64_t ldx, void *y, int64_t ldy, void *hip_stream);
size_t qp_rotate_linear_static_max_bytes(void);

/* One-time conversion canonical -> native.  `canonical` describes device codes in
 * canonical layout; native_codes is a device buffer of `bytes` >=
 * qp_native_bytes(canonical) bytes, 16-byte aligned, not overlapping the source.
 * On success *native_out is a copy of the descriptor with layout, codes and
 * row_stride (0) updated; lut and scales are shared with the source. */
qp_status qp_repack(const qp_weight *canonical, qp_weight *native_out, void *native_codes, size_t bytes,
                    void *hip_stream);

/* Quantization: targets -> packed codes, canonical layout (App. C.1 / C.2 / C.3.1 / C.3.2
 * "Quantization"): the nearest table entry per weight (QP_SQ) or per pair (QP_VQ); for the trellis
 * schemes, per 256-weight tile, the bitstream whose decode is closest to the targets, found with
 * the Viterbi algorithm over the 2^16 states, the tail-biting condition met in two passes (an open
 * pass over the tile rotated by half its length fixes the 16 - s bits that both ends of the stream
 * share; a second pass constrained to them gives the stream: optimal for those bits).  Half-TCQ
 * encodes its two halves with their own bitwidths.
 * w: scheme, shape, code_bits, vec, window_bits, tile, tlut_bits, lut (device, 16-byte aligned) and
 * row_stride describe the result, layout must be canonical; codes and scales are not read.
 * Supported: every layer that qp_linear supports; N % 16 == 0.  W: device fp16 [M, ldw], the
 * weights as they should decode (rotated and divided by the per-row scale by the caller),
 * 16-byte aligned, ldw % 8 == 0.  codes_out: device,
 * 16-byte aligned, M * row_stride bytes; only the row's code bytes are written.  tile_err:
 * optional device fp32 [M, N/256], the squared error of every tile (trellis schemes only; fp32
 * accumulation).  workspace (trellis schemes): device, 16-byte aligned; any size from one
 * workgroup's share, qp_encode_workspace_bytes(w) / min(256, tiles), upwards is accepted and decides
 * how many tiles are encoded at once.  Distances are computed in fp32 from the exact fp16 inputs;
 * ties go to the lower index. */
qp_status qp_encode(const qp_weight *w, const void *W, int64_t ldw, void *codes_out, float *tile_err,
                    void *workspace, size_t workspace_bytes, void *hip_stream);
/* Workspace that lets qp_encode use the whole chip (0 for QP_SQ / QP_VQ and for bad descriptors). */
size_t qp_encode_workspace_bytes(const qp_weight *w);

/* Per-output-channel scale of a (rotated) weight matrix (Section 3.3): for every row j of W,
 * device fp16 [M, ldw], s[j] = sqrt(mean_i W[j,i]^2) rounded to fp16 (1 for a row of zeros) is
 * written to scales (device fp16 [M]) and the row is divided by it in place (fp32 arithmetic,
 * one rounding to fp16), so that what is left is close to N(0,1) and ready for qp_encode.
 * The whole offline path of a layer with weights W [M, N] is then
 *   qp_hadamard(W, signs, M, N, block, ...)   rows of W rotated like the activations will be
 *   qp_row_normalize(...)                      s and W / s
 *   qp_encode(...), qp_repack(...)
 * after which qp_rotate_linear(x) = s (x R)(W R / s)^T approximates x W^T.
 * W 16-byte aligned, N % 8 == 0, ldw % 8 == 0, ldw >= N. */
qp_status qp_row_normalize(void *W, int64_t ldw, int32_t M, int32_t N, void *scales, void *hip_stream);

/* Code book construction by Lloyd's algorithm (App. C.1 / C.2 / C.3.1 "Codebook construction":
 * k-means of standard Gaussian samples; k = 2^b scalar levels, k = 2^(2b) 2-D points, or the
 * 2^tlut_bits pairs of the trellis quantizer's small table).  samples: device fp32 [n, d], d = 1
 * or 2, 4 d -byte aligned; centres: device fp32 [k, d], on entry the start (the caller's choice:
 * the paper does not fix it), on return the result; 1 <= k <= 4096.  Each iteration assigns every
 * sample to its nearest centre (fp32 distances, d = fma(dy, dy, dx dx); ties go to the lower index)
 * and moves every centre to the mean of its samples (fp32 partial sums per workgroup, added in a
 * fixed order in fp64; a centre without samples stays); the run ends with the update whose total
 * squared movement is <= tol, at the latest after max_iter (>= 1) updates.  All iterations are
 * enqueued at once; no host synchronisation.  Optional outputs (device, may be NULL): assign_out
 * int32 [n], the cluster of every sample at the last assignment step; centres_f16 fp16 [k, d],
 * the centres rounded to nearest even (the table format of qp_weight.lut); stats_out double [3]:
 * inertia of the last assignment step (sum of squared distances), updates made, movement of the
 * last update.  workspace: device, 16-byte aligned, qp_kmeans_workspace_bytes(k, d) bytes. */
qp_status qp_kmeans(const void *samples, int64_t n, int32_t d, void *centres, int32_t k, int32_t max_iter,
                    float tol, void *workspace, size_t workspace_bytes, int32_t *assign_out, void *centres_f16,
                    double *stats_out, void *hip_stream);
size_t qp_kmeans_workspace_bytes(int32_t k, int32_t d);   /* 0 for unsupported k, d */

/* Bytes of the native code buffer for this layer, 0 if it has no native form. */
size_t qp_native_bytes(const qp_weight *canonical);

/* Bytes of the optional workspace with which qp_linear runs (w, B) fastest: room for a copy of the
 * activations in the order the layer's kernel reads them (see qp_linear), a multiple of 256;
 * 0 where no copy is made (most layers at batch <= 4, small layers, bad arguments). */
size_t qp_linear_workspace_bytes(const qp_weight *w, int32_t B);

/* Process-wide tuning options (Appendix E.2 profiles every kernel on its own: these switches say
 * which of the library's kernels that is).  They exist for tests, which must reach every kernel
 * with layers of any size, and for measurements; the defaults are the measured best choices.
 * Plain integers read on the host when a call is dispatched - no environment variable is read and
 * a call costs nothing for them.  Set them while no other thread is inside the library;
 * qp_linear_workspace_bytes / qp_linear (and the rotate pair) must see the same values.
 *   QP_OPT_LINEAR_KERNEL   0 by shape (default), 1 one wavefront per row, 2 the 16 x 1024 block kernel
 *                          wherever the layer consists of whole blocks
 *   QP_OPT_DEQUANT_KERNEL  0 by shape, 1 layout-agnostic kernel, 2 block kernel (native layout)
 *   QP_OPT_ROTATE_SPLIT    1: qp_rotate_linear never rotates inside the layer's kernel
 *   QP_OPT_LINEAR_PACK     -1 by shape, 0 qp_linear never asks for a workspace, 1 always (block kernel)
 *   QP_OPT_LINEAR_SPLIT    -1 by shape, 0 / 1 the alternative form of the block kernel off / on where
 *                          it exists (two wavefronts per unit for the trellis schemes at batch <= 2:
 *                          only on request; for 5-bit VQ the sixteen-copy table of code pairs at
 *                          batch <= 2 and the per-wavefront table at batch 3 - 4: by shape)
 *   QP_OPT_WG_PER_CU       workgroups per compute unit of the block kernel (SQ / VQ; default 1)
 *   QP_OPT_NW              0 by shape, 4..16 wavefronts per workgroup of the block kernel (SQ / VQ)
 *   QP_OPT_TABLE_LATE_MAX  -1 by shape; units per workgroup up to which a shared table is built
 *                          after the first loads
 * qp_set_option: QP_ERR_UNSUPPORTED for an unknown option, QP_ERR_SHAPE for a value outside its
 * range; qp_get_option returns the current value (INT32_MIN for an unknown option);
 * qp_reset_options restores every default. */
typedef enum {
    QP_OPT_LINEAR_KERNEL = 0,
    QP_OPT_DEQUANT_KERNEL = 1,
    QP_OPT_ROTATE_SPLIT = 2,
    QP_OPT_LINEAR_PACK = 3,
    QP_OPT_LINEAR_SPLIT = 4,
    QP_OPT_WG_PER_CU = 5,
    QP_OPT_NW = 6,
    QP_OPT_TABLE_LATE_MAX = 7,
    QP_OPT_COUNT = 8
} qp_option;
qp_status qp_set_option(int32_t option, int32_t value);
int32_t qp_get_option(int32_t option);
void qp_reset_options(void);

/* Check a descriptor alone (what qp_linear / qp_dequant check first). */
qp_status qp_validate(const qp_weight *w);

/* Mixed-scheme selection on the host (Section 4.1 eq. (3) and the fusion-aware form, Section 4.2
 * eq. (4) with (C1), (C2)): n_classes classes, class c owning the options begin[c] .. begin[c+1]-1
 * (begin[0] = 0), option o with loss term loss[o] and profiled cost cost[o] >= 0 (latency or
 * memory).  Exactly one option per class is chosen so that the summed cost stays within budget
 * and the summed loss is least; choice[c] receives the option's index inside its class.  For the
 * fusion-aware problem a class is a cluster of layers sharing their input and an option a split
 * into fused groups with a quantizer per group (its loss: the sum over its layers; its cost: the
 * sum over its groups), which makes (C1) hold by construction.
 * Method: dynamic programming over the cost axis cut into `resolution` cells of budget/resolution;
 * costs are rounded up to whole cells (a cost that is a whole number of cells up to the rounding
 * of one floating-point multiplication counts as that number), so the result satisfies the true
 * budget up to that rounding - summed cost <= budget (1 + n_classes 2^-52) - and is optimal among
 * the selections whose rounded costs fit: exactly optimal when all costs are multiples of the
 * cell, otherwise no worse than the optimum for the budget reduced by n_classes cells.  Ties go to
 * the lower option index.  All pointers are host pointers; total_loss / total_cost (optional)
 * receive the sums of the true values.  QP_ERR_UNSUPPORTED: no selection fits; QP_ERR_MEMORY: the
 * tables (n_classes x (resolution + 1) cells) do not fit the host's memory.  1 <= resolution <= 2^22. */
qp_status qp_msq_solve(int32_t n_classes, const int32_t *begin, const double *loss, const double *cost,
                       double budget, int32_t resolution, int32_t *choice, double *total_loss,
                       double *total_cost);

/* The fusion-aware problem of Section 4.2, eq. (4), stated directly: n_blocks Transformer blocks of
 * seven linear layers each, in the order q, k, v, o, u (up), g (gate), d (down); the twelve fusible
 * groups of a block in the order {q} {k} {v} {q,k} {q,v} {k,v} {q,k,v} {o} {u} {g} {u,g} {d};
 * n_quant quantizers.  loss: host double [n_blocks][7][n_quant], the loss term of a layer under a
 * quantizer; cost: host double [n_blocks][12][n_quant], the profiled cost of a (fused) group under
 * a quantizer, >= 0.  Finds binary P[g, q] with every layer in exactly one active group (C1) and
 * the summed cost of the active groups within budget (C2) that minimises the summed loss terms of
 * the layers of the active groups: assign (host int32 [n_blocks][12]) receives the quantizer of
 * every active group and -1 for the others.  fusion == 0 restricts the groups to single layers
 * (the per-layer problem of Section 4.1, eq. (3)).  Method: every cluster of layers with a common
 * input ({q,k,v}, {o}, {u,g}, {d}) becomes a class of qp_msq_solve whose options are its splits into
 * groups with one quantizer per group, options that another one beats in both loss and cost
 * dropped; same guarantees, same error codes.  1 <= n_blocks <= 4096, 1 <= n_quant <= 16. */
qp_status qp_msq_solve_fused(int32_t n_blocks, int32_t n_quant, const double *loss, const double *cost,
                             double budget, int32_t resolution, int32_t fusion, int32_t *assign,
                             double *total_loss, double *total_cost);

/* Measurement aids, no part of the method (Appendix E.2 profiles each kernel alone; these give the
 * two yardsticks for such a profile on the machine at hand).  qp_bench_stream_read enqueues a kernel
 * that does nothing but read `bytes` bytes at `data` (device, 16-byte aligned, bytes a multiple of
 * 16) once, with 128-bit non-temporal loads, one contiguous KiB per wavefront and instruction, 256
 * workgroups: the time no kernel that has to read that many bytes of packed codes can beat.
 * sink: 4 bytes of device scratch (4-byte aligned).  qp_bench_empty_launch enqueues an empty kernel of
 * 256 workgroups x 1024 threads: the cost of a launch as such. */
qp_status qp_bench_stream_read(const void *data, size_t bytes, void *sink, void *hip_stream);
qp_status qp_bench_empty_launch(void *hip_stream);

const char *qp_status_string(qp_status s);
int32_t qp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* QP_H */
