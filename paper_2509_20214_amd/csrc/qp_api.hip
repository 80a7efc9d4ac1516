// C ABI: host-side validation and dispatch.  No device memory is allocated here and
// no call synchronises with the device.
#include <atomic>
#include <climits>
#include <cstring>
#include <new>

#include "qp_internal.h"

#define QP_VERSION 210

// ------------------------------------------------------------------ tuning options
// Plain process-wide integers (relaxed atomics: a read is an ordinary load); nothing here or
// elsewhere in the library reads the environment.
struct QpOptSpec { int32_t def, lo, hi; };
static const QpOptSpec kOptSpec[QP_OPT_COUNT] = {
    {0, 0, 2},       // QP_OPT_LINEAR_KERNEL
    {0, 0, 2},       // QP_OPT_DEQUANT_KERNEL
    {0, 0, 1},       // QP_OPT_ROTATE_SPLIT
    {-1, -1, 1},     // QP_OPT_LINEAR_PACK
    {-1, -1, 1},     // QP_OPT_LINEAR_SPLIT
    {1, 1, 4},       // QP_OPT_WG_PER_CU
    {0, 0, 16},      // QP_OPT_NW
    {-1, -1, 4096},  // QP_OPT_TABLE_LATE_MAX
};
static std::atomic<int32_t> g_opt[QP_OPT_COUNT] = {{0}, {0}, {0}, {-1}, {-1}, {1}, {0}, {-1}};

int32_t qp_opt(int option) { return g_opt[option].load(std::memory_order_relaxed); }

extern "C" qp_status qp_set_option(int32_t option, int32_t value) {
    if (option < 0 || option >= QP_OPT_COUNT) return QP_ERR_UNSUPPORTED;
    if (value < kOptSpec[option].lo || value > kOptSpec[option].hi) return QP_ERR_SHAPE;
    if (option == QP_OPT_NW && value != 0 && value < 4) return QP_ERR_SHAPE;
    g_opt[option].store(value, std::memory_order_relaxed);
    return QP_OK;
}

extern "C" int32_t qp_get_option(int32_t option) {
    if (option < 0 || option >= QP_OPT_COUNT) return INT32_MIN;
    return qp_opt(option);
}

extern "C" void qp_reset_options(void) {
    for (int o = 0; o < QP_OPT_COUNT; ++o) g_opt[o].store(kOptSpec[o].def, std::memory_order_relaxed);
}

static inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

static qp_status scheme_supported(const qp_weight *w) {
    switch (w->scheme) {
        case QP_SQ:
            return (w->vec == 1 && w->code_bits == 4) ? QP_OK : QP_ERR_UNSUPPORTED;
        case QP_VQ:
            return (w->vec == 2 && (w->code_bits == 5 || w->code_bits == 7)) ? QP_OK : QP_ERR_UNSUPPORTED;
        case QP_TCQ:
            return (w->vec == 1 && w->window_bits == 16 && w->tile == 256 && w->code_bits >= 2 &&
                    w->code_bits <= 4)
                       ? QP_OK
                       : QP_ERR_UNSUPPORTED;
        case QP_TCQH:
            // table size follows the bitwidth as in the paper: 2^9 pairs up to 4 bits, 2^10 at 4.5, 2^11 at 5
            return (w->vec == 2 && w->window_bits == 16 && w->tile == 256 && w->code_bits >= 3 &&
                    w->code_bits <= 10 &&
                    w->tlut_bits == (w->code_bits <= 8 ? 9 : w->code_bits == 9 ? 10 : 11))
                       ? QP_OK
                       : QP_ERR_UNSUPPORTED;
        case QP_TCQHH: {
            // s on the first half of the input channels, s + 1 on the second; the table of s + 1
            const int top = w->code_bits + 1;
            return (w->vec == 2 && w->window_bits == 16 && w->tile == 256 && w->code_bits >= 3 &&
                    w->code_bits <= 9 && w->tlut_bits == (top <= 8 ? 9 : top == 9 ? 10 : 11))
                       ? QP_OK
                       : QP_ERR_UNSUPPORTED;
        }
        default:
            return QP_ERR_UNSUPPORTED;
    }
}

static inline int64_t row_bytes(const qp_weight *w) {
    if (w->scheme == QP_TCQHH) return (int64_t)w->N / 4 * (2 * w->code_bits + 1) / 8;
    return ((int64_t)w->N / w->vec * w->code_bits + 7) / 8;   // a row of 5- or 7-bit codes may end inside a byte
}
static inline int span_bytes(const qp_weight *w) { return 32 * w->code_bits / w->vec; }

extern "C" qp_status qp_validate(const qp_weight *w) {
    if (!w) return QP_ERR_NULL;
    qp_status s = scheme_supported(w);
    if (s != QP_OK) return s;
    if (w->M <= 0 || w->N <= 0) return QP_ERR_SHAPE;
    if (w->N % 8 != 0) return QP_ERR_SHAPE;
    if ((w->scheme == QP_TCQ || w->scheme == QP_TCQH) && w->N % w->tile != 0) return QP_ERR_SHAPE;
    if (w->scheme == QP_TCQHH && w->N % (2 * w->tile) != 0) return QP_ERR_SHAPE;
    if (!w->codes || !w->lut || !w->scales) return QP_ERR_NULL;
    if (w->layout == QP_LAYOUT_CANONICAL) {
        if (w->row_stride % 16 != 0) return QP_ERR_ALIGN;
        if (w->row_stride < row_bytes(w)) return QP_ERR_SHAPE;
        if ((int64_t)w->row_stride * w->M > ((int64_t)1 << 40)) return QP_ERR_SHAPE;
    } else if (w->layout == QP_LAYOUT_NATIVE) {
        // whole 16 x 256 spans; a last column block of fewer than 1024 columns is padded with zero bytes
        if (w->M % 16 != 0 || w->N % 256 != 0) return QP_ERR_LAYOUT;
        if (w->scheme == QP_TCQHH && w->N % 2048 != 0) return QP_ERR_LAYOUT;
    } else {
        return QP_ERR_LAYOUT;
    }
    if (!aligned(w->codes, 16) || !aligned(w->lut, 4) || !aligned(w->scales, 2)) return QP_ERR_ALIGN;
    return QP_OK;
}

static QpW make_dev(const qp_weight *w) {
    QpW d;
    d.codes = static_cast<const uint8_t *>(w->codes);
    d.lut = static_cast<const uint16_t *>(w->lut);
    d.scales = static_cast<const uint16_t *>(w->scales);
    d.M = w->M;
    d.N = w->N;
    d.row_stride = w->row_stride;
    d.layout = w->layout;
    d.nbc = (w->N + 1023) / 1024;
    d.tlut_bits = w->tlut_bits;
    return d;
}

// Which kernel runs a layer.  QP_OPT_LINEAR_KERNEL = 1 / 2 forces the row / the block kernel (used
// by the tests to cover both on weights of any size); 0 lets shape, scheme and batch decide.
// The block kernel needs whole 16 x 1024 blocks; everything else goes to the row kernel.  Below one
// block per compute unit the row kernel still wins where a row is short and the batch is small
// (us per call, row / block kernel): 4 bit scalar 1024x1024 batch 1 3.15 / 3.45, batch 2 3.9 / 3.5,
// batch 8 7.5 / 3.6; pairs at 2.5 bits 256x1024 3.3 / 3.6 but 1024x2048 5.0 / 3.7 and 256x4096
// 7.5 / 3.7; the V = 1 trellis, whose block kernel first stages a 128 KiB table, 1024x1024 at 3 bits
// batch 1 / 2 / 4 4.7 / 5.5 / 6.5 against 6.2 / 6.25 / 6.6 and 1024x2048 batch 1 5.9 / 6.6, batch 2
// 7.55 / 6.6; the V = 2 trellis never (1024x1024 at 3 bits 6.3 / 4.4, 1024x3072 14.1 / 4.7).
static bool use_rowwave(const qp_weight *w, int B) {
    const int nbc = (w->N + 1023) / 1024;
    const int force = qp_opt(QP_OPT_LINEAR_KERNEL);
    const int64_t blocks = (int64_t)(w->M / 16) * nbc;
    // the block kernel reads whole blocks from either layout (in the canonical one a lane's pieces
    // are consecutive in its row instead of one KiB per piece); the last column block may stop
    // after one, two or three of its four spans of 256 columns (N = 11008, 13824 ...)
    const bool fits = w->M % 16 == 0 && w->N % 256 == 0 && nbc <= 32 &&
                      !(w->scheme == QP_TCQHH && w->N % 2048 != 0);
    if (!fits || force == 1) return true;
    if (force == 2 || blocks >= 256) return false;
    if (w->scheme == QP_SQ || w->scheme == QP_VQ) return nbc == 1 && B == 1;
    if (w->scheme == QP_TCQ) return (nbc == 1 && B <= 4) || (nbc == 2 && B == 1);
    return false;
}

static inline int pow2_at_least(int B) { return B <= 1 ? 1 : B <= 2 ? 2 : B <= 4 ? 4 : B <= 8 ? 8 : 16; }

static inline size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }
// columns of the activations in fragment order: whole blocks of 1024
static inline size_t padded_cols(const qp_weight *w) { return ((size_t)w->N + 1023) / 1024 * 1024; }

// Whether qp_linear first copies the activations into the fragment order of the matrix-core
// kernel (one more small launch; every activation load of the layer is then a contiguous KiB
// instead of 16 - 64 byte pieces of 8 - 16 rows).  Measured, layer alone, row-major / copied:
// batch 16 VQ 5 bit 57344x8192 130 / 67 us, 4096x14336 23.6 / 13.1 us, TCQ 3 bit 4096x14336
// 29 / 22 us; batch 9 VQ 7 bit 8192x28672 55 / 41 us, but 4096x4096 6.3 / 8.1 us; batch 8 VQ 7 bit
// 8192x28672 38 / 31 us, SQ 57344x8192 62 / 52 us, but VQ 7 bit 10240x8192 14.6 / 16 us and the
// V = 1 trellis (bound by its table lookups) never at batch <= 8.  At batch 1 - 4 the largest
// layers seem to gain 4 - 10 % as well, but a plain copy of x in front of the unchanged kernel
// gains the same: launches of large kernels back to back cost more than the same launches with
// any small kernel between them - an effect of the launch sequence, not of the layout.
static bool pack_pays(const qp_weight *w, int B) {
    if (use_rowwave(w, B)) return false;
    if (const int force = qp_opt(QP_OPT_LINEAR_PACK); force >= 0) return force == 1;   // always / never
    const int64_t weights = (int64_t)w->M * w->N;
    if (B > 8) return weights >= ((int64_t)1 << 25);
    if (B > 4) return w->scheme != QP_TCQ && weights >= ((int64_t)1 << 27);
    return false;
}

extern "C" size_t qp_linear_workspace_bytes(const qp_weight *w, int32_t B) {
    if (!w || B < 1 || B > QP_MAX_BATCH || w->N <= 0 || w->M <= 0) return 0;
    return pack_pays(w, B) ? round256((size_t)pow2_at_least(B) * padded_cols(w) * 2) : 0;
}

extern "C" qp_status qp_linear(const qp_weight *w, const void *x, int32_t B, int64_t ldx, void *y, int64_t ldy,
                               void *workspace, size_t workspace_bytes, void *hip_stream) {
    qp_status s = qp_validate(w);
    if (s != QP_OK) return s;
    if (!x || !y) return QP_ERR_NULL;
    if (B < 1 || B > QP_MAX_BATCH) return QP_ERR_SHAPE;
    if (ldx < w->N || ldx > QP_MAX_LDX || ldy < w->M || ldx % 8 != 0) return QP_ERR_SHAPE;
    if (!aligned(x, 16) || !aligned(y, 2)) return QP_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    QpW d = make_dev(w);
    if (use_rowwave(w, B)) return qp_launch_linear_rowwave(d, w->scheme, w->code_bits, x, B, ldx, y, ldy, st);
    // The workspace is optional: without one (or with one that is too small or not 256-byte
    // aligned) the layer reads the activations where they are - same result, bit for bit.
    const size_t need = qp_linear_workspace_bytes(w, B);
    if (need && workspace && workspace_bytes >= need && aligned(workspace, 256)) {
        s = qp_launch_pack_x(x, B, w->N, ldx, workspace, pow2_at_least(B), st);
        if (s != QP_OK) return s;
        return qp_launch_linear_mfma(d, w->scheme, w->code_bits, workspace, B, w->N, y, ldy, 1, nullptr, 0, st);
    }
    return qp_launch_linear_mfma(d, w->scheme, w->code_bits, x, B, ldx, y, ldy, 0, nullptr, 0, st);
}

extern "C" size_t qp_rotate_linear_workspace_bytes(const qp_weight *w, int32_t B) {
    if (!w || B < 1 || B > QP_MAX_BATCH || w->N <= 0) return 0;
    return round256((size_t)pow2_at_least(B) * padded_cols(w) * 2);
}

// Whether qp_rotate_linear would rotate inside the layer's kernel (one launch).
static bool rotates_in_kernel(const qp_weight *w, int B, int block) {
    if (B != 1 || qp_opt(QP_OPT_ROTATE_SPLIT)) return false;
    if (use_rowwave(w, B)) return qp_rowwave_rotates(w->scheme, w->code_bits, w->N, block);
    if (block == w->N) return block >= 1024 && block <= 8192 && w->scheme != QP_TCQ;
    return qp_linear_rotates_blocks(w->scheme, w->M, w->N, block);
}

extern "C" int32_t qp_rotate_linear_launches(const qp_weight *w, int32_t B, int32_t block) {
    if (!w) return 0;
    return rotates_in_kernel(w, B, block) ? 1 : 2;
}

extern "C" qp_status qp_rotate_linear(const qp_weight *w, const void *x, const int8_t *signs, int32_t block,
                                      int32_t B, int64_t ldx, void *y, int64_t ldy, void *workspace,
                                      size_t workspace_bytes, void *hip_stream) {
    qp_status s = qp_validate(w);
    if (s != QP_OK) return s;
    if (!x || !signs || !y || !workspace) return QP_ERR_NULL;
    if (B < 1 || B > QP_MAX_BATCH) return QP_ERR_SHAPE;
    if (ldx < w->N || ldx > QP_MAX_LDX || ldy < w->M || ldx % 8 != 0) return QP_ERR_SHAPE;
    if (block < 2 || block > 16384 || (block & (block - 1)) != 0 || w->N % block != 0) return QP_ERR_SHAPE;
    if (!aligned(x, 16) || !aligned(y, 2) || !aligned(workspace, 256) || !aligned(signs, 16)) return QP_ERR_ALIGN;
    if (workspace_bytes < qp_rotate_linear_workspace_bytes(w, B)) return QP_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    QpW d = make_dev(w);
    // Two launches; the rotated activations pass through the workspace.  For the block kernel
    // the rotation writes them in the order that kernel loads its B-operand fragments, so that
    // every one of its activation loads is a contiguous KiB whatever the batch; the results
    // are the same bit for bit (same values, same order of operations, other addresses).
    if (use_rowwave(w, B)) {
        // a tiny layer at batch 1: the row kernel rotates the activations itself where it can
        if (rotates_in_kernel(w, B, block))
            return qp_launch_linear_rowwave_rot(d, w->scheme, w->code_bits, x, signs, block, y, st);
        s = qp_launch_hadamard(x, signs, B, w->N, block, ldx, workspace, w->N, 0, st);
        if (s != QP_OK) return s;
        return qp_launch_linear_rowwave(d, w->scheme, w->code_bits, workspace, B, w->N, y, ldy, st);
    }
    // Batch 1 and either one rotation block (N a power of two up to 8192) or several blocks of 1024 in a
    // layer of at most 4096 x 16384 (N = 14336 ...): the layer's kernel rotates the activations itself
    // while its first weights are on their way - every workgroup repeats the small transform, and the
    // second launch is saved.  Not the V = 1 trellis (beside its 128 KiB table the transform has no room
    // of its own in LDS).  QP_OPT_ROTATE_SPLIT forces two launches.
    if (rotates_in_kernel(w, B, block))
        return qp_launch_linear_mfma(d, w->scheme, w->code_bits, x, 1, ldx, y, ldy, 0, signs, block, st);
    s = qp_launch_hadamard(x, signs, B, w->N, block, ldx, workspace, w->N, pow2_at_least(B), st);
    if (s != QP_OK) return s;
    return qp_launch_linear_mfma(d, w->scheme, w->code_bits, workspace, B, w->N, y, ldy, 1, nullptr, 0, st);
}

// ------------------------------------------------------------------ a decoder block as one unit
static qp_status block_item_check(const qp_block_item &it) {
    if (!it.w) return QP_ERR_NULL;
    qp_status s = qp_validate(it.w);
    if (s != QP_OK) return s;
    if (!it.x || !it.signs || !it.y) return QP_ERR_NULL;
    if (it.B < 1 || it.B > QP_MAX_BATCH) return QP_ERR_SHAPE;
    if (it.ldx < it.w->N || it.ldx > QP_MAX_LDX || it.ldy < it.w->M || it.ldx % 8 != 0) return QP_ERR_SHAPE;
    if (it.block < 2 || it.block > 16384 || (it.block & (it.block - 1)) != 0 || it.w->N % it.block != 0) return QP_ERR_SHAPE;
    if (!aligned(it.x, 16) || !aligned(it.y, 2) || !aligned(it.signs, 16)) return QP_ERR_ALIGN;
    return QP_OK;
}

static bool block_same_input(const qp_block_item &a, const qp_block_item &b) {
    return a.x == b.x && a.signs == b.signs && a.block == b.block && a.B == b.B && a.ldx == b.ldx && a.w->N == b.w->N;
}

extern "C" size_t qp_block_workspace_bytes(const qp_block_item *items, int32_t n) {
    if (!items || n < 1) return 0;
    size_t need = 0;
    for (int i = 0; i < n; ++i) {
        if (!items[i].w) return 0;
        const size_t one = qp_rotate_linear_workspace_bytes(items[i].w, items[i].B);
        if (one > need) need = one;
    }
    return 2 * need;   // a shared rotation may be needed in fragment order and row-major at once
}

extern "C" qp_status qp_block_enqueue(const qp_block_item *items, int32_t n, void *workspace, size_t workspace_bytes,
                                      void *hip_stream) {
    if (!items || !workspace) return QP_ERR_NULL;
    if (n < 1 || n > 4096) return QP_ERR_SHAPE;
    for (int i = 0; i < n; ++i) {
        const qp_status s = block_item_check(items[i]);
        if (s != QP_OK) return s;
    }
    if (!aligned(workspace, 256)) return QP_ERR_ALIGN;
    const size_t need = qp_block_workspace_bytes(items, n);
    if (workspace_bytes < need) return QP_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    void *ws_packed = workspace, *ws_rows = static_cast<char *>(workspace) + need / 2;
    for (int i = 0; i < n;) {
        int j = i + 1;
        while (j < n && block_same_input(items[i], items[j])) ++j;
        const qp_block_item &a = items[i];
        // One rotation for the whole group costs a launch of its own (about 2 us); rotating inside every
        // layer's kernel costs each of them about 1 us where that form exists (batch 1), and a launch
        // each where it does not.
        bool all_in_kernel = true;
        for (int k = i; k < j; ++k) all_in_kernel = all_in_kernel && rotates_in_kernel(items[k].w, a.B, a.block);
        const bool share = (j - i >= 2) && (!all_in_kernel || j - i >= 3);
        if (!share) {
            for (int k = i; k < j; ++k) {
                const qp_block_item &it = items[k];
                const qp_status s = qp_rotate_linear(it.w, it.x, it.signs, it.block, it.B, it.ldx, it.y, it.ldy, workspace,
                                                     workspace_bytes, hip_stream);
                if (s != QP_OK) return s;
            }
        } else {
            bool any_rows = false, any_blocks = false;
            for (int k = i; k < j; ++k) (use_rowwave(items[k].w, a.B) ? any_rows : any_blocks) = true;
            const int N = a.w->N;
            qp_status s = QP_OK;
            if (any_blocks) s = qp_launch_hadamard(a.x, a.signs, a.B, N, a.block, a.ldx, ws_packed, N, pow2_at_least(a.B), st);
            if (s == QP_OK && any_rows) s = qp_launch_hadamard(a.x, a.signs, a.B, N, a.block, a.ldx, ws_rows, N, 0, st);
            for (int k = i; k < j && s == QP_OK; ++k) {
                const qp_block_item &it = items[k];
                const QpW d = make_dev(it.w);
                if (use_rowwave(it.w, it.B)) s = qp_launch_linear_rowwave(d, it.w->scheme, it.w->code_bits, ws_rows, it.B, N, it.y, it.ldy, st);
                else s = qp_launch_linear_mfma(d, it.w->scheme, it.w->code_bits, ws_packed, it.B, N, it.y, it.ldy, 1, nullptr, 0, st);
            }
            if (s != QP_OK) return s;
        }
        i = j;
    }
    return QP_OK;
}

struct qp_block {
    hipGraphExec_t exec;
};

extern "C" qp_status qp_block_create(const qp_block_item *items, int32_t n, void *workspace, size_t workspace_bytes,
                                     qp_block **out) {
    if (!out) return QP_ERR_NULL;
    *out = nullptr;
    if (!items || !workspace) return QP_ERR_NULL;
    if (n < 1 || n > 4096) return QP_ERR_SHAPE;
    for (int i = 0; i < n; ++i) {   // refuse before anything is created
        const qp_status s = block_item_check(items[i]);
        if (s != QP_OK) return s;
    }
    if (!aligned(workspace, 256)) return QP_ERR_ALIGN;
    if (workspace_bytes < qp_block_workspace_bytes(items, n)) return QP_ERR_WORKSPACE;
    hipStream_t cs = nullptr;
    if (hipStreamCreateWithFlags(&cs, hipStreamNonBlocking) != hipSuccess) return QP_ERR_DEVICE;
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    qp_status s = QP_ERR_DEVICE;
    if (hipStreamBeginCapture(cs, hipStreamCaptureModeThreadLocal) == hipSuccess) {
        s = qp_block_enqueue(items, n, workspace, workspace_bytes, cs);
        const hipError_t e = hipStreamEndCapture(cs, &graph);   // always ends the capture, also after an error
        if (s == QP_OK && (e != hipSuccess || !graph)) s = QP_ERR_DEVICE;
        if (s == QP_OK && hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0) != hipSuccess) s = QP_ERR_DEVICE;
    }
    if (graph) (void)hipGraphDestroy(graph);
    (void)hipStreamDestroy(cs);
    if (s != QP_OK) {
        (void)hipGetLastError();
        return s;
    }
    qp_block *b = new (std::nothrow) qp_block{exec};
    if (!b) {
        (void)hipGraphExecDestroy(exec);
        return QP_ERR_MEMORY;
    }
    *out = b;
    return QP_OK;
}

extern "C" qp_status qp_block_run(const qp_block *blk, void *hip_stream) {
    if (!blk) return QP_ERR_NULL;
    return hipGraphLaunch(blk->exec, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? QP_OK : QP_ERR_DEVICE;
}

extern "C" qp_status qp_block_destroy(qp_block *blk) {
    if (!blk) return QP_ERR_NULL;
    const hipError_t e = hipGraphExecDestroy(blk->exec);
    delete blk;
    return e == hipSuccess ? QP_OK : QP_ERR_DEVICE;
}

// ------------------------------------------------------------------ the entry point that allocates nothing
// qp_rotate_linear for callers that cannot allocate: the rotated activations pass through this fixed
// array instead of a caller's workspace.  One copy per GPU, there until the process ends.  The array's
// name is only a handle on the host; its device address is looked up once per device.
#define QP_STATIC_SCRATCH_BYTES ((size_t)QP_MAX_BATCH * 32 * 1024 * 2)   // batch 16 x N = 32768 fp16
#define QP_MAX_DEVICES 64
static __device__ __align__(256) unsigned char scratch[QP_STATIC_SCRATCH_BYTES];
static std::atomic<void *> g_scratch_ptr[QP_MAX_DEVICES];

// Device address of `scratch` on the current device; nullptr when it cannot be had.
static void *scratch_address() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= QP_MAX_DEVICES) return nullptr;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
        (void)hipGetLastError();
        return nullptr;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // (two threads racing here store the same address)
    return p;
}

extern "C" size_t qp_rotate_linear_static_max_bytes(void) { return QP_STATIC_SCRATCH_BYTES; }

extern "C" qp_status qp_rotate_linear_static(const qp_weight *w, const void *x, const int8_t *signs, int32_t block,
                                             int32_t B, int64_t ldx, void *y, int64_t ldy, void *hip_stream) {
    qp_status s = qp_validate(w);
    if (s != QP_OK) return s;
    if (B < 1 || B > QP_MAX_BATCH) return QP_ERR_SHAPE;
    const size_t need = qp_rotate_linear_workspace_bytes(w, B);
    if (need == 0 || need > QP_STATIC_SCRATCH_BYTES) return QP_ERR_WORKSPACE;   // layer too wide for the fixed array
    void *ws = scratch_address();
    if (!ws) return QP_ERR_DEVICE;
    // Nothing has to be cleared between calls: the rotation writes the B batch rows that the layer's
    // results depend on; what the layer reads of the padding rows (B rounded up to a power of two) is
    // whatever an earlier call left and only reaches accumulator columns that are never stored.
    return qp_rotate_linear(w, x, signs, block, B, ldx, y, ldy, ws, QP_STATIC_SCRATCH_BYTES, hip_stream);
}

extern "C" qp_status qp_dequant(const qp_weight *w, void *W_out, void *hip_stream) {
    qp_status s = qp_validate(w);
    if (s != QP_OK) return s;
    if (!W_out) return QP_ERR_NULL;
    if (!aligned(W_out, 16)) return QP_ERR_ALIGN;
    // Native layout: one block per wavefront with the fused kernel's decoders, unless the layer
    // has fewer blocks than the chip has CUs (its table set-up would dominate: 1024 x 1024
    // takes 6.5 us there, 2.9 us on the layout-agnostic kernel).  QP_OPT_DEQUANT_KERNEL = 1 / 2
    // forces the layout-agnostic / the block kernel (the tests cover both on weights of any size).
    const int force = qp_opt(QP_OPT_DEQUANT_KERNEL);
    const bool small = (int64_t)(w->M / 16) * ((w->N + 1023) / 1024) < 256 && force != 2;
    if (w->layout == QP_LAYOUT_NATIVE && !small && force != 1)
        return qp_launch_dequant_blocks(make_dev(w), w->scheme, w->code_bits, W_out,
                                        static_cast<hipStream_t>(hip_stream));
    return qp_launch_dequant(make_dev(w), w->scheme, w->code_bits, W_out, static_cast<hipStream_t>(hip_stream));
}

extern "C" qp_status qp_hadamard(const void *x, const int8_t *signs, int32_t B, int32_t n, int32_t block,
                                 int64_t ldx, void *xr, int64_t ldxr, void *hip_stream) {
    if (!x || !signs || !xr) return QP_ERR_NULL;
    if (B < 1 || n < 1) return QP_ERR_SHAPE;
    if (block < 2 || block > 16384 || (block & (block - 1)) != 0 || n % block != 0) return QP_ERR_SHAPE;
    if (ldx < n || ldxr < n) return QP_ERR_SHAPE;
    if ((int64_t)B * (n / block) > 0x7fffffffLL) return QP_ERR_SHAPE;
    if (!aligned(x, 2) || !aligned(xr, 2)) return QP_ERR_ALIGN;
    if (x != xr || ldx != ldxr) {
        // partial overlap is not allowed
        const char *a = static_cast<const char *>(x), *b = static_cast<const char *>(xr);
        int64_t ea = ((int64_t)(B - 1) * ldx + n) * 2, eb = ((int64_t)(B - 1) * ldxr + n) * 2;
        if (a < b + eb && b < a + ea) return QP_ERR_ALIGN;
    }
    return qp_launch_hadamard(x, signs, B, n, block, ldx, xr, ldxr, 0, static_cast<hipStream_t>(hip_stream));
}

extern "C" size_t qp_native_bytes(const qp_weight *c) {
    if (!c || scheme_supported(c) != QP_OK) return 0;
    if (c->M <= 0 || c->N <= 0 || c->M % 16 != 0 || c->N % 256 != 0) return 0;
    if (c->scheme == QP_TCQHH) return c->N % 2048 != 0 ? 0 : (size_t)c->M * (size_t)row_bytes(c);
    // whole blocks of 16 x 1024: a last column block of fewer columns is padded
    return (size_t)c->M * (padded_cols(c) / 256) * (size_t)span_bytes(c);
}

extern "C" qp_status qp_repack(const qp_weight *c, qp_weight *native_out, void *native_codes, size_t bytes,
                               void *hip_stream) {
    if (!c || !native_out || !native_codes) return QP_ERR_NULL;
    qp_status s = qp_validate(c);
    if (s != QP_OK) return s;
    if (c->layout != QP_LAYOUT_CANONICAL) return QP_ERR_LAYOUT;
    size_t need = qp_native_bytes(c);
    if (need == 0) return QP_ERR_LAYOUT;
    if (bytes < need) return QP_ERR_SHAPE;
    if (!aligned(native_codes, 16)) return QP_ERR_ALIGN;
    {
        const char *a = static_cast<const char *>(c->codes), *b = static_cast<const char *>(native_codes);
        int64_t ea = (int64_t)c->row_stride * c->M;
        if (a < b + (int64_t)need && b < a + ea) return QP_ERR_ALIGN;
    }
    if (c->scheme == QP_TCQHH)
        s = qp_launch_repack_half(make_dev(c), c->code_bits, native_codes, static_cast<hipStream_t>(hip_stream));
    else
        s = qp_launch_repack(make_dev(c), span_bytes(c), native_codes, static_cast<hipStream_t>(hip_stream));
    if (s != QP_OK) return s;
    *native_out = *c;
    native_out->layout = QP_LAYOUT_NATIVE;
    native_out->codes = native_codes;
    native_out->row_stride = 0;
    return QP_OK;
}

// What the encoders support: every scheme that qp_linear does.
static qp_status encode_check(const qp_weight *w) {
    if (!w) return QP_ERR_NULL;
    qp_status s = scheme_supported(w);
    if (s != QP_OK) return s;
    if (w->M <= 0 || w->N <= 0) return QP_ERR_SHAPE;
    if (w->N % 16 != 0) return QP_ERR_SHAPE;
    if ((w->scheme == QP_TCQ || w->scheme == QP_TCQH) && w->N % 256 != 0) return QP_ERR_SHAPE;
    if (w->scheme == QP_TCQHH && w->N % 512 != 0) return QP_ERR_SHAPE;
    if (!w->lut) return QP_ERR_NULL;
    if (w->layout != QP_LAYOUT_CANONICAL) return QP_ERR_LAYOUT;
    if (w->row_stride % 16 != 0) return QP_ERR_ALIGN;
    if (w->row_stride < row_bytes(w)) return QP_ERR_SHAPE;
    if (!aligned(w->lut, 16)) return QP_ERR_ALIGN;
    return QP_OK;
}

extern "C" size_t qp_encode_workspace_bytes(const qp_weight *w) {
    if (encode_check(w) != QP_OK) return 0;
    const size_t per_wg = qp_encode_min_workspace(w->scheme, w->code_bits);
    int64_t tiles = (int64_t)w->M * (w->N / 256);
    if (w->scheme == QP_TCQHH) tiles /= 2;
    const int64_t wgs = tiles < 256 ? tiles : 256;
    return per_wg * (size_t)wgs;
}

extern "C" qp_status qp_encode(const qp_weight *w, const void *W, int64_t ldw, void *codes_out, float *tile_err,
                               void *workspace, size_t workspace_bytes, void *hip_stream) {
    qp_status s = encode_check(w);
    if (s != QP_OK) return s;
    if (!W || !codes_out) return QP_ERR_NULL;
    if (ldw < w->N || ldw % 8 != 0) return QP_ERR_SHAPE;
    if (!aligned(W, 16) || !aligned(codes_out, 16) || (tile_err && !aligned(tile_err, 4))) return QP_ERR_ALIGN;
    const size_t per_wg = qp_encode_min_workspace(w->scheme, w->code_bits);
    if (per_wg && (!workspace || workspace_bytes < per_wg)) return QP_ERR_WORKSPACE;
    if (per_wg && !aligned(workspace, 16)) return QP_ERR_ALIGN;
    return qp_launch_encode(w->scheme, w->code_bits, w->tlut_bits, w->M, w->N, static_cast<const uint16_t *>(w->lut), W, ldw,
                            codes_out, w->row_stride, workspace, workspace_bytes, tile_err,
                            static_cast<hipStream_t>(hip_stream));
}

extern "C" qp_status qp_row_normalize(void *W, int64_t ldw, int32_t M, int32_t N, void *scales, void *hip_stream) {
    if (!W || !scales) return QP_ERR_NULL;
    if (M < 1 || N < 8 || N % 8 != 0 || ldw < N || ldw % 8 != 0) return QP_ERR_SHAPE;
    if (!aligned(W, 16) || !aligned(scales, 2)) return QP_ERR_ALIGN;
    return qp_launch_row_normalize(W, ldw, M, N, scales, static_cast<hipStream_t>(hip_stream));
}

extern "C" size_t qp_kmeans_workspace_bytes(int32_t k, int32_t d) {
    if (k < 1 || k > 4096 || (d != 1 && d != 2)) return 0;
    return qp_kmeans_workspace(k, d);
}

extern "C" qp_status qp_kmeans(const void *samples, int64_t n, int32_t d, void *centres, int32_t k, int32_t max_iter,
                               float tol, void *workspace, size_t workspace_bytes, int32_t *assign_out,
                               void *centres_f16, double *stats_out, void *hip_stream) {
    if (!samples || !centres || !workspace) return QP_ERR_NULL;
    if (d != 1 && d != 2) return QP_ERR_UNSUPPORTED;
    if (k < 1 || k > 4096) return QP_ERR_UNSUPPORTED;
    if (n < 1 || max_iter < 1 || !(tol >= 0.0f)) return QP_ERR_SHAPE;
    if (!aligned(samples, 4 * d) || !aligned(centres, 4 * d) || !aligned(workspace, 16) ||
        (assign_out && !aligned(assign_out, 4)) || (centres_f16 && !aligned(centres_f16, 2 * d)) ||
        (stats_out && !aligned(stats_out, 8)))
        return QP_ERR_ALIGN;
    if (workspace_bytes < qp_kmeans_workspace(k, d)) return QP_ERR_WORKSPACE;
    return qp_launch_kmeans(static_cast<const float *>(samples), n, d, static_cast<float *>(centres), k, max_iter, tol,
                            workspace, assign_out, static_cast<uint16_t *>(centres_f16), stats_out,
                            static_cast<hipStream_t>(hip_stream));
}

extern "C" const char *qp_status_string(qp_status s) {
    switch (s) {
        case QP_OK: return "ok";
        case QP_ERR_NULL: return "null pointer";
        case QP_ERR_SHAPE: return "bad shape";
        case QP_ERR_UNSUPPORTED: return "unsupported quantizer";
        case QP_ERR_ALIGN: return "bad alignment or overlap";
        case QP_ERR_LAYOUT: return "bad layout";
        case QP_ERR_DEVICE: return "device launch error";
        case QP_ERR_WORKSPACE: return "workspace too small";
        case QP_ERR_MEMORY: return "host memory exhausted";
        default: return "unknown status";
    }
}

extern "C" int32_t qp_version(void) { return QP_VERSION; }
