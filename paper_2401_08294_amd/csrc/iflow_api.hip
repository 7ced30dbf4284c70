// C-ABI entry points of libiflow.so: argument validation on the host, then one launcher call.
// Nothing here allocates, synchronises or keeps state between calls (except the thread-local
// record of the last HIP error).
#include <algorithm>

#include "iflow_common.h"

namespace {

// smallest batch that goes to the 16-wide MFMA kernel (below it, the vector kernel with that many columns is faster:
// measured on 4096 x 4096, 8-bit at four columns 7.9 us on the vector units against 10.6 us on the matrix cores)
constexpr int64_t IFLOW_SMALL_MFMA_MIN_BATCH = 3, IFLOW_SMALL_MFMA_MIN_BATCH_Q8 = 5;

thread_local int g_last_hip_error = 0;

// From 32 vectors on there are two ways to run a product: the dense kernel (a workgroup per 64 weight rows and 64 or 128
// vectors walks the whole reduction length, about 0.39 / 0.53 us per 64 columns; the part runs one such workgroup per compute
// unit at full speed) or passes of sixteen vectors through the streaming MFMA kernel (about 2.5 us per pass plus the packed
// bytes at 2.6 TB/s, a third slower when a row spans several 4096-column strips).  With few vectors and long rows the dense
// kernel leaves most of the part idle for a long time - 4096 x 11008 at 32 vectors: 63 us against 28 us in two passes - so
// the cheaper of the two is taken, by this model of them (constants measured on 7B shapes; the choice depends on shapes,
// format and the number of compute units only, so a call always takes the same path on the same device).
bool passes_beat_dense(const iflow::FormatInfo &fi, int64_t rows, int64_t cols, int64_t batch, int cus)
{
    const double packed = (double)rows * (double)(cols / fi.block) * (fi.code_bytes + 4);
    const double pass_us = 2.5 + packed / 2.6e6 * (cols > 4096 ? 1.35 : 1.0);
    const double passes_us = (double)((batch + 15) / 16) * pass_us;
    const int64_t bm = batch <= 64 ? 64 : 128;
    const double wgs = (double)((rows + 63) / 64) * (double)((batch + bm - 1) / bm);
    const double dense_us = (double)(cols / 64) * (batch <= 64 ? 0.39 : 0.53) * (wgs > cus ? wgs / cus : 1.0);
    return passes_us < dense_us;
}

iflow_status_t device_status(hipError_t e)
{
    if (e == hipSuccess) return IFLOW_OK;
    g_last_hip_error = (int)e;
    return IFLOW_ERR_DEVICE;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool overlaps(const void *p, int64_t pn, const void *q, int64_t qn)
{
    const uintptr_t a0 = (uintptr_t)p, b0 = (uintptr_t)q;
    return a0 < b0 + (uintptr_t)qn && b0 < a0 + (uintptr_t)pn;
}

// Shape rules shared by every call: positive sizes, cols a whole number of blocks, and sizes that
// keep every kernel index inside 32-bit block/row counters.
iflow_status_t check_shape(iflow_format_t f, int64_t rows, int64_t cols, iflow::FormatInfo *fi)
{
    if (!iflow::format_info((int)f, fi)) return IFLOW_ERR_FORMAT;
    if (rows <= 0 || cols <= 0) return IFLOW_ERR_SHAPE;
    if (cols % fi->block != 0) return IFLOW_ERR_SHAPE;
    if (rows > (1LL << 30) || cols > (1LL << 30)) return IFLOW_ERR_SHAPE;
    return IFLOW_OK;
}

size_t packed_size(const iflow::FormatInfo &fi, int64_t rows, int64_t cols)
{
    return (size_t)rows * (size_t)(cols / fi.block) * (size_t)(fi.code_bytes + 4);
}

}  // namespace

extern "C" {

int iflow_layout_version(void) { return 1; }

const char *iflow_status_string(iflow_status_t status)
{
    switch (status) {
    case IFLOW_OK: return "ok";
    case IFLOW_ERR_NULL: return "null pointer argument";
    case IFLOW_ERR_FORMAT: return "unknown format";
    case IFLOW_ERR_SHAPE: return "bad shape: sizes must be positive and cols a multiple of the block size";
    case IFLOW_ERR_SIZE: return "output buffer too small";
    case IFLOW_ERR_ALIGN: return "device pointer not 16-byte aligned";
    case IFLOW_ERR_DEVICE: return "HIP call failed (see iflow_last_hip_error)";
    case IFLOW_ERR_TIMEOUT: return "a chained launch gave up waiting for an earlier phase's output";
    default: return "unknown status";
    }
}

int iflow_last_hip_error(void) { return g_last_hip_error; }

int iflow_format_block(iflow_format_t format)
{
    iflow::FormatInfo fi;
    return iflow::format_info((int)format, &fi) ? fi.block : -1;
}

int iflow_format_levels(iflow_format_t format)
{
    iflow::FormatInfo fi;
    return iflow::format_info((int)format, &fi) ? fi.L + 1 : -1;
}

iflow_status_t iflow_packed_bytes(iflow_format_t format, int64_t rows, int64_t cols, size_t *bytes)
{
    iflow::FormatInfo fi;
    if (!bytes) return IFLOW_ERR_NULL;
    iflow_status_t st = check_shape(format, rows, cols, &fi);
    if (st != IFLOW_OK) return st;
    *bytes = packed_size(fi, rows, cols);
    return IFLOW_OK;
}

iflow_status_t iflow_quantize(iflow_format_t format, const float *w, int64_t rows, int64_t cols,
                              void *packed, size_t packed_bytes, void *stream)
{
    iflow::FormatInfo fi;
    iflow_status_t st = check_shape(format, rows, cols, &fi);
    if (st != IFLOW_OK) return st;
    if (!w || !packed) return IFLOW_ERR_NULL;
    if (packed_bytes < packed_size(fi, rows, cols)) return IFLOW_ERR_SIZE;
    if (!aligned16(w) || !aligned16(packed)) return IFLOW_ERR_ALIGN;
    return device_status(iflow::launch_quantize((int)format, w, rows, cols, packed, (hipStream_t)stream));
}

iflow_status_t iflow_dequant(iflow_format_t format, const void *packed, int64_t rows, int64_t cols,
                             uint16_t *w16, void *stream)
{
    iflow::FormatInfo fi;
    iflow_status_t st = check_shape(format, rows, cols, &fi);
    if (st != IFLOW_OK) return st;
    if (!packed || !w16) return IFLOW_ERR_NULL;
    if (!aligned16(packed) || !aligned16(w16)) return IFLOW_ERR_ALIGN;
    return device_status(iflow::launch_dequant((int)format, packed, rows, cols, w16, (hipStream_t)stream));
}

iflow_status_t iflow_unpack_logical(iflow_format_t format, const void *packed, int64_t rows, int64_t cols,
                                    uint8_t *levels, uint16_t *scale16, uint16_t *offset16, void *stream)
{
    iflow::FormatInfo fi;
    iflow_status_t st = check_shape(format, rows, cols, &fi);
    if (st != IFLOW_OK) return st;
    if (!packed || !levels || !scale16 || !offset16) return IFLOW_ERR_NULL;
    if (!aligned16(packed) || !aligned16(levels) || !aligned16(scale16) || !aligned16(offset16)) return IFLOW_ERR_ALIGN;
    return device_status(iflow::launch_unpack((int)format, packed, rows, cols, levels, scale16, offset16, (hipStream_t)stream));
}

iflow_status_t iflow_unpack_pair_codes(iflow_format_t format, const void *packed, int64_t rows, int64_t cols, uint8_t *codes, void *stream)
{
    iflow::FormatInfo fi;
    iflow_status_t st = check_shape(format, rows, cols, &fi);
    if (st != IFLOW_OK) return st;
    if (format != IFLOW_Q3H_B64) return IFLOW_ERR_FORMAT;      // only the 3.5-bit format stores pair codes
    if (!packed || !codes) return IFLOW_ERR_NULL;
    if (!aligned16(packed) || !aligned16(codes)) return IFLOW_ERR_ALIGN;
    return device_status(iflow::launch_unpack_pair_codes(packed, rows, cols, codes, (hipStream_t)stream));
}

iflow_status_t iflow_qgemm(iflow_format_t format, const void *packed, int64_t rows, int64_t cols,
                           const uint16_t *X, int64_t batch, uint16_t *Y, void *stream)
{
    iflow::FormatInfo fi;
    iflow_status_t st = check_shape(format, rows, cols, &fi);
    if (st != IFLOW_OK) return st;
    if (batch <= 0 || batch > (1LL << 30)) return IFLOW_ERR_SHAPE;
    if (!packed || !X || !Y) return IFLOW_ERR_NULL;
    if (!aligned16(packed) || !aligned16(X) || !aligned16(Y)) return IFLOW_ERR_ALIGN;
    // One backend, three kernels chosen by batch: a few activation vectors ride along with the weight stream on the
    // vector units; up to 31 vectors the weights stream once per 16 vectors through 16x16x16 MFMAs; from 32 vectors
    // on the product is a dense contraction on LDS tiles (64-column chunks), unless passes of the streaming kernel are
    // cheaper (few vectors, long rows: see passes_beat_dense).  Column counts that are not a multiple
    // of 64 (possible with the 32-wide blocks) stay on the vector kernel, four vectors per pass.
    hipStream_t hs = (hipStream_t)stream;
    bool dense = batch >= 32 && cols % 64 == 0;
    if (dense && batch <= 256) {                              // (beyond that the dense kernel always wins)
        int cus = 0;
        const hipError_t e = iflow::device_compute_units(&cus);
        if (e != hipSuccess) return device_status(e);
        dense = !passes_beat_dense(fi, rows, cols, batch, cus);
    }
    if (dense)
        return device_status(iflow::launch_qgemm_mfma((int)format, packed, rows, cols, X, batch, Y, hs));
    if (cols % 64 == 0 && batch >= (format == IFLOW_Q8_B32 || format == IFLOW_Q8_B64 ? IFLOW_SMALL_MFMA_MIN_BATCH_Q8 : IFLOW_SMALL_MFMA_MIN_BATCH)) {
        for (int64_t b0 = 0; b0 < batch; b0 += 16) {
            const int64_t nb = batch - b0 < 16 ? batch - b0 : 16;
            hipError_t e = iflow::launch_qgemm_small((int)format, packed, rows, cols, X + b0 * cols, nb, Y + b0 * rows, hs);
            if (e != hipSuccess) return device_status(e);
        }
        return IFLOW_OK;
    }
    return device_status(iflow::launch_qgemv((int)format, packed, rows, cols, X, batch, Y, hs));
}

iflow_status_t iflow_qgemv_multi(iflow_format_t format, int count, const void *const *packed, const int64_t *rows,
                                 int64_t cols, const uint16_t *x, uint16_t *const *y, void *stream)
{
    iflow::FormatInfo fi;
    if (!iflow::format_info((int)format, &fi)) return IFLOW_ERR_FORMAT;
    if (count < 1 || count > 8) return IFLOW_ERR_SHAPE;
    if (!packed || !rows || !x || !y) return IFLOW_ERR_NULL;
    if (!aligned16(x)) return IFLOW_ERR_ALIGN;
    for (int i = 0; i < count; ++i) {
        iflow_status_t st = check_shape(format, rows[i], cols, &fi);
        if (st != IFLOW_OK) return st;
        if (!packed[i] || !y[i]) return IFLOW_ERR_NULL;
        if (!aligned16(packed[i]) || !aligned16(y[i])) return IFLOW_ERR_ALIGN;
    }
    return device_status(iflow::launch_qgemv_multi((int)format, count, packed, rows, cols, x, y, (hipStream_t)stream));
}

iflow_status_t iflow_qgemv_fused(iflow_format_t format, int count, const void *const *packed, const int64_t *rows,
                                 int64_t cols, const uint16_t *x, iflow_x_op_t x_op, const uint16_t *aux, float eps,
                                 const uint16_t *const *residual, uint16_t *const *y, void *stream)
{
    iflow::FormatInfo fi;
    if (!iflow::format_info((int)format, &fi)) return IFLOW_ERR_FORMAT;
    if (count < 1 || count > 8) return IFLOW_ERR_SHAPE;
    if (x_op != IFLOW_X_PLAIN && x_op != IFLOW_X_RMS_GAIN && x_op != IFLOW_X_SILU_MUL) return IFLOW_ERR_SHAPE;
    if (!packed || !rows || !x || !y) return IFLOW_ERR_NULL;
    if ((x_op == IFLOW_X_PLAIN) != (aux == nullptr)) return IFLOW_ERR_NULL;
    if (x_op == IFLOW_X_RMS_GAIN && !(eps >= 0.0f && eps < 3.0e38f)) return IFLOW_ERR_SHAPE;
    if (!aligned16(x) || (aux && !aligned16(aux))) return IFLOW_ERR_ALIGN;
    for (int i = 0; i < count; ++i) {
        iflow_status_t st = check_shape(format, rows[i], cols, &fi);
        if (st != IFLOW_OK) return st;
        if (!packed[i] || !y[i]) return IFLOW_ERR_NULL;
        if (!aligned16(packed[i]) || !aligned16(y[i])) return IFLOW_ERR_ALIGN;
        // outputs are written while other workgroups still read x and aux
        if (overlaps(y[i], rows[i] * 2, x, cols * 2) || (aux && overlaps(y[i], rows[i] * 2, aux, cols * 2))) return IFLOW_ERR_SHAPE;
        if (residual && residual[i]) {
            if (((uintptr_t)residual[i] & 1u) != 0) return IFLOW_ERR_ALIGN;
            // a residual is read by the wavefront that later writes the same rows: equal to y[i] is fine, a shifted overlap is not
            if (residual[i] != y[i] && overlaps(residual[i], rows[i] * 2, y[i], rows[i] * 2)) return IFLOW_ERR_SHAPE;
            for (int j = 0; j < count; ++j)
                if (j != i && y[j] && overlaps(residual[i], rows[i] * 2, y[j], rows[j] * 2)) return IFLOW_ERR_SHAPE;
        }
    }
    if (format != IFLOW_Q3H_B64) {
        const hipError_t e = iflow::launch_qgemv_rows_fused((int)format, count, packed, rows, cols, x, (int)x_op, aux, eps, residual, y,
                                                            (hipStream_t)stream);
        return e == hipErrorNotSupported ? IFLOW_ERR_SHAPE : device_status(e);   // (rows too long for the staged activations)
    }
    return device_status(iflow::launch_qgemv_fused(count, packed, rows, cols, x, (int)x_op, aux, eps, residual, y, (hipStream_t)stream));
}

iflow_status_t iflow_qgemm_fused(iflow_format_t format, const void *packed, int64_t rows, int64_t cols, const uint16_t *X, int64_t batch,
                                 iflow_x_op_t x_op, const uint16_t *aux, float eps, const uint16_t *residual, uint16_t *Y, void *stream)
{
    iflow::FormatInfo fi;
    if (!iflow::format_info((int)format, &fi)) return IFLOW_ERR_FORMAT;
    if (batch < 1 || batch > 16) return IFLOW_ERR_SHAPE;
    if (x_op != IFLOW_X_PLAIN && x_op != IFLOW_X_RMS_GAIN && x_op != IFLOW_X_SILU_MUL) return IFLOW_ERR_SHAPE;
    if (!packed || !X || !Y) return IFLOW_ERR_NULL;
    if ((x_op == IFLOW_X_PLAIN) != (aux == nullptr)) return IFLOW_ERR_NULL;
    if (x_op == IFLOW_X_RMS_GAIN && !(eps >= 0.0f && eps < 3.0e38f)) return IFLOW_ERR_SHAPE;
    iflow_status_t st = check_shape(format, rows, cols, &fi);
    if (st != IFLOW_OK) return st;
    if (cols % 64 != 0) return IFLOW_ERR_SHAPE;                // (the 32-wide formats too: the batch kernel works on 64-column groups)
    if (!aligned16(packed) || !aligned16(X) || !aligned16(Y) || (aux && !aligned16(aux))) return IFLOW_ERR_ALIGN;
    const int64_t aux_len = x_op == IFLOW_X_SILU_MUL ? batch * cols : cols;
    // outputs are written while other workgroups still read X and aux
    if (overlaps(Y, batch * rows * 2, X, batch * cols * 2) || (aux && overlaps(Y, batch * rows * 2, aux, aux_len * 2))) return IFLOW_ERR_SHAPE;
    if (residual) {
        if (((uintptr_t)residual & 1u) != 0) return IFLOW_ERR_ALIGN;
        // a residual element is read by the thread that writes the same output element: equal to Y is fine, a shifted overlap is not
        if (residual != Y && overlaps(residual, batch * rows * 2, Y, batch * rows * 2)) return IFLOW_ERR_SHAPE;
    }
    if (batch == 1) {
        const void *pk[1] = {packed};
        const int64_t rw[1] = {rows};
        const uint16_t *rs[1] = {residual};
        uint16_t *ys[1] = {Y};
        return iflow_qgemv_fused(format, 1, pk, rw, cols, X, x_op, aux, eps, rs, ys, stream);
    }
    return device_status(iflow::launch_qgemm_small_fused((int)format, packed, rows, cols, X, batch, (int)x_op, aux, eps, residual, Y,
                                                         (hipStream_t)stream));
}

iflow_status_t iflow_qgemv_gated(iflow_format_t format, const void *packed_gate, const void *packed_up, int64_t rows, int64_t cols,
                                 const uint16_t *x, iflow_x_op_t x_op, const uint16_t *aux, float eps, uint16_t *y, void *stream)
{
    iflow::FormatInfo fi;
    if (!iflow::format_info((int)format, &fi)) return IFLOW_ERR_FORMAT;
    if (x_op != IFLOW_X_PLAIN && x_op != IFLOW_X_RMS_GAIN) return IFLOW_ERR_SHAPE;
    if (!packed_gate || !packed_up || !x || !y) return IFLOW_ERR_NULL;
    if ((x_op == IFLOW_X_PLAIN) != (aux == nullptr)) return IFLOW_ERR_NULL;
    if (x_op == IFLOW_X_RMS_GAIN && !(eps >= 0.0f && eps < 3.0e38f)) return IFLOW_ERR_SHAPE;
    iflow_status_t st = check_shape(format, rows, cols, &fi);
    if (st != IFLOW_OK) return st;
    if (!aligned16(packed_gate) || !aligned16(packed_up) || !aligned16(x) || !aligned16(y) || (aux && !aligned16(aux))) return IFLOW_ERR_ALIGN;
    // outputs are written while other workgroups still read x and aux
    if (overlaps(y, rows * 2, x, cols * 2) || (aux && overlaps(y, rows * 2, aux, cols * 2))) return IFLOW_ERR_SHAPE;
    const hipError_t e = iflow::launch_qgemv_gated((int)format, packed_gate, packed_up, rows, cols, x, (int)x_op, aux, eps, y,
                                                   (hipStream_t)stream);
    return e == hipErrorNotSupported ? IFLOW_ERR_SHAPE : device_status(e);       // (rows too long for the staged activations)
}

iflow_status_t iflow_attn_decode_workspace_bytes(int n_heads, size_t *bytes)
{
    if (!bytes) return IFLOW_ERR_NULL;
    if (n_heads < 1 || n_heads > 512) return IFLOW_ERR_SHAPE;
    *bytes = iflow::attn_workspace_bytes(n_heads);
    return IFLOW_OK;
}

iflow_status_t iflow_attn_decode(const uint16_t *q, const uint16_t *k_cache, const uint16_t *v_cache, int n_heads,
                                 int n_kv_heads, int head_dim, int64_t seq_len, int64_t max_seq, float scale,
                                 uint16_t *out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (head_dim != 64 && head_dim != 128) return IFLOW_ERR_SHAPE;
    if (n_kv_heads < 1 || n_kv_heads > 64 || n_heads < 1 || n_heads > 512 || n_heads % n_kv_heads != 0) return IFLOW_ERR_SHAPE;
    if (seq_len < 1 || max_seq < seq_len || max_seq > (1LL << 20)) return IFLOW_ERR_SHAPE;
    if (!(scale > 0.0f && scale < 3.0e38f)) return IFLOW_ERR_SHAPE;
    if (!q || !k_cache || !v_cache || !out || !workspace) return IFLOW_ERR_NULL;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out) || !aligned16(workspace)) return IFLOW_ERR_ALIGN;
    if (workspace_bytes < iflow::attn_workspace_bytes(n_heads)) return IFLOW_ERR_SIZE;
    return device_status(iflow::launch_attn_decode(q, k_cache, v_cache, n_heads, n_kv_heads, head_dim, seq_len, max_seq, scale, out, workspace,
                                                   (hipStream_t)stream));
}

iflow_status_t iflow_attn_decode_static(const uint16_t *q, const uint16_t *k_cache, const uint16_t *v_cache, int n_heads,
                                        int n_kv_heads, int head_dim, int64_t seq_len, int64_t max_seq, float scale,
                                        uint16_t *out, void *stream)
{
    if (head_dim != 64 && head_dim != 128) return IFLOW_ERR_SHAPE;
    if (n_kv_heads < 1 || n_kv_heads > 64 || n_heads < 1 || n_heads > 512 || n_heads % n_kv_heads != 0) return IFLOW_ERR_SHAPE;
    if (seq_len < 1 || max_seq < seq_len || max_seq > (1LL << 20)) return IFLOW_ERR_SHAPE;
    if (!(scale > 0.0f && scale < 3.0e38f)) return IFLOW_ERR_SHAPE;
    if (!q || !k_cache || !v_cache || !out) return IFLOW_ERR_NULL;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out)) return IFLOW_ERR_ALIGN;
    if (n_heads > IFLOW_ATTN_STATIC_MAX_HEADS) return IFLOW_ERR_SIZE;      // more partial results than the library's own array holds
    return device_status(iflow::launch_attn_decode_static(q, k_cache, v_cache, n_heads, n_kv_heads, head_dim, seq_len, max_seq, scale, out,
                                                          (hipStream_t)stream));
}

iflow_status_t iflow_rope_append(uint16_t *q, const uint16_t *k_new, const uint16_t *v_new, int n_heads, int n_kv_heads,
                                 int head_dim, int64_t position, int64_t max_seq, float base, iflow_rope_pairing_t pair_mode,
                                 uint16_t *k_cache, uint16_t *v_cache, void *stream)
{
    if (head_dim < 16 || head_dim > 256 || head_dim % 8 != 0) return IFLOW_ERR_SHAPE;   // rows of the caches stay 16-byte aligned
    if (n_heads < 1 || n_heads > 65536 || n_kv_heads < 1 || n_kv_heads > 65536) return IFLOW_ERR_SHAPE;
    if (position < 0 || position >= max_seq || max_seq > (1LL << 20)) return IFLOW_ERR_SHAPE;
    if (!(base > 1.0f && base < 3.0e38f)) return IFLOW_ERR_SHAPE;
    if (pair_mode != IFLOW_ROPE_ADJACENT && pair_mode != IFLOW_ROPE_HALVES) return IFLOW_ERR_SHAPE;
    if (!q || !k_new || !v_new || !k_cache || !v_cache) return IFLOW_ERR_NULL;
    if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache)) return IFLOW_ERR_ALIGN;
    return device_status(iflow::launch_rope_append(q, k_new, v_new, n_heads, n_kv_heads, head_dim, position, max_seq, (double)base, (int)pair_mode,
                                                   k_cache, v_cache, (hipStream_t)stream));
}

// ---- the chained launch ---------------------------------------------------------------------------------------------
namespace {

// Everything that can be checked about a chain on the host; fills the index arrays the plan builder wants.
struct ChainOps {                      // the modules around the products; every pointer may be null (bare products)
    const iflow_x_op_t *x_op;
    const uint16_t *const *aux;
    const float *eps;
    const int *gated;
    const uint16_t *const *residual;
};

iflow_status_t chain_validate(iflow_format_t format, int nphases, const int *counts, const int64_t *cols, const uint16_t *const *x,
                              const void *const *packed, const int64_t *rows, uint16_t *const *y, const ChainOps &ops,
                              std::vector<int> &first, std::vector<int> &x_src, std::vector<int> &residual_src, int *nmatrices)
{
    iflow::FormatInfo fi;
    if (!iflow::format_info((int)format, &fi)) return IFLOW_ERR_FORMAT;
    if (!iflow::chain_supports_format((int)format)) return IFLOW_ERR_FORMAT;
    if (nphases < 1 || nphases > IFLOW_CHAIN_MAX_PHASES) return IFLOW_ERR_SHAPE;
    if (!counts || !cols || !x || !packed || !rows || !y) return IFLOW_ERR_NULL;
    int total = 0;
    first.assign(nphases, 0);
    for (int p = 0; p < nphases; ++p) {
        if (counts[p] < 1 || counts[p] > IFLOW_CHAIN_MAX_GROUP || counts[p] > IFLOW_CHAIN_MAX_MATRICES - total) return IFLOW_ERR_SHAPE;
        first[p] = total;
        total += counts[p];
    }
    *nmatrices = total;
    x_src.assign(nphases, -1);
    for (int p = 0; p < nphases; ++p) {
        if (!x[p]) return IFLOW_ERR_NULL;
        if (!aligned16(x[p])) return IFLOW_ERR_ALIGN;
        if (cols[p] > iflow::chain_max_cols((int)format)) return IFLOW_ERR_SHAPE;   // a row's activations have to fit the kernel's LDS
        const bool gated = ops.gated && ops.gated[p];
        if (gated && (counts[p] != 2 || rows[first[p]] != rows[first[p] + 1])) return IFLOW_ERR_SHAPE;   // a gate and an up matrix of equal size
        for (int m = first[p]; m < first[p] + counts[p]; ++m) {
            iflow_status_t st = check_shape(format, rows[m], cols[p], &fi);
            if (st != IFLOW_OK) return st;
            const bool no_output = gated && m == first[p] + 1;                   // the up matrix of a gated pair has no output of its own
            if (!packed[m] || (!y[m] && !no_output)) return IFLOW_ERR_NULL;
            if (no_output && y[m]) return IFLOW_ERR_SHAPE;
            if (!aligned16(packed[m]) || (y[m] && !aligned16(y[m]))) return IFLOW_ERR_ALIGN;
            if (gated && ops.residual && ops.residual[m]) return IFLOW_ERR_SHAPE;
        }
        if (ops.x_op) {
            if (ops.x_op[p] == IFLOW_X_RMS_GAIN) {
                if (!ops.aux || !ops.aux[p] || !ops.eps) return IFLOW_ERR_NULL;
                if (!aligned16(ops.aux[p])) return IFLOW_ERR_ALIGN;
                if (!(ops.eps[p] >= 0.0f && ops.eps[p] < 3.0e38f)) return IFLOW_ERR_SHAPE;
            } else if (ops.x_op[p] != IFLOW_X_PLAIN) {
                return IFLOW_ERR_SHAPE;                                          // (the gated input comes from a gated phase, not from an x_op)
            }
        }
    }
    // Outputs must not overlap each other.  An activation vector is either exactly the whole output of a matrix of an
    // EARLIER phase (then the phase waits for it inside the launch), or memory that no output of the whole call touches:
    // workgroups run ahead of each other, so a later phase's output may be written before a slow workgroup has read
    // an earlier phase's input.
    for (int i = 0; i < total; ++i)
        for (int j = i + 1; j < total; ++j)
            if (y[i] && y[j] && overlaps(y[i], rows[i] * 2, y[j], rows[j] * 2)) return IFLOW_ERR_SHAPE;
    for (int p = 0; p < nphases; ++p) {
        for (int i = 0; i < total; ++i) {
            if (!y[i]) continue;
            if (ops.x_op && ops.x_op[p] == IFLOW_X_RMS_GAIN && overlaps(ops.aux[p], cols[p] * 2, y[i], rows[i] * 2)) return IFLOW_ERR_SHAPE;
            if (!overlaps(x[p], cols[p] * 2, y[i], rows[i] * 2)) continue;
            if (i < first[p] && static_cast<const void *>(x[p]) == static_cast<const void *>(y[i]) && rows[i] == cols[p] && x_src[p] < 0) x_src[p] = i;
            else return IFLOW_ERR_SHAPE;
        }
    }
    // a residual is an input of the launch that no output overlaps, or exactly the output of a matrix of an earlier phase
    residual_src.assign(total, -1);
    for (int p = 0; p < nphases && ops.residual; ++p) {
        for (int m = first[p]; m < first[p] + counts[p]; ++m) {
            if (!ops.residual[m]) continue;
            if ((reinterpret_cast<uintptr_t>(ops.residual[m]) & 3u) != 0) return IFLOW_ERR_ALIGN;
            for (int i = 0; i < total; ++i) {
                if (!y[i] || !overlaps(ops.residual[m], rows[m] * 2, y[i], rows[i] * 2)) continue;
                if (i < first[p] && static_cast<const void *>(ops.residual[m]) == static_cast<const void *>(y[i]) && rows[i] == rows[m] &&
                    residual_src[m] < 0) residual_src[m] = i;
                else return IFLOW_ERR_SHAPE;
            }
        }
    }
    return IFLOW_OK;
}

}  // namespace

iflow_status_t iflow_qgemv_chain_workspace_bytes(int nmatrices, const int64_t *rows, size_t *bytes)
{
    if (!rows || !bytes) return IFLOW_ERR_NULL;
    if (nmatrices < 1 || nmatrices > IFLOW_CHAIN_MAX_MATRICES) return IFLOW_ERR_SHAPE;
    for (int i = 0; i < nmatrices; ++i)
        if (rows[i] <= 0 || rows[i] > (1LL << 30)) return IFLOW_ERR_SHAPE;
    *bytes = iflow::chain_workspace_bytes(nmatrices, rows);
    return IFLOW_OK;
}

iflow_status_t iflow_qgemv_chain_plan_bytes(int nphases, int nmatrices, size_t *bytes)
{
    if (!bytes) return IFLOW_ERR_NULL;
    if (nphases < 1 || nphases > IFLOW_CHAIN_MAX_PHASES || nmatrices < nphases || nmatrices > IFLOW_CHAIN_MAX_MATRICES) return IFLOW_ERR_SHAPE;
    *bytes = iflow::chain_plan_bytes(nphases, nmatrices);
    return IFLOW_OK;
}

iflow_status_t iflow_qgemv_chain_plan_fused(iflow_format_t format, int nphases, const int *counts, const int64_t *cols,
                                            const uint16_t *const *x, const iflow_x_op_t *x_op, const uint16_t *const *aux,
                                            const float *eps, const int *gated, const void *const *packed, const int64_t *rows,
                                            const uint16_t *const *residual, uint16_t *const *y, void *plan, size_t plan_bytes,
                                            void *workspace, size_t workspace_bytes, void *stream, iflow_chain_t *chain)
{
    std::vector<int> first, x_src, residual_src;
    int total = 0;
    const ChainOps ops = {x_op, aux, eps, gated, residual};
    iflow_status_t st = chain_validate(format, nphases, counts, cols, x, packed, rows, y, ops, first, x_src, residual_src, &total);
    if (st != IFLOW_OK) return st;
    if (!plan || !workspace || !chain) return IFLOW_ERR_NULL;
    if (!aligned16(plan) || !aligned16(workspace)) return IFLOW_ERR_ALIGN;
    const size_t ws_need = iflow::chain_workspace_bytes(total, rows);
    if (workspace_bytes < ws_need || plan_bytes < iflow::chain_plan_bytes(nphases, total)) return IFLOW_ERR_SIZE;
    int grid = 0;
    hipError_t e = iflow::chain_grid_for_device(&grid);
    if (e != hipSuccess) return device_status(e);
    std::vector<int> xop_int(nphases, IFLOW_X_PLAIN);
    for (int p = 0; p < nphases && x_op; ++p) xop_int[p] = (int)x_op[p];
    iflow::ChainSpec spec = {(int)format, nphases, counts, first.data(), cols, x, x_src.data(), packed, rows, y,
                             xop_int.data(), aux, eps, gated, residual, residual_src.data(), nullptr, nullptr, 0, nullptr};
    std::vector<uint8_t> host;
    if (!iflow::chain_build_plan(spec, grid, host)) return IFLOW_ERR_SHAPE;   // more rows than the kernel's 32-bit indices cover
    hipStream_t s = (hipStream_t)stream;
    e = hipMemsetAsync(workspace, 0, ws_need, s);
    if (e == hipSuccess) e = hipMemcpyAsync(plan, host.data(), host.size(), hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);          // (the host copy of the plan goes away when this call returns)
    if (e != hipSuccess) return device_status(e);
    int max_strips = 1;
    for (int p = 0; p < nphases; ++p) max_strips = std::max(max_strips, iflow::chain_strips((int)format, cols[p]));
    bool fused = false;
    for (int p = 0; p < nphases; ++p) fused = fused || (x_op && x_op[p] != IFLOW_X_PLAIN) || (gated && gated[p]);
    for (int m = 0; m < total && residual; ++m) fused = fused || residual[m] != nullptr;
    chain->plan = plan; chain->workspace = workspace;
    chain->grid = grid; chain->max_strips = max_strips;
    chain->magic = IFLOW_CHAIN_MAGIC; chain->fused = fused ? 1u : 0u;
    chain->format = (int32_t)format; chain->lds_bytes = iflow::chain_lds_bytes((int)format, max_strips);
    chain->max_seq = 0;
    return IFLOW_OK;
}

iflow_status_t iflow_qgemv_chain_plan(iflow_format_t format, int nphases, const int *counts, const int64_t *cols,
                                      const uint16_t *const *x, const void *const *packed, const int64_t *rows,
                                      uint16_t *const *y, void *plan, size_t plan_bytes, void *workspace,
                                      size_t workspace_bytes, void *stream, iflow_chain_t *chain)
{
    return iflow_qgemv_chain_plan_fused(format, nphases, counts, cols, x, nullptr, nullptr, nullptr, nullptr, packed, rows, nullptr, y,
                                        plan, plan_bytes, workspace, workspace_bytes, stream, chain);
}

iflow_status_t iflow_qgemv_chain_launch(const iflow_chain_t *chain, void *stream)
{
    if (!chain || !chain->plan || !chain->workspace) return IFLOW_ERR_NULL;
    if (chain->magic != IFLOW_CHAIN_MAGIC || chain->max_seq != 0) return IFLOW_ERR_SHAPE;   // (a decoder stack's plan needs a position)
    hipError_t e = iflow::launch_chain(chain->plan, chain->workspace, chain->grid, chain->lds_bytes, chain->fused != 0, (int)chain->format, -1,
                                       (hipStream_t)stream);
    if (e == hipErrorInvalidValue) return IFLOW_ERR_SHAPE;     // planned for a device with another number of compute units
    return device_status(e);
}

iflow_status_t iflow_qgemv_chain_check(const iflow_chain_t *chain, void *stream)
{
    if (!chain || !chain->workspace) return IFLOW_ERR_NULL;
    uint32_t head[2] = {0, 0};
    hipError_t e = hipMemcpyAsync(head, chain->workspace, sizeof(head), hipMemcpyDeviceToHost, (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) return device_status(e);
    return head[1] ? IFLOW_ERR_TIMEOUT : IFLOW_OK;
}

// ---- a decoder stack's decode step as one chained launch ---------------------------------------------------------------------
namespace {

constexpr int STACK_MATS = 8, STACK_PHASES = 6;               // per layer: Wq Wk Wv, the attention's output, Wo, Wgate Wup, Wdown
constexpr int STACK_MAX_LAYERS = 128;

inline int64_t round128(int64_t n) { return (n + 127) / 128 * 128; }

// element offsets of a layer's intermediate vectors inside its share of the scratch buffer
struct StackLayout {
    int64_t q, k, v, t, h1, a, h2, per_layer;
};
StackLayout stack_layout(const iflow_decode_stack_t &d)
{
    const int64_t kvd = (int64_t)d.n_kv_heads * 128;
    StackLayout L;
    L.q = 0; L.k = L.q + round128(d.hidden); L.v = L.k + round128(kvd); L.t = L.v + round128(kvd);
    L.h1 = L.t + round128(d.hidden); L.a = L.h1 + round128(d.hidden); L.h2 = L.a + round128(d.ffn);
    L.per_layer = L.h2 + round128(d.hidden);
    return L;
}

iflow_status_t stack_check_shape(const iflow_decode_stack_t *d)
{
    if (!d) return IFLOW_ERR_NULL;
    if (!iflow::chain_supports_format((int)d->format)) return IFLOW_ERR_FORMAT;
    if (d->n_layers < 1 || d->n_layers > STACK_MAX_LAYERS) return IFLOW_ERR_SHAPE;
    if (d->head_dim != 128 || d->n_heads < 1 || d->n_kv_heads < 1 || d->n_heads % d->n_kv_heads != 0) return IFLOW_ERR_SHAPE;
    const int group = d->n_heads / d->n_kv_heads;
    if (group != 1 && (group & 1)) return IFLOW_ERR_SHAPE;
    if ((int64_t)d->n_heads * 128 != d->hidden) return IFLOW_ERR_SHAPE;
    const int64_t max_cols = iflow::chain_max_cols((int)d->format);
    if (d->hidden % 64 != 0 || d->ffn < 64 || d->ffn % 64 != 0 || d->hidden > max_cols || d->ffn > max_cols) return IFLOW_ERR_SHAPE;
    if (d->max_seq < 1 || d->max_seq > (1LL << 20)) return IFLOW_ERR_SHAPE;
    if (d->rope_pairing != IFLOW_ROPE_ADJACENT && d->rope_pairing != IFLOW_ROPE_HALVES) return IFLOW_ERR_SHAPE;
    if (!(d->eps >= 0.0f) || !(d->rope_base > 1.0f)) return IFLOW_ERR_SHAPE;
    return IFLOW_OK;
}

// rows of the eight matrix entries of every layer
void stack_rows(const iflow_decode_stack_t &d, std::vector<int64_t> &rows)
{
    const int64_t kvd = (int64_t)d.n_kv_heads * 128;
    rows.resize((size_t)d.n_layers * STACK_MATS);
    for (int l = 0; l < d.n_layers; ++l) {
        int64_t *r = rows.data() + (size_t)l * STACK_MATS;
        r[0] = d.hidden; r[1] = kvd; r[2] = kvd; r[3] = d.hidden; r[4] = d.hidden; r[5] = d.ffn; r[6] = d.ffn; r[7] = d.hidden;
    }
}

size_t stack_workspace_bytes(const iflow_decode_stack_t &d, const std::vector<int64_t> &rows, int grid)
{
    return iflow::chain_workspace_bytes((int)rows.size(), rows.data()) +
           (size_t)d.n_layers * iflow::chain_attn_workspace_bytes(d.n_heads, d.n_kv_heads, grid);
}

}  // namespace

iflow_status_t iflow_decode_stack_sizes(const iflow_decode_stack_t *stack, size_t *scratch_bytes, size_t *plan_bytes, size_t *workspace_bytes)
{
    iflow_status_t st = stack_check_shape(stack);
    if (st != IFLOW_OK) return st;
    if (!scratch_bytes || !plan_bytes || !workspace_bytes) return IFLOW_ERR_NULL;
    int grid = 0;
    hipError_t e = iflow::chain_grid_for_device(&grid);
    if (e != hipSuccess) return device_status(e);
    if (stack->n_kv_heads > grid) return IFLOW_ERR_SHAPE;
    std::vector<int64_t> rows;
    stack_rows(*stack, rows);
    *scratch_bytes = (size_t)stack->n_layers * (size_t)stack_layout(*stack).per_layer * 2;
    *plan_bytes = iflow::chain_plan_bytes(stack->n_layers * STACK_PHASES, stack->n_layers * STACK_MATS, stack->n_layers);
    *workspace_bytes = stack_workspace_bytes(*stack, rows, grid);
    return IFLOW_OK;
}

iflow_status_t iflow_decode_stack_plan(const iflow_decode_stack_t *stack, void *plan, size_t plan_bytes, void *workspace,
                                       size_t workspace_bytes, void *stream, iflow_chain_t *chain)
{
    iflow_status_t st = stack_check_shape(stack);
    if (st != IFLOW_OK) return st;
    const iflow_decode_stack_t &d = *stack;
    if (!d.layers || !d.h_in || !d.h_out || !d.scratch || !plan || !workspace || !chain) return IFLOW_ERR_NULL;
    if (!aligned16(d.h_in) || !aligned16(d.h_out) || !aligned16(d.scratch) || !aligned16(plan) || !aligned16(workspace)) return IFLOW_ERR_ALIGN;
    const StackLayout L = stack_layout(d);
    const size_t scratch_bytes = (size_t)d.n_layers * (size_t)L.per_layer * 2;
    if (overlaps(d.h_in, (size_t)d.hidden * 2, d.h_out, (size_t)d.hidden * 2) || overlaps(d.h_in, (size_t)d.hidden * 2, d.scratch, scratch_bytes) ||
        overlaps(d.h_out, (size_t)d.hidden * 2, d.scratch, scratch_bytes)) return IFLOW_ERR_SHAPE;
    // what the launch writes (scratch, h_out, the caches' rows) must not overlap anything else it reads or writes: workgroups
    // run ahead of each other, so no order between a write and an unrelated read can be relied on
    const int64_t cache_bytes = (int64_t)d.n_kv_heads * d.max_seq * 128 * 2;
    auto hits_an_output = [&](const void *p, int64_t n) {
        return overlaps(p, n, d.scratch, (int64_t)scratch_bytes) || overlaps(p, n, d.h_out, (int64_t)d.hidden * 2);
    };
    for (int l = 0; l < d.n_layers; ++l) {
        const iflow_decode_layer_t &y = d.layers[l];
        const void *ptrs[] = {y.wq, y.wk, y.wv, y.wo, y.w_gate, y.w_up, y.w_down, y.norm1, y.norm2, y.k_cache, y.v_cache};
        for (const void *p : ptrs) {
            if (!p) return IFLOW_ERR_NULL;
            if (!aligned16(p)) return IFLOW_ERR_ALIGN;
        }
        if (hits_an_output(y.norm1, (int64_t)d.hidden * 2) || hits_an_output(y.norm2, (int64_t)d.hidden * 2) ||
            hits_an_output(y.k_cache, cache_bytes) || hits_an_output(y.v_cache, cache_bytes) ||
            overlaps(y.k_cache, cache_bytes, y.v_cache, cache_bytes) || overlaps(y.k_cache, cache_bytes, d.h_in, (int64_t)d.hidden * 2) ||
            overlaps(y.v_cache, cache_bytes, d.h_in, (int64_t)d.hidden * 2)) return IFLOW_ERR_SHAPE;
        for (int m = 0; m < l; ++m) {                          // every layer has caches of its own
            const iflow_decode_layer_t &z = d.layers[m];
            if (overlaps(y.k_cache, cache_bytes, z.k_cache, cache_bytes) || overlaps(y.k_cache, cache_bytes, z.v_cache, cache_bytes) ||
                overlaps(y.v_cache, cache_bytes, z.k_cache, cache_bytes) || overlaps(y.v_cache, cache_bytes, z.v_cache, cache_bytes))
                return IFLOW_ERR_SHAPE;
        }
    }
    int grid = 0;
    hipError_t e = iflow::chain_grid_for_device(&grid);
    if (e != hipSuccess) return device_status(e);
    if (d.n_kv_heads > grid) return IFLOW_ERR_SHAPE;
    std::vector<int64_t> rows;
    stack_rows(d, rows);
    const int nphases = d.n_layers * STACK_PHASES, nmat = d.n_layers * STACK_MATS;
    const size_t ws_need = stack_workspace_bytes(d, rows, grid);
    if (workspace_bytes < ws_need || plan_bytes < iflow::chain_plan_bytes(nphases, nmat, d.n_layers)) return IFLOW_ERR_SIZE;

    // the chain: per layer   [norm1 -> Wq Wk Wv] [attention, first half] [second half] [Wo + h] [norm2 -> gate, up] [Wdown + h1]
    std::vector<int> counts(nphases), first(nphases), x_src(nphases), x_op(nphases), gated(nphases), kind(nphases), attn_of(nphases);
    std::vector<int64_t> cols(nphases);
    std::vector<const uint16_t *> x(nphases, nullptr), aux(nphases, nullptr), residual(nmat, nullptr);
    std::vector<float> eps(nphases, 0.0f);
    std::vector<const void *> packed(nmat, nullptr);
    std::vector<uint16_t *> y(nmat, nullptr);
    std::vector<int> residual_src(nmat, -1);
    std::vector<iflow::ChainAttnSpec> attn(d.n_layers);
    for (int l = 0; l < d.n_layers; ++l) {
        const iflow_decode_layer_t &w = d.layers[l];
        const int p0 = l * STACK_PHASES, m0 = l * STACK_MATS;
        uint16_t *base = d.scratch + (int64_t)l * L.per_layer;
        const uint16_t *h = l == 0 ? d.h_in : d.scratch + (int64_t)(l - 1) * L.per_layer + L.h2;
        const int h_src = l == 0 ? -1 : m0 - 1;               // the layer's input: the launch's, or the layer before's Wdown
        const int cnt[STACK_PHASES] = {3, 1, 0, 1, 2, 1};
        int m = m0;
        for (int j = 0; j < STACK_PHASES; ++j) {
            counts[p0 + j] = cnt[j]; first[p0 + j] = m; m += cnt[j];
            x_src[p0 + j] = -1; x_op[p0 + j] = IFLOW_X_PLAIN; gated[p0 + j] = 0; kind[p0 + j] = 0; attn_of[p0 + j] = l;
            cols[p0 + j] = d.hidden;
        }
        // Wq, Wk, Wv on the normalized input
        x[p0] = h; x_src[p0] = h_src; x_op[p0] = IFLOW_X_RMS_GAIN; aux[p0] = w.norm1; eps[p0] = d.eps;
        packed[m0 + 0] = w.wq; y[m0 + 0] = base + L.q;
        packed[m0 + 1] = w.wk; y[m0 + 1] = base + L.k;
        packed[m0 + 2] = w.wv; y[m0 + 2] = base + L.v;
        // attention
        kind[p0 + 1] = 1; kind[p0 + 2] = 2;
        y[m0 + 3] = base + L.t;
        attn[l] = {nullptr, nullptr, nullptr, m0 + 0, m0 + 1, m0 + 2, w.k_cache, w.v_cache, d.n_heads, d.n_kv_heads, (int)d.max_seq,
                   (int)d.rope_pairing, 1.0f / sqrtf(128.0f), d.rope_base};
        // Wo, plus the layer's input
        x[p0 + 3] = base + L.t; x_src[p0 + 3] = m0 + 3;
        packed[m0 + 4] = w.wo; y[m0 + 4] = base + L.h1; residual[m0 + 4] = h; residual_src[m0 + 4] = h_src;
        // the gated feed-forward on the normalized h1
        x[p0 + 4] = base + L.h1; x_src[p0 + 4] = m0 + 4; x_op[p0 + 4] = IFLOW_X_RMS_GAIN; aux[p0 + 4] = w.norm2; eps[p0 + 4] = d.eps;
        gated[p0 + 4] = 1;
        packed[m0 + 5] = w.w_gate; y[m0 + 5] = base + L.a;
        packed[m0 + 6] = w.w_up; y[m0 + 6] = nullptr;
        x[p0 + 5] = base + L.a; x_src[p0 + 5] = m0 + 5; cols[p0 + 5] = d.ffn;
        packed[m0 + 7] = w.w_down; y[m0 + 7] = l == d.n_layers - 1 ? d.h_out : base + L.h2;
        residual[m0 + 7] = base + L.h1; residual_src[m0 + 7] = m0 + 4;
    }
    iflow::ChainSpec spec = {(int)d.format, nphases, counts.data(), first.data(), cols.data(), x.data(), x_src.data(), packed.data(), rows.data(),
                             y.data(), x_op.data(), aux.data(), eps.data(), gated.data(), residual.data(), residual_src.data(),
                             kind.data(), attn_of.data(), d.n_layers, attn.data()};
    std::vector<uint8_t> host;
    if (!iflow::chain_build_plan(spec, grid, host)) return IFLOW_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    e = hipMemsetAsync(workspace, 0, ws_need, s);
    if (e == hipSuccess) e = hipMemcpyAsync(plan, host.data(), host.size(), hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return device_status(e);
    const int max_strips = std::max(iflow::chain_strips((int)d.format, d.hidden), iflow::chain_strips((int)d.format, d.ffn));
    chain->plan = plan; chain->workspace = workspace;
    chain->grid = grid; chain->max_strips = max_strips;
    chain->magic = IFLOW_CHAIN_MAGIC; chain->fused = 1u;
    chain->format = (int32_t)d.format; chain->lds_bytes = iflow::chain_lds_bytes((int)d.format, max_strips);
    chain->max_seq = d.max_seq;
    return IFLOW_OK;
}

iflow_status_t iflow_decode_stack_launch(const iflow_chain_t *chain, int64_t position, void *stream)
{
    if (!chain || !chain->plan || !chain->workspace) return IFLOW_ERR_NULL;
    if (chain->magic != IFLOW_CHAIN_MAGIC || chain->max_seq < 1 || chain->fused == 0) return IFLOW_ERR_SHAPE;
    if (position < 0 || position >= chain->max_seq) return IFLOW_ERR_SHAPE;
    hipError_t e = iflow::launch_chain(chain->plan, chain->workspace, chain->grid, chain->lds_bytes, true, (int)chain->format, (int)position,
                                       (hipStream_t)stream);
    if (e == hipErrorInvalidValue) return IFLOW_ERR_SHAPE;
    return device_status(e);
}

iflow_status_t iflow_calibration_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (!src || !dst) return IFLOW_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0) return IFLOW_ERR_SHAPE;
    if (!aligned16(src) || !aligned16(dst)) return IFLOW_ERR_ALIGN;
    return device_status(iflow::launch_calibration_copy(src, dst, bytes, (hipStream_t)stream));
}

iflow_status_t iflow_calibration_read(const void *src, size_t bytes, void *sink, void *stream)
{
    if (!src || !sink) return IFLOW_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0) return IFLOW_ERR_SHAPE;
    if (!aligned16(src) || !aligned16(sink)) return IFLOW_ERR_ALIGN;
    return device_status(iflow::launch_calibration_read(src, bytes, sink, (hipStream_t)stream));
}

iflow_status_t iflow_qgemv(iflow_format_t format, const void *packed, int64_t rows, int64_t cols,
                           const uint16_t *x, uint16_t *y, void *stream)
{
    return iflow_qgemm(format, packed, rows, cols, x, 1, y, stream);
}

}  // extern "C"
