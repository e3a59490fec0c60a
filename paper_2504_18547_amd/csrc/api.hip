// C ABI of libvitq.so: argument validation on the host, then kernel launches.
// No allocation, no synchronization; the only state is the per-device address of the static
// scratch array that vq_attention_block_static uses.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <atomic>

#include "../../include/vitq.h"
#include "attention.h"
#include "gemm.h"
#include "gemm_f6.h"
#include "layernorm.h"
#include "quantize.h"

using namespace vitq;

namespace {

constexpr int kMaxDevices = 64;

bool good_step(float s) { return isfinite(s) && s > 0.0f; }

int64_t row_bytes(const vq_qmat *m) { return (m->cols * m->storage_bits + 7) / 8; }
int64_t row_bytes16(const vq_qmat *m) { return (row_bytes(m) + 15) / 16 * 16; }

// Structural checks of a packed-matrix descriptor.
vq_status check_qmat(const vq_qmat *m, int want_unsigned) {
    if (!m) return VQ_ERR_NULL;
    if (m->rows < 0 || m->cols <= 0 || m->rows > INT32_MAX || m->cols > INT32_MAX) return VQ_ERR_SHAPE;
    if (m->storage_bits != 2 && m->storage_bits != 4 && m->storage_bits != 8) return VQ_ERR_BITS;
    if (m->bits < 2 || m->bits > 8 || m->bits > m->storage_bits) return VQ_ERR_BITS;
    if ((m->is_unsigned != 0) != (want_unsigned != 0)) return VQ_ERR_BITS;
    if (m->row_stride <= 0 || m->row_stride % 16 != 0 || m->row_stride < row_bytes(m)) return VQ_ERR_STRIDE;
    if (m->rows > 0 && !m->data) return VQ_ERR_NULL;
    if (((uintptr_t)m->data) % 16 != 0) return VQ_ERR_STRIDE;
    return VQ_OK;
}

void level_range(int bits, float *qminf, float *qmaxf) {
    *qminf = -(float)(1 << (bits - 1));
    *qmaxf = (float)((1 << (bits - 1)) - 1);
}

bool pair_supported(int wb, int ab) {
    return (wb == 4 && ab == 4) || (wb == 2 && ab == 4) || (wb == 8 && ab == 8);
}

struct LinearExtra {      // head-major output of the QKV linear inside the block
    int head_major = 0;
    int D = 0, dh = 0, Ntok = 0, Bimg = 0, Hh = 0;
    float s_q = 0, s_k = 0, s_v = 0;
    uint8_t *dst = nullptr; int sb = 0; int bits = 0;
    const float *hn_gamma = nullptr, *hn_beta = nullptr; float hn_eps = 0;   // per-head LayerNorm on Q, K
};

// Shared by vq_linear and vq_attention_block; all descriptors already validated.
vq_status run_linear(const vq_qmat *xq, float s_x, const vq_qmat *wq, const float *s_w,
                     int per_channel, const float *bias, int act, int32_t *acc_out, float *y_out,
                     float s_y, const vq_qmat *yq_out, const LinearExtra *ex, hipStream_t stream,
                     const void *wp = nullptr, const float *res = nullptr) {
    GemmParams p{};
    p.res = res;
    p.x = (const uint8_t *)xq->data; p.x_stride = xq->row_stride; p.M = (int)xq->rows;
    p.w = (const uint8_t *)wq->data; p.w_stride = wq->row_stride; p.Nout = (int)wq->rows;
    p.K = (int)xq->cols;
    p.kbytes_x16 = (int)row_bytes16(xq);
    p.kbytes_w16 = (int)row_bytes16(wq);
    p.s_x = s_x; p.s_w = s_w; p.s_w_per_channel = per_channel; p.bias = bias; p.act = act;
    p.acc_out = acc_out; p.y_out = y_out; p.vec_ok = (p.Nout % 4 == 0) ? 1 : 0;
    if (((uintptr_t)acc_out) % 16 || ((uintptr_t)y_out) % 16) p.vec_ok = 0;
    if (ex && ex->head_major) {
        p.head_major = 1;
        p.D = ex->D; p.dh = ex->dh; p.Ntok = ex->Ntok; p.Bimg = ex->Bimg; p.Hh = ex->Hh;
        p.s_y[0] = ex->s_q; p.s_y[1] = ex->s_k; p.s_y[2] = ex->s_v;
        p.hn_gamma = ex->hn_gamma; p.hn_beta = ex->hn_beta; p.hn_eps = ex->hn_eps;
        p.yq = ex->dst; p.yq_sb = ex->sb; p.yq_stride = (int64_t)ex->dh * ex->sb / 8;
        p.yq_row_bytes16 = (int)p.yq_stride;
        level_range(ex->bits, &p.qminf, &p.qmaxf);
    } else if (yq_out) {
        p.yq = (uint8_t *)yq_out->data; p.yq_stride = yq_out->row_stride; p.yq_sb = yq_out->storage_bits;
        p.yq_row_bytes16 = (int)row_bytes16(yq_out);
        p.s_y[0] = p.s_y[1] = p.s_y[2] = s_y;
        level_range(yq_out->bits, &p.qminf, &p.qmaxf);
    }
    if (p.M == 0 || p.Nout == 0) return VQ_OK;
    int wb = wq->storage_bits;
    if (wp && xq->storage_bits == 4 && (wb == 2 || wb == 4)) {
        // expanded int8 copy of the same weights: same products, no unpacking of W in the tiles
        const int64_t kp = (wq->cols + 15) / 16 * 16;
        p.w = (const uint8_t *)wp; p.w_stride = kp; p.kbytes_w16 = (int)kp;
        wb = 8;
    }
    hipError_t e = gemm_launch(p, wb, xq->storage_bits, stream);
    return e == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

vq_status check_linear_operands(const vq_qmat *xq, const vq_qmat *wq) {
    vq_status st;
    if ((st = check_qmat(xq, 0)) != VQ_OK) return st;
    if ((st = check_qmat(wq, 0)) != VQ_OK) return st;
    if (xq->cols != wq->cols) return VQ_ERR_SHAPE;
    if (xq->cols > 65536) return VQ_ERR_SHAPE;
    // the kernels keep a lane's operand offset inside a tile (up to 255 rows) in 32 bits
    if (xq->row_stride >= (1 << 24) || wq->row_stride >= (1 << 24)) return VQ_ERR_STRIDE;
    if (!pair_supported(wq->storage_bits, xq->storage_bits)) return VQ_ERR_UNSUPPORTED;
    return VQ_OK;
}

int pick_qsplit(int64_t heads, int N) {
    const int nqb = (N + 15) / 16;
    const int max_split = (nqb + 3) / 4;
    if (heads >= 512) return 1;
    int64_t want = (512 + heads - 1) / heads;
    if (want > max_split) want = max_split;
    return want < 1 ? 1 : (int)want;
}

// alpha = ((s_q*s_k)*scale)*log2(e) in fp32, then divided by the 2^shift operand factor.
// The division by a power of two must be exact for the kernel's product to round like the
// definition's; it is unless alpha is subnormal-small.
bool scaled_alpha(float s_q, float s_k, float scale, int shift, AttnParams *p) {
    const float kLog2e = 0x1.715476p+0f;
    float alpha = ((s_q * s_k) * scale) * kLog2e;
    if (!good_step(alpha)) return false;
    float scaled = ldexpf(alpha, -shift);
    if (!(ldexpf(scaled, shift) == alpha) || !isnormal(scaled)) return false;
    p->alpha_scaled = scaled;
    p->alpha = alpha;
    // Exponential table for 4-bit operands: the score difference d = max - S is an integer in
    // [0, 8192].  Beyond alpha*d >= 22.5 the fixed-point value is 0 (the shift is >= 22 and the
    // mantissa is < 2^22), so the table ends there with one shared zero entry.
    // The table is cut at kLutCap entries (filling it is per-workgroup work and it occupies LDS);
    // with very small alpha it then ends before the exponential reaches 0, and the kernel
    // computes the rare rows with a larger score spread directly.
    p->lut_n = 0;
    p->lut_full = 1;
    if (shift == 8) {
        const int kLutCap = 2048;
        double need = 22.5 / (double)alpha + 2.0;
        int n = need > 8193.0 ? 8193 : (int)need;
        if (n > kLutCap) { n = kLutCap; p->lut_full = 0; }
        p->lut_n = n + 1;
    }
    return true;
}

}  // namespace

extern "C" {

const char *vq_status_string(vq_status s) {
    switch (s) {
        case VQ_OK: return "ok";
        case VQ_ERR_NULL: return "required pointer is NULL";
        case VQ_ERR_SHAPE: return "bad or mismatching dimensions";
        case VQ_ERR_BITS: return "bad bit width / storage width / signedness";
        case VQ_ERR_STRIDE: return "row stride too small or stride/pointer not 16-byte aligned";
        case VQ_ERR_STEP: return "step size not a positive finite number";
        case VQ_ERR_UNSUPPORTED: return "no kernel for this combination";
        case VQ_ERR_WORKSPACE: return "workspace missing or too small";
        case VQ_ERR_HIP: return "HIP launch failed";
    }
    return "unknown status";
}

vq_status vq_weight_steps(const float *w, int64_t rows, int64_t cols, int64_t ld, int32_t bits,
                          float *step_out, void *stream) {
    if (rows < 0 || cols <= 0 || ld < cols) return VQ_ERR_SHAPE;
    if (bits < 2 || bits > 8) return VQ_ERR_BITS;
    if (rows == 0) return VQ_OK;
    if (!w || !step_out) return VQ_ERR_NULL;
    float qminf, qmaxf;
    level_range(bits, &qminf, &qmaxf);
    hipError_t e = weight_steps_launch(w, rows, cols, ld, qmaxf, step_out, (hipStream_t)stream);
    return e == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

vq_status vq_quantize(const float *x, int64_t rows, int64_t cols, int64_t ld, float step,
                      const float *step_per_row, const vq_qmat *out, void *stream) {
    vq_status st = check_qmat(out, 0);
    if (st != VQ_OK) return st;
    if (rows < 0 || cols <= 0 || ld < cols) return VQ_ERR_SHAPE;
    if (out->rows != rows || out->cols != cols) return VQ_ERR_SHAPE;
    if (!step_per_row && !good_step(step)) return VQ_ERR_STEP;
    if (rows == 0) return VQ_OK;
    if (!x) return VQ_ERR_NULL;
    QuantParams p{};
    p.x = x; p.rows = rows; p.cols = cols; p.ld = ld; p.step = step; p.step_per_row = step_per_row;
    p.out = (uint8_t *)out->data; p.out_stride = out->row_stride; p.sb = out->storage_bits;
    p.row_bytes16 = (int)row_bytes16(out);
    level_range(out->bits, &p.qminf, &p.qmaxf);
    hipError_t e = quantize_launch(p, (hipStream_t)stream);
    return e == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

vq_status vq_linear(const vq_qmat *xq, float s_x, const vq_qmat *wq, const float *s_w,
                    int32_t s_w_per_channel, const float *bias, int32_t act, int32_t *acc_out,
                    float *y_out, float s_y, const vq_qmat *yq_out, void *stream) {
    vq_status st = check_linear_operands(xq, wq);
    if (st != VQ_OK) return st;
    if (!s_w) return VQ_ERR_NULL;
    if (!acc_out && !y_out && !yq_out) return VQ_ERR_NULL;
    if (act != 0 && act != 1) return VQ_ERR_UNSUPPORTED;
    if (!good_step(s_x)) return VQ_ERR_STEP;
    if (yq_out) {
        if ((st = check_qmat(yq_out, 0)) != VQ_OK) return st;
        if (yq_out->rows != xq->rows || yq_out->cols != wq->rows) return VQ_ERR_SHAPE;
        if (!good_step(s_y)) return VQ_ERR_STEP;
    }
    return run_linear(xq, s_x, wq, s_w, s_w_per_channel ? 1 : 0, bias, act, acc_out, y_out, s_y, yq_out,
                      nullptr, (hipStream_t)stream);
}

// ---- absorbed mode: equivalent integer bias, integer comparator references -------------------
// Host arithmetic in double precision, in the stated order (one multiply, one divide per
// reference), so that any IEEE-754 host reproduces the same integers.
vq_status vq_absorb_thresholds(float s_x, const float *s_w, int32_t s_w_per_channel, const float *bias,
                               int64_t out_features, const float *s_y, int32_t s_y_per_channel, int32_t bits,
                               int32_t *b_int, int32_t *thr) {
    if (!s_w || !s_y || !b_int || !thr) return VQ_ERR_NULL;
    if (bits < 2 || bits > 8) return VQ_ERR_BITS;
    if (out_features < 0) return VQ_ERR_SHAPE;
    if (!good_step(s_x)) return VQ_ERR_STEP;
    const int qmin = -(1 << (bits - 1)), qmax = (1 << (bits - 1)) - 1;
    const int nthr = qmax - qmin;
    const double lo = -2147483648.0, hi = 2147483647.0;
    for (int64_t c = 0; c < out_features; ++c) {
        const float sw = s_w[s_w_per_channel ? c : 0], sy = s_y[s_y_per_channel ? c : 0];
        if (!good_step(sw) || !good_step(sy)) return VQ_ERR_STEP;
        const float scale32 = s_x * sw;                 // Eq. 2's post-scale, the fp32 product
        if (!good_step(scale32)) return VQ_ERR_STEP;
        const double scale = (double)scale32, step = (double)sy;
        double bi = bias ? std::rint((double)bias[c] / scale) : 0.0;     // nearest integer, ties to even
        bi = bi > hi ? hi : (bi < lo ? lo : bi);
        b_int[c] = (int32_t)bi;
        for (int t = 0; t < nthr; ++t) {
            const double kk = (double)(qmin + 1 + t) - 0.5;
            const double prod = kk * step;
            double T = std::floor(prod / scale);        // a > theta  <=>  a > floor(theta) for integer a
            T = T > hi ? hi : (T < lo ? lo : T);
            thr[c * nthr + t] = (int32_t)T;
        }
    }
    return VQ_OK;
}

vq_status vq_linear_absorbed(const vq_qmat *xq, const vq_qmat *wq, const int32_t *b_int, const int32_t *thr,
                             int32_t *acc_out, const vq_qmat *yq_out, void *stream) {
    vq_status st = check_linear_operands(xq, wq);
    if (st != VQ_OK) return st;
    if (!thr || !yq_out) return VQ_ERR_NULL;
    if ((st = check_qmat(yq_out, 0)) != VQ_OK) return st;
    if (yq_out->rows != xq->rows || yq_out->cols != wq->rows) return VQ_ERR_SHAPE;
    if (yq_out->storage_bits != 4 && yq_out->storage_bits != 8) return VQ_ERR_UNSUPPORTED;
    if (wq->rows % 16 != 0) return VQ_ERR_UNSUPPORTED;
    if (((uintptr_t)thr) % 4 != 0 || ((uintptr_t)b_int) % 4 != 0 || ((uintptr_t)acc_out) % 4 != 0) return VQ_ERR_STRIDE;
    if (xq->rows == 0 || wq->rows == 0) return VQ_OK;
    GemmParams p{};
    p.x = (const uint8_t *)xq->data; p.x_stride = xq->row_stride; p.M = (int)xq->rows;
    p.w = (const uint8_t *)wq->data; p.w_stride = wq->row_stride; p.Nout = (int)wq->rows;
    p.K = (int)xq->cols;
    p.kbytes_x16 = (int)row_bytes16(xq);
    p.kbytes_w16 = (int)row_bytes16(wq);
    hipStream_t stream_ = (hipStream_t)stream;
    if (acc_out) {
        // the accumulators on request (a parity aid): a separate pass through the plain epilogue
        GemmParams pa = p;
        pa.acc_out = acc_out;
        pa.s_x = 1.0f;
        pa.vec_ok = (p.Nout % 4 == 0 && ((uintptr_t)acc_out) % 16 == 0) ? 1 : 0;
        if (gemm_launch(pa, wq->storage_bits, xq->storage_bits, stream_) != hipSuccess) return VQ_ERR_HIP;
    }
    p.yq = (uint8_t *)yq_out->data; p.yq_stride = yq_out->row_stride; p.yq_sb = yq_out->storage_bits;
    p.yq_row_bytes16 = (int)row_bytes16(yq_out);
    level_range(yq_out->bits, &p.qminf, &p.qmaxf);
    p.ab_bint = b_int; p.ab_thr = thr; p.ab_nthr = (1 << yq_out->bits) - 1;
    return gemm_launch(p, wq->storage_bits, xq->storage_bits, stream_) == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

// ---- experimental 6-bit-float operand path ------------------------------------------------------
vq_status vq_recode_e3m2_bytes(const vq_qmat *m, size_t *bytes) {
    if (!bytes) return VQ_ERR_NULL;
    vq_status st = check_qmat(m, 0);
    if (st != VQ_OK) return st;
    if (m->storage_bits != 4) return VQ_ERR_UNSUPPORTED;
    *bytes = (size_t)(m->rows * f6_row_bytes(m->cols));
    return VQ_OK;
}

vq_status vq_recode_e3m2(const vq_qmat *m, void *out, size_t out_bytes, void *stream) {
    size_t need = 0;
    vq_status st = vq_recode_e3m2_bytes(m, &need);
    if (st != VQ_OK) return st;
    if (need == 0) return VQ_OK;
    if (!out) return VQ_ERR_NULL;
    if (((uintptr_t)out) % 16 != 0) return VQ_ERR_STRIDE;
    if (out_bytes < need) return VQ_ERR_WORKSPACE;
    RecodeParams p{};
    p.in = (const uint8_t *)m->data; p.in_stride = m->row_stride; p.in_row_bytes16 = (int)row_bytes16(m);
    p.rows = m->rows; p.cols = m->cols;
    p.out = (uint8_t *)out; p.out_stride = f6_row_bytes(m->cols);
    return recode_e3m2_launch(p, (hipStream_t)stream) == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

vq_status vq_linear_e3m2(const void *x6, int64_t rows, const void *w6, int64_t out_features, int64_t cols,
                         float s_x, const float *s_w, int32_t s_w_per_channel, const float *bias, float *y_out,
                         void *stream) {
    if (rows < 0 || out_features < 0 || cols <= 0 || cols > 65536) return VQ_ERR_SHAPE;
    if (rows > INT32_MAX || out_features > INT32_MAX) return VQ_ERR_SHAPE;
    if (!good_step(s_x)) return VQ_ERR_STEP;
    if (rows == 0 || out_features == 0) return VQ_OK;
    if (!x6 || !w6 || !s_w || !y_out) return VQ_ERR_NULL;
    if (((uintptr_t)x6) % 16 != 0 || ((uintptr_t)w6) % 16 != 0 || ((uintptr_t)y_out) % 4 != 0) return VQ_ERR_STRIDE;
    F6Params p{};
    p.x = (const uint8_t *)x6; p.x_stride = f6_row_bytes(cols); p.M = (int)rows;
    p.w = (const uint8_t *)w6; p.w_stride = f6_row_bytes(cols); p.Nout = (int)out_features;
    p.K = (int)cols;
    p.s_x = s_x; p.s_w = s_w; p.s_w_per_channel = s_w_per_channel ? 1 : 0; p.bias = bias; p.y_out = y_out;
    return gemm_f6_launch(p, (hipStream_t)stream) == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

vq_status vq_layernorm_quantize(const float *x, const float *residual, float *sum_out, int64_t rows,
                                int64_t cols, int64_t ld, const float *gamma, const float *beta, float eps,
                                float step, const vq_qmat *out, void *stream) {
    vq_status st = check_qmat(out, 0);
    if (st != VQ_OK) return st;
    if (rows < 0 || cols <= 0 || ld < cols || cols > (1 << 24)) return VQ_ERR_SHAPE;
    if (out->rows != rows || out->cols != cols) return VQ_ERR_SHAPE;
    if (!good_step(step) || !(eps >= 0.0f) || !isfinite(eps)) return VQ_ERR_STEP;
    if (rows == 0) return VQ_OK;
    if (!x || !gamma || !beta) return VQ_ERR_NULL;
    LnParams p{};
    p.x = x; p.res = residual; p.sum_out = sum_out; p.rows = rows; p.cols = cols; p.ld = ld;
    p.gamma = gamma; p.beta = beta; p.eps = eps; p.step = step;
    p.out = (uint8_t *)out->data; p.out_stride = out->row_stride; p.sb = out->storage_bits;
    p.row_bytes16 = (int)row_bytes16(out);
    p.qmin = -(1 << (out->bits - 1)); p.qmax = (1 << (out->bits - 1)) - 1;
    hipError_t e = layernorm_quantize_launch(p, (hipStream_t)stream);
    return e == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

vq_status vq_qkv_headnorm(const float *y, int64_t ld, int32_t B, int32_t H, int32_t N, const float *gamma,
                          const float *beta, float eps, float s_q, float s_k, float s_v, int32_t bits,
                          int32_t storage_bits, void *out, void *stream) {
    if (B < 0 || H <= 0 || N <= 0 || ld < 3 * 64 * (int64_t)H || ld % 4 != 0) return VQ_ERR_SHAPE;
    if ((int64_t)B * N * 3 * H > INT32_MAX) return VQ_ERR_SHAPE;
    if (storage_bits != 4 && storage_bits != 8) return VQ_ERR_BITS;
    if (bits < 2 || bits > storage_bits) return VQ_ERR_BITS;
    if (!good_step(s_q) || !good_step(s_k) || !good_step(s_v) || !(eps >= 0.0f) || !isfinite(eps))
        return VQ_ERR_STEP;
    if (B == 0) return VQ_OK;
    if (!y || !gamma || !beta || !out) return VQ_ERR_NULL;
    if (((uintptr_t)y) % 16 || ((uintptr_t)out) % 16 || ((uintptr_t)gamma) % 16 || ((uintptr_t)beta) % 16)
        return VQ_ERR_STRIDE;
    HeadNormParams hp{};
    hp.y = y; hp.ld = ld; hp.B = B; hp.H = H; hp.N = N; hp.D = 64 * H;
    hp.gamma = gamma; hp.beta = beta; hp.eps = eps; hp.s_q = s_q; hp.s_k = s_k; hp.s_v = s_v;
    hp.out = (uint8_t *)out; hp.sb = storage_bits; hp.qmin = -(1 << (bits - 1)); hp.qmax = (1 << (bits - 1)) - 1;
    return qkv_headnorm_launch(hp, (hipStream_t)stream) == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

vq_status vq_prepack_weight_bytes(const vq_qmat *w, size_t *bytes) {
    if (!bytes) return VQ_ERR_NULL;
    vq_status st = check_qmat(w, 0);
    if (st != VQ_OK) return st;
    if (w->storage_bits != 2 && w->storage_bits != 4) return VQ_ERR_UNSUPPORTED;
    *bytes = (size_t)w->rows * (size_t)((w->cols + 15) / 16 * 16);
    return VQ_OK;
}

vq_status vq_prepack_weight(const vq_qmat *w, void *out, size_t out_bytes, void *stream) {
    size_t need = 0;
    vq_status st = vq_prepack_weight_bytes(w, &need);
    if (st != VQ_OK) return st;
    if (need == 0) return VQ_OK;
    if (!out) return VQ_ERR_NULL;
    if (out_bytes < need || ((uintptr_t)out) % 16 != 0) return VQ_ERR_WORKSPACE;
    hipError_t e = prepack_launch((const uint8_t *)w->data, w->rows, w->cols, w->row_stride, w->storage_bits,
                                  (int8_t *)out, (w->cols + 15) / 16 * 16, (hipStream_t)stream);
    return e == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

vq_status vq_linear_prepacked(const vq_qmat *xq, float s_x, const vq_qmat *wq, const void *wp,
                              const float *s_w, int32_t s_w_per_channel, const float *bias, int32_t act,
                              int32_t *acc_out, float *y_out, float s_y, const vq_qmat *yq_out,
                              void *stream) {
    vq_status st = check_linear_operands(xq, wq);
    if (st != VQ_OK) return st;
    if (!s_w || !wp) return VQ_ERR_NULL;
    if (xq->storage_bits != 4 || (wq->storage_bits != 2 && wq->storage_bits != 4)) return VQ_ERR_UNSUPPORTED;
    if (((uintptr_t)wp) % 16 != 0) return VQ_ERR_STRIDE;
    if (!acc_out && !y_out && !yq_out) return VQ_ERR_NULL;
    if (act != 0 && act != 1) return VQ_ERR_UNSUPPORTED;
    if (!good_step(s_x)) return VQ_ERR_STEP;
    if (yq_out) {
        if ((st = check_qmat(yq_out, 0)) != VQ_OK) return st;
        if (yq_out->rows != xq->rows || yq_out->cols != wq->rows) return VQ_ERR_SHAPE;
        if (!good_step(s_y)) return VQ_ERR_STEP;
    }
    return run_linear(xq, s_x, wq, s_w, s_w_per_channel ? 1 : 0, bias, act, acc_out, y_out, s_y, yq_out,
                      nullptr, (hipStream_t)stream, wp);
}

vq_status vq_matmul_qk(const vq_qmat *q, const vq_qmat *k, int32_t B, int32_t H, int32_t N,
                       float s_q, float s_k, float scale, int32_t *s_acc_out,
                       const vq_qmat *p_out, void *stream) {
    vq_status st;
    if ((st = check_qmat(q, 0)) != VQ_OK) return st;
    if ((st = check_qmat(k, 0)) != VQ_OK) return st;
    if (B < 0 || H <= 0 || N <= 0) return VQ_ERR_SHAPE;
    const int64_t rows = (int64_t)B * H * N;
    if (rows > INT32_MAX) return VQ_ERR_SHAPE;
    if (q->cols != 64 || k->cols != 64) return VQ_ERR_UNSUPPORTED;
    if (q->rows != rows || k->rows != rows) return VQ_ERR_SHAPE;
    if (q->storage_bits != k->storage_bits) return VQ_ERR_BITS;
    if (q->storage_bits != 4 && q->storage_bits != 8) return VQ_ERR_UNSUPPORTED;
    if (N > 592) return VQ_ERR_UNSUPPORTED;
    if (!s_acc_out && !p_out) return VQ_ERR_NULL;
    if (!good_step(s_q) || !good_step(s_k) || !good_step(scale)) return VQ_ERR_STEP;
    AttnParams p{};
    p.pmax = 15; p.p_sb = 4;
    if (p_out) {
        if ((st = check_qmat(p_out, 1)) != VQ_OK) return st;
        if (p_out->rows != rows || p_out->cols != N) return VQ_ERR_SHAPE;
        if (p_out->storage_bits != 4 && p_out->storage_bits != 8) return VQ_ERR_UNSUPPORTED;
        p.pmax = (1 << p_out->bits) - 1;
        p.p_sb = p_out->storage_bits;
        p.p_out = (uint8_t *)p_out->data; p.p_out_stride = p_out->row_stride;
        p.p_out_row_bytes16 = (int)row_bytes16(p_out);
    }
    if (!scaled_alpha(s_q, s_k, scale, q->storage_bits == 4 ? 8 : 0, &p)) return VQ_ERR_STEP;
    if (rows == 0) return VQ_OK;
    p.q = (const uint8_t *)q->data; p.k = (const uint8_t *)k->data;
    p.q_stride = q->row_stride; p.k_stride = k->row_stride; p.sb = q->storage_bits;
    p.B = B; p.H = H; p.N = N;
    p.s_acc_out = s_acc_out;
    p.qsplit = pick_qsplit((int64_t)B * H, N);
    hipError_t e = attention_launch(p, kAttnQKOnly, (hipStream_t)stream);
    return e == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

vq_status vq_matmul_pv(const vq_qmat *pm, const vq_qmat *v, int32_t B, int32_t H, int32_t N,
                       float s_p, float s_v, int32_t *o_acc_out, float *o_out, float s_o,
                       const vq_qmat *oq_out, void *stream) {
    vq_status st;
    if ((st = check_qmat(pm, 1)) != VQ_OK) return st;
    if ((st = check_qmat(v, 0)) != VQ_OK) return st;
    if (B < 0 || H <= 0 || N <= 0) return VQ_ERR_SHAPE;
    const int64_t rows = (int64_t)B * H * N;
    if (rows > INT32_MAX) return VQ_ERR_SHAPE;
    if (v->cols != 64) return VQ_ERR_UNSUPPORTED;
    if (v->rows != rows || pm->rows != rows || pm->cols != N) return VQ_ERR_SHAPE;
    if (v->storage_bits != 4 && v->storage_bits != 8) return VQ_ERR_UNSUPPORTED;
    if (pm->storage_bits != 4 && pm->storage_bits != 8) return VQ_ERR_UNSUPPORTED;
    if (N > 592) return VQ_ERR_UNSUPPORTED;
    if (!o_acc_out && !o_out && !oq_out) return VQ_ERR_NULL;
    if (!good_step(s_p) || !good_step(s_v)) return VQ_ERR_STEP;
    if (((uintptr_t)o_acc_out) % 16 || ((uintptr_t)o_out) % 16) return VQ_ERR_STRIDE;
    AttnParams p{};
    if (oq_out) {
        if ((st = check_qmat(oq_out, 0)) != VQ_OK) return st;
        if (oq_out->rows != (int64_t)B * N || oq_out->cols != (int64_t)H * 64) return VQ_ERR_SHAPE;
        if (oq_out->storage_bits != 4 && oq_out->storage_bits != 8) return VQ_ERR_UNSUPPORTED;
        if (!good_step(s_o)) return VQ_ERR_STEP;
        p.oq = (uint8_t *)oq_out->data; p.oq_stride = oq_out->row_stride; p.oq_sb = oq_out->storage_bits;
        level_range(oq_out->bits, &p.qminf, &p.qmaxf);
        p.s_o = s_o;
    } else {
        p.s_o = 1.0f; p.qminf = -8.0f; p.qmaxf = 7.0f;
    }
    if (rows == 0) return VQ_OK;
    p.v = (const uint8_t *)v->data; p.v_stride = v->row_stride; p.sb = v->storage_bits;
    p.p_in = (const uint8_t *)pm->data; p.p_in_stride = pm->row_stride;
    p.p_in_row_bytes16 = (int)row_bytes16(pm);
    p.p_sb = pm->storage_bits; p.pmax = (1 << pm->bits) - 1;
    p.B = B; p.H = H; p.N = N;
    p.spv = s_p * s_v;
    p.o_acc_out = o_acc_out; p.o_out = o_out;
    p.qsplit = pick_qsplit((int64_t)B * H, N);
    p.r_o = 1.0f / p.s_o; p.eps_o = ldexpf(1.0f, (p.qmaxf > 7.5f ? 8 : 4) - 22);
    hipError_t e = attention_launch(p, kAttnPVOnly, (hipStream_t)stream);
    return e == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

// ---- the whole block ----------------------------------------------------------------------

namespace {

struct BlockLayout {
    int64_t M; int sa; int dh;
    size_t qkv_off, o_off, x2_off, h_off, y3_off, total;
    int64_t qkv_bytes, act_row, h_row;
};

size_t align256(size_t v) { return (v + 255) / 256 * 256; }

vq_status block_check(const vq_block_desc *d, int64_t B, BlockLayout *L) {
    if (!d) return VQ_ERR_NULL;
    if (d->D <= 0 || d->H <= 0 || d->N <= 0 || d->hidden < 0 || B < 0) return VQ_ERR_SHAPE;
    if (d->D % d->H != 0) return VQ_ERR_SHAPE;
    if (d->D / d->H != 64) return VQ_ERR_UNSUPPORTED;
    if (d->N > 592) return VQ_ERR_UNSUPPORTED;
    if (d->hidden % 64 != 0) return VQ_ERR_SHAPE;
    if (d->storage_a != 4 && d->storage_a != 8) return VQ_ERR_BITS;
    if (d->bits_a < 2 || d->bits_a > d->storage_a) return VQ_ERR_BITS;
    if (d->bits_p < 2 || d->bits_p > d->storage_a) return VQ_ERR_BITS;
    if ((int64_t)B * d->N > INT32_MAX / 4 || (int64_t)B * d->H * d->N > INT32_MAX / 4) return VQ_ERR_SHAPE;
    // the head-major store of the QKV linear splits a token row into (image, token) with an fp32
    // reciprocal that is exact below 2^22 rows
    if ((int64_t)B * d->N >= (1 << 22)) return VQ_ERR_SHAPE;
    L->M = B * d->N; L->sa = d->storage_a; L->dh = 64;
    L->act_row = (int64_t)d->D * L->sa / 8;
    L->h_row = (int64_t)d->hidden * L->sa / 8;
    L->qkv_bytes = 3 * B * d->H * d->N * (64 * L->sa / 8);
    size_t off = 0;
    L->qkv_off = off; off += align256((size_t)L->qkv_bytes);
    L->o_off = off;   off += align256((size_t)(L->M * L->act_row));
    L->x2_off = off;  off += d->hidden ? align256((size_t)(L->M * L->act_row)) : 0;
    L->h_off = off;   off += d->hidden ? align256((size_t)(L->M * L->h_row)) : 0;
    L->y3_off = off;  off += d->qk_gamma ? align256((size_t)L->M * 3 * d->D * sizeof(float)) : 0;   // fp32 QKV
    L->total = off;
    return VQ_OK;
}

vq_status weight_check(const vq_qmat *w, int64_t rows, int64_t cols, int sa, const float *sw) {
    vq_status st = check_qmat(w, 0);
    if (st != VQ_OK) return st;
    if (w->rows != rows || w->cols != cols) return VQ_ERR_SHAPE;
    if (!pair_supported(w->storage_bits, sa)) return VQ_ERR_UNSUPPORTED;
    if (!sw) return VQ_ERR_NULL;
    return VQ_OK;
}

void block_qkv_extra(const vq_block_desc *d, const BlockLayout &L, int64_t B, uint8_t *qkv, LinearExtra &ex) {
    ex.head_major = 1; ex.D = d->D; ex.dh = 64; ex.Ntok = d->N; ex.Bimg = (int)B; ex.Hh = d->H;
    ex.s_q = d->s_q; ex.s_k = d->s_k; ex.s_v = d->s_v; ex.dst = qkv; ex.sb = L.sa; ex.bits = d->bits_a;
}

void block_attention_params(const vq_block_desc *d, const BlockLayout &L, const AttnParams &ap, int64_t B,
                            uint8_t *qkv, uint8_t *obuf, AttnParams &p) {
    const int64_t BHN = B * d->H * d->N;
    const int64_t hrow = 64 * L.sa / 8;
    p = ap;
    p.q = qkv; p.k = qkv + BHN * hrow; p.v = qkv + 2 * BHN * hrow;
    p.q_stride = p.k_stride = p.v_stride = hrow;
    p.sb = L.sa; p.B = (int)B; p.H = d->H; p.N = d->N;
    p.pmax = (1 << d->bits_p) - 1;
    p.p_sb = L.sa;
    p.spv = (1.0f / (float)p.pmax) * d->s_v;
    p.s_o = d->s_o;
    level_range(d->bits_a, &p.qminf, &p.qmaxf);
    p.oq = obuf; p.oq_stride = L.act_row; p.oq_sb = L.sa;
    p.qsplit = pick_qsplit((int64_t)B * d->H, d->N);
    p.r_o = 1.0f / p.s_o; p.eps_o = ldexpf(1.0f, (p.qmaxf > 7.5f ? 8 : 4) - 22);
}

// QKV stage of both block entry points: the linear with the head-major requantizing epilogue
// (plain quantizers, or the per-head LayerNorm quantizers of Q and K inside that epilogue), or,
// for steps the fused epilogue does not take, the linear in fp32 and then vq_qkv_headnorm's kernel.
vq_status run_qkv_stage(const vq_block_desc *d, const BlockLayout &L, const vq_qmat *xq, int64_t B, uint8_t *qkv,
                        uint8_t *ws, hipStream_t stream) {
    // With 64-channel heads the per-head LayerNorm quantizers run inside the linear's epilogue
    // (its fast paths need steps whose reciprocals are ordinary numbers).
    auto ordinary = [](float s) { const float r = 1.0f / s; return r > 0x1p-100f && r < 0x1p100f; };
    const bool fused_norm = d->qk_gamma && d->D % 64 == 0 && ordinary(d->s_q) && ordinary(d->s_k) && ordinary(d->s_v);
    if (!d->qk_gamma || fused_norm) {
        LinearExtra ex;
        block_qkv_extra(d, L, B, qkv, ex);
        if (fused_norm) { ex.hn_gamma = d->qk_gamma; ex.hn_beta = d->qk_beta; ex.hn_eps = d->qk_eps; }
        return run_linear(xq, d->s_x, &d->w_qkv, d->sw_qkv, 1, d->b_qkv, 0, nullptr, nullptr, 0.0f, nullptr, &ex,
                          stream, d->wp_qkv);
    }
    float *y3 = reinterpret_cast<float *>(ws + L.y3_off);
    vq_status st = run_linear(xq, d->s_x, &d->w_qkv, d->sw_qkv, 1, d->b_qkv, 0, nullptr, y3, 0.0f, nullptr,
                              nullptr, stream, d->wp_qkv);
    if (st != VQ_OK) return st;
    HeadNormParams hp{};
    hp.y = y3; hp.ld = 3 * (int64_t)d->D; hp.B = (int)B; hp.H = d->H; hp.N = d->N; hp.D = d->D;
    hp.gamma = d->qk_gamma; hp.beta = d->qk_beta; hp.eps = d->qk_eps;
    hp.s_q = d->s_q; hp.s_k = d->s_k; hp.s_v = d->s_v;
    hp.out = qkv; hp.sb = L.sa; hp.qmin = -(1 << (d->bits_a - 1)); hp.qmax = (1 << (d->bits_a - 1)) - 1;
    return qkv_headnorm_launch(hp, stream) == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

// Checks shared by the two block entry points (weights, steps, prepacked copies, dumps).
vq_status block_args_check(const vq_block_desc *d, const BlockLayout &L, AttnParams *ap) {
    vq_status st;
    if ((st = weight_check(&d->w_qkv, 3 * (int64_t)d->D, d->D, L.sa, d->sw_qkv)) != VQ_OK) return st;
    if ((st = weight_check(&d->w_proj, d->D, d->D, L.sa, d->sw_proj)) != VQ_OK) return st;
    if (d->hidden) {
        if ((st = weight_check(&d->w_fc1, d->hidden, d->D, L.sa, d->sw_fc1)) != VQ_OK) return st;
        if ((st = weight_check(&d->w_fc2, d->D, d->hidden, L.sa, d->sw_fc2)) != VQ_OK) return st;
        if (!good_step(d->s_x2) || !good_step(d->s_h)) return VQ_ERR_STEP;
    }
    if (!good_step(d->s_x) || !good_step(d->s_q) || !good_step(d->s_k) || !good_step(d->s_v) ||
        !good_step(d->s_o) || !good_step(d->scale))
        return VQ_ERR_STEP;
    if (!scaled_alpha(d->s_q, d->s_k, d->scale, L.sa == 4 ? 8 : 0, ap)) return VQ_ERR_STEP;
    for (void *dp : {d->dump_qkv, d->dump_o, d->dump_x2, d->dump_h})
        if (((uintptr_t)dp) % 16 != 0) return VQ_ERR_STRIDE;
    if ((d->qk_gamma == nullptr) != (d->qk_beta == nullptr)) return VQ_ERR_NULL;
    if (d->qk_gamma && (!(d->qk_eps >= 0.0f) || !isfinite(d->qk_eps))) return VQ_ERR_STEP;
    const int have = (d->wp_qkv != nullptr) + (d->wp_proj != nullptr) + (d->wp_fc1 != nullptr) +
                     (d->wp_fc2 != nullptr);
    if (have != 0 && have != (d->hidden ? 4 : 2)) return VQ_ERR_NULL;
    if (have != 0 && (!d->wp_qkv || !d->wp_proj)) return VQ_ERR_NULL;
    for (const void *wp : {d->wp_qkv, d->wp_proj, d->wp_fc1, d->wp_fc2})
        if (((uintptr_t)wp) % 16 != 0) return VQ_ERR_STRIDE;
    return VQ_OK;
}

}  // namespace

vq_status vq_attention_block_workspace(const vq_block_desc *desc, int64_t B, size_t *bytes) {
    if (!bytes) return VQ_ERR_NULL;
    BlockLayout L;
    vq_status st = block_check(desc, B, &L);
    if (st != VQ_OK) return st;
    *bytes = L.total;
    return VQ_OK;
}

namespace {

// Body of both block entry points: every check on the host first, then the launches.
vq_status run_attention_block(const vq_block_desc *d, const vq_qmat *xq, int64_t B, float *y_out,
                              void *workspace, size_t workspace_bytes, void *stream_) {
    BlockLayout L;
    vq_status st = block_check(d, B, &L);
    if (st != VQ_OK) return st;
    hipStream_t stream = (hipStream_t)stream_;
    if ((st = check_qmat(xq, 0)) != VQ_OK) return st;
    if (xq->rows != L.M || xq->cols != d->D || xq->storage_bits != L.sa) return VQ_ERR_SHAPE;
    AttnParams ap{};
    if ((st = block_args_check(d, L, &ap)) != VQ_OK) return st;
    if (B == 0) return VQ_OK;
    if (!y_out) return VQ_ERR_NULL;
    if (!workspace || workspace_bytes < L.total) return VQ_ERR_WORKSPACE;
    if (((uintptr_t)workspace) % 256 != 0) return VQ_ERR_WORKSPACE;
    if (((uintptr_t)y_out) % 16 != 0) return VQ_ERR_STRIDE;

    uint8_t *ws = (uint8_t *)workspace;
    uint8_t *qkv = d->dump_qkv ? (uint8_t *)d->dump_qkv : ws + L.qkv_off;
    uint8_t *obuf = d->dump_o ? (uint8_t *)d->dump_o : ws + L.o_off;
    uint8_t *x2buf = d->dump_x2 ? (uint8_t *)d->dump_x2 : ws + L.x2_off;
    uint8_t *hbuf = d->dump_h ? (uint8_t *)d->dump_h : ws + L.h_off;

    int ev = 0;
    auto mark = [&]() {
        if (d->stage_events) (void)hipEventRecord((hipEvent_t)d->stage_events[ev], stream);
        ++ev;
    };
    mark();
    // 1. QKV linear; the epilogue requantizes Q, K, V with their own steps, head-major
    st = run_qkv_stage(d, L, xq, B, qkv, ws, stream);
    if (st != VQ_OK) return st;
    mark();

    // 2. fused attention: scores and P never leave the chip
    vq_qmat oq{};
    oq.data = obuf; oq.bits = d->bits_a; oq.storage_bits = L.sa; oq.rows = L.M; oq.cols = d->D;
    oq.row_stride = L.act_row;
    {
        AttnParams p;
        block_attention_params(d, L, ap, B, qkv, obuf, p);
        if (attention_launch(p, kAttnFused, stream) != hipSuccess) return VQ_ERR_HIP;
    }
    mark();

    // 3. projection (fp32 out, or requantized for the MLP)
    if (!d->hidden) {
        st = run_linear(&oq, d->s_o, &d->w_proj, d->sw_proj, 1, d->b_proj, 0, nullptr, y_out, 0.0f, nullptr,
                        nullptr, stream, d->wp_proj);
        mark();
        return st;
    }
    vq_qmat x2{};
    x2.data = x2buf; x2.bits = d->bits_a; x2.storage_bits = L.sa; x2.rows = L.M; x2.cols = d->D;
    x2.row_stride = L.act_row;
    st = run_linear(&oq, d->s_o, &d->w_proj, d->sw_proj, 1, d->b_proj, 0, nullptr, nullptr, d->s_x2, &x2, nullptr,
                    stream, d->wp_proj);
    if (st != VQ_OK) return st;
    mark();
    // 4. fc1 + GELU + requant, 5. fc2
    vq_qmat hq{};
    hq.data = hbuf; hq.bits = d->bits_a; hq.storage_bits = L.sa; hq.rows = L.M; hq.cols = d->hidden;
    hq.row_stride = L.h_row;
    st = run_linear(&x2, d->s_x2, &d->w_fc1, d->sw_fc1, 1, d->b_fc1, 1, nullptr, nullptr, d->s_h, &hq, nullptr,
                    stream, d->wp_fc1);
    if (st != VQ_OK) return st;
    mark();
    st = run_linear(&hq, d->s_h, &d->w_fc2, d->sw_fc2, 1, d->b_fc2, 0, nullptr, y_out, 0.0f, nullptr, nullptr,
                    stream, d->wp_fc2);
    mark();
    return st;
}

// The intermediates of vq_attention_block_static (packed Q/K/V, O, X2, H): one array per GPU, held
// until the process ends.  The name below is a host-side handle only; the device address comes
// from hipGetSymbolAddress, once per device, and that pointer is what the kernels receive.
static __device__ __align__(256) unsigned char scratch[VQ_STATIC_SCRATCH_BYTES];
std::atomic<void *> g_scratch_ptr[kMaxDevices];

vq_status static_scratch(void **out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return VQ_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return VQ_ERR_UNSUPPORTED;
    void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return VQ_ERR_HIP;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);     // (racing first calls store the same address)
    }
    *out = ptr;
    return VQ_OK;
}

}  // namespace

vq_status vq_attention_block(const vq_block_desc *d, const vq_qmat *xq, int64_t B, float *y_out,
                             void *workspace, size_t workspace_bytes, void *stream) {
    return run_attention_block(d, xq, B, y_out, workspace, workspace_bytes, stream);
}

vq_status vq_attention_block_static(const vq_block_desc *d, const vq_qmat *xq, int64_t B, float *y_out,
                                    void *stream) {
    BlockLayout L;
    vq_status st = block_check(d, B, &L);
    if (st != VQ_OK) return st;
    if (d->qk_gamma) return VQ_ERR_UNSUPPORTED;                   // (its fallback stages an fp32 QKV matrix)
    if (L.total > (size_t)VQ_STATIC_SCRATCH_BYTES) return VQ_ERR_WORKSPACE;
    void *ws = nullptr;
    if ((st = static_scratch(&ws)) != VQ_OK) return st;
    return run_attention_block(d, xq, B, y_out, ws, (size_t)VQ_STATIC_SCRATCH_BYTES, stream);
}

vq_status vq_vit_block_workspace(const vq_preln_desc *desc, int64_t B, size_t *bytes) {
    if (!bytes) return VQ_ERR_NULL;
    if (!desc) return VQ_ERR_NULL;
    BlockLayout L;
    vq_status st = block_check(&desc->block, B, &L);
    if (st != VQ_OK) return st;
    if (desc->block.hidden <= 0) return VQ_ERR_SHAPE;
    *bytes = L.total + align256((size_t)(L.M * L.act_row));      // + the LayerNorm-1 output X_q
    return VQ_OK;
}

namespace {

// Every host-side check of vq_vit_block (nothing is launched here).
vq_status vit_block_check(const vq_preln_desc *desc, const float *x, int64_t B, const float *y_out,
                          const void *workspace, size_t workspace_bytes, BlockLayout *L, AttnParams *ap) {
    if (!desc) return VQ_ERR_NULL;
    const vq_block_desc *d = &desc->block;
    vq_status st = block_check(d, B, L);
    if (st != VQ_OK) return st;
    if (d->hidden <= 0) return VQ_ERR_SHAPE;
    if ((st = block_args_check(d, *L, ap)) != VQ_OK) return st;
    if (!(desc->ln_eps >= 0.0f) || !isfinite(desc->ln_eps)) return VQ_ERR_STEP;
    if (!desc->ln1_gamma || !desc->ln1_beta || !desc->ln2_gamma || !desc->ln2_beta) return VQ_ERR_NULL;
    if (B == 0) return VQ_OK;
    if (!x || !y_out) return VQ_ERR_NULL;
    {   // in place is fine (x is last read as the residual, element by element, by the lane that then
        // writes x1 there); any other overlap is not
        const uintptr_t xa = (uintptr_t)x, ya = (uintptr_t)y_out;
        const uintptr_t bytes = (uintptr_t)L->M * (uintptr_t)d->D * sizeof(float);
        if (xa != ya && xa < ya + bytes && ya < xa + bytes) return VQ_ERR_STRIDE;
    }
    const size_t xq_bytes = align256((size_t)(L->M * L->act_row));
    if (!workspace || workspace_bytes < L->total + xq_bytes) return VQ_ERR_WORKSPACE;
    if (((uintptr_t)workspace) % 256 != 0) return VQ_ERR_WORKSPACE;
    if (((uintptr_t)y_out) % 16 != 0 || ((uintptr_t)x) % 16 != 0 || ((uintptr_t)desc->dump_xq) % 16 != 0)
        return VQ_ERR_STRIDE;
    return VQ_OK;
}

// The launches of vq_vit_block, after vit_block_check has passed.
vq_status vit_block_run(const vq_preln_desc *desc, const BlockLayout &L, const AttnParams &ap, const float *x,
                        int64_t B, float *y_out, void *workspace, hipStream_t stream) {
    const vq_block_desc *d = &desc->block;
    vq_status st;
    uint8_t *ws = (uint8_t *)workspace;
    uint8_t *qkv = d->dump_qkv ? (uint8_t *)d->dump_qkv : ws + L.qkv_off;
    uint8_t *obuf = d->dump_o ? (uint8_t *)d->dump_o : ws + L.o_off;
    uint8_t *x2buf = d->dump_x2 ? (uint8_t *)d->dump_x2 : ws + L.x2_off;
    uint8_t *hbuf = d->dump_h ? (uint8_t *)d->dump_h : ws + L.h_off;
    uint8_t *xqbuf = desc->dump_xq ? (uint8_t *)desc->dump_xq : ws + L.total;
    auto act = [&](uint8_t *data, int64_t cols, int64_t stride) {
        vq_qmat m{};
        m.data = data; m.bits = d->bits_a; m.storage_bits = L.sa; m.rows = L.M; m.cols = cols; m.row_stride = stride;
        return m;
    };
    const vq_qmat xq = act(xqbuf, d->D, L.act_row), oq = act(obuf, d->D, L.act_row);
    const vq_qmat x2 = act(x2buf, d->D, L.act_row), hq = act(hbuf, d->hidden, L.h_row);
    int qmin = -(1 << (d->bits_a - 1)), qmax = (1 << (d->bits_a - 1)) - 1;
    auto lnq = [&](const float *src, const float *gamma, const float *beta, float step, const vq_qmat &out) {
        LnParams p{};
        p.x = src; p.rows = L.M; p.cols = d->D; p.ld = d->D; p.gamma = gamma; p.beta = beta;
        p.eps = desc->ln_eps; p.step = step;
        p.out = (uint8_t *)out.data; p.out_stride = out.row_stride; p.sb = out.storage_bits;
        p.row_bytes16 = (int)row_bytes16(&out); p.qmin = qmin; p.qmax = qmax;
        return layernorm_quantize_launch(p, stream) == hipSuccess ? VQ_OK : VQ_ERR_HIP;
    };

    // 1. X_q = LayerNorm-1 quantizer of the stream
    if ((st = lnq(x, desc->ln1_gamma, desc->ln1_beta, d->s_x, xq)) != VQ_OK) return st;
    // 2. QKV linear, fused attention
    st = run_qkv_stage(d, L, &xq, B, qkv, ws, stream);
    if (st != VQ_OK) return st;
    {
        AttnParams p;
        block_attention_params(d, L, ap, B, qkv, obuf, p);
        if (attention_launch(p, kAttnFused, stream) != hipSuccess) return VQ_ERR_HIP;
    }
    // 3. x1 = proj(O_q) + x, written to y_out
    st = run_linear(&oq, d->s_o, &d->w_proj, d->sw_proj, 1, d->b_proj, 0, nullptr, y_out, 0.0f, nullptr, nullptr,
                    stream, d->wp_proj, x);
    if (st != VQ_OK) return st;
    if (desc->dump_x1) {
        if (hipMemcpyAsync(desc->dump_x1, y_out, (size_t)L.M * d->D * sizeof(float), hipMemcpyDeviceToDevice,
                           stream) != hipSuccess)
            return VQ_ERR_HIP;
    }
    // 4. X2_q = LayerNorm-2 quantizer of x1
    if ((st = lnq(y_out, desc->ln2_gamma, desc->ln2_beta, d->s_x2, x2)) != VQ_OK) return st;
    // 5. fc1 + GELU + requant, 6. y = fc2(H_q) + x1, in place
    st = run_linear(&x2, d->s_x2, &d->w_fc1, d->sw_fc1, 1, d->b_fc1, 1, nullptr, nullptr, d->s_h, &hq, nullptr,
                    stream, d->wp_fc1);
    if (st != VQ_OK) return st;
    return run_linear(&hq, d->s_h, &d->w_fc2, d->sw_fc2, 1, d->b_fc2, 0, nullptr, y_out, 0.0f, nullptr, nullptr,
                      stream, d->wp_fc2, y_out);
}

}  // namespace

vq_status vq_vit_block(const vq_preln_desc *desc, const float *x, int64_t B, float *y_out, void *workspace,
                       size_t workspace_bytes, void *stream) {
    BlockLayout L;
    AttnParams ap{};
    vq_status st = vit_block_check(desc, x, B, y_out, workspace, workspace_bytes, &L, &ap);
    if (st != VQ_OK || B == 0) return st;
    return vit_block_run(desc, L, ap, x, B, y_out, workspace, (hipStream_t)stream);
}

vq_status vq_vit_encoder_workspace(const vq_preln_desc *layers, int32_t n_layers, int64_t B, size_t *bytes) {
    if (!layers || !bytes) return VQ_ERR_NULL;
    if (n_layers < 1) return VQ_ERR_SHAPE;
    size_t need = 0;
    for (int32_t i = 0; i < n_layers; ++i) {
        size_t n = 0;
        vq_status st = vq_vit_block_workspace(&layers[i], B, &n);
        if (st != VQ_OK) return st;
        need = n > need ? n : need;
        const vq_block_desc &a = layers[0].block, &b = layers[i].block;
        if (a.D != b.D || a.H != b.H || a.N != b.N || a.bits_a != b.bits_a || a.bits_p != b.bits_p ||
            a.storage_a != b.storage_a)
            return VQ_ERR_SHAPE;
    }
    *bytes = need;
    return VQ_OK;
}

vq_status vq_vit_encoder(const vq_preln_desc *layers, int32_t n_layers, const float *x, int64_t B, float *y_out,
                         void *workspace, size_t workspace_bytes, void *stream) {
    size_t need = 0;
    vq_status st = vq_vit_encoder_workspace(layers, n_layers, B, &need);
    if (st != VQ_OK) return st;
    if (workspace_bytes < need) return VQ_ERR_WORKSPACE;
    // every layer's whole argument check first: nothing is enqueued, and y_out stays untouched,
    // unless all of them pass
    for (int32_t i = 0; i < n_layers; ++i) {
        BlockLayout L;
        AttnParams ap{};
        st = vit_block_check(&layers[i], i == 0 ? x : y_out, B, y_out, workspace, workspace_bytes, &L, &ap);
        if (st != VQ_OK) return st;
    }
    if (B == 0) return VQ_OK;
    for (int32_t i = 0; i < n_layers; ++i) {
        BlockLayout L;
        AttnParams ap{};
        (void)vit_block_check(&layers[i], i == 0 ? x : y_out, B, y_out, workspace, workspace_bytes, &L, &ap);
        st = vit_block_run(&layers[i], L, ap, i == 0 ? x : y_out, B, y_out, workspace, (hipStream_t)stream);
        if (st != VQ_OK) return st;
    }
    return VQ_OK;
}

}  // extern "C"
