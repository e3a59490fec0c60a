/*
 * vqo -- CPU oracle for the integerized ViT block (operand reordering).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, obviously-correct
 * statement of what the GPU library must compute.  It shares no code, header,
 * table or constant generator with the HIP path, and only the tests, the smoke
 * check and the benchmark's CPU-baseline leg may load it.  It is never tuned.
 *
 * Conventions
 *   - "Unpacked" quantized matrices are row-major, one value per element:
 *     int8_t for signed levels, uint8_t for the unsigned attention matrix P.
 *   - Every fp32 value that feeds a quantizer is produced by a fixed sequence
 *     of correctly rounded IEEE-754 binary32 primitives (convert, add, sub,
 *     mul, fmaf, divide, floorf, rintf, ldexpf, compare).  Build with
 *     -ffp-contract=off so the compiler neither fuses nor splits them.
 *   - All reductions (accumulators, row max, row sum) are integer and hence
 *     independent of summation order.
 *
 * What follows the paper, and where:
 *   quantizer levels/thresholds ........ Sec. IV-B (3-bit reference list), Sec. IV-C
 *   dequantize-first linear ............ Eq. 1 (first line)           [cross-check]
 *   reordered linear ................... Eq. 2
 *   equivalent bias, absorbed scales ... Eq. 2 (second form), Sec. IV-B
 *   Q.K^T and softmax .................. Eq. 3
 *   shift-based exponential ............ Eq. 4
 *   row-sum-scaled comparator .......... Sec. IV-B, Fig. 4 caption
 *   P.V with scales absorbed ........... Sec. IV-B (weighted sum of values)
 *   LayerNorm + comparator quantizer ... Sec. IV-C, Eq. 5, Fig. 5
 * Where the paper is silent the reading taken is stated at the function.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py
 * against printed values, closed forms, brute force or library routines,
 * except the *choice* of tie direction in vqo_quantize, the fixed-point width
 * in vqo_softmax_row and the GELU definition, which the paper does not fix
 * (conventions; "parity unpinned by the paper", pinned to their own closed
 * forms only), and the whole-chain vqo_attention_block, for which the paper
 * prints no worked example ("parity unpinned"; each stage is pinned instead).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* Level range of a b-bit quantizer.  Signed: [-2^(b-1), 2^(b-1)-1] -- the    */
/* 2^b levels separated by the 2^b-1 inner thresholds (k-1/2)*step of         */
/* Sec. IV-B / IV-C.  Unsigned (attention matrix P only): [0, 2^b-1].         */
/* ------------------------------------------------------------------------ */
int vqo_qrange(int bits, int is_unsigned, int *qmin, int *qmax)
{
    if (bits < 2 || bits > 8) return 1;
    if (is_unsigned) { *qmin = 0; *qmax = (1 << bits) - 1; }
    else { *qmin = -(1 << (bits - 1)); *qmax = (1 << (bits - 1)) - 1; }
    return 0;
}

/* One value through the uniform quantizer: level = clamp(round(x/step)).      */
/* Thresholds sit at (k-1/2)*step (Sec. IV-B, IV-C).  Reading where the paper  */
/* is silent: x/step is an fp32 division and an exact half rounds to the even  */
/* level (rintf in the default rounding mode).                                 */
static int quantize_one(float x, float step, int qmin, int qmax)
{
    float t = x / step;
    float r = rintf(t);
    r = fmaxf(r, (float)qmin);
    r = fminf(r, (float)qmax);
    return (int)r;
}

/* x: [rows x cols] fp32 with leading dimension ld.  step: one value, or one   */
/* per row when step_per_row != 0 (per-output-channel weight steps).           */
int vqo_quantize(const float *x, int64_t rows, int64_t cols, int64_t ld,
                 const float *step, int step_per_row, int bits, int8_t *q)
{
    int qmin, qmax;
    if (vqo_qrange(bits, 0, &qmin, &qmax)) return 1;
    for (int64_t r = 0; r < rows; ++r) {
        float s = step_per_row ? step[r] : step[0];
        for (int64_t c = 0; c < cols; ++c)
            q[r * cols + c] = (int8_t)quantize_one(x[r * ld + c], s, qmin, qmax);
    }
    return 0;
}

/* Per-output-channel weight step: max|w_c| / qmax in fp32; an all-zero row    */
/* gets step 1.  (The benchmark configurations state this rule; the paper      */
/* takes its steps from a trained low-bit checkpoint.)                         */
int vqo_weight_steps(const float *w, int64_t rows, int64_t cols, int64_t ld,
                     int bits, float *s_w)
{
    int qmin, qmax;
    if (vqo_qrange(bits, 0, &qmin, &qmax)) return 1;
    for (int64_t r = 0; r < rows; ++r) {
        float m = 0.0f;
        for (int64_t c = 0; c < cols; ++c) {
            float a = fabsf(w[r * ld + c]);
            if (a > m) m = a;
        }
        s_w[r] = (m == 0.0f) ? 1.0f : m / (float)qmax;
    }
    return 0;
}

/* Dequantize: level * step (the multipliers of Eq. 1).                        */
void vqo_dequantize(const int8_t *q, int64_t rows, int64_t cols,
                    const float *step, int step_per_row, float *x)
{
    for (int64_t r = 0; r < rows; ++r) {
        float s = step_per_row ? step[r] : step[0];
        for (int64_t c = 0; c < cols; ++c)
            x[r * cols + c] = (float)q[r * cols + c] * s;
    }
}

/* ------------------------------------------------------------------------ */
/* Packed storage (the paper only gives model sizes; the format is the         */
/* interchange format of the library): element c of a row occupies             */
/* storage_bits bits at byte (c*sb)/8, bit offset (c*sb)%8, i.e. element 0 in  */
/* the least-significant field; two's complement; pad bytes are zero.          */
/* storage_bits is 2, 4 or 8 (3-bit levels live in 4-bit fields).              */
/* ------------------------------------------------------------------------ */
static int pack_generic(const void *q, int is_u8, int64_t rows, int64_t cols,
                        int storage_bits, uint8_t *out, int64_t row_stride)
{
    if (storage_bits != 2 && storage_bits != 4 && storage_bits != 8) return 1;
    if (row_stride * 8 < cols * storage_bits) return 2;
    unsigned mask = (1u << storage_bits) - 1u;
    memset(out, 0, (size_t)(rows * row_stride));
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            int v = is_u8 ? (int)((const uint8_t *)q)[r * cols + c]
                          : (int)((const int8_t *)q)[r * cols + c];
            int64_t bit = c * storage_bits;
            out[r * row_stride + bit / 8] |= (uint8_t)(((unsigned)v & mask) << (bit % 8));
        }
    return 0;
}

int vqo_pack(const int8_t *q, int64_t rows, int64_t cols, int storage_bits,
             uint8_t *out, int64_t row_stride)
{
    return pack_generic(q, 0, rows, cols, storage_bits, out, row_stride);
}

int vqo_pack_u8(const uint8_t *q, int64_t rows, int64_t cols, int storage_bits,
                uint8_t *out, int64_t row_stride)
{
    return pack_generic(q, 1, rows, cols, storage_bits, out, row_stride);
}

int vqo_unpack(const uint8_t *in, int64_t rows, int64_t cols, int storage_bits,
               int64_t row_stride, int8_t *q)
{
    if (storage_bits != 2 && storage_bits != 4 && storage_bits != 8) return 1;
    unsigned mask = (1u << storage_bits) - 1u;
    unsigned sign = 1u << (storage_bits - 1);
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            int64_t bit = c * storage_bits;
            unsigned f = ((unsigned)in[r * row_stride + bit / 8] >> (bit % 8)) & mask;
            int v = (f & sign) ? (int)f - (int)(mask + 1u) : (int)f;
            q[r * cols + c] = (int8_t)v;
        }
    return 0;
}

int vqo_unpack_u8(const uint8_t *in, int64_t rows, int64_t cols, int storage_bits,
                  int64_t row_stride, uint8_t *q)
{
    if (storage_bits != 2 && storage_bits != 4 && storage_bits != 8) return 1;
    unsigned mask = (1u << storage_bits) - 1u;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            int64_t bit = c * storage_bits;
            q[r * cols + c] = (uint8_t)(((unsigned)in[r * row_stride + bit / 8] >> (bit % 8)) & mask);
        }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Integer contractions: the plain definition, accumulated in int64 and        */
/* checked to fit int32 (the inner term X_q W_q^T of Eq. 2; Q K^T of Eq. 3;    */
/* the weighted sum of values of Sec. IV-B).  Return value: number of          */
/* accumulators that did not fit int32 (0 on every supported shape).           */
/* ------------------------------------------------------------------------ */
/* acc[m][n] = sum_k a[m][k] * b[n][k]        a: [M x K], b: [N x K]           */
int64_t vqo_matmul_nt(const int8_t *a, const int8_t *b, int64_t M, int64_t N,
                      int64_t K, int32_t *acc)
{
    int64_t bad = 0;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += (int64_t)a[m * K + k] * (int64_t)b[n * K + k];
            if (s > INT32_MAX || s < INT32_MIN) ++bad;
            acc[m * N + n] = (int32_t)s;
        }
    return bad;
}

/* acc[m][n] = sum_k p[m][k] * v[k][n]        p: [M x K] unsigned, v: [K x N]  */
int64_t vqo_matmul_nn_u8(const uint8_t *p, const int8_t *v, int64_t M, int64_t N,
                         int64_t K, int32_t *acc)
{
    int64_t bad = 0;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += (int64_t)p[m * K + k] * (int64_t)v[k * N + n];
            if (s > INT32_MAX || s < INT32_MIN) ++bad;
            acc[m * N + n] = (int32_t)s;
        }
    return bad;
}

/* ------------------------------------------------------------------------ */
/* GELU between the two MLP linears.  The paper integerizes self-attention     */
/* only and says the same principle extends to the rest of the block; it       */
/* gives no GELU.  Reading taken: the tanh form                                */
/*     g(y) = 0.5*y*(1 + tanh(u)),  u = sqrt(2/pi)*(y + 0.044715*y^3),         */
/* with tanh(u) = 1 - 2/(1 + 2^(2*u*log2 e)) and 2^t evaluated reproducibly:   */
/* t = n + x with n = rint(t), x in [-1/2, 1/2], 2^x by the degree-7 Taylor    */
/* polynomial of e^(x ln 2) in Horner form with fmaf, scaled by ldexpf.        */
/* ------------------------------------------------------------------------ */
static float exp2_reproducible(float t)
{
    /* (ln 2)^k / k!, k = 0..7, each rounded to binary32 */
    const float c0 = 0x1.000000p+0f, c1 = 0x1.62e430p-1f, c2 = 0x1.ebfbe0p-3f,
                c3 = 0x1.c6b08ep-5f, c4 = 0x1.3b2ab6p-7f, c5 = 0x1.5d87fep-10f,
                c6 = 0x1.430912p-13f, c7 = 0x1.ffcbfcp-17f;
    float n = rintf(t);
    float x = t - n;
    float p = c7;
    p = fmaf(p, x, c6);
    p = fmaf(p, x, c5);
    p = fmaf(p, x, c4);
    p = fmaf(p, x, c3);
    p = fmaf(p, x, c2);
    p = fmaf(p, x, c1);
    p = fmaf(p, x, c0);
    return ldexpf(p, (int)n);
}

float vqo_gelu(float y)
{
    const float kSqrt2OverPi = 0x1.988454p-1f; /* 0.7978845608 */
    const float kCubic = 0x1.6e4e26p-5f;       /* 0.044715     */
    const float kLog2e = 0x1.715476p+0f;       /* 1.44269504   */
    float y3 = (y * y) * y;
    float inner = fmaf(kCubic, y3, y);
    float u = kSqrt2OverPi * inner;
    float t = (2.0f * u) * kLog2e;
    t = fmaxf(t, -126.0f);
    t = fminf(t, 126.0f);
    float X = exp2_reproducible(t);
    float th = 1.0f - 2.0f / (1.0f + X);
    return (0.5f * y) * (1.0f + th);
}

void vqo_gelu_array(const float *y, int64_t n, float *g)
{
    for (int64_t i = 0; i < n; ++i) g[i] = vqo_gelu(y[i]);
}

/* ------------------------------------------------------------------------ */
/* Reordered (integerized) linear, Eq. 2 with a scalar activation step:        */
/*   acc[m][c] = sum_k xq[m][k]*wq[c][k]                    (exact integer)    */
/*   y[m][c]   = fmaf((float)acc, s_x*s_w[c], bias[c])      (post-scaling)     */
/* The bias is added after the scaling (same value, in exact arithmetic, as    */
/* Eq. 2's equivalent bias b/(s_x*s_w) added before it).  act = 1 applies      */
/* vqo_gelu to y.  If yq_out is given, the result is requantized with the      */
/* next operand's per-tensor step s_y to bits_y bits.                          */
/* Any of acc_out / y_out / yq_out may be NULL.  Returns overflow count.       */
/* ------------------------------------------------------------------------ */
int64_t vqo_linear(const int8_t *xq, int64_t M, int64_t K, float s_x,
                   const int8_t *wq, int64_t Nout, const float *s_w, int s_w_per_channel,
                   const float *bias, int act,
                   int32_t *acc_out, float *y_out,
                   float s_y, int bits_y, int8_t *yq_out)
{
    int qmin = 0, qmax = 0;
    if (yq_out && vqo_qrange(bits_y, 0, &qmin, &qmax)) return -1;
    int64_t bad = 0;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t c = 0; c < Nout; ++c) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += (int64_t)xq[m * K + k] * (int64_t)wq[c * K + k];
            if (s > INT32_MAX || s < INT32_MIN) ++bad;
            int32_t acc = (int32_t)s;
            float scale = s_x * (s_w_per_channel ? s_w[c] : s_w[0]);
            float y = fmaf((float)acc, scale, bias ? bias[c] : 0.0f);
            if (act == 1) y = vqo_gelu(y);
            if (acc_out) acc_out[m * Nout + c] = acc;
            if (y_out) y_out[m * Nout + c] = y;
            if (yq_out) yq_out[m * Nout + c] = (int8_t)quantize_one(y, s_y, qmin, qmax);
        }
    return bad;
}

/* ------------------------------------------------------------------------ */
/* Scale absorption for a linear that feeds a quantizer directly (Eq. 2 in its */
/* second form; Sec. IV-B on absorbing the scales into the quantizer).          */
/*                                                                            */
/* Eq. 2 factors the post-scale s_x*s_w[c] out of the sum AND the bias: the     */
/* bias becomes an "equivalent bias" b[c]/(s_x*s_w[c]) added in the integer     */
/* domain.  The quantizer that follows is a bank of comparators against the     */
/* references (k-1/2)*s_y (Sec. IV-B, IV-C); dividing both sides of every       */
/* comparison by the positive post-scale moves it into the references too, so   */
/* the whole linear + quantizer is integer:                                     */
/*     a     = acc + b_int[c]                                                   */
/*     level = qmin + #{ k in qmin+1..qmax : a > T[c][k] }                      */
/* Readings (the paper gives the algebra, not the number formats):              */
/*   - scale_c = s_x*s_w[c] is the fp32 product of Eq. 2's path, then taken as  */
/*     the real number it is;                                                   */
/*   - the equivalent bias is rounded to the nearest integer (ties to even),    */
/*     b_int[c] = rint(b[c]/scale_c) in double precision -- it has to be an     */
/*     integer to be added to integer accumulators;                             */
/*   - theta = ((double)k - 0.5)*(double)s_y / scale_c in double precision      */
/*     (one multiply, one divide), T = floor(theta): for an integer a,          */
/*     a > theta  <=>  a > floor(theta).  The comparator is strict, so a tie    */
/*     goes to the lower level.  T is clamped to the int32 range.               */
/* This mode is NOT bit-identical to vqo_linear's requantized output: that one  */
/* rounds y to fp32 and adds the bias unrounded; the two differ by at most one  */
/* level and only near a reference.                                             */
/* s_y: one step, or one per output channel (s_y_per_channel).                  */
/* ------------------------------------------------------------------------ */
int vqo_absorb(float s_x, const float *s_w, int s_w_per_channel, const float *bias,
               int64_t Nout, const float *s_y, int s_y_per_channel, int bits,
               int32_t *b_int, int32_t *thr)
{
    int qmin = 0, qmax = 0;
    if (vqo_qrange(bits, 0, &qmin, &qmax)) return -1;
    const int nthr = qmax - qmin;
    for (int64_t c = 0; c < Nout; ++c) {
        const float scale32 = s_x * (s_w_per_channel ? s_w[c] : s_w[0]);
        const double scale = (double)scale32;
        const double step = (double)(s_y_per_channel ? s_y[c] : s_y[0]);
        if (!(scale > 0.0) || !(step > 0.0)) return -1;
        double bi = bias ? rint((double)bias[c] / scale) : 0.0;
        if (bi > 2147483647.0) bi = 2147483647.0;
        if (bi < -2147483648.0) bi = -2147483648.0;
        b_int[c] = (int32_t)bi;
        for (int t = 0; t < nthr; ++t) {
            const int k = qmin + 1 + t;
            const double theta = ((double)k - 0.5) * step / scale;
            double T = floor(theta);
            if (T > 2147483647.0) T = 2147483647.0;
            if (T < -2147483648.0) T = -2147483648.0;
            thr[c * nthr + t] = (int32_t)T;
        }
    }
    return 0;
}

/* The integer-only linear + quantizer.  acc_out and yq_out may be NULL.        */
/* Returns the number of int32 overflows (of acc, or of acc + b_int).           */
int64_t vqo_linear_absorbed(const int8_t *xq, int64_t M, int64_t K, const int8_t *wq,
                            int64_t Nout, const int32_t *b_int, const int32_t *thr, int bits,
                            int32_t *acc_out, int8_t *yq_out)
{
    int qmin = 0, qmax = 0;
    if (vqo_qrange(bits, 0, &qmin, &qmax)) return -1;
    const int nthr = qmax - qmin;
    int64_t bad = 0;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t c = 0; c < Nout; ++c) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += (int64_t)xq[m * K + k] * (int64_t)wq[c * K + k];
            if (s > INT32_MAX || s < INT32_MIN) ++bad;
            const int64_t a = s + (b_int ? (int64_t)b_int[c] : 0);
            if (a > INT32_MAX || a < INT32_MIN) ++bad;
            int level = qmin;
            for (int t = 0; t < nthr; ++t)
                if (a > (int64_t)thr[c * nthr + t]) ++level;
            if (acc_out) acc_out[m * Nout + c] = (int32_t)s;
            if (yq_out) yq_out[m * Nout + c] = (int8_t)level;
        }
    return bad;
}

/* ------------------------------------------------------------------------ */
/* Softmax of one integer score row, quantized to unsigned levels 0..pmax      */
/* (step 1/pmax), Eq. 3-4 and the row-sum-scaled comparator of Sec. IV-B.      */
/*                                                                            */
/*  alpha = s_q*s_k*scale*log2(e) turns an integer score difference into a     */
/*  base-2 exponent.  Readings where the paper is silent: the integer row max  */
/*  is subtracted first (so every shift is a right shift and the largest term  */
/*  is exactly 2^20); (1+r) carries 20 fractional bits; right shifts           */
/*  truncate; the comparator is strict (an exact tie goes to the lower         */
/*  level), and exp_j is compared with (k-1/2)*(1/pmax)*sum instead of being   */
/*  divided by the sum.                                                        */
/* ------------------------------------------------------------------------ */
float vqo_alpha(float s_q, float s_k, float scale)
{
    const float kLog2e = 0x1.715476p+0f;
    return ((s_q * s_k) * scale) * kLog2e;
}

/* fixed-point value of (1+r) << floor(alpha*d), d <= 0 an integer difference  */
uint32_t vqo_shift_exp(int32_t d, float alpha)
{
    float t = alpha * (float)d;
    float f = floorf(t);
    float r = t - f;
    uint32_t u = (uint32_t)((1.0f + r) * 1048576.0f);
    float nf = -f;
    int sh = (nf >= 31.0f) ? 31 : (int)nf;
    return u >> sh;
}

void vqo_softmax_row(const int32_t *s, int64_t n, float alpha, int pmax, uint8_t *p,
                     uint32_t *e_out /* nullable [n] */, uint64_t *sum_out /* nullable */)
{
    int32_t mx = s[0];
    for (int64_t j = 1; j < n; ++j) if (s[j] > mx) mx = s[j];
    uint64_t sum = 0;
    uint32_t *e = (uint32_t *)malloc((size_t)n * sizeof(uint32_t));
    for (int64_t j = 0; j < n; ++j) {
        e[j] = vqo_shift_exp(s[j] - mx, alpha);
        sum += e[j];
    }
    for (int64_t j = 0; j < n; ++j) {
        int level = 0;
        for (int k = 1; k <= pmax; ++k)
            if ((uint64_t)2 * (uint64_t)pmax * (uint64_t)e[j] > (uint64_t)(2 * k - 1) * sum)
                ++level;
        p[j] = (uint8_t)level;
    }
    if (e_out) memcpy(e_out, e, (size_t)n * sizeof(uint32_t));
    if (sum_out) *sum_out = sum;
    free(e);
}

/* Q.K^T per (image, head) then the quantized softmax.                         */
/* q, k: [B][H][N][dh] levels.  s_acc_out: [B][H][N][N] or NULL.               */
/* p_out: [B][H][N][N] unsigned levels or NULL.  scale is 1/sqrt(dh).          */
int64_t vqo_matmul_qk(const int8_t *q, const int8_t *k, int64_t B, int64_t H, int64_t N,
                      int64_t dh, float s_q, float s_k, float scale, int bits_p,
                      int32_t *s_acc_out, uint8_t *p_out)
{
    int qmin, pmax;
    if (vqo_qrange(bits_p, 1, &qmin, &pmax)) return -1;
    float alpha = vqo_alpha(s_q, s_k, scale);
    int64_t bad = 0;
    int32_t *S = (int32_t *)malloc((size_t)(N * N) * sizeof(int32_t));
    for (int64_t bh = 0; bh < B * H; ++bh) {
        bad += vqo_matmul_nt(q + bh * N * dh, k + bh * N * dh, N, N, dh, S);
        if (s_acc_out) memcpy(s_acc_out + bh * N * N, S, (size_t)(N * N) * sizeof(int32_t));
        if (p_out)
            for (int64_t i = 0; i < N; ++i)
                vqo_softmax_row(S + i * N, N, alpha, pmax, p_out + bh * N * N + i * N, NULL, NULL);
    }
    free(S);
    return bad;
}

/* P.V per (image, head); both input scales are absorbed next to the output    */
/* quantizer (Sec. IV-B):  o = (float)acc * (s_p*s_v);  O_q = quantize(o,s_o). */
/* p: [B][H][N][N] unsigned, v: [B][H][N][dh].  o_acc_out: [B][H][N][dh].      */
/* o_out / oq_out: [B*N][H*dh] (heads concatenated along the channel axis).    */
int64_t vqo_matmul_pv(const uint8_t *p, const int8_t *v, int64_t B, int64_t H, int64_t N,
                      int64_t dh, float s_p, float s_v,
                      int32_t *o_acc_out, float *o_out,
                      float s_o, int bits_o, int8_t *oq_out)
{
    int qmin = 0, qmax = 0;
    if (oq_out && vqo_qrange(bits_o, 0, &qmin, &qmax)) return -1;
    float spv = s_p * s_v;
    int64_t bad = 0;
    int32_t *O = (int32_t *)malloc((size_t)(N * dh) * sizeof(int32_t));
    for (int64_t b = 0; b < B; ++b)
        for (int64_t h = 0; h < H; ++h) {
            int64_t bh = b * H + h;
            bad += vqo_matmul_nn_u8(p + bh * N * N, v + bh * N * dh, N, dh, N, O);
            for (int64_t i = 0; i < N; ++i)
                for (int64_t d = 0; d < dh; ++d) {
                    int32_t acc = O[i * dh + d];
                    float o = (float)acc * spv;
                    int64_t at = (b * N + i) * (H * dh) + h * dh + d;
                    if (o_acc_out) o_acc_out[bh * N * dh + i * dh + d] = acc;
                    if (o_out) o_out[at] = o;
                    if (oq_out) oq_out[at] = (int8_t)quantize_one(o, s_o, qmin, qmax);
                }
        }
    free(O);
    return bad;
}

/* ------------------------------------------------------------------------ */
/* The whole block, image by image:                                            */
/*   X_q -> QKV linear -> requant Q,K,V (own steps) -> Q.K^T -> softmax->P_q   */
/*       -> P.V -> requant O_q -> projection                                   */
/*       [-> requant X2_q -> fc1 + GELU -> requant H_q -> fc2] -> fp32 Y       */
/* Output channel c of the QKV linear maps to (which, head, d) =                */
/* (c / D, (c % D) / dh, c % dh).  No residual and no second LayerNorm are     */
/* part of this chain.  Images are independent; the loop over images is the    */
/* only parallel loop (OpenMP, when compiled with it).                         */
/* ------------------------------------------------------------------------ */
int vqo_layernorm_quantize(const float *x, const float *res, float *sum_out, int64_t rows,
                           int64_t cols, int64_t ld, const float *gamma, const float *beta,
                           float eps, float step, int bits, int8_t *q, float *mu_out,
                           float *m2_out);

typedef struct vqo_block {
    int64_t D, H, N, hidden;   /* hidden = 0: attention only                  */
    int32_t bits_a, bits_p;    /* activation bits (signed), P bits (unsigned) */
    const int8_t *w_qkv;  const float *sw_qkv;  const float *b_qkv;   /* [3D x D]      */
    const int8_t *w_proj; const float *sw_proj; const float *b_proj;  /* [D x D]       */
    const int8_t *w_fc1;  const float *sw_fc1;  const float *b_fc1;   /* [hidden x D]  */
    const int8_t *w_fc2;  const float *sw_fc2;  const float *b_fc2;   /* [D x hidden]  */
    float s_x, s_q, s_k, s_v, s_o, s_x2, s_h, scale;
} vqo_block;

typedef struct vqo_block_dumps {  /* all nullable; sizes for B images          */
    int8_t *q, *k, *v;     /* [B][H][N][dh]                                   */
    uint8_t *p;            /* [B][H][N][N]                                    */
    int8_t *o;             /* [B*N][D]                                        */
    float *y_attn;         /* [B*N][D]  projection output (fp32)              */
    int8_t *x2;            /* [B*N][D]                                        */
    int8_t *h;             /* [B*N][hidden]                                   */
} vqo_block_dumps;

/* Per-head LayerNorm of Q and K (Sec. III, Fig. 1(b); Table I lists a LayerNorm */
/* of 2 x O elements after the Q and the K linear, none after V): gamma, beta    */
/* are [2D] (the Q channels, then the K channels), each head's 64 channels are   */
/* normalised on their own by vqo_layernorm_quantize; s_q, s_k are then the      */
/* steps of those quantizers.  NULL: the plain requantization of the block.      */
typedef struct vqo_qkln {
    const float *gamma, *beta;
    float eps;
} vqo_qkln;

static int64_t block_one_image_ln(const vqo_block *blk, const vqo_qkln *qkln, const int8_t *xq,
                                  int64_t b, float *y_out, const vqo_block_dumps *dmp);

static int64_t block_one_image(const vqo_block *blk, const int8_t *xq, int64_t b,
                               float *y_out, const vqo_block_dumps *dmp)
{
    return block_one_image_ln(blk, NULL, xq, b, y_out, dmp);
}

static int64_t block_one_image_ln(const vqo_block *blk, const vqo_qkln *qkln, const int8_t *xq,
                                  int64_t b, float *y_out, const vqo_block_dumps *dmp)
{
    const int64_t D = blk->D, H = blk->H, N = blk->N, dh = D / H, Hd = blk->hidden;
    int64_t bad = 0;
    int8_t *hm = (int8_t *)malloc((size_t)(3 * H * N * dh));       /* head-major Q,K,V */
    uint8_t *P = (uint8_t *)malloc((size_t)(H * N * N));
    int8_t *O = (int8_t *)malloc((size_t)(N * D));
    float *Y = (float *)malloc((size_t)(N * 3 * D) * sizeof(float));
    int qmin, qmax;
    vqo_qrange(blk->bits_a, 0, &qmin, &qmax);

    /* QKV linear (fp32 y), then each third requantized with its own step */
    bad += vqo_linear(xq, N, D, blk->s_x, blk->w_qkv, 3 * D, blk->sw_qkv, 1, blk->b_qkv, 0,
                      NULL, Y, 0.0f, 0, NULL);
    for (int64_t n = 0; n < N; ++n)
        for (int64_t c = 0; c < 3 * D; ++c) {
            int64_t which = c / D, h = (c % D) / dh, d = c % dh;
            float step = which == 0 ? blk->s_q : (which == 1 ? blk->s_k : blk->s_v);
            if (qkln && which < 2) continue;          /* Q and K: LayerNorm quantizer, below */
            hm[((which * H + h) * N + n) * dh + d] =
                (int8_t)quantize_one(Y[n * 3 * D + c], step, qmin, qmax);
        }
    if (qkln) {
        /* one head of one token at a time: dh consecutive channels of the row, own statistics */
        for (int64_t which = 0; which < 2; ++which)
            for (int64_t h = 0; h < H; ++h)
                vqo_layernorm_quantize(Y + which * D + h * dh, NULL, NULL, N, dh, 3 * D,
                                       qkln->gamma + which * D + h * dh, qkln->beta + which * D + h * dh,
                                       qkln->eps, which == 0 ? blk->s_q : blk->s_k, blk->bits_a,
                                       hm + (which * H + h) * N * dh, NULL, NULL);
    }
    const int8_t *Q = hm, *K = hm + H * N * dh, *V = hm + 2 * H * N * dh;

    bad += vqo_matmul_qk(Q, K, 1, H, N, dh, blk->s_q, blk->s_k, blk->scale, blk->bits_p, NULL, P);
    {
        int pmin, pmax;
        vqo_qrange(blk->bits_p, 1, &pmin, &pmax);
        float s_p = 1.0f / (float)pmax;
        bad += vqo_matmul_pv(P, V, 1, H, N, dh, s_p, blk->s_v, NULL, NULL, blk->s_o, blk->bits_a, O);
    }
    if (dmp) {
        if (dmp->q) memcpy(dmp->q + b * H * N * dh, Q, (size_t)(H * N * dh));
        if (dmp->k) memcpy(dmp->k + b * H * N * dh, K, (size_t)(H * N * dh));
        if (dmp->v) memcpy(dmp->v + b * H * N * dh, V, (size_t)(H * N * dh));
        if (dmp->p) memcpy(dmp->p + b * H * N * N, P, (size_t)(H * N * N));
        if (dmp->o) memcpy(dmp->o + b * N * D, O, (size_t)(N * D));
    }

    if (Hd == 0) {
        bad += vqo_linear(O, N, D, blk->s_o, blk->w_proj, D, blk->sw_proj, 1, blk->b_proj, 0,
                          NULL, y_out + b * N * D, 0.0f, 0, NULL);
        if (dmp && dmp->y_attn)
            memcpy(dmp->y_attn + b * N * D, y_out + b * N * D, (size_t)(N * D) * sizeof(float));
    } else {
        int8_t *X2 = (int8_t *)malloc((size_t)(N * D));
        int8_t *Hq = (int8_t *)malloc((size_t)(N * Hd));
        bad += vqo_linear(O, N, D, blk->s_o, blk->w_proj, D, blk->sw_proj, 1, blk->b_proj, 0,
                          NULL, (dmp && dmp->y_attn) ? dmp->y_attn + b * N * D : NULL,
                          blk->s_x2, blk->bits_a, X2);
        bad += vqo_linear(X2, N, D, blk->s_x2, blk->w_fc1, Hd, blk->sw_fc1, 1, blk->b_fc1, 1,
                          NULL, NULL, blk->s_h, blk->bits_a, Hq);
        bad += vqo_linear(Hq, N, Hd, blk->s_h, blk->w_fc2, D, blk->sw_fc2, 1, blk->b_fc2, 0,
                          NULL, y_out + b * N * D, 0.0f, 0, NULL);
        if (dmp) {
            if (dmp->x2) memcpy(dmp->x2 + b * N * D, X2, (size_t)(N * D));
            if (dmp->h) memcpy(dmp->h + b * N * Hd, Hq, (size_t)(N * Hd));
        }
        free(X2);
        free(Hq);
    }
    free(hm); free(P); free(O); free(Y);
    return bad;
}

/* xq: [B*N][D] levels.  y_out: [B*N][D] fp32.  Returns overflow count.        */
int64_t vqo_attention_block(const vqo_block *blk, const int8_t *xq, int64_t B,
                            float *y_out, const vqo_block_dumps *dmp)
{
    if (blk->D % blk->H) return -1;
    int64_t bad = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : bad)
#endif
    for (int64_t b = 0; b < B; ++b)
        bad += block_one_image(blk, xq + b * blk->N * blk->D, b, y_out, dmp);
    return bad;
}

/* The same chain with the per-head LayerNorm quantizers on Q and K.             */
int64_t vqo_attention_block_qkln(const vqo_block *blk, const vqo_qkln *qkln, const int8_t *xq,
                                 int64_t B, float *y_out, const vqo_block_dumps *dmp)
{
    if (blk->D % blk->H) return -1;
    int64_t bad = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : bad)
#endif
    for (int64_t b = 0; b < B; ++b)
        bad += block_one_image_ln(blk, qkln, xq + b * blk->N * blk->D, b, y_out, dmp);
    return bad;
}

#ifdef _OPENMP
#include <omp.h>
int vqo_num_threads(void) { return omp_get_max_threads(); }
void vqo_set_num_threads(int n) { omp_set_num_threads(n); }
#else
int vqo_num_threads(void) { return 1; }
void vqo_set_num_threads(int n) { (void)n; }
#endif

/* ------------------------------------------------------------------------ */
/* Exact-math cross-checks (used by the invariants tests only, never by the    */
/* parity gate).                                                               */
/* ------------------------------------------------------------------------ */
/* Eq. 1, first line: dequantize both operands, multiply and sum in double.    */
void vqo_x_linear_dequant_first(const int8_t *xq, int64_t M, int64_t K, float s_x,
                                const int8_t *wq, int64_t Nout, const float *s_w,
                                int s_w_per_channel, const float *bias, double *y)
{
    for (int64_t m = 0; m < M; ++m)
        for (int64_t c = 0; c < Nout; ++c) {
            double sw = (double)(s_w_per_channel ? s_w[c] : s_w[0]);
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k)
                s += ((double)xq[m * K + k] * (double)s_x) * ((double)wq[c * K + k] * sw);
            y[m * Nout + c] = s + (bias ? (double)bias[c] : 0.0);
        }
}

/* True softmax of a*(s_j) in double, rounded to the nearest of 0..pmax.       */
void vqo_x_softmax_true(const int32_t *s, int64_t n, double a, int pmax, uint8_t *p,
                        double *prob_out /* nullable [n] */)
{
    int32_t mx = s[0];
    for (int64_t j = 1; j < n; ++j) if (s[j] > mx) mx = s[j];
    double sum = 0.0;
    for (int64_t j = 0; j < n; ++j) sum += exp(a * (double)(s[j] - mx));
    for (int64_t j = 0; j < n; ++j) {
        double pr = exp(a * (double)(s[j] - mx)) / sum;
        if (prob_out) prob_out[j] = pr;
        double lv = floor(pr * (double)pmax + 0.5);
        if (lv > (double)pmax) lv = (double)pmax;
        p[j] = (uint8_t)lv;
    }
}

/* ------------------------------------------------------------------------ */
/* LayerNorm followed by a quantizer, without division by sigma and without    */
/* square root (Sec. IV-C, Eq. 5, Fig. 5).                                     */
/*                                                                            */
/* Row statistics: the incremental recurrences of Eq. 5 in fp32, elements in   */
/* order i = 1..n, mu_0 = 0, M_0 = 0:                                          */
/*     d1 = x_i - mu;  mu = mu + d1 / (float)i;  d2 = x_i - mu;                */
/*     M  = M + d1 * d2            (a multiply, then an add)                   */
/* M_n is the SUM of squared deviations (Eq. 5 has no 1/i in its second line), */
/* so variance = M_n / n; the n is folded into the comparison below.           */
/* An optional eps (reading: the usual LayerNorm stabiliser, which the paper   */
/* does not mention; 0 switches it off) enters as V = M_n + (float)n * eps.    */
/*                                                                            */
/* Quantizer: level = qmin + #{k = qmin+1 .. qmax : y_j > (k - 1/2) * step}     */
/* with y_j = (x_j - mu) / sigma * gamma_j + beta_j, decided in the comparator  */
/* form of Fig. 5(b): both sides are multiplied by sigma > 0 and squared with   */
/* the sign kept (the "sign logic"), ssq(v) = v * |v|:                          */
/*     a = x_j - mu;  g = a * gamma_j;  L = (g * |g|) * (float)n               */
/*     r = ((float)k - 0.5f) * step;  c = r - beta_j;  R = (c * |c|) * V        */
/*     y_j > r   <=>   L > R                                                   */
/* Reading: Fig. 5(b) scales the REFERENCE by 1/gamma; here the data side is    */
/* scaled by gamma instead, which needs no reciprocal and stays valid for       */
/* gamma <= 0.  A row with V == 0 (constant row, eps == 0) has no defined       */
/* normalisation; every comparison is then "0 > +-0" = false and the row gets   */
/* qmin.  With a residual input the element is first x_j = x_j + res_j (fp32),  */
/* optionally returned in sum_out.                                              */
/* Outputs: q [rows x cols] levels; mu_out, m2_out [rows] (nullable).           */
/* ------------------------------------------------------------------------ */
int vqo_layernorm_quantize(const float *x, const float *res, float *sum_out, int64_t rows,
                           int64_t cols, int64_t ld, const float *gamma, const float *beta,
                           float eps, float step, int bits, int8_t *q, float *mu_out,
                           float *m2_out)
{
    int qmin, qmax;
    if (vqo_qrange(bits, 0, &qmin, &qmax)) return 1;
    float *row = (float *)malloc((size_t)(cols > 0 ? cols : 1) * sizeof(float));
    if (!row) return 2;
    for (int64_t r_ = 0; r_ < rows; ++r_) {
        for (int64_t j = 0; j < cols; ++j) {
            float v = x[r_ * ld + j];
            if (res) v = v + res[r_ * ld + j];
            row[j] = v;
            if (sum_out) sum_out[r_ * ld + j] = v;
        }
        float mu = 0.0f, m2 = 0.0f;
        for (int64_t i = 1; i <= cols; ++i) {
            float xi = row[i - 1];
            float d1 = xi - mu;
            mu = mu + d1 / (float)i;
            float d2 = xi - mu;
            float pr = d1 * d2;
            m2 = m2 + pr;
        }
        if (mu_out) mu_out[r_] = mu;
        if (m2_out) m2_out[r_] = m2;
        float nf = (float)cols;
        float ne = nf * eps;
        float V = m2 + ne;
        for (int64_t j = 0; j < cols; ++j) {
            float a = row[j] - mu;
            float g = a * gamma[j];
            float gs = g * fabsf(g);
            float L = gs * nf;
            int level = qmin;
            for (int k = qmin + 1; k <= qmax; ++k) {
                float rk = ((float)k - 0.5f) * step;
                float c = rk - beta[j];
                float cs = c * fabsf(c);
                float R = cs * V;
                if (L > R) level += 1;
            }
            q[r_ * cols + j] = (int8_t)level;
        }
    }
    free(row);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* A whole pre-LayerNorm ViT block on the fp32 residual stream, composed of    */
/* the pieces above (the paper integerizes the attention part, Sec. III, and   */
/* gives the LayerNorm quantizer of Sec. IV-C as the module in front of it;    */
/* the residual wiring is the standard pre-LN transformer block):              */
/*   X_q  = LNQ1(x)                      vqo_layernorm_quantize, step s_x      */
/*   a    = proj(attention(X_q))         block_one_image with hidden = 0       */
/*   x1   = a + x                        fp32 add                              */
/*   X2_q = LNQ2(x1)                     step s_x2                             */
/*   H_q  = requant(GELU(fc1(X2_q)))     step s_h                              */
/*   y    = fc2(H_q) + x1                fp32 add                              */
/* x, y_out, x1_out: [B*N][D] fp32.  Dumps (nullable): xq_out, x2_out [B*N][D],*/
/* h_out [B*N][hidden], plus the attention dumps of dmp.                       */
/* ------------------------------------------------------------------------ */
typedef struct vqo_ln_params {
    const float *g1, *b1, *g2, *b2;   /* [D] each */
    float eps;
} vqo_ln_params;

int64_t vqo_vit_block_preln(const vqo_block *blk, const vqo_ln_params *ln, const float *x,
                            int64_t B, float *y_out, float *x1_out, int8_t *xq_out,
                            int8_t *x2_out, int8_t *h_out, const vqo_block_dumps *dmp)
{
    if (blk->D % blk->H || blk->hidden <= 0) return -1;
    const int64_t D = blk->D, N = blk->N, Hd = blk->hidden;
    int64_t bad = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : bad)
#endif
    for (int64_t b = 0; b < B; ++b) {
        vqo_block att = *blk;
        att.hidden = 0;                               /* attention + projection, fp32 out */
        int8_t *Xq = (int8_t *)malloc((size_t)(N * D));
        int8_t *X2 = (int8_t *)malloc((size_t)(N * D));
        int8_t *Hq = (int8_t *)malloc((size_t)(N * Hd));
        float *A = (float *)malloc((size_t)(N * D) * sizeof(float));
        float *X1 = (float *)malloc((size_t)(N * D) * sizeof(float));
        float *T = (float *)malloc((size_t)(N * D) * sizeof(float));
        const float *xb = x + b * N * D;
        vqo_layernorm_quantize(xb, NULL, NULL, N, D, D, ln->g1, ln->b1, ln->eps, blk->s_x,
                               blk->bits_a, Xq, NULL, NULL);
        /* block_one_image indexes its outputs by image; hand it image-0 views */
        vqo_block_dumps d0;
        const vqo_block_dumps *dp = NULL;
        if (dmp) {
            const int64_t dh = D / blk->H, H = blk->H;
            d0 = *dmp;
            if (d0.q) d0.q += b * H * N * dh;
            if (d0.k) d0.k += b * H * N * dh;
            if (d0.v) d0.v += b * H * N * dh;
            if (d0.p) d0.p += b * H * N * N;
            if (d0.o) d0.o += b * N * D;
            if (d0.y_attn) d0.y_attn += b * N * D;
            d0.x2 = NULL; d0.h = NULL;
            dp = &d0;
        }
        bad += block_one_image(&att, Xq, 0, A, dp);
        /* x1 = a + x, then the second LayerNorm quantizer on x1 */
        vqo_layernorm_quantize(A, xb, X1, N, D, D, ln->g2, ln->b2, ln->eps, blk->s_x2,
                               blk->bits_a, X2, NULL, NULL);
        bad += vqo_linear(X2, N, D, blk->s_x2, blk->w_fc1, Hd, blk->sw_fc1, 1, blk->b_fc1, 1,
                          NULL, NULL, blk->s_h, blk->bits_a, Hq);
        bad += vqo_linear(Hq, N, Hd, blk->s_h, blk->w_fc2, D, blk->sw_fc2, 1, blk->b_fc2, 0,
                          NULL, T, 0.0f, 0, NULL);
        for (int64_t i = 0; i < N * D; ++i) y_out[b * N * D + i] = T[i] + X1[i];
        if (x1_out) memcpy(x1_out + b * N * D, X1, (size_t)(N * D) * sizeof(float));
        if (xq_out) memcpy(xq_out + b * N * D, Xq, (size_t)(N * D));
        if (x2_out) memcpy(x2_out + b * N * D, X2, (size_t)(N * D));
        if (h_out) memcpy(h_out + b * N * Hd, Hq, (size_t)(N * Hd));
        free(Xq); free(X2); free(Hq); free(A); free(X1); free(T);
    }
    return bad;
}

/* Cross-check: the direct form of Fig. 5(a) in double -- two-pass mean and    */
/* variance, y = (x - mean) / sqrt(var + eps) * gamma + beta -- returned as y.  */
void vqo_x_layernorm(const float *x, int64_t rows, int64_t cols, int64_t ld, const float *gamma,
                     const float *beta, double eps, double *y)
{
    for (int64_t r_ = 0; r_ < rows; ++r_) {
        double m = 0.0, v = 0.0;
        for (int64_t j = 0; j < cols; ++j) m += (double)x[r_ * ld + j];
        m /= (double)cols;
        for (int64_t j = 0; j < cols; ++j) { double d = (double)x[r_ * ld + j] - m; v += d * d; }
        v /= (double)cols;
        for (int64_t j = 0; j < cols; ++j)
            y[r_ * cols + j] = ((double)x[r_ * ld + j] - m) / sqrt(v + eps) * (double)gamma[j] + (double)beta[j];
    }
}

/* erf-form GELU in double.                                                    */
double vqo_x_gelu_erf(double y) { return 0.5 * y * (1.0 + erf(y / sqrt(2.0))); }
