/*
 * vitq -- integerized ViT block matmuls (operand reordering) for AMD MI355X (gfx950).
 *
 * C ABI of libvitq.so.  Every matrix operation of a ViT block (QKV / projection / MLP
 * linears, Q.K^T, P.V) runs directly on packed b-bit integer operands with exact int32
 * accumulation; dequantization is moved AFTER the matmul and fused, with bias, activation and
 * requantization, into the kernel epilogue (paper: Sec. III-A, Eq. 2; Sec. IV-B, Eq. 3-4).
 *
 * General conventions
 *   - All data pointers are DEVICE pointers unless a parameter says "host".  Every buffer
 *     (inputs, outputs, workspace) is owned by the caller; the library allocates and frees
 *     nothing and keeps no state.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue
 *     work on it and return without synchronizing.
 *   - Errors are reported by return code only.  All argument checks run on the host before
 *     anything is launched; a failed check leaves every output untouched.
 *   - Nullable outputs select what the epilogue writes.
 *
 * Quantizer (paper: Sec. IV-B lists the 3-bit comparator references -3.5..2.5 x step;
 * Sec. IV-C gives the general (k - 1/2) x step): level = clamp(round(x / step), qmin, qmax)
 * with qmin = -2^(b-1), qmax = 2^(b-1)-1; x/step is an IEEE fp32 division and exact halves
 * round to the even level.  The attention matrix P is unsigned: levels 0..2^b-1, step
 * 1/(2^b-1).
 */
#ifndef VITQ_H
#define VITQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum vq_status {
    VQ_OK = 0,
    VQ_ERR_NULL = 1,        /* a required pointer is NULL                                  */
    VQ_ERR_SHAPE = 2,       /* dimensions non-positive, mismatching or too large           */
    VQ_ERR_BITS = 3,        /* bits / storage_bits / signedness not valid for this operand */
    VQ_ERR_STRIDE = 4,      /* row_stride too small, or stride / pointer not 16-B aligned  */
    VQ_ERR_STEP = 5,        /* a host-visible step size is not a positive finite number    */
    VQ_ERR_UNSUPPORTED = 6, /* valid request this build has no kernel for                  */
    VQ_ERR_WORKSPACE = 7,   /* workspace NULL or too small                                 */
    VQ_ERR_HIP = 8          /* the HIP runtime refused a launch                            */
} vq_status;

/*
 * A packed quantized matrix in device memory (the interchange format).
 * Element (r, c) occupies `storage_bits` bits at byte r*row_stride + (c*storage_bits)/8,
 * bit offset (c*storage_bits)%8 -- element 0 sits in the least-significant field; signed
 * levels are two's complement.  storage_bits is 2, 4 or 8; `bits` (2..8, <= storage_bits) is
 * the level range (3-bit levels live in 4-bit fields).  Rows are packed along `cols`, which is
 * the contraction dimension whenever the matrix is a matmul operand.
 * row_stride is in bytes and a multiple of 16; `data` is 16-byte aligned.  In an INPUT, the
 * bytes from ceil(cols*storage_bits/8) up to the next multiple of 16 must be zero.  In an
 * OUTPUT, the library writes bytes [0, that multiple of 16) of every row (zeros in the pad)
 * and touches nothing beyond.
 */
typedef struct vq_qmat {
    void *data;
    int32_t bits;
    int32_t storage_bits;
    int32_t is_unsigned; /* 1 only for the attention matrix P */
    int32_t reserved;
    int64_t rows;
    int64_t cols;
    int64_t row_stride;
} vq_qmat;

const char *vq_status_string(vq_status s);

/*
 * Per-row (per-output-channel) weight steps: step_out[r] = max_c |w[r][c]| / qmax(bits) in
 * fp32, or 1 for an all-zero row.  (The benchmark configurations' rule; the paper takes its
 * steps from a trained low-bit checkpoint, Sec. V-A.)
 * w: device fp32 [rows x cols], leading dimension ld (elements).  step_out: device [rows].
 */
vq_status vq_weight_steps(const float *w, int64_t rows, int64_t cols, int64_t ld, int32_t bits,
                          float *step_out, void *stream);

/*
 * Uniform b-bit quantizer (see the top of this file), writing the packed format.
 * x: device fp32 [rows x cols], leading dimension ld.  `step` (host scalar) is the per-tensor
 * step; if step_per_row (device, [rows]) is non-NULL it overrides `step` row by row.
 * out: describes the destination (data, bits, storage_bits, rows, cols, row_stride are read;
 * is_unsigned must be 0).  Errors: NULL, SHAPE (rows/cols mismatch), BITS, STRIDE, STEP.
 */
vq_status vq_quantize(const float *x, int64_t rows, int64_t cols, int64_t ld, float step,
                      const float *step_per_row, const vq_qmat *out, void *stream);

/*
 * Reordered (integerized) linear layer, Eq. 2 with a scalar activation step:
 *     acc[m][c] = sum_k xq[m][k] * wq[c][k]                    exact, int32
 *     y[m][c]   = fma((float)acc, s_x * s_w[c], bias[c])       post-scaling, fp32
 *     act == 1:   y = gelu(y)   (tanh form, fixed fp32 operation sequence)
 *     yq        = quantize(y, s_y) packed with yq_out's bits
 * xq: [M x K]; wq: [Nout x K]; both packed along K.  s_w: device, [Nout] if s_w_per_channel
 * else [1].  bias: device [Nout] or NULL.  acc_out: device int32 [M x Nout] or NULL.
 * y_out: device fp32 [M x Nout] or NULL.  yq_out: destination descriptor or NULL
 * (rows = M, cols = Nout); s_y is its per-tensor step (host scalar).
 * Supported (weight storage, activation storage) pairs: (4,4), (2,4), (8,8).
 * Limits: K <= 65536; row strides of both operands below 2^24 bytes (VQ_ERR_STRIDE).
 * Errors: NULL, SHAPE (K mismatch, K > 65536, sizes overflowing int32 indexing), BITS,
 * STRIDE, STEP (s_x or s_y not positive finite), UNSUPPORTED.
 */
vq_status vq_linear(const vq_qmat *xq, float s_x, const vq_qmat *wq, const float *s_w,
                    int32_t s_w_per_channel, const float *bias, int32_t act, int32_t *acc_out,
                    float *y_out, float s_y, const vq_qmat *yq_out, void *stream);

/*
 * Q.K^T per (image, head) followed by the quantized softmax (Eq. 3-4 and the row-sum-scaled
 * comparator of Sec. IV-B):
 *     S[i][j] = sum_d q[i][d] * k[j][d]                        exact, int32
 *     alpha   = ((s_q*s_k)*scale)*log2(e)                      fp32, in this order
 *     e_j     = ((1+r) * 2^20) >> -floor(alpha*(S_ij - max_j S_ij)),  r the fractional part
 *     P[i][j] = #{ k in 1..pmax : 2*pmax*e_j > (2k-1) * sum_j e_j },  pmax = 2^bits - 1
 * q, k: packed [B*H*N x 64], head-major (row = (b*H + h)*N + token), signed, same bits.
 * s_acc_out: device int32 [B*H*N x N] or NULL.  p_out: unsigned destination [B*H*N x N] or
 * NULL.  Limits: head dimension 64, N <= 592.
 */
vq_status vq_matmul_qk(const vq_qmat *q, const vq_qmat *k, int32_t B, int32_t H, int32_t N,
                       float s_q, float s_k, float scale, int32_t *s_acc_out,
                       const vq_qmat *p_out, void *stream);

/*
 * P.V per (image, head) with both operand scales absorbed next to the output quantizer
 * (Sec. IV-B, weighted sum of values):
 *     O[i][d] = sum_j p[i][j] * v[j][d]                        exact, int32
 *     o       = (float)O * (s_p * s_v);     oq = quantize(o, s_o)
 * p: unsigned packed [B*H*N x N]; v: packed [B*H*N x 64] head-major.
 * o_acc_out: device int32 [B*H*N x 64] or NULL.  o_out: device fp32 [B*N x H*64] (heads
 * concatenated along the channel axis) or NULL.  oq_out: destination [B*N x H*64] or NULL.
 */
vq_status vq_matmul_pv(const vq_qmat *p, const vq_qmat *v, int32_t B, int32_t H, int32_t N,
                       float s_p, float s_v, int32_t *o_acc_out, float *o_out, float s_o,
                       const vq_qmat *oq_out, void *stream);

/*
 * One whole block: X_q -> QKV linear -> Q,K,V requantized with their own steps -> Q.K^T ->
 * quantized softmax -> P.V -> O_q -> projection [-> X2_q -> fc1 + GELU -> H_q -> fc2] -> Y.
 * Output channel c of the QKV linear is (q/k/v, head, d) = (c / D, (c % D) / 64, c % 64).
 * Scores and P never leave the chip.  hidden == 0 selects the attention-only chain.
 * No residual connection and no LayerNorm are part of the chain.
 */
typedef struct vq_block_desc {
    int32_t D, H, N, hidden;
    int32_t bits_a;               /* activation levels (signed): X, Q, K, V, O, X2, H      */
    int32_t bits_p;               /* attention levels (unsigned)                           */
    int32_t storage_a;            /* storage bits of every activation tensor: 4 or 8       */
    int32_t reserved;
    vq_qmat w_qkv, w_proj, w_fc1, w_fc2; /* [3D x D] [D x D] [hidden x D] [D x hidden]     */
    const float *sw_qkv, *b_qkv;  /* per-channel steps and biases, device                  */
    const float *sw_proj, *b_proj;
    const float *sw_fc1, *b_fc1;
    const float *sw_fc2, *b_fc2;
    float s_x, s_q, s_k, s_v, s_o, s_x2, s_h, scale; /* per-tensor steps; scale = 1/sqrt(64) */
    /* Optional copies of the intermediates (device, nullable).  When given, the stage writes
     * there instead of into the workspace -- same kernels, same code path.                  */
    void *dump_qkv;   /* packed [3][B*H*N][64*storage_a/8]  (Q, then K, then V; head-major)  */
    void *dump_o;     /* packed [B*N][D*storage_a/8]                                         */
    void *dump_x2;    /* packed [B*N][D*storage_a/8]        (hidden > 0 only)                */
    void *dump_h;     /* packed [B*N][hidden*storage_a/8]   (hidden > 0 only)                */
    /* Optional profiling hook (host array of hipEvent_t, nullable): event 0 is recorded on the
     * stream before the first stage and event i after stage i (1 QKV linear, 2 attention,
     * 3 projection, 4 fc1, 5 fc2); 4 events are used when hidden == 0, else 6.              */
    void **stage_events;
    /* Optional expanded copies of the four weight matrices made by vq_prepack_weight (device,
     * nullable, all four or none; hidden == 0: the first two).  With 4-bit activation storage
     * the linears then read these instead of unpacking the packed weights in every tile.     */
    const void *wp_qkv, *wp_proj, *wp_fc1, *wp_fc2;
    /* Optional per-head LayerNorm of Q and K (Fig. 1(b), Table I: a LayerNorm of 2 x O elements
     * after the Q and the K linear, none after V).  qk_gamma, qk_beta: device fp32 [2D] (Q
     * channels, then K channels), nullable together.  When given, s_q and s_k are the steps of
     * the two LayerNorm quantizers (the scalar s_x is cancelled by them); the packed Q, K, V
     * are those of the QKV linear in fp32 followed by vq_qkv_headnorm.  The quantizers run in
     * the linear's epilogue (the fp32 values stay in registers) unless 1/s_q, 1/s_k or 1/s_v
     * leaves [2^-100, 2^100]: then the fp32 matrix goes through the workspace.              */
    const float *qk_gamma, *qk_beta;
    float qk_eps;
    int32_t reserved2;
} vq_block_desc;

/*
 * Absorbed mode: the linear and the quantizer after it as integer arithmetic only (Eq. 2 in its
 * second form, Sec. IV-B on absorbing the scales into the quantizer).  Eq. 2 moves the bias into
 * the integer domain as an "equivalent bias" b[c]/(s_x*s_w[c]); the quantizer is a bank of
 * comparators against (k - 1/2)*s_y, and dividing those references by the positive post-scale
 * s_x*s_w[c] leaves
 *     level = qmin + #{ k = qmin+1 .. qmax : acc + b_int[c] > T[c][k] }      (strict: a tie stays below).
 *
 * vq_absorb_thresholds -- HOST pointers, plain host arithmetic, no GPU work: fills
 *   b_int[c]  = rint(bias[c] / scale_c)  (double precision, ties to even; 0 without a bias) and
 *   thr[c][t] = floor(((qmin+1+t) - 0.5) * s_y / scale_c)  (double: one multiply, one divide),
 * scale_c = s_x*s_w[c] the fp32 product of Eq. 2 taken as a real number; both clamped to int32.
 * thr is [out_features][2^bits - 1], non-decreasing along t.  s_w / s_y: one value or one per
 * channel (flags).  The caller copies both arrays to the device.
 * Errors: VQ_ERR_NULL, VQ_ERR_BITS (bits outside 2..8), VQ_ERR_STEP (a step or a product of
 * steps that is not positive and finite).
 *
 * vq_linear_absorbed -- DEVICE pointers: yq_out[m][c] = the level above for acc = sum_k xq*wq.
 * No floating-point value takes part in a decision.  b_int nullable (no bias); thr as above
 * with 2^(yq_out->bits) - 1 references per channel (the kernel only needs them non-decreasing);
 * acc_out nullable [rows x out_features] int32.  out_features must be a multiple of 16 and
 * yq_out use 4- or 8-bit storage (else VQ_ERR_UNSUPPORTED).  Not bit-identical to vq_linear's
 * requantized output: that one rounds y to fp32 and adds the bias unrounded; the two differ by
 * at most one level and only next to a reference.
 */
vq_status vq_absorb_thresholds(float s_x, const float *s_w, int32_t s_w_per_channel, const float *bias,
                               int64_t out_features, const float *s_y, int32_t s_y_per_channel, int32_t bits,
                               int32_t *b_int, int32_t *thr);
vq_status vq_linear_absorbed(const vq_qmat *xq, const vq_qmat *wq, const int32_t *b_int, const int32_t *thr,
                             int32_t *acc_out, const vq_qmat *yq_out, void *stream);

/*
 * Experimental: the reordered linear (Eq. 2) on the 6-bit-float matrix format.  CDNA4's scaled
 * MFMA takes E3M2 operands (1 sign, 3 exponent, 2 mantissa bits, bias 3: every integer in
 * [-8, 8] is a value) at twice the int8 rate with fp32 accumulation; sums of such integer
 * products stay far below 2^24, where that accumulation is exact, so the result is the same
 * integer contraction.  Operands must be stored as E3M2 codes in the kernel's operand order:
 * a row is a sequence of 96-byte stages of 128 values (padded with zero codes to whole
 * stages); quarter q = 2s + h (s, h in {0,1}) of a stage, values 32q..32q+31, is a 192-bit
 * string with value j at bits 6j..6j+5; its first 128 bits are the 16-byte piece 3h + s of the
 * stage and its last 64 bits are half s of piece 3h + 2.  vq_recode_e3m2 makes such a copy of a
 * packed matrix with 4-bit storage (levels of 2..4 bits).
 *   vq_recode_e3m2_bytes: size of that copy (rows * ceil(cols/128) * 96).
 *   vq_recode_e3m2: out device, 16-byte aligned, at least that size (else VQ_ERR_WORKSPACE).
 *   vq_linear_e3m2: y[m][c] = fma(sum_k x[m][k]*w[c][k], s_x*s_w[c], bias ? bias[c] : 0), fp32
 *     [rows x out_features]; x6 / w6 are re-coded matrices with `cols` values per row; s_w one
 *     value or one per channel; the fp32 output equals vq_linear's y_out bit for bit.
 * storage_bits other than 4: VQ_ERR_UNSUPPORTED.
 */
vq_status vq_recode_e3m2_bytes(const vq_qmat *m, size_t *bytes);
vq_status vq_recode_e3m2(const vq_qmat *m, void *out, size_t out_bytes, void *stream);
vq_status vq_linear_e3m2(const void *x6, int64_t rows, const void *w6, int64_t out_features, int64_t cols,
                         float s_x, const float *s_w, int32_t s_w_per_channel, const float *bias, float *y_out,
                         void *stream);

/*
 * Offline weight preparation (optional).  The packed format above is the interchange format;
 * the matrix cores consume int8, so a 2-/3-/4-bit weight matrix is expanded either inside every
 * GEMM tile that uses it, or once, here: `out` receives an int8 copy [rows x kp], kp = cols
 * rounded up to 16, values in the operand order of the GEMM kernels (opaque to the caller),
 * zero beyond cols.  The products, and therefore every result, are identical (Eq. 2 is an
 * exact integer contraction either way).
 * w: packed weights, storage_bits 2 or 4 (else VQ_ERR_UNSUPPORTED).  out: device, 16-byte
 * aligned, at least the size vq_prepack_weight_bytes reports (else VQ_ERR_WORKSPACE).
 */
vq_status vq_prepack_weight_bytes(const vq_qmat *w, size_t *bytes);
vq_status vq_prepack_weight(const vq_qmat *w, void *out, size_t out_bytes, void *stream);

/*
 * vq_linear with the expanded weight copy `wp` of the same `wq` (made by vq_prepack_weight).
 * xq must use 4-bit storage.  Everything else as vq_linear; results are identical to it.
 */
vq_status vq_linear_prepacked(const vq_qmat *xq, float s_x, const vq_qmat *wq, const void *wp,
                              const float *s_w, int32_t s_w_per_channel, const float *bias,
                              int32_t act, int32_t *acc_out, float *y_out, float s_y,
                              const vq_qmat *yq_out, void *stream);

/*
 * LayerNorm followed by the b-bit quantizer, free of division by sigma and of square roots
 * (Sec. IV-C: incremental statistics of Eq. 5, comparator of Fig. 5(b)); the glue between the
 * residual stream (fp32) and the next packed operand.
 *   t[r][c]  = x[r][c] (+ residual[r][c] when residual != NULL), fp32; written to sum_out when
 *              sum_out != NULL (the updated residual stream)
 *   mu, M    = Eq. 5 over c = 1..cols in this order, fp32 (M = sum of squared deviations)
 *   out[r][c]= qmin + #{k = qmin+1..qmax : ssq((t - mu)*gamma[c]) * cols
 *                                          > ssq((k - 1/2)*step - beta[c]) * (M + cols*eps)},
 *              ssq(v) = v*|v|  (the comparison "normalised value > reference" multiplied by
 *              sigma and squared with the sign kept)
 * x, residual, sum_out: device fp32 [rows x cols], leading dimension ld (elements); gamma, beta:
 * device fp32 [cols] (gamma may have any sign); eps >= 0 (0: none); step > 0; out: packed signed
 * levels [rows x cols].  A row whose M + cols*eps is 0 gets qmin everywhere.
 * Errors as elsewhere: host-side checks before the launch, outputs untouched on failure.
 */
vq_status vq_layernorm_quantize(const float *x, const float *residual, float *sum_out, int64_t rows,
                                int64_t cols, int64_t ld, const float *gamma, const float *beta,
                                float eps, float step, const vq_qmat *out, void *stream);

/*
 * Q, K, V of a QKV linear, y fp32 [B*N x 3D] (leading dimension ld, elements; D = 64*H), to the
 * packed head-major operands of the attention, out = [3][B][H][N][64*storage_bits/8] bytes:
 * every 64-channel head of Q and of K goes through the LayerNorm quantizer of
 * vq_layernorm_quantize on its own (statistics per token and head, gamma / beta [2D], steps
 * s_q / s_k), V through the plain quantizer with step s_v.
 */
vq_status vq_qkv_headnorm(const float *y, int64_t ld, int32_t B, int32_t H, int32_t N,
                          const float *gamma, const float *beta, float eps, float s_q, float s_k,
                          float s_v, int32_t bits, int32_t storage_bits, void *out, void *stream);

/* Bytes of workspace vq_attention_block needs for batch B (host computation only). */
vq_status vq_attention_block_workspace(const vq_block_desc *desc, int64_t B, size_t *bytes);

/*
 * xq: packed [B*N x D] tokens (step desc->s_x).  y_out: device fp32 [B*N x D].
 * workspace: device, 256-byte aligned, at least the size reported above.
 * Limits: 64-channel heads, N <= 592, B*N < 2^22 token rows (VQ_ERR_SHAPE beyond).
 */
vq_status vq_attention_block(const vq_block_desc *desc, const vq_qmat *xq, int64_t B,
                             float *y_out, void *workspace, size_t workspace_bytes,
                             void *stream);

/*
 * vq_attention_block for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, checks, kernels and results as vq_attention_block, but the intermediates (packed
 * Q/K/V, O, X2, H) live in an array of VQ_STATIC_SCRATCH_BYTES bytes that is part of the
 * library's device code: every GPU the library runs on holds one copy until the process ends.
 * The call allocates and frees nothing (no hipMalloc / hipFree, no allocating runtime routine);
 * the array's device address is looked up once per device, on the first call there.
 * Limits: vq_attention_block_workspace(desc, B) must not exceed VQ_STATIC_SCRATCH_BYTES (else
 * VQ_ERR_WORKSPACE, nothing launched; e.g. ViT-S attention up to B = 110, the ViT-B block up to
 * B = 24); desc->qk_gamma must be NULL (VQ_ERR_UNSUPPORTED).  All calls on one GPU share that
 * GPU's array, which keeps the previous call's contents (every byte a stage reads is written by
 * the stage before it, so nothing needs clearing): calls that overlap in time on one GPU -- two
 * streams, two threads -- race and must be serialised by the caller.
 */
#define VQ_STATIC_SCRATCH_BYTES (16u << 20)
vq_status vq_attention_block_static(const vq_block_desc *desc, const vq_qmat *xq, int64_t B,
                                    float *y_out, void *stream);

/*
 * A whole pre-LayerNorm ViT block on the fp32 residual stream, built from the stages above
 * (the LayerNorm quantizer of Sec. IV-C in front of the integerized attention of Sec. III-IV and,
 * by the same principle, in front of the MLP):
 *   X_q = LNQ1(x);  x1 = proj(attention(X_q)) + x;  X2_q = LNQ2(x1);
 *   y   = fc2(requant(GELU(fc1(X2_q)))) + x1
 * The two additions are fp32 adds fused into the projection / fc2 epilogues.
 * block: as for vq_attention_block with hidden > 0; block.s_x and block.s_x2 are the steps of
 * the two LayerNorm quantizers; block.stage_events is ignored.  ln*_gamma / ln*_beta: device
 * fp32 [D].  dump_xq (packed [B*N][D*storage_a/8]) and dump_x1 (fp32 [B*N][D]): optional copies.
 */
typedef struct vq_preln_desc {
    vq_block_desc block;
    const float *ln1_gamma, *ln1_beta, *ln2_gamma, *ln2_beta;
    float ln_eps;
    int32_t reserved;
    void *dump_xq;
    float *dump_x1;
} vq_preln_desc;

/* Bytes of workspace vq_vit_block needs for batch B (host computation only). */
vq_status vq_vit_block_workspace(const vq_preln_desc *desc, int64_t B, size_t *bytes);

/*
 * x: device fp32 [B*N x D], 16-byte aligned.  y_out: device fp32 [B*N x D] (holds x1 between the
 * stages); it may be x itself (the block then updates the stream in place: x is last read, as
 * the residual, by the very lanes that write x1 over it) but must not overlap it otherwise
 * (VQ_ERR_STRIDE).  workspace: device, 256-byte aligned.
 */
vq_status vq_vit_block(const vq_preln_desc *desc, const float *x, int64_t B, float *y_out,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * A stack of such blocks (an encoder: the paper's model is twelve of them): layer 0 reads x and
 * writes y_out, every further layer updates y_out in place.  layers: HOST array of n_layers
 * descriptors that agree in D, H, N, bit widths and storage (else VQ_ERR_SHAPE); the dump
 * pointers of the descriptors are honoured per layer.  The workspace is shared by the layers:
 * vq_vit_encoder_workspace reports the largest need.  x may be y_out (as above).  The argument
 * checks of ALL layers run before the first launch: a bad descriptor in any layer leaves y_out
 * untouched.
 */
vq_status vq_vit_encoder_workspace(const vq_preln_desc *layers, int32_t n_layers, int64_t B, size_t *bytes);
vq_status vq_vit_encoder(const vq_preln_desc *layers, int32_t n_layers, const float *x, int64_t B,
                         float *y_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Measurement aid (not part of the method): enqueues a register-resident loop of the int8 matrix
 * instruction the linears run on (v_mfma_i32_32x32x32_i8, operands of the kind the kernels feed,
 * no memory traffic) on every compute unit: `iters` x 4 instructions per wave, 4 waves per SIMD.
 * *ops_out (host, nullable) receives the integer operations the launch performs (2 per MAC);
 * timing it with events gives the matrix-core rate this machine sustains, which bench.py reports as
 * roofline.peak_measured next to the published peak.  sink: device int32[1] or NULL (never
 * written in practice).  Errors: VQ_ERR_SHAPE (iters outside 1..2^22), VQ_ERR_HIP.
 */
vq_status vq_probe_mfma_i8(int32_t iters, int32_t *sink, double *ops_out, void *stream);

/*
 * Measurement aid for the guard of fc1's GELU + requantizing epilogue (vq_linear with act = 1 and a
 * packed output only): that epilogue first evaluates the activation with the hardware exp2 / rcp
 * and accepts the level only when it lies further from a rounding boundary than the distance
 * 2^-21 * |y| / s_y between that value and the definition's (Sec. IV-B quantizer after the
 * activation; the GELU sequence itself is this build's reading).  This call runs through every
 * finite nonzero fp32 y on the GPU and writes max |fast(y) - definition(y)| / |y| to worst_out
 * (device, one fp32; 2^-22.40 on gfx950).  Errors: VQ_ERR_NULL, VQ_ERR_HIP.
 */
vq_status vq_probe_gelu_distance(float *worst_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* VITQ_H */
