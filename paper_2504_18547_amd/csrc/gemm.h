// Host-visible parameter block and launcher of the integer GEMM kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vitq {

struct GemmParams {
    // operands (packed along K)
    const uint8_t *x; int64_t x_stride; int M;       // tokens    [M x K]
    const uint8_t *w; int64_t w_stride; int Nout;    // weights   [Nout x K]
    int K;
    int kbytes_x16, kbytes_w16;                      // valid bytes per row, rounded up to 16
    // dequantization
    float s_x; const float *s_w; int s_w_per_channel; const float *bias; int act;
    // outputs (each nullable)
    int32_t *acc_out; float *y_out; int vec_ok;      // vec_ok: Nout % 4 == 0 (aligned rows)
    const float *res;                                // nullable [M x Nout]: added to y (may alias y_out)
    uint8_t *yq; int64_t yq_stride; int yq_sb; int yq_row_bytes16;
    float s_y[3]; float qminf, qmaxf;
    // constants of the guarded fast requantization (see gemm.hip): 1/s_y, the guard widths
    float r_y[3]; float eps0; float gelu_guard;
    // head-major output of the QKV linear: channel -> (q/k/v, head, d), token -> (image, n)
    int head_major; int D, dh, Ntok, Bimg, Hh;
    int dh_shift; float inv_ntok;                    // filled by gemm_launch
    // per-head LayerNorm quantizers on Q and K inside the head-major epilogue (Sec. IV-C): gamma
    // and beta are [2*D] (Q then K), the steps are s_y[0], s_y[1]; V keeps the plain quantizer.
    // Needs dh == 64.  Null: plain quantizers on all three.
    const float *hn_gamma, *hn_beta; float hn_eps;
    // integer-only epilogue (Eq. 2 with the equivalent bias in the integer domain, scales absorbed
    // into the comparator references): level = qmin + #{t : acc + ab_bint[c] > ab_thr[c][t]}.
    // ab_thr [Nout][ab_nthr] non-decreasing per channel, ab_bint [Nout] nullable; s_x, s_w, bias,
    // s_y are not read.  Null ab_thr: the floating-point epilogues.
    const int32_t *ab_bint, *ab_thr; int ab_nthr;
};

// wb / ab: storage bits of the weight / activation operand.  Supported: (4,4) (2,4) (8,8).
// Fills the fast-path constants of p itself.
hipError_t gemm_launch(GemmParams p, int wb, int ab, hipStream_t stream);

}  // namespace vitq
