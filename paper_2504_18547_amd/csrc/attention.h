// Host-visible parameter block and launcher of the attention kernels
// (Q.K^T -> quantized shift-softmax -> P.V, fused or as separate stages).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vitq {

enum AttnMode { kAttnFused = 0, kAttnQKOnly = 1, kAttnPVOnly = 2 };

struct AttnParams {
    // operands, packed head-major [B*H*N x 64]
    const uint8_t *q, *k, *v;
    int64_t q_stride, k_stride, v_stride;
    int sb;                      // storage bits of q, k, v (4 or 8)
    int B, H, N;
    // softmax
    float alpha_scaled;          // ((s_q*s_k)*scale)*log2(e), divided by the operand scale 2^8 at 4 bits
    float alpha;                 // the same, unscaled (fills the exponential table)
    int lut_n;                   // entries of the exponential table (0: compute directly)
    int lut_full;                // 1: the table reaches the point where the exponential is 0 (its last
                                 // entry stands for every larger difference); 0: it was cut short, and
                                 // rows whose score spread exceeds it are computed directly
    int pmax;                    // 2^bits_p - 1
    // P as an input (PV-only) or output (QK-only), packed unsigned [B*H*N x N]
    const uint8_t *p_in; int64_t p_in_stride; int p_in_row_bytes16;
    uint8_t *p_out; int64_t p_out_stride; int p_out_row_bytes16;
    int p_sb;                    // storage bits of P (4 or 8)
    int32_t *s_acc_out;          // [B*H*N x N] or null
    // output side of P.V
    float spv;                   // s_p * s_v
    float s_o, qminf, qmaxf;
    float r_o, eps_o;            // 1/s_o and the guard width of the fast requantization
    int32_t *o_acc_out;          // [B*H*N x 64] or null
    float *o_out;                // [B*N x H*64] or null
    uint8_t *oq; int64_t oq_stride; int oq_sb;   // packed [B*N x H*64] or null
    int qsplit;                  // workgroups per (image, head)
};

// Returns hipErrorInvalidValue for combinations without a kernel (N > 592, sb not 4/8).
hipError_t attention_launch(const AttnParams &p, AttnMode mode, hipStream_t stream);

}  // namespace vitq
