// Launcher of the LayerNorm + comparator-quantizer kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vitq {

struct LnParams {
    const float *x; const float *res; float *sum_out;   // [rows x cols], leading dimension ld
    int64_t rows, cols, ld;
    const float *gamma, *beta;                           // [cols]
    float eps, step;
    uint8_t *out; int64_t out_stride; int sb; int row_bytes16;
    int qmin, qmax;
};

hipError_t layernorm_quantize_launch(const LnParams &p, hipStream_t stream);

// Q, K, V of the QKV linear (fp32 [M x 3D], leading dimension ld) -> packed head-major levels
// [3][B][H][N][64]: each 64-channel head of Q and K through the LayerNorm quantizer (own
// statistics per token and head; gamma, beta [2D]), V through the plain quantizer.
struct HeadNormParams {
    const float *y; int64_t ld;
    int B, H, N, D;
    const float *gamma, *beta;
    float eps, s_q, s_k, s_v;
    uint8_t *out; int sb; int qmin, qmax;
};

hipError_t qkv_headnorm_launch(const HeadNormParams &p, hipStream_t stream);

}  // namespace vitq
