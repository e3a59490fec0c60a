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

}  // namespace vitq
