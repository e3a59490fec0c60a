// Launchers of the element-wise quantizer kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vitq {

struct QuantParams {
    const float *x; int64_t rows, cols, ld;
    float step; const float *step_per_row;
    uint8_t *out; int64_t out_stride; int sb; int row_bytes16;
    float qminf, qmaxf;
};

hipError_t quantize_launch(const QuantParams &p, hipStream_t stream);
hipError_t weight_steps_launch(const float *w, int64_t rows, int64_t cols, int64_t ld, float qmaxf,
                               float *step_out, hipStream_t stream);

}  // namespace vitq
