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

// Expanded int8 copy of a packed 2- or 4-bit matrix: row r of `out` (stride kp = cols rounded up
// to 16 bytes) holds, in byte 16*j + p, the value of column 16*j + perm[p] with
// perm = {0,2,4,6, 1,3,5,7, 8,10,12,14, 9,11,13,15} -- the order in which the GEMM kernels
// unpack sixteen 4-bit activations into one MFMA operand.  Columns beyond `cols` are zero.
hipError_t prepack_launch(const uint8_t *w, int64_t rows, int64_t cols, int64_t w_stride, int sb,
                          int8_t *out, int64_t kp, hipStream_t stream);

}  // namespace vitq
