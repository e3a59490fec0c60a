// Host-visible parameter blocks and launchers of the experimental 6-bit-float operand path:
// the reordered linear of Eq. 2 with both operands re-coded as E3M2 ("BF6") values, which hold
// the integers -8..8 exactly, contracted by the scaled-MFMA instruction at twice the int8 rate.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vitq {

// bytes of one re-coded row: 128 values -> 96 bytes, rows padded to whole groups of 128
inline int64_t f6_row_bytes(int64_t cols) { return (cols + 127) / 128 * 96; }

struct RecodeParams {
    const uint8_t *in; int64_t in_stride; int in_row_bytes16;   // packed 4-bit fields (two's complement)
    int64_t rows, cols;
    uint8_t *out; int64_t out_stride;                            // f6_row_bytes(cols) per row
};
hipError_t recode_e3m2_launch(const RecodeParams &p, hipStream_t stream);

struct F6Params {
    const uint8_t *x; int64_t x_stride; int M;        // tokens  [M x K]  re-coded
    const uint8_t *w; int64_t w_stride; int Nout;     // weights [Nout x K] re-coded
    int K;
    float s_x; const float *s_w; int s_w_per_channel; const float *bias;
    float *y_out;                                     // [M x Nout] fp32
};
hipError_t gemm_f6_launch(const F6Params &p, hipStream_t stream);

}  // namespace vitq
