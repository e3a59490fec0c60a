// Measurement aid: what the matrix cores of this machine deliver to a register-resident loop of
// v_mfma_i32_32x32x32_i8 (no memory, no LDS, no other arithmetic), with operands of the kind the
// GEMM kernels feed (int8 values whose low nibble is zero).  bench.py times it and reports the
// rate beside the published peak.  Second aid: the exhaustive distance between the fast GELU of the
// linear's epilogue and the definition's, which is what that epilogue's guard rests on.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/vitq.h"
#include "vitq_dev.h"

namespace vitq {
namespace {

constexpr int kProbeWavesPerSimd = 4;

__global__ __launch_bounds__(256) void mfma_probe_kernel(int iters, int32_t *sink) {
    const int t = threadIdx.x;
    // sixteen 4-bit levels per operand, each moved to the top of its byte (16 * level)
    v4i a, b;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = (int)(((u32)(t * 2654435761u + i * 40503u)) & 0xF0F0F0F0u);
        b[i] = (int)(((u32)(t * 2246822519u + i * 69069u + blockIdx.x)) & 0xF0F0F0F0u);
    }
    v16i c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(b, a, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(b, a, c3, 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) s += c0[r] ^ c1[r] ^ c2[r] ^ c3[r];
    if (s == 0x7fffffff && sink) sink[0] = s;        // keeps the loop alive; practically never true
}

// Largest |gelu_fast(y) - gelu_tanh(y)| / |y| over every finite nonzero fp32 y (bit patterns are strided
// over the grid; the maximum is taken on the bit patterns, where unsigned order is float order).
__global__ __launch_bounds__(256) void gelu_distance_kernel(u32 *worst) {
    u32 m = 0;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t b = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; b < (1ull << 32); b += stride) {
        const float y = __uint_as_float((u32)b);
        if (!(fabsf(y) < 3.0e38f) || y == 0.0f) continue;
        const float r = fabsf(gelu_fast(y) - gelu_tanh(y)) / fabsf(y);
        if (r == r) m = max(m, __float_as_uint(r));
    }
    atomicMax(worst, m);
}

}  // namespace
}  // namespace vitq

extern "C" vq_status vq_probe_mfma_i8(int32_t iters, int32_t *sink, double *ops_out, void *stream) {
    if (iters < 1 || iters > (1 << 22)) return VQ_ERR_SHAPE;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return VQ_ERR_HIP;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return VQ_ERR_HIP;
    const int blocks = cus * vitq::kProbeWavesPerSimd;                  // 4 waves per block: one per SIMD
    hipLaunchKernelGGL(vitq::mfma_probe_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, iters, sink);
    if (hipGetLastError() != hipSuccess) return VQ_ERR_HIP;
    if (ops_out) *ops_out = (double)blocks * 4.0 * (double)iters * 4.0 * 65536.0;   // 2 * 32*32*32 per instruction
    return VQ_OK;
}

extern "C" vq_status vq_probe_gelu_distance(float *worst_out, void *stream) {
    if (!worst_out) return VQ_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    if (hipMemsetAsync(worst_out, 0, sizeof(float), st) != hipSuccess) return VQ_ERR_HIP;
    hipLaunchKernelGGL(vitq::gelu_distance_kernel, dim3(4096), dim3(256), 0, st, reinterpret_cast<vitq::u32 *>(worst_out));
    return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}
