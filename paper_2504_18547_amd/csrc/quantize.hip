// Uniform b-bit quantizer writing the packed format, and the absmax weight-step rule.
// Both are streaming kernels bound by HBM: the quantizer reads 4 bytes and writes b/8 bytes
// per element.
#include "quantize.h"
#include "vitq_dev.h"

namespace vitq {

namespace {

// One thread produces one 32-bit word of a packed row (32/SB consecutive levels), so a wave
// reads a contiguous run of fp32 values and writes 256 contiguous bytes.
template <int SB>
__global__ __launch_bounds__(256) void quantize_kernel(QuantParams p) {
    constexpr int PER = 32 / SB;
    const int words_per_row = p.row_bytes16 / 4;
    const int64_t total = p.rows * words_per_row;
    for (int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; id < total;
         id += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = id / words_per_row;
        const int wi = (int)(id - r * words_per_row);
        const float s = p.step_per_row ? p.step_per_row[r] : p.step;
        const float *src = p.x + r * p.ld;
        const int64_t c0 = (int64_t)wi * PER;
        u32 word = 0;
        if (c0 + PER <= p.cols && (((uintptr_t)(src + c0)) & 15) == 0) {
            float f[PER];
#pragma unroll
            for (int j = 0; j < PER / 4; ++j) {
                float4 v = reinterpret_cast<const float4 *>(src + c0)[j];
                f[4 * j] = v.x; f[4 * j + 1] = v.y; f[4 * j + 2] = v.z; f[4 * j + 3] = v.w;
            }
            // Guarded fast path (the same scheme as the linear's requantizing epilogue): with r = RN(1/s),
            // g = 2^(bits-22) and C = -qmin + 1/2 - g, u = fma(x, r, C) is within g of x/s - qmin + 1/2 - g
            // for |x/s| <= qmax + 2; unless fract(u) >= 1 - 2g the level is floor(u), clamped.  A thread with
            // an element inside the guard (or a NaN, whose fraction compares above everything as a bit
            // pattern) redoes its word with the division.
            const float r = 1.0f / s;
            const bool fast = r > 0x1p-100f && r < 0x1p100f;
            const float g = (p.qmaxf > 7.5f) ? 0x1p-14f : 0x1p-18f;
            const float C = (0.5f - p.qminf) - g;
            const float top = p.qmaxf - p.qminf;
            u32 worst = fast ? 0u : 0x7F800000u;
            int lv[PER];
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const float u = fmaf(f[i], r, C);
                const float z = __builtin_amdgcn_fractf(u);
                worst = max(worst, __float_as_uint(z));
                lv[i] = (int)__builtin_amdgcn_fmed3f(u - z, 0.0f, top) + (int)p.qminf;
            }
            if (worst > __float_as_uint(1.0f - 2.0f * g) - 1u) {
#pragma unroll
                for (int i = 0; i < PER; ++i) lv[i] = quantize_level(f[i], s, p.qminf, p.qmaxf);
            }
#pragma unroll
            for (int i = 0; i < PER; ++i) word |= ((u32)lv[i] & ((1u << SB) - 1u)) << (SB * i);
        } else {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                if (c0 + i < p.cols) {
                    int q = quantize_level(src[c0 + i], s, p.qminf, p.qmaxf);
                    word |= ((u32)q & ((1u << SB) - 1u)) << (SB * i);
                }
            }
        }
        *reinterpret_cast<u32 *>(p.out + r * p.out_stride + (int64_t)wi * 4) = word;
    }
}

// One wave per row: max |w| by a butterfly over the 64 lanes (max is order-independent).
__global__ __launch_bounds__(256) void weight_steps_kernel(const float *w, int64_t rows, int64_t cols,
                                                           int64_t ld, float qmaxf, float *step_out) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * (blockDim.x / 64) + (threadIdx.x >> 6);
    if (row >= rows) return;
    const float *src = w + row * ld;
    float m = 0.0f;
    for (int64_t c = lane; c < cols; c += 64) m = fmaxf(m, fabsf(src[c]));
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if (lane == 0) step_out[row] = (m == 0.0f) ? 1.0f : m / qmaxf;
}

}  // namespace

// one thread per group of sixteen columns
__global__ __launch_bounds__(256) void prepack_kernel(const uint8_t *w, int64_t rows, int64_t cols,
                                                      int64_t w_stride, int sb, int8_t *out, int64_t kp) {
    const int64_t groups = kp / 16;
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= rows * groups) return;
    const int64_t r = id / groups, j = id % groups;
    int v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int64_t c = 16 * j + i;
        int q = 0;
        if (c < cols) {
            const int64_t bit = c * sb;
            const int field = (w[r * w_stride + (bit >> 3)] >> (bit & 7)) & ((1 << sb) - 1);
            q = (field << (32 - sb)) >> (32 - sb);      // sign extension of the sb-bit field
        }
        v[i] = q;
    }
    const int perm[16] = {0, 2, 4, 6, 1, 3, 5, 7, 8, 10, 12, 14, 9, 11, 13, 15};
    u32 o[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        u32 x = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) x |= ((u32)v[perm[4 * d + b]] & 0xFFu) << (8 * b);
        o[d] = x;
    }
    *reinterpret_cast<uint4 *>(out + r * kp + 16 * j) = make_uint4(o[0], o[1], o[2], o[3]);
}

hipError_t quantize_launch(const QuantParams &p, hipStream_t stream) {
    const int64_t total = p.rows * (p.row_bytes16 / 4);
    if (total == 0) return hipSuccess;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    if (p.sb == 4) hipLaunchKernelGGL(quantize_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, stream, p);
    else if (p.sb == 8) hipLaunchKernelGGL(quantize_kernel<8>, dim3((unsigned)blocks), dim3(256), 0, stream, p);
    else hipLaunchKernelGGL(quantize_kernel<2>, dim3((unsigned)blocks), dim3(256), 0, stream, p);
    return hipGetLastError();
}

hipError_t weight_steps_launch(const float *w, int64_t rows, int64_t cols, int64_t ld, float qmaxf,
                               float *step_out, hipStream_t stream) {
    if (rows == 0) return hipSuccess;
    int64_t blocks = (rows + 3) / 4;
    hipLaunchKernelGGL(weight_steps_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, w, rows, cols, ld,
                       qmaxf, step_out);
    return hipGetLastError();
}

hipError_t prepack_launch(const uint8_t *w, int64_t rows, int64_t cols, int64_t w_stride, int sb,
                          int8_t *out, int64_t kp, hipStream_t stream) {
    const int64_t n = rows * (kp / 16);
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(prepack_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, w, rows, cols,
                       w_stride, sb, out, kp);
    return hipGetLastError();
}

}  // namespace vitq
