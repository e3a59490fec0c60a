// Device-side helpers shared by the vitq kernels (gfx950 only).
//
// Every fp32 value that reaches a quantizer is produced by an explicit, fixed sequence of
// correctly rounded operations (v_div via '/', v_fma via fmaf, v_rndne, v_floor, v_ldexp);
// the translation units are compiled with -ffp-contract=off so nothing is fused or split.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <utility>

namespace vitq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int u32;

constexpr int kWave = 64;

// Compile-time loop: the body receives std::integral_constant indices, so register arrays are
// only ever indexed by constants (a run-time index would push them to scratch memory).
template <int... I, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F &&f) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
    static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

// ---------------------------------------------------------------------------------------
// Uniform quantizer: clamp(round-half-even(y / s), qmin, qmax).  (Sec. IV-B / IV-C thresholds
// at (k - 1/2) * step.)  The division is the correctly rounded IEEE one.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ int quantize_level(float y, float s, float qminf, float qmaxf) {
    float t = y / s;
    float r = rintf(t);
    r = fmaxf(r, qminf);
    r = fminf(r, qmaxf);
    return (int)r;
}

// ---------------------------------------------------------------------------------------
// GELU, tanh form, with 2^t evaluated by range reduction and a degree-7 polynomial so that
// the result is the same on any IEEE machine.  The paper gives no GELU (it integerizes
// self-attention and notes the idea extends to the rest of the block, Sec. III).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float exp2_poly(float t) {
    float n = rintf(t);
    float x = t - n;
    float p = 0x1.ffcbfcp-17f;
    p = fmaf(p, x, 0x1.430912p-13f);
    p = fmaf(p, x, 0x1.5d87fep-10f);
    p = fmaf(p, x, 0x1.3b2ab6p-7f);
    p = fmaf(p, x, 0x1.c6b08ep-5f);
    p = fmaf(p, x, 0x1.ebfbe0p-3f);
    p = fmaf(p, x, 0x1.62e430p-1f);
    p = fmaf(p, x, 1.0f);
    return ldexpf(p, (int)n);
}

__device__ __forceinline__ float gelu_tanh(float y) {
    float y3 = (y * y) * y;
    float inner = fmaf(0x1.6e4e26p-5f, y3, y);
    float u = 0x1.988454p-1f * inner;
    float t = (2.0f * u) * 0x1.715476p+0f;
    t = fmaxf(t, -126.0f);
    t = fminf(t, 126.0f);
    float X = exp2_poly(t);
    float th = 1.0f - 2.0f / (1.0f + X);
    return (0.5f * y) * (1.0f + th);
}

// The same activation from the hardware transcendentals, for a first guess that a guard then accepts or
// sends to gelu_tanh: 0.5*y*(1+tanh(u)) = y - y/(1 + 2^(2u*log2 e)) with 2u*log2e = y*(k0 + k1*y^2).
// Over every finite fp32 y its distance from gelu_tanh(y) is at most 2^-22.40 * |y| (exhaustive run on
// the GPU; vq_probe_gelu_distance repeats it), so kGeluFastBound = 2^-21 * |y| bounds it with room.
__device__ __forceinline__ float gelu_fast(float y) {
    const float y2 = y * y;
    const float w = fmaf(y2, 0x1.a5a7d0p-4f, 0x1.26aec2p+1f);
    const float X = __builtin_amdgcn_exp2f(w * y);
    const float rc = __builtin_amdgcn_rcpf(1.0f + X);
    return fmaf(-y, rc, y);
}
constexpr float kGeluFastBound = 0x1p-21f;

// ---------------------------------------------------------------------------------------
// Unpacking packed low-bit fields into int8 MFMA operands WITHOUT sign extension: a signed
// b-bit field moved to the top b bits of a byte is the int8 value 2^(8-b) * q.  The products
// then carry a known power-of-two factor that the epilogue removes with an exact shift.
// The order of the 16 values inside one lane's operand is permuted; both operands of a
// contraction use the same permutation, which leaves the sum unchanged.
// ---------------------------------------------------------------------------------------
// 8 nibbles n0..n7 -> lo = 16*{n0,n2,n4,n6}, hi = 16*{n1,n3,n5,n7}
__device__ __forceinline__ void nib_split(u32 w, int &lo, int &hi) {
    lo = (int)((w << 4) & 0xF0F0F0F0u);
    hi = (int)(w & 0xF0F0F0F0u);
}

// two packed words (16 nibbles) -> one MFMA operand, value order (0,2,4,6 | 1,3,5,7 | 8,.. | 9,..)
__device__ __forceinline__ v4i unpack4_x16(u32 w0, u32 w1) {
    v4i r;
    int a, b, c, d;
    nib_split(w0, a, b);
    nib_split(w1, c, d);
    r[0] = a; r[1] = b; r[2] = c; r[3] = d;
    return r;
}

// one packed word of 16 two-bit fields c0..c15 -> 64*{c0,c4,c8,c12 | c1,c5,.. | c2,.. | c3,..}
__device__ __forceinline__ v4i unpack2_x64(u32 w) {
    v4i r;
    r[0] = (int)((w << 6) & 0xC0C0C0C0u);
    r[1] = (int)((w << 4) & 0xC0C0C0C0u);
    r[2] = (int)((w << 2) & 0xC0C0C0C0u);
    r[3] = (int)(w & 0xC0C0C0C0u);
    return r;
}

// two packed nibble words -> operand in the value order of unpack2_x64:
// (0,4,8,12 | 1,5,9,13 | 2,6,10,14 | 3,7,11,15), each value times 16
__device__ __forceinline__ v4i unpack4_x16_order2(u32 w0, u32 w1) {
    int lo0, hi0, lo1, hi1;
    nib_split(w0, lo0, hi0);   // lo0 = {n0,n2,n4,n6}, hi0 = {n1,n3,n5,n7}
    nib_split(w1, lo1, hi1);   // lo1 = {n8,n10,n12,n14}, hi1 = {n9,n11,n13,n15}
    v4i r;
    // v_perm_b32(src0, src1, sel): selector values 0..3 pick bytes of src1, 4..7 bytes of src0
    r[0] = (int)__builtin_amdgcn_perm((u32)lo1, (u32)lo0, 0x06040200u);  // n0,n4,n8,n12
    r[1] = (int)__builtin_amdgcn_perm((u32)hi1, (u32)hi0, 0x06040200u);  // n1,n5,n9,n13
    r[2] = (int)__builtin_amdgcn_perm((u32)lo1, (u32)lo0, 0x07050301u);  // n2,n6,n10,n14
    r[3] = (int)__builtin_amdgcn_perm((u32)hi1, (u32)hi0, 0x07050301u);  // n3,n7,n11,n15
    return r;
}

// Pack sixteen levels (already clamped) into storage fields, element 0 in the low field.
template <int SB>
__device__ __forceinline__ void pack16(const int (&q)[16], u32 (&out)[4]) {
    if constexpr (SB == 4) {
        u32 a = 0, b = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a |= ((u32)q[i] & 0xFu) << (4 * i);
            b |= ((u32)q[8 + i] & 0xFu) << (4 * i);
        }
        out[0] = a; out[1] = b; out[2] = 0; out[3] = 0;
    } else if constexpr (SB == 8) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            u32 a = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) a |= ((u32)q[4 * j + i] & 0xFFu) << (8 * i);
            out[j] = a;
        }
    } else {
        u32 a = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) a |= ((u32)q[i] & 0x3u) << (2 * i);
        out[0] = a; out[1] = 0; out[2] = 0; out[3] = 0;
    }
}

}  // namespace vitq
