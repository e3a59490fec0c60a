// Integer GEMM with fused dequant / bias / GELU / requant epilogue (reordered linear, Eq. 2).
//
//   acc[m][c] = sum_k xq[m][k] * wq[c][k]      int8 MFMA (v_mfma_i32_32x32x32_i8), int32 exact
//   y         = fma((float)acc, s_x*s_w[c], b[c]);  optional GELU;  optional requantization
//
// Both operands stay PACKED (b-bit fields) in HBM and in LDS; a lane unpacks its fragment to
// int8 in registers right before the MFMA (2^(8-b)-scaled values, see vitq_dev.h), and the
// epilogue removes the scale exactly.
//
// MFMA roles: the A operand (32 rows) carries WEIGHT rows (output channels), the B operand
// (32 columns) carries TOKEN rows, so a lane of the 32x32 result holds 16 output channels of
// ONE token.  Weight rows are placed in LDS in a permuted slot order so that those 16 channels
// are consecutive: the lane then packs them into one 8-byte (4-bit) store of the token's
// output row, which is exactly the packed operand layout the next linear reads.
//
// Epilogues.  The definition of a requantized output is level = clamp(rint(y / s)) with an IEEE
// division.  The throughput epilogues evaluate a cheaper expression (multiplication by 1/s,
// hardware exp2/rcp inside GELU) whose distance from the definition is bounded; an element
// whose cheap value lies within that bound of a rounding boundary is recomputed with the exact
// operation sequence.  The result is therefore always the definition's, bit for bit.
#include "gemm.h"
#include <type_traits>
#include "launch_util.h"
#include "vitq_dev.h"

namespace vitq {

namespace {

#ifndef VITQ_TC
#define VITQ_TC 128
#define VITQ_TT 256
#define VITQ_WC 2
#define VITQ_WT 4
#define VITQ_BK44 128
#define VITQ_S44 3
#define VITQ_OCC44 4
#endif
#ifndef VITQ_BK88
#define VITQ_BK88 64
#define VITQ_S88 3
#define VITQ_OCC88 3
#endif
#ifndef VITQ_BK84
#define VITQ_BK84 128
#define VITQ_S84 2
#define VITQ_OCC84 4
#endif
enum Epi { kEpiGeneric = 0, kEpiF32 = 1, kEpiQuant = 2, kEpiQuantGelu = 3, kEpiHeadNorm = 4, kEpiAbsorbed = 5, kEpiAbsorbedBig = 6 };   // Big: more than 15 references per channel

// channel c (0..31 within a 32-block) -> MFMA row slot, chosen so that a lane's sixteen
// accumulator registers (rows 8*(r/4) + 4*(lane/32) + r%4) are channels 16*(lane/32) + r
__device__ __forceinline__ int slot_of_channel(int c) {
    return 8 * ((c & 15) >> 2) + 4 * (c >> 4) + (c & 3);
}

template <int WB, int AB>
struct Shift {
    // (8,4): weights expanded to plain int8 beforehand, activations unpacked to 16*x
    static constexpr int value = (WB == 4 && AB == 4) ? 8 : (WB == 2 && AB == 4) ? 10 : (WB == 8 && AB == 4) ? 4 : 0;
};

template <int SB>
__device__ __forceinline__ void store_packed16(uint8_t *dst, const int (&q)[16]) {
    u32 w[4];
    pack16<SB>(q, w);
    if constexpr (SB == 4) {
        *reinterpret_cast<uint2 *>(dst) = make_uint2(w[0], w[1]);
    } else if constexpr (SB == 8) {
        *reinterpret_cast<uint4 *>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
    } else {
        *reinterpret_cast<u32 *>(dst) = w[0];
    }
}

// Destination of a lane's 16 packed levels = yq + token part + channel part (the address is
// linear in both).  Head-major mode: channel -> (q/k/v, head, d), token -> (image, n).  The two
// divisions avoid the integer-division expansion: the channel one by comparisons (3D channels)
// and a shift when the head size is a power of two; the token one by an fp32 reciprocal with a
// one-step correction (exact for m < 2^22).  A negative part marks "nothing to store".
__device__ __forceinline__ int64_t packed_token_part(const GemmParams &p, int m) {
    if (m >= p.M) return -1;
    if (p.head_major) {
        int b = (int)((float)m * p.inv_ntok);
        int n = m - b * p.Ntok;
        if (n < 0) { b -= 1; n += p.Ntok; }
        if (n >= p.Ntok) { b += 1; n -= p.Ntok; }
        return ((int64_t)b * p.Hh * p.Ntok + n) * p.yq_stride;
    }
    return (int64_t)m * p.yq_stride;
}
__device__ __forceinline__ int64_t packed_channel_part(const GemmParams &p, int cb, int &which) {
    which = 0;
    if (p.head_major) {
        if (cb >= p.Nout) return -1;
        which = (cb >= p.D ? 1 : 0) + (cb >= 2 * p.D ? 1 : 0);
        const int rem = cb - which * p.D;
        int h, d;
        if (p.dh_shift >= 0) { h = rem >> p.dh_shift; d = rem & (p.dh - 1); }
        else { h = rem / p.dh; d = rem - h * p.dh; }
        return (((int64_t)which * p.Bimg * p.Hh + h) * p.Ntok) * p.yq_stride + ((d * p.yq_sb) >> 3);
    }
    if (((cb * p.yq_sb) >> 3) >= p.yq_row_bytes16) return -1;
    return (cb * p.yq_sb) >> 3;
}
__device__ __forceinline__ uint8_t *packed_dst(const GemmParams &p, int m, int cb, int &which) {
    const int64_t t = packed_token_part(p, m), c = packed_channel_part(p, cb, which);
    if (t < 0 || c < 0) return nullptr;
    return p.yq + t + c;
}

// ---- exact epilogue: every output kind, the definition's operation sequence ------------------
__device__ __forceinline__ void epilogue_generic(const GemmParams &p, const v16i &acc, int shift,
                                                 int m, int cb) {
    if (m >= p.M) return;
    const int nvalid = p.Nout - cb;  // may be <= 0 for a group that only exists as padding
    const bool full = nvalid >= 16;
    float y[16];
    int a[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int c = cb + r;
        const bool ok = c < p.Nout;
        // (an accumulators-only call carries no scales)
        const float sc = p.s_x * ((ok && p.s_w) ? p.s_w[p.s_w_per_channel ? c : 0] : 1.0f);
        const float bsr = (ok && p.bias) ? p.bias[c] : 0.0f;
        a[r] = acc[r] >> shift;
        float v = fmaf((float)a[r], sc, bsr);
        if (p.act == 1) v = gelu_tanh(v);
        if (p.res && ok && m < p.M) v = v + p.res[(int64_t)m * p.Nout + c];
        y[r] = v;
    }
    const bool vec = full && p.vec_ok;
    if (p.acc_out) {
        int32_t *dst = p.acc_out + (int64_t)m * p.Nout + cb;
        if (vec) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                reinterpret_cast<int4 *>(dst)[j] = make_int4(a[4 * j], a[4 * j + 1], a[4 * j + 2], a[4 * j + 3]);
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (r < nvalid) dst[r] = a[r];
        }
    }
    if (p.y_out) {
        float *dst = p.y_out + (int64_t)m * p.Nout + cb;
        if (vec) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                reinterpret_cast<float4 *>(dst)[j] = make_float4(y[4 * j], y[4 * j + 1], y[4 * j + 2], y[4 * j + 3]);
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (r < nvalid) dst[r] = y[r];
        }
    }
    if (p.yq) {
        int which;
        uint8_t *dst = packed_dst(p, m, cb, which);
        if (!dst) return;
        const float sy0 = p.s_y[0], sy1 = p.s_y[1], sy2 = p.s_y[2];
        const float s_y = which == 0 ? sy0 : (which == 1 ? sy1 : sy2);
        int q[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int lv = quantize_level(y[r], s_y, p.qminf, p.qmaxf);
            q[r] = (r < nvalid) ? lv : 0;
        }
        if (p.yq_sb == 4) store_packed16<4>(dst, q);
        else if (p.yq_sb == 8) store_packed16<8>(dst, q);
        else store_packed16<2>(dst, q);
    }
}

// ---- fp32-only epilogue (Nout % 16 == 0) -------------------------------------------------------
// This epilogue runs with the MFMA roles SWAPPED (tokens on the A side, weight rows on the B
// side, weight rows unpermuted in LDS): a lane then holds ONE channel of sixteen tokens, and
// register r of the wave is 32 consecutive channels (one full 128-byte line) of tokens
// m0 + 8*(r/4) + r%4 (+4 for the upper half-wave).  Every store instruction therefore writes
// two complete lines instead of 64 scattered 16-byte pieces.
// The caller passes the folded scale (sc * 2^-shift exactly, so fma((float)acc_scaled, scs, b) ==
// fma((float)acc, sc, b)) with shift 0, or, when the fold was inexact, the plain one and the shift.
template <bool FULL, bool RES>   // FULL: the whole tile lies inside the matrix (no per-element tests); RES: residual given
__device__ __forceinline__ void epilogue_f32(const GemmParams &p, const v16i &acc, int shift, int m0, int ch,
                                             float sc, float bs, const float (&rv)[16]) {
    if (!FULL && ch >= p.Nout) return;
    float *out = p.y_out + (int64_t)m0 * p.Nout + ch;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int dm = 8 * (r >> 2) + (r & 3);
        if (FULL || m0 + dm < p.M) {
            float y = fmaf((float)(acc[r] >> shift), sc, bs);
            if constexpr (RES) y = y + rv[r];               // residual stream
            out[(int64_t)dm * p.Nout] = y;
        }
    }
}
// The residual elements of one 32x32 block, in the register order of epilogue_f32 (each element
// is read by the lane that later writes it, so the stream may be updated in place).
template <bool FULL>
__device__ __forceinline__ void load_residual(const GemmParams &p, int m0, int ch, float (&rv)[16]) {
    if (!FULL && ch >= p.Nout) return;
    const float *res = p.res + (int64_t)m0 * p.Nout + ch;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int dm = 8 * (r >> 2) + (r & 3);
        if (FULL || m0 + dm < p.M) rv[r] = res[(int64_t)dm * p.Nout];
    }
}

// Packs sixteen levels (floats holding level - qmin, i.e. 0 .. qmax - qmin) into 4- or 8-bit
// two's-complement fields and stores them: 8 or 16 bytes at dst.
__device__ __forceinline__ void pack_store16(const GemmParams &p, uint8_t *dst, const float (&lv)[16], float bias8) {
    if (p.yq_sb == 4) {
        // even-indexed levels in the low nibbles of one word, odd-indexed shifted into the high
        u32 ev0 = 0, od0 = 0, ev1 = 0, od1 = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            ev0 = __builtin_amdgcn_cvt_pk_u8_f32(lv[2 * i], i, ev0);
            od0 = __builtin_amdgcn_cvt_pk_u8_f32(lv[2 * i + 1], i, od0);
            ev1 = __builtin_amdgcn_cvt_pk_u8_f32(lv[8 + 2 * i], i, ev1);
            od1 = __builtin_amdgcn_cvt_pk_u8_f32(lv[8 + 2 * i + 1], i, od1);
        }
        // stored levels are biased by -qmin = 2^(bits-1); remove it per nibble, modulo 16 and
        // without borrows across nibbles (for 4-bit levels this is a flip of bit 3)
        const u32 a0 = ev0 | (od0 << 4), a1 = ev1 | (od1 << 4);
        u32 w0, w1;
        if (bias8 == 8.0f) {                 // (uniform) 4-bit levels: subtracting 8 modulo 16 flips bit 3
            w0 = a0 ^ 0x88888888u;
            w1 = a1 ^ 0x88888888u;
        } else {
            const u32 fix = 0x11111111u * ((u32)bias8 & 0xFu);
            w0 = ((a0 | 0x88888888u) - (fix & 0x77777777u)) ^ ((a0 ^ ~fix) & 0x88888888u);
            w1 = ((a1 | 0x88888888u) - (fix & 0x77777777u)) ^ ((a1 ^ ~fix) & 0x88888888u);
        }
        *reinterpret_cast<uint2 *>(dst) = make_uint2(w0, w1);
    } else {
        // 8-bit storage: the bias -qmin = 2^(bits-1) is removed modulo 256
        const u32 fix = 0x01010101u * ((u32)bias8 & 0xFFu);
        u32 w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            u32 v = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) v = __builtin_amdgcn_cvt_pk_u8_f32(lv[4 * j + i], i, v);
            // per-byte subtraction of the bias: (v - fix) without borrows across bytes
            w[j] = ((v | 0x80808080u) - (fix & 0x7F7F7F7Fu)) ^ ((v ^ ~fix) & 0x80808080u);
        }
        *reinterpret_cast<uint4 *>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// Eight levels (floats holding level - qmin) -> one word of 4-bit fields (w[0]) or two words of
// 8-bit fields, two's complement, bias removed.
__device__ __forceinline__ void pack8(const GemmParams &p, const float (&lv)[8], float bias8, u32 (&w)[2]) {
    if (p.yq_sb == 4) {
        u32 ev = 0, od = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            ev = __builtin_amdgcn_cvt_pk_u8_f32(lv[2 * i], i, ev);
            od = __builtin_amdgcn_cvt_pk_u8_f32(lv[2 * i + 1], i, od);
        }
        const u32 a = ev | (od << 4);
        if (bias8 == 8.0f) {                 // (uniform) 4-bit levels: subtracting 8 modulo 16 flips bit 3
            w[0] = a ^ 0x88888888u;
        } else {
            const u32 fix = 0x11111111u * ((u32)bias8 & 0xFu);
            w[0] = ((a | 0x88888888u) - (fix & 0x77777777u)) ^ ((a ^ ~fix) & 0x88888888u);
        }
        w[1] = 0;
    } else {
        const u32 fix = 0x01010101u * ((u32)bias8 & 0xFFu);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            u32 v = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) v = __builtin_amdgcn_cvt_pk_u8_f32(lv[4 * j + i], i, v);
            w[j] = ((v | 0x80808080u) - (fix & 0x7F7F7F7Fu)) ^ ((v ^ ~fix) & 0x80808080u);
        }
    }
}

// A 16-channel group that lies wholly beyond the last output channel but inside the 16-byte
// padded row: the packed format wants zero bytes there.
__device__ __forceinline__ void store_zero_group(const GemmParams &p, uint8_t *dst) {
    if (!dst) return;
    if (p.yq_sb == 4) *reinterpret_cast<uint2 *>(dst) = make_uint2(0u, 0u);
    else *reinterpret_cast<uint4 *>(dst) = make_uint4(0u, 0u, 0u, 0u);
}

// ---- guarded fast requantization (Nout % 16 == 0; 4- or 8-bit storage) ------------------------
// Definition: level = clamp(rint(T)), T = RN(y / s).  Cheap value: with r = RN(1/s), g = eps0 =
// 2^(bits-22) and C = -qmin + 1/2 - g (exactly representable),
//     u = fma(y, r, C),   |u - (T - qmin + 1/2 - g)| <= |T| * 2^-23 + ulp(u)/2  <  g   for |T| <= qmax + 2.
// If fract(u) < 1 - 2g then T - qmin + 1/2 lies strictly inside (floor(u), floor(u) + 1): it is not
// a tie and rint(T) - qmin = floor(u) = u - fract(u) (an exact subtraction).  Otherwise the element
// sits within the error bound of a rounding boundary and is redone with the definition's own
// operations.  Beyond |T| = qmax + 2 both clamp to the same level; a NaN or infinity gives a NaN
// fraction, whose bit pattern compares above every threshold, so it is redone too.
// With GELU the cheap activation (gelu_fast: hardware exp2 / rcp) is within kGeluFastBound * |y| of the
// definition's, which widens the guard per element (there the test is on |t - rint(t)|).
// The sixteen channels of a lane are done in two halves of eight (each with its own test and, if
// need be, its own exact redo): the working set stays small enough for four waves per SIMD.
// lscs / lbs: this lane's sixteen folded scales and biases in LDS.
template <bool GELU>
__device__ __forceinline__ void epilogue_quant(const GemmParams &p, const v16i &acc, int shift, uint8_t *dst,
                                               float s_y, float r_y, int cb, const float *lscs, const float *lbs,
                                               bool force_exact) {
    if (!dst) return;
    const float bias8 = -p.qminf;
    const float top = p.qmaxf - p.qminf;
    u32 words[4];
    static_for<2>([&](auto H) {
        constexpr int h = decltype(H)::value;
        float scs[8], bs[8];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const float4 a = *reinterpret_cast<const float4 *>(lscs + 8 * h + 4 * j);
            const float4 b = *reinterpret_cast<const float4 *>(lbs + 8 * h + 4 * j);
            scs[4 * j] = a.x; scs[4 * j + 1] = a.y; scs[4 * j + 2] = a.z; scs[4 * j + 3] = a.w;
            bs[4 * j] = b.x; bs[4 * j + 1] = b.y; bs[4 * j + 2] = b.z; bs[4 * j + 3] = b.w;
        }
        float lv[8];
        // worst = max over the elements of a non-negative per-element figure, taken on the bit
        // patterns: there unsigned order is float order and a NaN compares above everything (so
        // it is caught, which a float max would drop)
        u32 worst = force_exact ? 0x7F800000u : 0u;
        u32 fig[8];
        u32 limit;
        if constexpr (GELU) {
            const float gguard = p.gelu_guard * r_y;
            limit = __float_as_uint(0.5f - p.eps0);
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const float y = fmaf((float)acc[8 * h + r], scs[r], bs[r]);        // the definition's y, exactly
                const float g = gelu_fast(y);
                const float t8 = fmaf(g, r_y, bias8);
                const float q8 = rintf(t8);
                fig[r] = __float_as_uint(fmaf(fabsf(y), gguard, fabsf(t8 - q8)));
                lv[r] = __builtin_amdgcn_fmed3f(q8, 0.0f, top);
            }
        } else {
            const float C = (bias8 + 0.5f) - p.eps0;
            limit = __float_as_uint(1.0f - 2.0f * p.eps0) - 1u;              // risky: fract(u) >= 1 - 2g
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const float y = fmaf((float)acc[8 * h + r], scs[r], bs[r]);        // the definition's y, exactly
                const float u = fmaf(y, r_y, C);
                const float z = __builtin_amdgcn_fractf(u);
                fig[r] = __float_as_uint(z);
                lv[r] = __builtin_amdgcn_fmed3f(u - z, 0.0f, top);
            }
        }
#pragma unroll
        for (int r = 0; r < 8; r += 2) worst = max(worst, max(fig[r], fig[r + 1]));
        const bool risky = worst > limit;
        if (__builtin_amdgcn_ballot_w64(risky) != 0) {
            // some element of these eight channels x 32 tokens sits within the error bound of a rounding
            // boundary: redo them with the definition's exact operation sequence (rare)
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                // (re-read the channel's step: the folded copy may be inexact when force_exact is set)
                const float sc = p.s_x * p.s_w[p.s_w_per_channel ? cb + 8 * h + r : 0];
                float ye = fmaf((float)(acc[8 * h + r] >> shift), sc, bs[r]);
                if constexpr (GELU) ye = gelu_tanh(ye);
                const float te = rintf(ye / s_y) + bias8;
                lv[r] = __builtin_amdgcn_fmed3f(te, 0.0f, top);
            }
        }
        u32 w2[2];
        pack8(p, lv, bias8, w2);
        words[2 * h] = w2[0];
        words[2 * h + 1] = w2[1];
    });
    if (p.yq_sb == 4) *reinterpret_cast<uint2 *>(dst) = make_uint2(words[0], words[2]);
    else *reinterpret_cast<uint4 *>(dst) = make_uint4(words[0], words[1], words[2], words[3]);
}

// ---- per-head LayerNorm quantizers of Q and K in the QKV epilogue (Sec. IV-C, Table I) ----------
// Heads are 64 channels and a wave's tile is 64 channels x 64 tokens, so a wave holds whole
// (token, head) groups: after the accumulation, lanes l and l+32 own the two 16-channel halves
// of each 32-channel block of token l (first token block) and of token 32+l (second block).
// One v_permlane32_swap per register pair trades those halves, after which lane (l, g) owns all
// 64 channels of ONE token (block g) and can walk them in order, as Eq. 5 requires: the mean and
// the sum of squared deviations are the fp32 recurrences in element order, and every level is
// the sigma-free comparator's: a guess from the hardware reciprocal square root stands when it is
// provably far from every boundary, and otherwise picks which two comparisons are evaluated.
// The fp32 linear output never leaves registers.
// gamma / beta / the folded scales are wave-uniform: staged in LDS once per tile and read as
// broadcasts.
constexpr float kHnGuard = 0x1p-21f;   // unit of the guard that lets a guessed level stand (see the LayerNorm kernel)
template <int SB, int NTK, int PAIR>   // PAIR: token blocks 2*PAIR and 2*PAIR + 1 of the wave's NTK
__device__ __forceinline__ void epilogue_headnorm(const GemmParams &p, v16i (&acc)[2][NTK], int shift, uint8_t *dst,
                                                  const float *scs64, const float *bs64, float step,
                                                  const float *gp, const float *bp) {
    // trade halves: afterwards sw[0] is channel 32*ci + r and sw[1] channel 32*ci + 16 + r of this
    // lane's token.  The definition's y = fma((float)acc, s_x*s_w[c], b[c]); the caller passes
    // either the folded scales (which carry 2^-shift exactly) with shift 0, or the plain ones.
    float v[64];
    auto to_y = [&](int a, int i) { return fmaf((float)(a >> shift), scs64[i], bs64[i]); };
#pragma unroll
    for (int ci = 0; ci < 2; ++ci) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const auto sw = __builtin_amdgcn_permlane32_swap(acc[ci][2 * PAIR][r], acc[ci][2 * PAIR + 1][r], false, false);
            v[32 * ci + r] = to_y((int)sw[0], 32 * ci + r);
            v[32 * ci + 16 + r] = to_y((int)sw[1], 32 * ci + 16 + r);
        }
        __builtin_amdgcn_sched_barrier(0);   // the two accumulator tiles are dead before the next pair is touched
    }
    float mu = 0.0f, m2 = 0.0f;
#pragma unroll
    for (int i = 0; i < 64; ++i) {
        const float d1 = v[i] - mu;
        mu = mu + d1 / (float)(i + 1);
        const float d2 = v[i] - mu;
        const float pr = d1 * d2;
        m2 = m2 + pr;
    }
    const float nf = 64.0f;
    const float ne = nf * p.hn_eps;
    const float V = m2 + ne;
    const float rs = __builtin_amdgcn_rsqf(V / nf);          // for the guess only
    const float rstep = __builtin_amdgcn_rcpf(step);         // for the guess only
    const bool stats_ok = step >= 0x1p-20f && step <= 0x1p10f && V >= 0x1p-40f && V <= 0x1p30f;
    const float qminf = p.qminf, qmaxf = p.qmaxf;
    const int span = (int)(qmaxf - qminf);
    const float bias8 = -qminf;
#pragma unroll
    for (int i = 0; i < 64; ++i) {
        const float gm = gp[i], bt = bp[i];
        const float a = v[i] - mu;
        const float g = a * gm;
        const float gs = g * fabsf(g);
        const float L = gs * nf;
        auto above = [&](float k) {
            const float rk = (k - 0.5f) * step;
            const float cc = rk - bt;
            const float cs = cc * fabsf(cc);
            const float R = cs * V;
            return L > R;
        };
        // The guess tp is within (|g/(sigma*step)| + |beta/step|) * 2^-21 of the exact-arithmetic value the
        // comparator tests, and the comparator's own fp32 evaluation moves a boundary by at most
        // (2|level| + |beta/step| + 1) * 2^-22: a guess further than 2^-21 * (4|tp| + 3|beta/step| + 3) from every
        // half-integer is the level the comparator would count, and it is not run (stats_ok: the squares stay
        // ordinary numbers, which that error model needs).  A NaN figure fails the test and is verified.
        const float tp = fmaf(g, rs, bt) * rstep;
        const float tt = rintf(tp);
        float c = (tt == tt) ? __builtin_amdgcn_fmed3f(tt, qminf, qmaxf) : qminf;
        const float cgi = fmaf(fabsf(bt * rstep), 3.0f * kHnGuard, 3.0f * kHnGuard);
        const float fig = fmaf(fabsf(tp), 4.0f * kHnGuard, fabsf(tp - tt)) + cgi;
        if (!(stats_ok && fig <= 0.5f)) {
            for (int it = 0; it <= span; ++it) {
                const bool low_ok = (c <= qminf) || above(c);
                const bool high_ok = (c >= qmaxf) || !above(c + 1.0f);
                if (low_ok && high_ok) break;
                c = c + (!low_ok ? -1.0f : 1.0f);
            }
        }
        v[i] = c + bias8;                                  // stored biased: 0 .. qmax - qmin
        if ((i & 3) == 3) __builtin_amdgcn_sched_barrier(0);
    }
    if (!dst) return;
    if constexpr (SB == 4) {
        const u32 fix = 0x11111111u * ((u32)bias8 & 0xFu);
        u32 w[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            u32 ev = 0, od = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ev = __builtin_amdgcn_cvt_pk_u8_f32(v[8 * j + 2 * i], i, ev);
                od = __builtin_amdgcn_cvt_pk_u8_f32(v[8 * j + 2 * i + 1], i, od);
            }
            const u32 a0 = ev | (od << 4);
            w[j] = ((a0 | 0x88888888u) - (fix & 0x77777777u)) ^ ((a0 ^ ~fix) & 0x88888888u);
        }
        *reinterpret_cast<uint4 *>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
        *reinterpret_cast<uint4 *>(dst + 16) = make_uint4(w[4], w[5], w[6], w[7]);
    } else {
        const u32 fix = 0x01010101u * ((u32)bias8 & 0xFFu);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            u32 w[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                u32 x = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) x = __builtin_amdgcn_cvt_pk_u8_f32(v[16 * q + 4 * j + i], i, x);
                w[j] = ((x | 0x80808080u) - (fix & 0x7F7F7F7Fu)) ^ ((x ^ ~fix) & 0x80808080u);
            }
            *reinterpret_cast<uint4 *>(dst + 16 * q) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
}

// ---- integer-only epilogue: equivalent bias + comparator references with the scales absorbed ----
// (Eq. 2, second form; Sec. IV-B.)  level = qmin + #{t : acc + b_int[c] > T[c][t]}, T non-decreasing
// in t, so the count is found by bisection: 4 integer comparisons for up to 15 references, 8 for up
// to 255, no branch, no floating point.  The tile keeps rows of kAbsRow entries in LDS (INT32_MAX
// -- never exceeded -- beyond the last reference): the references themselves when there are at
// most 15 per channel, else every sixteenth one (T[15], T[31], ...), which settles the first four
// strides; the last four then probe one 16-entry stretch of the caller's table in global memory.
constexpr int kAbsRow = 17;
// WIDE: acc + b_int may leave 32 bits (see the staging of the biases): sums and comparisons in 64 bits.
template <bool TBL_LDS, bool WIDE>
__device__ __forceinline__ void epilogue_absorbed(const GemmParams &p, const v16i &acc, int shift, uint8_t *dst,
                                                  const int *lds_tbl, const int *glb_tbl, int64_t glb_row, const int *bint) {
    if (!dst) return;
    using sum_t = std::conditional_t<WIDE, int64_t, int>;
    const int nthr = p.ab_nthr;
    float lv[16];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int4 b4 = *reinterpret_cast<const int4 *>(bint + 4 * q);
        const int bq[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = 4 * q + i;
            const sum_t a = (sum_t)(acc[r] >> shift) + (sum_t)bq[i];
            int pos = 0;                                // references known to be exceeded
            if constexpr (TBL_LDS) {
                // (a missing reference is INT32_MAX "never exceeded": a 64-bit sum above it can only
                // occur with every real reference exceeded too, and pos is capped at their number)
#pragma unroll
                for (int step = 8; step >= 1; step >>= 1) {
                    const int t = pos + step - 1;
                    pos += ((!WIDE || t < nthr) && a > (sum_t)lds_tbl[r * kAbsRow + t]) ? step : 0;
                }
            } else {
                // strides 128..16 probe T[16(i+1) - 1]: entry i of the LDS row; strides 8..1 finish
                // inside one 16-entry stretch of the caller's table
#pragma unroll
                for (int step = 128; step >= 16; step >>= 1) {
                    const int t = pos + step - 1;
                    pos += ((!WIDE || t < nthr) && a > (sum_t)lds_tbl[r * kAbsRow + ((pos + step) >> 4) - 1]) ? step : 0;
                }
#pragma unroll
                for (int step = 8; step >= 1; step >>= 1) {
                    const int t = pos + step - 1;
                    const int v = glb_tbl[(int64_t)r * glb_row + min(t, nthr - 1)];
                    pos += (a > (t >= nthr ? (sum_t)INT32_MAX : (sum_t)v) && (!WIDE || t < nthr)) ? step : 0;
                }
            }
            lv[r] = (float)pos;
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    pack_store16(p, dst, lv, -p.qminf);
}

// ---- direct global -> LDS loads ----------------------------------------------------------------
// global_load_lds_dwordx4: lane i of the wave writes its 16 bytes to LDS address M0 + 16*i; no
// VGPRs are used for the data, so several k-stages can be in flight at once.  The compiler does
// not see these loads: completion is tracked by hand with s_waitcnt vmcnt(n) (loads retire in
// order), followed by a workgroup barrier before any lane reads the stage.
__device__ __forceinline__ u32 lds_address(const void *p) {
    return (u32)(uintptr_t)(const __attribute__((address_space(3))) uint8_t *)p;
}
// address = sbase (uniform) + voff (per lane)
__device__ __forceinline__ void dma16(u32 voff, const uint8_t *sbase, u32 lds_dst) {
    u32 keep;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %1, %2\n\ts_mov_b32 m0, %0"
                 : "=&s"(keep) : "v"(voff), "s"(sbase), "s"(lds_dst) : "memory");
}
// address = per-lane pointer
__device__ __forceinline__ void dma16_ptr(const uint8_t *ptr, u32 lds_dst) {
    u32 keep;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(keep) : "v"(ptr), "s"(lds_dst) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// sixteen zero bytes: the source of operand chunks that lie beyond the end of a row (K tail)
__device__ __attribute__((aligned(16))) const u32 g_zero16[4] = {0u, 0u, 0u, 0u};

// XOR swizzle of the 16-byte chunk index inside an LDS row of CH chunks (rows are stored without
// padding): spreads the rows that consecutive lanes read over all banks.
template <int CH>
__device__ __forceinline__ int swz(int row) {
    if constexpr (CH == 4) return ((row >> 2) & 3) ^ (row & 2);
    else if constexpr (CH == 8) return row & 7;
    else if constexpr (CH == 2) return (row >> 3) & 1;
    else return 0;
}

// inverse of slot_of_channel
__device__ __forceinline__ int channel_of_slot(int s) {
    return 16 * ((s >> 2) & 1) + 4 * (s >> 3) + (s & 3);
}

// marks every fragment of a set as used (and possibly modified) here: an anchor for the scheduler
template <int N>
__device__ __forceinline__ void pin_frags(v4i (&f)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+v"(f[i]));
}

template <int WB, int AB, int TC, int TT, int WAVES_C, int WAVES_T, int BK, int S, int OCC, int EPI>
__global__ __launch_bounds__(WAVES_C *WAVES_T * 64, OCC)
void gemm_kernel(GemmParams p) {
    constexpr int NT = WAVES_C * WAVES_T * 64;                // S = k-stages resident in LDS
    constexpr int WROW = BK * WB / 8, XROW = BK * AB / 8;     // bytes per row per stage
    constexpr int WCH = WROW / 16, XCH = XROW / 16;           // 16-byte chunks per row
    constexpr int W_ITERS = TC * WCH / NT, X_ITERS = TT * XCH / NT;
    static_assert((TC * WCH) % NT == 0 && (TT * XCH) % NT == 0, "tile/threads mismatch");
    constexpr int LOADS = W_ITERS + X_ITERS;                  // loads per lane per stage
    constexpr int WC = TC / WAVES_C, WT = TT / WAVES_T;       // wave tile
    constexpr int NC = WC / 32, NTK = WT / 32;                // 32x32 blocks per wave
    static_assert(WC % 32 == 0 && WT % 32 == 0 && TC % 64 == 0 && BK % 64 == 0, "wave tile");
    constexpr int WBUF = TC * WROW, XBUF = TT * XROW, STAGE = WBUF + XBUF;
    constexpr bool SWAP = (EPI == kEpiF32);   // tokens as the MFMA A operand (see epilogue_f32)
    constexpr bool ABSORBED = (EPI == kEpiAbsorbed || EPI == kEpiAbsorbedBig);   // integer-only epilogue

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    float *s_scs = reinterpret_cast<float *>(smem + S * STAGE);           // [TC] folded scales
    float *s_bs = s_scs + TC;                                             // [TC] biases
    int *s_fold_bad = reinterpret_cast<int *>(s_bs + TC);                 // [1] flag
    [[maybe_unused]] float *s_raw = s_bs + TC + 4;                        // [TC] plain scales (fp32, head-norm epilogues)
    [[maybe_unused]] float *s_hg = s_raw + TC, *s_hb = s_raw + 2 * TC;    // [TC] each: gamma, beta of the head-norm epilogue

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_c = wave % WAVES_C;
    const int wave_t = wave / WAVES_C;
    const int li = lane & 31;   // MFMA row / column index of this lane
    const int g = lane >> 5;    // k-group of this lane

    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Re-number them so
    // that the workgroups of one XCD walk consecutive tiles: the channel tiles of one token tile
    // then share that XCD's L2 copy of the activations.
    const int n_ct = (p.Nout + TC - 1) / TC;
    int logical;
    {
        const int total = gridDim.x, id = blockIdx.x;
        const int xcd = id & 7, slot = id >> 3;
        const int per = total >> 3, rem = total & 7;
        logical = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + slot;
    }
    const int ct = logical % n_ct;
    const int tt = logical / n_ct;
    const int c0 = ct * TC;
    const int t0 = tt * TT;

    // ---- stage loads: what each lane fetches is fixed; only the k offset (uniform) advances ----
    // LDS position pos (16-byte units) of a tile holds row pos / CH, chunk (pos % CH) ^ swz(row).
    // Weight rows sit in permuted slots (slot_of_channel) unless the roles are swapped.  Rows
    // beyond the matrix are clamped to its last row: their products land in accumulators that
    // are never stored.
    const int nk = (p.K + BK - 1) / BK;
    const bool ktail = (nk * WROW > p.kbytes_w16) || (nk * XROW > p.kbytes_x16);
    const uint8_t *wbase = p.w + (int64_t)c0 * p.w_stride;
    const uint8_t *xbase = p.x + (int64_t)t0 * p.x_stride;
    u32 w_off[W_ITERS], x_off[X_ITERS];
    int w_kb[W_ITERS], x_kb[X_ITERS];
#pragma unroll
    for (int it = 0; it < W_ITERS; ++it) {
        const int pos = it * NT + tid;
        const int slot = pos / WCH;
        const int chunk = (pos % WCH) ^ swz<WCH>(slot);
        int row = SWAP ? slot : ((slot & ~31) | channel_of_slot(slot & 31));
        row = min(row, p.Nout - 1 - c0);
        w_off[it] = (u32)row * (u32)p.w_stride + (u32)chunk * 16u;
        w_kb[it] = chunk * 16;
    }
#pragma unroll
    for (int it = 0; it < X_ITERS; ++it) {
        const int pos = it * NT + tid;
        int row = pos / XCH;
        const int chunk = (pos % XCH) ^ swz<XCH>(row);
        row = min(row, p.M - 1 - t0);
        x_off[it] = (u32)row * (u32)p.x_stride + (u32)chunk * 16u;
        x_kb[it] = chunk * 16;
    }
    const u32 lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem)) + (u32)wave * 1024u;
    // The LOADS loads of a stage (weights first, then tokens) are issued in kParts groups: a burst of
    // all of them from all four waves queues up in the CU's one address path and stalls every wave
    // for hundreds of cycles, so the main loop spreads the groups over several MFMA steps.
    constexpr int kParts = 3;
    constexpr int kPartLoads = (LOADS + kParts - 1) / kParts;
    auto issue_part = [&](int kt, auto PART) {
        constexpr int lo = decltype(PART)::value * kPartLoads;
        constexpr int hi = (lo + kPartLoads < LOADS) ? lo + kPartLoads : LOADS;
        const u32 dst = lds0 + (u32)(kt % S) * STAGE;
        if (ktail && kt == nk - 1) {
            // last stage of a K that does not fill it: chunks past the row end come from zeros
            static_for<(hi > lo ? hi - lo : 0)>([&](auto I) {
                constexpr int l = lo + decltype(I)::value;
                if constexpr (l < W_ITERS) {
                    const uint8_t *src = wbase + (int64_t)kt * WROW + w_off[l];
                    if (kt * WROW + w_kb[l] >= p.kbytes_w16) src = reinterpret_cast<const uint8_t *>(g_zero16);
                    dma16_ptr(src, dst + l * (NT * 16));
                } else {
                    constexpr int it = l - W_ITERS;
                    const uint8_t *src = xbase + (int64_t)kt * XROW + x_off[it];
                    if (kt * XROW + x_kb[it] >= p.kbytes_x16) src = reinterpret_cast<const uint8_t *>(g_zero16);
                    dma16_ptr(src, dst + WBUF + it * (NT * 16));
                }
            });
        } else {
            const uint8_t *wk = wbase + (int64_t)kt * WROW;
            const uint8_t *xk = xbase + (int64_t)kt * XROW;
            static_for<(hi > lo ? hi - lo : 0)>([&](auto I) {
                constexpr int l = lo + decltype(I)::value;
                if constexpr (l < W_ITERS) dma16(w_off[l], wk, dst + l * (NT * 16));
                else dma16(x_off[l - W_ITERS], xk, dst + WBUF + (l - W_ITERS) * (NT * 16));
            });
        }
    };
    auto issue = [&](int kt) {
        static_for<kParts>([&](auto P) { issue_part(kt, P); });
    };
    // Integer-only epilogue: this lane's share of the tile's comparator references is requested
    // now, ahead of every operand load (loads retire in order, so the hand-counted waits of the
    // main loop are unaffected), and parked in registers until the pipeline buffers are free.
    constexpr int ABS_ITERS = ABSORBED ? (TC * kAbsRow + NT - 1) / NT : 1;
    [[maybe_unused]] int abs_ref[ABS_ITERS];
    if constexpr (ABSORBED) {
        const int nthr = p.ab_nthr;
#pragma unroll
        for (int k = 0; k < ABS_ITERS; ++k) {
            const int i = min(k * NT + tid, TC * kAbsRow - 1);
            const int c = i / kAbsRow, e = i - kAbsRow * c;              // entry e of channel c
            const int t = (EPI == kEpiAbsorbed) ? e : 16 * (e + 1) - 1;  // the reference it holds
            const int ch = min(c0 + c, p.Nout - 1);
            abs_ref[k] = p.ab_thr[(int64_t)ch * nthr + min(t, nthr - 1)];               // (pads: replaced when stored)
        }
    }
#pragma unroll
    for (int st = 0; st < S - 1; ++st)
        if (st < nk) issue(st);

    // Per-channel epilogue constants, staged once per tile while the first operand loads are in
    // flight: sc = s_x*s_w[c] (the definition's exact product) with the operand factor 2^shift
    // folded in.  The fold is exact unless the result is subnormal; a flag then sends the whole
    // tile through the exact operation sequence.
    if constexpr (ABSORBED) {
        // per channel: the equivalent bias.  |acc| stays below 2^23 (K <= 65536), so acc + b_int fits
        // 32 bits unless a bias lies within 2^23 of the int32 limits (a near-dead channel): such a
        // tile takes the 64-bit form of the comparisons.
        if (tid == 0) s_fold_bad[0] = 0;
        __syncthreads();
        for (int c = tid; c < TC; c += NT) {
            const int b = p.ab_bint ? p.ab_bint[min(c0 + c, p.Nout - 1)] : 0;
            reinterpret_cast<int *>(s_raw)[c] = b;
            if (b > INT32_MAX - (1 << 23) || b < INT32_MIN + (1 << 23)) s_fold_bad[0] = 1;
        }
    } else if constexpr (EPI != kEpiGeneric) {
        if (tid == 0) s_fold_bad[0] = 0;
        __syncthreads();
        for (int c = tid; c < TC; c += NT) {
            const int ch = c0 + c;
            const bool ok = ch < p.Nout;
            const float sw = ok ? p.s_w[p.s_w_per_channel ? ch : 0] : 1.0f;
            const float sc = p.s_x * sw;
            const float folded = ldexpf(sc, -Shift<WB, AB>::value);
            s_scs[c] = folded;
            if constexpr (EPI == kEpiHeadNorm || EPI == kEpiF32) s_raw[c] = sc;
            if constexpr (EPI == kEpiHeadNorm) {
                const bool qk = ch < 2 * p.D;          // V channels have no LayerNorm
                s_hg[c] = qk ? p.hn_gamma[ch] : 0.0f;
                s_hb[c] = qk ? p.hn_beta[ch] : 0.0f;
            }
            s_bs[c] = (ok && p.bias) ? p.bias[ch] : 0.0f;
            if (!(ldexpf(folded, Shift<WB, AB>::value) == sc)) s_fold_bad[0] = 1;
        }
    }

    v16i acc[NC][NTK];
#pragma unroll
    for (int i = 0; i < NC; ++i)
#pragma unroll
        for (int j = 0; j < NTK; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // Byte offsets (inside a stage) of this lane's operand reads.  In sub-step ss the lane owns the
    // 32 values [64*ss + 32*g, +32) of its row: two MFMA operands of 16 values each.
    constexpr int NSS = BK / 64;
    constexpr int WRD = (WB == 8) ? 2 : 1, XRD = (AB == 8) ? 2 : 1;      // 16-byte reads per sub-step
    u32 w_rd[NSS][WRD], x_rd[NSS][XRD];
    {
        const int wrow = wave_c * WC + li, xrow = wave_t * WT + li;
#pragma unroll
        for (int ss = 0; ss < NSS; ++ss) {
            const int wbo = ((ss * 64 + g * 32) * WB) / 8, xbo = ((ss * 64 + g * 32) * AB) / 8;
#pragma unroll
            for (int j = 0; j < WRD; ++j)
                w_rd[ss][j] = (u32)((wrow * WCH + (((wbo >> 4) + j) ^ swz<WCH>(wrow))) * 16 + (wbo & 15));
#pragma unroll
            for (int j = 0; j < XRD; ++j)
                x_rd[ss][j] = (u32)(WBUF + (xrow * XCH + (((xbo >> 4) + j) ^ swz<XCH>(xrow))) * 16 + (xbo & 15));
        }
    }
    // ---- main loop, software-pipelined by hand -------------------------------------------------
    // A k-stage is NSS sub-steps of 64 values; a sub-step is two MFMA steps s = 0, 1 of 32 values.
    // Per sub-step a lane fetches one packed piece per operand block ("raw": 32 values each) and
    // unpacks half of it per MFMA step into int8 fragments ("frag").  Fragments are double
    // buffered: while the NC*NTK MFMAs of one step run on one set, the VALU fills the other set,
    // and the LDS reads of the next sub-step are issued as soon as the current raw registers have
    // been unpacked, so their latency hides behind the MFMAs that follow.  The wait for the next
    // k-stage, the workgroup barrier and the issue of the stage after it sit in the middle of the
    // last sub-step (not between k-steps), where the matrix pipe still holds queued work.
    constexpr int WRAW = (32 * WB) / 32, XRAW = (32 * AB) / 32;   // dwords of raw data per lane, block and sub-step
    u32 wr[NC][WRAW], xr[NTK][XRAW];
    v4i wf[2][NC], xf[2][NTK];
    auto load_raw = [&](int buf, auto SS) {
        constexpr int ss = decltype(SS)::value;
        const uint8_t *stage = smem + buf * STAGE;
#pragma unroll
        for (int ci = 0; ci < NC; ++ci) {
            const uint8_t *src = stage + w_rd[ss][0] + ci * 32 * WROW;
            if constexpr (WB == 4) {
                uint4 v = *reinterpret_cast<const uint4 *>(src);
                wr[ci][0] = v.x; wr[ci][1] = v.y; wr[ci][2] = v.z; wr[ci][3] = v.w;
            } else if constexpr (WB == 2) {
                uint2 v = *reinterpret_cast<const uint2 *>(src);
                wr[ci][0] = v.x; wr[ci][1] = v.y;
            } else {
                uint4 v0 = *reinterpret_cast<const uint4 *>(src);
                uint4 v1 = *reinterpret_cast<const uint4 *>(stage + w_rd[ss][WRD - 1] + ci * 32 * WROW);
                wr[ci][0] = v0.x; wr[ci][1] = v0.y; wr[ci][2] = v0.z; wr[ci][3] = v0.w;
                wr[ci][4] = v1.x; wr[ci][5] = v1.y; wr[ci][6] = v1.z; wr[ci][7] = v1.w;
            }
        }
#pragma unroll
        for (int ti = 0; ti < NTK; ++ti) {
            const uint8_t *src = stage + x_rd[ss][0] + ti * 32 * XROW;
            if constexpr (AB == 4) {
                uint4 v = *reinterpret_cast<const uint4 *>(src);
                xr[ti][0] = v.x; xr[ti][1] = v.y; xr[ti][2] = v.z; xr[ti][3] = v.w;
            } else {
                uint4 v0 = *reinterpret_cast<const uint4 *>(src);
                uint4 v1 = *reinterpret_cast<const uint4 *>(stage + x_rd[ss][XRD - 1] + ti * 32 * XROW);
                xr[ti][0] = v0.x; xr[ti][1] = v0.y; xr[ti][2] = v0.z; xr[ti][3] = v0.w;
                xr[ti][4] = v1.x; xr[ti][5] = v1.y; xr[ti][6] = v1.z; xr[ti][7] = v1.w;
            }
        }
    };
    // raw -> fragment set `fb` for MFMA step s of the current sub-step
    auto unpack = [&](auto S_, auto FB) {
        constexpr int s = decltype(S_)::value, fb = decltype(FB)::value;
#pragma unroll
        for (int ci = 0; ci < NC; ++ci) {
            if constexpr (WB == 4) wf[fb][ci] = unpack4_x16(wr[ci][2 * s], wr[ci][2 * s + 1]);
            else if constexpr (WB == 2) wf[fb][ci] = unpack2_x64(wr[ci][s]);
            else { wf[fb][ci][0] = (int)wr[ci][4 * s]; wf[fb][ci][1] = (int)wr[ci][4 * s + 1];
                   wf[fb][ci][2] = (int)wr[ci][4 * s + 2]; wf[fb][ci][3] = (int)wr[ci][4 * s + 3]; }
        }
#pragma unroll
        for (int ti = 0; ti < NTK; ++ti) {
            if constexpr (AB == 4) {
                if constexpr (WB == 2) xf[fb][ti] = unpack4_x16_order2(xr[ti][2 * s], xr[ti][2 * s + 1]);
                else xf[fb][ti] = unpack4_x16(xr[ti][2 * s], xr[ti][2 * s + 1]);
            } else {
                xf[fb][ti][0] = (int)xr[ti][4 * s]; xf[fb][ti][1] = (int)xr[ti][4 * s + 1];
                xf[fb][ti][2] = (int)xr[ti][4 * s + 2]; xf[fb][ti][3] = (int)xr[ti][4 * s + 3];
            }
        }
    };
    auto mma = [&](auto FB) {
        constexpr int fb = decltype(FB)::value;
#pragma unroll
        for (int ci = 0; ci < NC; ++ci)
#pragma unroll
            for (int ti = 0; ti < NTK; ++ti) {
                if constexpr (SWAP)
                    acc[ci][ti] = __builtin_amdgcn_mfma_i32_32x32x32_i8(xf[fb][ti], wf[fb][ci], acc[ci][ti], 0, 0, 0);
                else
                    acc[ci][ti] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[fb][ci], xf[fb][ti], acc[ci][ti], 0, 0, 0);
            }
    };
    // Interleave pattern of one MFMA step: NC*NTK matrix instructions with the unpack arithmetic of
    // the next step spread evenly between them (then, where given, the LDS reads of the next sub-step).
    constexpr int kMma = NC * NTK;
    constexpr int kUnpackOps = (WB == 8 ? 0 : (WB == 4 ? 6 : 7) * NC) + (AB == 8 ? 0 : (WB == 2 ? 10 : 6) * NTK);
    constexpr int kValuPerMma = (kUnpackOps + kMma - 1) / kMma;
    constexpr int kRawReads = NC * WRD + NTK * XRD;
    auto pattern = [&](bool reads_after) {
#pragma unroll
        for (int i = 0; i < kMma; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                 // one MFMA
            if (kValuPerMma > 0) __builtin_amdgcn_sched_group_barrier(0x002, kValuPerMma, 0);   // its share of VALU
        }
        if (reads_after) __builtin_amdgcn_sched_group_barrier(0x100, kRawReads, 0);              // DS reads
    };
    // Stage j is complete once all but the loads of the (at most S-2) younger stages have retired;
    // the barrier then also tells that every wave has finished reading stage j-1, whose buffer the
    // next issue overwrites.
    auto sync_stage = [&](int j) {
        const int younger = nk - 1 - j;
        if (younger >= S - 2) wait_vmcnt<(S - 2) * LOADS>();
        else if (younger == 1) wait_vmcnt<LOADS>();
        else wait_vmcnt<0>();
        __syncthreads();
        if (j + S - 1 < nk) {
            if (j == 0) issue(j + S - 1);
            else issue_part(j + S - 1, std::integral_constant<int, 0>{});
        }
    };
    // The fragments of a set are made "used" at the end of the step that fills them, so the
    // compiler cannot sink their arithmetic past the branches of the synchronisation code (where
    // it would no longer overlap with any MFMA).
    auto pin = [&](auto FB) {
        constexpr int fb = decltype(FB)::value;
        pin_frags(wf[fb]);
        pin_frags(xf[fb]);
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    sync_stage(0);
    load_raw(0, I0{});
    unpack(I0{}, I0{});
    // One k-stage.  NEXT: another stage follows (its synchronisation, the issue of a later stage and
    // the first raw reads of the next stage are part of this one); the last stage is a separate
    // instantiation, so that neither copy carries a branch between an MFMA step and its unpacking.
    auto kstep = [&](int kt, auto NEXT_) {
        constexpr bool NEXT = decltype(NEXT_)::value;
        const int buf = kt % S;
        static_for<NSS>([&](auto SS) {
            constexpr int ss = decltype(SS)::value;
            constexpr bool last_ss = (ss + 1 == NSS);
            // the rest of the stage whose first loads followed the previous synchronisation
            // (a stage's groups must enter the load queue in order and ahead of the next stage's first
            // group, which the synchronisation below issues: the waits count loads from the youngest.
            // With a single sub-step per stage that leaves no later slot for the last group.)
            if constexpr (ss == 0) {
                if (kt >= 1 && kt + S - 1 < nk) {
                    issue_part(kt + S - 1, I1{});
                    if constexpr (NSS == 1) issue_part(kt + S - 1, std::integral_constant<int, 2>{});
                }
            }
            // step s = 0 runs; step s = 1 is unpacked; then the raw registers are free
            __builtin_amdgcn_sched_barrier(0);
            mma(I0{});
            unpack(I1{}, I1{});
            if constexpr (!last_ss) {
                load_raw(buf, std::integral_constant<int, (last_ss ? 0 : ss + 1)>{});
                pattern(true);
                pin(I1{});
                __builtin_amdgcn_sched_barrier(0);
            } else {
                pattern(false);
                pin(I1{});
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (NEXT) {
                    sync_stage(kt + 1);
                    load_raw((kt + 1) % S, I0{});
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if constexpr (ss == 0 && NSS > 1) {
                if (kt >= 1 && kt + S - 1 < nk) issue_part(kt + S - 1, std::integral_constant<int, 2>{});
                __builtin_amdgcn_sched_barrier(0);
            }
            // step s = 1 runs; step s = 0 of the next sub-step is unpacked
            mma(I1{});
            if constexpr (!last_ss || NEXT) {
                unpack(I0{}, I0{});
                pattern(false);
                pin(I0{});
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    for (int kt = 0; kt < nk - 1; ++kt) kstep(kt, std::true_type{});
    kstep(nk - 1, std::false_type{});
    __syncthreads();


    // ---- epilogue -------------------------------------------------------------------------
    constexpr int shift = Shift<WB, AB>::value;
    const bool fold_ok = (EPI != kEpiGeneric && !ABSORBED) && (s_fold_bad[0] == 0);
    if constexpr (SWAP) {
        // Blocks in turn; the residual of the next block is requested before the current block is
        // stored, so its loads never queue behind those stores.
        auto block_pos = [&](int b, int &m0, int &cl) {
            const int ci = b / NTK, ti = b % NTK;
            cl = wave_c * WC + ci * 32 + li;               // this lane's channel inside the tile
            m0 = t0 + wave_t * WT + ti * 32 + 4 * g;
        };
        auto run = [&](auto FULLT, auto REST) {
            constexpr bool FULL = decltype(FULLT)::value, RES = decltype(REST)::value;
            float rbuf[2][16];                 // residual of the current / the next block
#pragma unroll
            for (int r = 0; r < 16; ++r) rbuf[0][r] = rbuf[1][r] = 0.0f;
            if constexpr (RES) {
                int m0, cl;
                block_pos(0, m0, cl);
                load_residual<FULL>(p, m0, c0 + cl, rbuf[0]);
            }
            static_for<NC * NTK>([&](auto BI) {
                constexpr int b = decltype(BI)::value;
                int m0, cl;
                if constexpr (RES && b + 1 < NC * NTK) {
                    block_pos(b + 1, m0, cl);
                    load_residual<FULL>(p, m0, c0 + cl, rbuf[(b + 1) & 1]);
                }
                block_pos(b, m0, cl);
                epilogue_f32<FULL, RES>(p, acc[b / NTK][b % NTK], fold_ok ? 0 : shift, m0, c0 + cl,
                                        fold_ok ? s_scs[cl] : s_raw[cl], s_bs[cl], rbuf[b & 1]);
            });
        };
        // tiles wholly inside the matrix (all but the last row / column of tiles) skip the bounds tests
        const bool full = t0 + TT <= p.M && c0 + TC <= p.Nout;
        if (p.res) { if (full) run(std::true_type{}, std::true_type{}); else run(std::false_type{}, std::true_type{}); }
        else { if (full) run(std::true_type{}, std::false_type{}); else run(std::false_type{}, std::false_type{}); }
    } else {
        if constexpr (EPI == kEpiHeadNorm) {
            // Q and K tiles: per-head LayerNorm quantizer; V tiles fall through to the plain one
            const int cbw = c0 + wave_c * WC;                       // the wave's head starts here
            if (cbw < 2 * p.D) {
                static_assert(EPI != kEpiHeadNorm || (NC == 2 && NTK % 2 == 0 && WC == 64), "one head per wave");
                int which;
                const int64_t ch_part = packed_channel_part(p, cbw, which);
                const float step = which == 0 ? p.s_y[0] : p.s_y[1];
                // folded scales unless folding was inexact somewhere in the tile: then the plain
                // ones (kept behind the flag word) and the explicit shift
                const float *sc64 = (fold_ok ? s_scs : s_raw) + wave_c * WC;
                const int sh = fold_ok ? 0 : shift;
                if constexpr (EPI == kEpiHeadNorm) {
                    static_for<NTK / 2>([&](auto PI) {
                        constexpr int pair = decltype(PI)::value;
                        const int64_t tk = packed_token_part(p, t0 + wave_t * WT + 64 * pair + 32 * g + li);
                        uint8_t *dst = (ch_part >= 0 && tk >= 0) ? p.yq + tk + ch_part : nullptr;
                        if (p.yq_sb == 4)
                            epilogue_headnorm<4, NTK, pair>(p, acc, sh, dst, sc64, s_bs + wave_c * WC, step, s_hg + wave_c * WC, s_hb + wave_c * WC);
                        else
                            epilogue_headnorm<8, NTK, pair>(p, acc, sh, dst, sc64, s_bs + wave_c * WC, step, s_hg + wave_c * WC, s_hb + wave_c * WC);
                    });
                }
                return;
            }
        }
        if constexpr (ABSORBED) {
            // The pipeline buffers are free now: the tile's LDS table (see epilogue_absorbed) goes there.
            const int nthr = p.ab_nthr;
            constexpr bool in_lds = (EPI == kEpiAbsorbed);
            const bool wide = s_fold_bad[0] != 0;          // (read before the barrier below, written before the main loop)
            int *s_tbl = reinterpret_cast<int *>(smem);
            static_assert(TC * kAbsRow * 4 <= S * STAGE, "reference table exceeds the pipeline buffers");
#pragma unroll
            for (int k = 0; k < ABS_ITERS; ++k) {
                const int i = k * NT + tid;
                const int e = i % kAbsRow;
                const int t = in_lds ? e : 16 * (e + 1) - 1;
                if (i < TC * kAbsRow) s_tbl[i] = t >= nthr ? INT32_MAX : abs_ref[k];
            }
            __syncthreads();
            int64_t tok_part[NTK];
#pragma unroll
            for (int ti = 0; ti < NTK; ++ti) tok_part[ti] = packed_token_part(p, t0 + wave_t * WT + ti * 32 + li);
            static_for<NC>([&](auto CI) {
                constexpr int ci = decltype(CI)::value;
                const int cl = wave_c * WC + ci * 32 + 16 * g;
                const int cb = c0 + cl;
                int which;
                const int64_t ch_part = packed_channel_part(p, cb, which);
                const int *bint = reinterpret_cast<const int *>(s_raw) + cl;
                static_for<NTK>([&](auto TI) {
                    constexpr int ti = decltype(TI)::value;
                    uint8_t *dst = (ch_part >= 0 && tok_part[ti] >= 0) ? p.yq + tok_part[ti] + ch_part : nullptr;
                    if (cb >= p.Nout)
                        store_zero_group(p, dst);
                    else if (wide)
                        epilogue_absorbed<in_lds, true>(p, acc[ci][ti], shift, dst, s_tbl + cl * kAbsRow,
                                                        p.ab_thr + (int64_t)min(cb, p.Nout - 16) * nthr, nthr, bint);
                    else
                        epilogue_absorbed<in_lds, false>(p, acc[ci][ti], shift, dst, s_tbl + cl * kAbsRow,
                                                         p.ab_thr + (int64_t)min(cb, p.Nout - 16) * nthr, nthr, bint);
                });
            });
            return;
        }
        constexpr bool QUANT = (EPI == kEpiQuant || EPI == kEpiQuantGelu || EPI == kEpiHeadNorm);
        int64_t tok_part[NTK];
        if constexpr (QUANT) {
#pragma unroll
            for (int ti = 0; ti < NTK; ++ti)
                tok_part[ti] = packed_token_part(p, t0 + wave_t * WT + ti * 32 + li);
        }
        static_for<NC>([&](auto CI) {
            constexpr int ci = decltype(CI)::value;
            const int cl = wave_c * WC + ci * 32 + 16 * g;     // channel offset inside the tile
            const int cb = c0 + cl;
            int64_t ch_part = -1;
            float s_y = 1.0f, r_y = 1.0f;
            if constexpr (EPI != kEpiGeneric) {
                int which;
                ch_part = packed_channel_part(p, cb, which);
                const float sy0 = p.s_y[0], sy1 = p.s_y[1], sy2 = p.s_y[2];
                const float ry0 = p.r_y[0], ry1 = p.r_y[1], ry2 = p.r_y[2];
                s_y = which == 0 ? sy0 : (which == 1 ? sy1 : sy2);
                r_y = which == 0 ? ry0 : (which == 1 ? ry1 : ry2);
            }
            static_for<NTK>([&](auto TI) {
                constexpr int ti = decltype(TI)::value;
                if constexpr (QUANT) {
                    uint8_t *dst = (ch_part >= 0 && tok_part[ti] >= 0) ? p.yq + tok_part[ti] + ch_part : nullptr;
                    if (cb >= p.Nout) store_zero_group(p, dst);
                    else epilogue_quant<EPI == kEpiQuantGelu>(p, acc[ci][ti], shift, dst, s_y, r_y, cb, s_scs + cl, s_bs + cl, !fold_ok);
                } else {
                    const int m = t0 + wave_t * WT + ti * 32 + li;
                    epilogue_generic(p, acc[ci][ti], shift, m, cb);
                }
            });
        });
    }
}

template <int WB, int AB, int TC, int TT, int WAVES_C, int WAVES_T, int BK, int S, int OCC, int EPI>
hipError_t launch(const GemmParams &p, hipStream_t stream) {
    constexpr size_t lds = S * ((size_t)TC * (BK * WB / 8) + (size_t)TT * (BK * AB / 8)) + 2 * TC * sizeof(float) + 16 +
                           ((EPI == kEpiHeadNorm || EPI == kEpiF32 || EPI == kEpiAbsorbed || EPI == kEpiAbsorbedBig) ? TC * sizeof(float) : 0) +
                           (EPI == kEpiHeadNorm ? 2 * TC * sizeof(float) : 0);
    auto kern = gemm_kernel<WB, AB, TC, TT, WAVES_C, WAVES_T, BK, S, OCC, EPI>;
    if (lds > 48 * 1024) {
        static std::atomic<uint64_t> allowed{0};        // (one per instantiation)
        hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds, allowed);
        if (e != hipSuccess) return e;
    }
    const int n_ct = (p.Nout + TC - 1) / TC;
    const int n_tt = (p.M + TT - 1) / TT;
    const int64_t blocks = (int64_t)n_ct * n_tt;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(WAVES_C * WAVES_T * 64), lds, stream, p);
    return hipGetLastError();
}

template <int WB, int AB, int TC, int TT, int WAVES_C, int WAVES_T, int BK, int S, int OCC>
hipError_t launch_epi(const GemmParams &p, int epi, hipStream_t stream) {
    switch (epi) {
        case kEpiF32: return launch<WB, AB, TC, TT, WAVES_C, WAVES_T, BK, S, OCC, kEpiF32>(p, stream);
        case kEpiQuant: return launch<WB, AB, TC, TT, WAVES_C, WAVES_T, BK, S, OCC, kEpiQuant>(p, stream);
        case kEpiQuantGelu: return launch<WB, AB, TC, TT, WAVES_C, WAVES_T, BK, S, OCC, kEpiQuantGelu>(p, stream);
        case kEpiHeadNorm: {
            // this epilogue keeps a token's whole 64-channel head in registers on top of the
            // accumulators: it runs with two waves per SIMD (256 registers) on 64x128 wave tiles
            constexpr int stage = 128 * BK * WB / 8 + 256 * BK * AB / 8;
            constexpr int S_HN = (3 * stage <= 80 * 1024) ? 3 : 2;
            return launch<WB, AB, 128, 256, 2, 2, BK, S_HN, 2, kEpiHeadNorm>(p, stream);
        }
        case kEpiAbsorbed: return launch<WB, AB, TC, TT, WAVES_C, WAVES_T, BK, S, OCC, kEpiAbsorbed>(p, stream);
        case kEpiAbsorbedBig: return launch<WB, AB, TC, TT, WAVES_C, WAVES_T, BK, S, OCC, kEpiAbsorbedBig>(p, stream);
        default: return launch<WB, AB, TC, TT, WAVES_C, WAVES_T, BK, S, OCC, kEpiGeneric>(p, stream);
    }
}

}  // namespace

hipError_t gemm_launch(GemmParams p, int wb, int ab, hipStream_t stream) {
    // pick the epilogue: the specialised ones need full 16-channel groups and a single output
    int epi = kEpiGeneric;
    const bool aligned = (p.Nout % 16 == 0);
    if (!p.acc_out && p.y_out && !p.yq && p.act == 0) epi = kEpiF32;     // any Nout
    if (aligned && !p.acc_out) {
        if (p.yq && !p.y_out && (p.yq_sb == 4 || p.yq_sb == 8)) epi = p.act == 1 ? kEpiQuantGelu : kEpiQuant;
    }
    if (p.ab_thr) {
        // integer-only epilogue: packed output only, whole 16-channel groups, 4- or 8-bit storage
        if (!aligned || p.acc_out || p.y_out || !p.yq || (p.yq_sb != 4 && p.yq_sb != 8) || p.act != 0 ||
            p.ab_nthr < 1 || p.ab_nthr > 255 || p.hn_gamma)
            return hipErrorInvalidValue;
        epi = p.ab_nthr <= 15 ? kEpiAbsorbed : kEpiAbsorbedBig;
    }
    if (p.hn_gamma) {
        // the fused per-head LayerNorm quantizers need whole 64-channel heads per wave tile
        if (epi != kEpiQuant || !p.head_major || p.dh != 64 || p.D % 64 != 0 || p.Nout != 3 * p.D || !p.hn_beta)
            return hipErrorInvalidValue;
        epi = kEpiHeadNorm;
    }
    // per-lane operand offsets inside a tile are kept in 32 bits (127 rows * stride + 112)
    if (p.x_stride >= (1 << 24) || p.w_stride >= (1 << 24) || p.M < 1 || p.Nout < 1) return hipErrorInvalidValue;
    if (p.head_major) {
        p.inv_ntok = 1.0f / (float)p.Ntok;
        p.dh_shift = -1;
        for (int sft = 0; sft < 16; ++sft)
            if ((1 << sft) == p.dh) p.dh_shift = sft;
        if (p.M >= (1 << 22)) return hipErrorInvalidValue;
    }
    if (p.yq && epi != kEpiAbsorbed && epi != kEpiAbsorbedBig) {
        for (int i = 0; i < 3; ++i) p.r_y[i] = 1.0f / p.s_y[i];
        p.eps0 = ldexpf(1.0f, (p.qmaxf > 7.5f ? 8 : 4) - 22);
        p.gelu_guard = kGeluFastBound;
        // a step so small that 1/s overflows, or so large that it underflows, takes the exact path
        for (int i = 0; i < 3; ++i)
            if (!(p.r_y[i] > 0x1p-100f && p.r_y[i] < 0x1p100f)) {
                if (epi == kEpiHeadNorm) return hipErrorInvalidValue;
                epi = (epi == kEpiF32) ? epi : kEpiGeneric;
            }
    }
    if (wb == 4 && ab == 4) return launch_epi<4, 4, VITQ_TC, VITQ_TT, VITQ_WC, VITQ_WT, VITQ_BK44, VITQ_S44, VITQ_OCC44>(p, epi, stream);
    if (wb == 2 && ab == 4) return launch_epi<2, 4, 128, 128, 2, 2, 128, 2, 4>(p, epi, stream);
    if (wb == 8 && ab == 8) {
        // 8-bit operands are read from LDS at twice the bytes per product and need no unpacking: a long
        // contraction is bound by those reads and gains from 64x128 wave tiles (a quarter fewer fragment
        // reads per product, at two waves per SIMD); a short one is dominated by its epilogue, which wants
        // four waves per SIMD.
        if (p.K >= 2048 && (epi == kEpiF32 || epi == kEpiQuant || epi == kEpiQuantGelu))
            return launch_epi<8, 8, 128, 256, 2, 2, 64, 3, 2>(p, epi, stream);
        return launch_epi<8, 8, 128, 128, 2, 2, VITQ_BK88, VITQ_S88, VITQ_OCC88>(p, epi, stream);
    }
    if (wb == 8 && ab == 4) return launch_epi<8, 4, VITQ_TC, VITQ_TT, VITQ_WC, VITQ_WT, VITQ_BK84, VITQ_S84, VITQ_OCC84>(p, epi, stream);
    return hipErrorInvalidValue;
}

}  // namespace vitq
