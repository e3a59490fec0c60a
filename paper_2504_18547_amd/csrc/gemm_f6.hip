// Experimental 6-bit-float operand path for the reordered linear (Eq. 2).
//
// CDNA4's scaled-MFMA instruction takes 6-bit E3M2 operands ("BF6": 1 sign, 3 exponent, 2
// mantissa bits, bias 3) at twice the rate of int8 and accumulates in fp32.  Every integer in
// [-8, 8] is an E3M2 value, so b-bit levels (b <= 4) can be handed to the matrix core as they
// are -- no unpacking instruction in the main loop -- provided they are STORED as those codes.
// Products are integers <= 64 in magnitude and the sums stay far below 2^24, where the fp32
// accumulation of integers was found exact on the hardware (the parity tests compare the fp32
// outputs of this path with the integer definition bit for bit).
//
//   recode_e3m2_kernel   packed 4-bit two's-complement rows  ->  rows of 6-bit codes
//                        (128 values = 96 bytes in the piece order described below; rows padded
//                        with zero codes to whole groups of 128)
//   gemm_f6_kernel       y[m][c] = fma(sum_k x[m][k]*w[c][k], s_x*s_w[c], b[c])     fp32 out
//
// Operand layout in registers (v_mfma_scale_f32_32x32x64_f8f6f4, 6-bit formats): lane l holds
// row l % 32 of its operand, k = 32*(l / 32) .. +31, as 192 consecutive bits (value j at bits
// 6j .. 6j+5) in six VGPRs: 24 bytes, one and a half 16-byte pieces.
//
// Storage format of a re-coded row ("stage" = 128 values = 96 bytes = six 16-byte pieces).
// Quarter q = 2s + h of a stage (values 32q .. 32q+31; s = MFMA step, h = half-wave that
// consumes it) is a 192-bit string; its first 128 bits are piece 3h + s, its last 64 bits are
// half s of piece 3h + 2.  A lane of half-wave h therefore reads the three consecutive pieces
// 3h, 3h+1, 3h+2 of its row once per stage with 16-byte LDS reads and owns both of its MFMA
// operands: {piece 3h+s, half s of piece 3h+2}.
//
// LDS layout.  Operands arrive through direct global->LDS loads of 16 bytes per lane, lane i at
// M0 + 16*i: the kernel is free to choose which piece of which row a lane fetches.  The piece a
// row keeps at position `pos` is (pos - rot(row)) mod 6 with rot = bit 2 of the row index, which
// spreads the 24-word row pitch over the banks (without it rows r and r+4 collide).
//
// MFMA roles: tokens on the A side, weight rows on the B side, so that register r of the wave
// is 32 consecutive channels (a 128-byte line) of one token, as in the int8 kernel's fp32 epilogue.
#include "gemm_f6.h"
#include "launch_util.h"
#include "vitq_dev.h"

namespace vitq {

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

// ---- level -> E3M2 code -----------------------------------------------------------------------
// |v| in 1..8 as fp32 has exponent e = floor(log2 |v|) and the two mantissa bits E3M2 keeps in
// bits 22..21, so its code is (fp32 bits >> 21) - ((127 - 3) << 2); zero stays zero.
__device__ __forceinline__ u32 e3m2_of_nibble(u32 n) {
    const int v = ((int)(n << 28)) >> 28;                // two's-complement 4-bit field
    const int a = v < 0 ? -v : v;
    const u32 mag = a == 0 ? 0u : ((__float_as_uint((float)a) >> 21) - ((127u - 3u) << 2));
    return mag | (v < 0 ? 32u : 0u);
}

__global__ __launch_bounds__(256) void recode_e3m2_kernel(RecodeParams p) {
    // one thread per quarter of a stage: 32 values = four input dwords -> 128 + 64 output bits
    const int64_t quarters_per_row = p.out_stride / 24;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= p.rows * quarters_per_row) return;
    const int64_t row = t / quarters_per_row;
    const int64_t qi = t - row * quarters_per_row;       // quarter index along the row
    u32 w[4] = {0, 0, 0, 0};
    if (qi * 16 + 16 <= p.in_row_bytes16) {              // (input rows are zero beyond cols)
        const uint4 v = *reinterpret_cast<const uint4 *>(p.in + row * p.in_stride + qi * 16);
        w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
    }
    u32 o[6] = {0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        const u32 n = (w[j >> 3] >> (4 * (j & 7))) & 15u;
        const u32 c = (qi * 32 + j < p.cols) ? e3m2_of_nibble(n) : 0u;
        const int bit = 6 * j, d = bit >> 5, sh = bit & 31;
        o[d] |= c << sh;
        if (sh > 26) o[d + 1] |= c >> (32 - sh);
    }
    const int64_t stage = qi >> 2;
    const int q = (int)(qi & 3), s = q >> 1, h = q & 1;
    uint8_t *base = p.out + row * p.out_stride + stage * 96;
    *reinterpret_cast<uint4 *>(base + (3 * h + s) * 16) = make_uint4(o[0], o[1], o[2], o[3]);
    *reinterpret_cast<uint2 *>(base + (3 * h + 2) * 16 + 8 * s) = make_uint2(o[4], o[5]);
}

// ---- direct global -> LDS load (16 bytes per lane, lane i to M0 + 16*i) ---------------------------
__device__ __forceinline__ u32 lds_address_f6(const void *p) {
    return (u32)(uintptr_t)(const __attribute__((address_space(3))) uint8_t *)p;
}
__device__ __forceinline__ void dma16_f6(u32 voff, const uint8_t *sbase, u32 lds_dst) {
    u32 keep;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %1, %2\n\ts_mov_b32 m0, %0"
                 : "=&s"(keep) : "v"(voff), "s"(sbase), "s"(lds_dst) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt_f6() {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

constexpr int kRowB = 96;           // bytes of one row in one stage (128 values)
constexpr int kPieces = 6;          // 16-byte pieces per row and stage

__device__ __forceinline__ int rot_of(int row) { return (row >> 2) & 1; }

// TILE x TILE tokens x channels per workgroup, (TILE/64)^2 waves of 64 x 64 each, S stages in LDS.
// (TILE = 256 with 16 waves and three stages was measured as well: same results, same time --
// the bytes moved are not what bounds the kernel; 128 is what is launched.)
template <int TILE, int S, int OCC>
__global__ __launch_bounds__((TILE / 64) * (TILE / 64) * 64, OCC) void gemm_f6_kernel(F6Params p) {
    constexpr int kTile = TILE;
    constexpr int NWC = TILE / 64;                                // waves along the channels (and along the tokens)
    constexpr int kThreads = NWC * NWC * 64;
    constexpr int kStage = 2 * kTile * kRowB;                     // weights then tokens
    constexpr int kLoads = 2 * kTile * kPieces / kThreads;        // loads per lane and stage
    static_assert(2 * kTile * kPieces % kThreads == 0 && (kTile * kPieces) % 64 == 0, "tile / threads mismatch");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_c = wave % NWC, wave_t = wave / NWC;
    const int li = lane & 31, kh = lane >> 5;

    // workgroups of one XCD walk consecutive tiles (they share that XCD's L2 copy of the tokens)
    const int n_ct = (p.Nout + kTile - 1) / kTile;
    int logical;
    {
        const int total = gridDim.x, id = blockIdx.x;
        const int xcd = id & 7, slot = id >> 3;
        const int per = total >> 3, rem = total & 7;
        logical = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + slot;
    }
    const int c0 = (logical % n_ct) * kTile;
    const int t0 = (logical / n_ct) * kTile;
    const int nk = (p.K + 127) / 128;

    // ---- what each lane fetches per stage: slot = it*threads + tid; the first kTile*6 slots are
    // weight rows, the rest token rows (the boundary falls between waves, never inside one)
    const uint8_t *wbase = p.w + (int64_t)c0 * p.w_stride;
    const uint8_t *xbase = p.x + (int64_t)t0 * p.x_stride;
    u32 off[kLoads];
    bool from_w[kLoads];                                        // wave-uniform
#pragma unroll
    for (int it = 0; it < kLoads; ++it) {
        from_w[it] = it * kThreads + wave * 64 < kTile * kPieces;
        const int slot = it * kThreads + tid - (from_w[it] ? 0 : kTile * kPieces);
        const int row = slot / kPieces, pos = slot - row * kPieces;
        const int piece = (pos + kPieces - rot_of(row)) % kPieces;
        // rows beyond the matrix are clamped to its last row: their sums are never stored
        const int grow = from_w[it] ? min(row, p.Nout - 1 - c0) : min(row, p.M - 1 - t0);
        off[it] = (u32)grow * (u32)(from_w[it] ? p.w_stride : p.x_stride) + (u32)piece * 16u;
    }
    const u32 lds0 = __builtin_amdgcn_readfirstlane(lds_address_f6(smem)) + (u32)wave * 1024u;
    auto issue = [&](int kt) {
        const u32 dst = lds0 + (u32)(kt % S) * kStage;
        const uint8_t *wk = wbase + (int64_t)kt * kRowB;
        const uint8_t *xk = xbase + (int64_t)kt * kRowB;
#pragma unroll
        for (int it = 0; it < kLoads; ++it)
            dma16_f6(off[it], from_w[it] ? wk : xk, dst + it * (kThreads * 16));
    };
#pragma unroll
    for (int st = 0; st < S - 1; ++st)
        if (st < nk) issue(st);

    // this lane's channels (one per 32-channel block): scale and bias of the epilogue
    float sc[2], bs[2];
#pragma unroll
    for (int ci = 0; ci < 2; ++ci) {
        const int ch = min(c0 + wave_c * 64 + ci * 32 + li, p.Nout - 1);
        sc[ci] = p.s_x * p.s_w[p.s_w_per_channel ? ch : 0];
        bs[ci] = p.bias ? p.bias[ch] : 0.0f;
    }

    v16f acc[2][2];          // [token block][channel block]
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // Byte offsets (inside a stage, relative to the row) of this lane's three pieces 3*kh + j,
    // stored at position (3*kh + j + rot) mod 6.
    u32 rd[3];
    {
        const int rot = rot_of(li);
#pragma unroll
        for (int j = 0; j < 3; ++j) rd[j] = (u32)(((3 * kh + j + rot) % kPieces) * 16);
    }
    const u32 w_row = (u32)((wave_c * 64 + li) * kRowB);
    const u32 x_row = (u32)(kTile * kRowB + (wave_t * 64 + li) * kRowB);
    auto compute = [&](int buf) {
        const uint8_t *stage = smem + buf * kStage;
        uint4 wp[2][3], xp[2][3];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                wp[b][j] = *reinterpret_cast<const uint4 *>(stage + w_row + b * 32 * kRowB + rd[j]);
                xp[b][j] = *reinterpret_cast<const uint4 *>(stage + x_row + b * 32 * kRowB + rd[j]);
            }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            v8i wf[2], xf[2];
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const uint4 wa = wp[b][s], xa = xp[b][s];
                wf[b][0] = (int)wa.x; wf[b][1] = (int)wa.y; wf[b][2] = (int)wa.z; wf[b][3] = (int)wa.w;
                xf[b][0] = (int)xa.x; xf[b][1] = (int)xa.y; xf[b][2] = (int)xa.z; xf[b][3] = (int)xa.w;
                wf[b][4] = (int)(s ? wp[b][2].z : wp[b][2].x); wf[b][5] = (int)(s ? wp[b][2].w : wp[b][2].y);
                xf[b][4] = (int)(s ? xp[b][2].z : xp[b][2].x); xf[b][5] = (int)(s ? xp[b][2].w : xp[b][2].y);
                wf[b][6] = 0; wf[b][7] = 0; xf[b][6] = 0; xf[b][7] = 0;
            }
#pragma unroll
            for (int ti = 0; ti < 2; ++ti)
#pragma unroll
                for (int ci = 0; ci < 2; ++ci)
                    acc[ti][ci] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        xf[ti], wf[ci], acc[ti][ci], 3 /* A: E3M2 */, 3 /* B: E3M2 */, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
        }
    };

    for (int kt = 0; kt < nk; ++kt) {
        const int younger = nk - 1 - kt;
        if (younger >= S - 2) wait_vmcnt_f6<(S - 2) * kLoads>();
        else if (younger == 1) wait_vmcnt_f6<kLoads>();
        else wait_vmcnt_f6<0>();
        __syncthreads();
        if (kt + S - 1 < nk) issue(kt + S - 1);
        compute(kt % S);
    }

    // ---- epilogue: the sums are integers held exactly in fp32, so y is the definition's
    // fma((float)acc, s_x*s_w[c], b[c]) without a conversion
#pragma unroll
    for (int ci = 0; ci < 2; ++ci) {
        const int ch = c0 + wave_c * 64 + ci * 32 + li;
        if (ch >= p.Nout) continue;
#pragma unroll
        for (int ti = 0; ti < 2; ++ti) {
            const int m0 = t0 + wave_t * 64 + ti * 32 + 4 * kh;
            float *out = p.y_out + (int64_t)m0 * p.Nout + ch;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int dm = 8 * (r >> 2) + (r & 3);
                if (m0 + dm < p.M) out[(int64_t)dm * p.Nout] = fmaf(acc[ti][ci][r], sc[ci], bs[ci]);
            }
        }
    }
}

template <int TILE, int S, int OCC>
hipError_t launch_f6(const F6Params &p, hipStream_t stream) {
    constexpr size_t lds = (size_t)S * 2 * TILE * kRowB;
    constexpr int threads = (TILE / 64) * (TILE / 64) * 64;
    auto kern = gemm_f6_kernel<TILE, S, OCC>;
    static std::atomic<uint64_t> allowed{0};            // (one per instantiation)
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds, allowed);
    if (e != hipSuccess) return e;
    const int64_t blocks = (int64_t)((p.Nout + TILE - 1) / TILE) * ((p.M + TILE - 1) / TILE);
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(threads), lds, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t recode_e3m2_launch(const RecodeParams &p, hipStream_t stream) {
    const int64_t threads = p.rows * (p.out_stride / 24);
    if (threads == 0) return hipSuccess;
    hipLaunchKernelGGL(recode_e3m2_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream, p);
    return hipGetLastError();
}

#ifndef VITQ_F6_S
#define VITQ_F6_S 2      // stages in LDS (24 KB each); with 2, three workgroups share a CU
#define VITQ_F6_OCC 3
#endif
hipError_t gemm_f6_launch(const F6Params &p, hipStream_t stream) {
    // per-lane operand offsets inside a tile are kept in 32 bits (255 rows * stride + 80)
    if (p.M < 1 || p.Nout < 1 || p.K < 1 || p.x_stride >= (1 << 23) || p.w_stride >= (1 << 23)) return hipErrorInvalidValue;
    return launch_f6<128, VITQ_F6_S, VITQ_F6_OCC>(p, stream);
}

}  // namespace vitq
