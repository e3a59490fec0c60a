// Integer GEMM with fused dequant / bias / GELU / requant epilogue (reordered linear, Eq. 2).
//
//   acc[m][c] = sum_k xq[m][k] * wq[c][k]      int8 MFMA (v_mfma_i32_32x32x32_i8), int32 exact
//   y         = fma((float)acc, s_x*s_w[c], b[c]);  optional GELU;  optional requantization
//
// Both operands stay PACKED (b-bit fields) in HBM and in LDS; a lane unpacks its fragment to
// int8 in registers right before the MFMA (2^(8-b)-scaled values, see vitq_dev.h), and the
// epilogue removes the scale with an exact arithmetic shift.
//
// MFMA roles: the A operand (32 rows) carries WEIGHT rows (output channels), the B operand
// (32 columns) carries TOKEN rows, so a lane of the 32x32 result holds 16 output channels of
// ONE token.  Weight rows are placed in LDS in a permuted slot order so that those 16 channels
// are consecutive: the lane then packs them into one 8-byte (4-bit) store of the token's
// output row, which is exactly the packed operand layout the next linear reads.
#include "gemm.h"
#include "vitq_dev.h"

namespace vitq {

namespace {

constexpr int kBK = 128;  // contraction values staged per LDS buffer

// channel c (0..31 within a 32-block) -> MFMA row slot, chosen so that a lane's sixteen
// accumulator registers (rows 8*(r/4) + 4*(lane/32) + r%4) are channels 16*(lane/32) + r
__device__ __forceinline__ int slot_of_channel(int c) {
    return 8 * ((c & 15) >> 2) + 4 * (c >> 4) + (c & 3);
}

template <int WB, int AB>
struct Shift {
    static constexpr int value = (WB == 4 && AB == 4) ? 8 : (WB == 2 && AB == 4) ? 10 : 0;
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

// Epilogue for one 32x32 accumulator block: this lane owns token m and channels cb..cb+15.
__device__ __forceinline__ void epilogue_block(const GemmParams &p, const v16i &acc, int shift,
                                               int m, int cb, const float (&sc)[16],
                                               const float (&bs)[16]) {
    if (m >= p.M) return;
    const int nvalid = p.Nout - cb;  // may be <= 0 for a group that only exists as padding
    const bool full = nvalid >= 16;
    float y[16];
    int a[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        a[r] = acc[r] >> shift;
        float v = fmaf((float)a[r], sc[r], bs[r]);
        if (p.act == 1) v = gelu_tanh(v);
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
        float s_y = p.s_y[0];
        uint8_t *dst;
        if (p.head_major) {
            if (nvalid <= 0) return;
            // channel -> (q/k/v, head, d); token -> (image, n)
            int which = cb / p.D;
            int rem = cb - which * p.D;
            int h = rem / p.dh;
            int d = rem - h * p.dh;
            int b = m / p.Ntok;
            int n = m - b * p.Ntok;
            s_y = which == 0 ? p.s_y[0] : (which == 1 ? p.s_y[1] : p.s_y[2]);
            int64_t row = (((int64_t)which * p.Bimg + b) * p.Hh + h) * p.Ntok + n;
            dst = p.yq + row * p.yq_stride + ((d * p.yq_sb) >> 3);
        } else {
            if (((cb * p.yq_sb) >> 3) >= p.yq_row_bytes16) return;
            dst = p.yq + (int64_t)m * p.yq_stride + ((cb * p.yq_sb) >> 3);
        }
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

template <int WB, int AB, int TC, int TT, int WAVES_C, int WAVES_T>
__global__ __launch_bounds__(WAVES_C *WAVES_T * 64) void gemm_kernel(GemmParams p) {
    constexpr int NT = WAVES_C * WAVES_T * 64;
    constexpr int WROW = kBK * WB / 8, XROW = kBK * AB / 8;   // bytes per row per stage
    constexpr int WPITCH = WROW + 16, XPITCH = XROW + 16;     // LDS row pitch (bank spread)
    constexpr int WCH = WROW / 16, XCH = XROW / 16;           // 16-byte chunks per row
    constexpr int W_ITERS = TC * WCH / NT, X_ITERS = TT * XCH / NT;
    static_assert((TC * WCH) % NT == 0 && (TT * XCH) % NT == 0, "tile/threads mismatch");
    constexpr int WC = TC / WAVES_C, WT = TT / WAVES_T;       // wave tile
    constexpr int NC = WC / 32, NTK = WT / 32;                // 32x32 blocks per wave
    static_assert(WC % 32 == 0 && WT % 32 == 0 && TC % 64 == 0, "wave tile");
    constexpr int WBUF = TC * WPITCH, XBUF = TT * XPITCH;

    __shared__ __attribute__((aligned(16))) uint8_t smem[2 * (WBUF + XBUF)];
    uint8_t *sW = smem;
    uint8_t *sX = smem + 2 * WBUF;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wave_c = wave % WAVES_C;
    const int wave_t = wave / WAVES_C;
    const int li = lane & 31;   // MFMA row / column index of this lane
    const int g = lane >> 5;    // k-group of this lane

    const int n_ct = (p.Nout + TC - 1) / TC;
    const int ct = blockIdx.x % n_ct;
    const int tt = blockIdx.x / n_ct;
    const int c0 = ct * TC;
    const int t0 = tt * TT;

    v16i acc[NC][NTK];
#pragma unroll
    for (int i = 0; i < NC; ++i)
#pragma unroll
        for (int j = 0; j < NTK; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    uint4 wreg[W_ITERS], xreg[X_ITERS];

    auto gload = [&](int kt) {
#pragma unroll
        for (int it = 0; it < W_ITERS; ++it) {
            int id = it * NT + tid;
            int row = id / WCH, ch = id % WCH;
            int gr = c0 + row;
            int kb = kt * WROW + ch * 16;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (gr < p.Nout && kb < p.kbytes_w16)
                v = *reinterpret_cast<const uint4 *>(p.w + (int64_t)gr * p.w_stride + kb);
            wreg[it] = v;
        }
#pragma unroll
        for (int it = 0; it < X_ITERS; ++it) {
            int id = it * NT + tid;
            int row = id / XCH, ch = id % XCH;
            int gr = t0 + row;
            int kb = kt * XROW + ch * 16;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (gr < p.M && kb < p.kbytes_x16)
                v = *reinterpret_cast<const uint4 *>(p.x + (int64_t)gr * p.x_stride + kb);
            xreg[it] = v;
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int it = 0; it < W_ITERS; ++it) {
            int id = it * NT + tid;
            int row = id / WCH, ch = id % WCH;
            int slot = (row & ~31) | slot_of_channel(row & 31);
            *reinterpret_cast<uint4 *>(sW + buf * WBUF + slot * WPITCH + ch * 16) = wreg[it];
        }
#pragma unroll
        for (int it = 0; it < X_ITERS; ++it) {
            int id = it * NT + tid;
            int row = id / XCH, ch = id % XCH;
            *reinterpret_cast<uint4 *>(sX + buf * XBUF + row * XPITCH + ch * 16) = xreg[it];
        }
    };
    auto compute = [&](int buf) {
        const uint8_t *bw = sW + buf * WBUF + (wave_c * WC + li) * WPITCH;
        const uint8_t *bx = sX + buf * XBUF + (wave_t * WT + li) * XPITCH;
#pragma unroll
        for (int ss = 0; ss < kBK / 64; ++ss) {
            // lane g owns values [64*ss + 32*g, +32): two MFMA operands of 16 values each
            v4i wf[NC][2], xf[NTK][2];
#pragma unroll
            for (int ci = 0; ci < NC; ++ci) {
                const uint8_t *src = bw + ci * 32 * WPITCH + ((ss * 64 + g * 32) * WB) / 8;
                if constexpr (WB == 4) {
                    uint4 v = *reinterpret_cast<const uint4 *>(src);
                    wf[ci][0] = unpack4_x16(v.x, v.y);
                    wf[ci][1] = unpack4_x16(v.z, v.w);
                } else if constexpr (WB == 2) {
                    uint2 v = *reinterpret_cast<const uint2 *>(src);
                    wf[ci][0] = unpack2_x64(v.x);
                    wf[ci][1] = unpack2_x64(v.y);
                } else {
                    wf[ci][0] = *reinterpret_cast<const v4i *>(src);
                    wf[ci][1] = *reinterpret_cast<const v4i *>(src + 16);
                }
            }
#pragma unroll
            for (int ti = 0; ti < NTK; ++ti) {
                const uint8_t *src = bx + ti * 32 * XPITCH + ((ss * 64 + g * 32) * AB) / 8;
                if constexpr (AB == 4) {
                    uint4 v = *reinterpret_cast<const uint4 *>(src);
                    if constexpr (WB == 2) {
                        xf[ti][0] = unpack4_x16_order2(v.x, v.y);
                        xf[ti][1] = unpack4_x16_order2(v.z, v.w);
                    } else {
                        xf[ti][0] = unpack4_x16(v.x, v.y);
                        xf[ti][1] = unpack4_x16(v.z, v.w);
                    }
                } else {
                    xf[ti][0] = *reinterpret_cast<const v4i *>(src);
                    xf[ti][1] = *reinterpret_cast<const v4i *>(src + 16);
                }
            }
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int ci = 0; ci < NC; ++ci)
#pragma unroll
                    for (int ti = 0; ti < NTK; ++ti)
                        acc[ci][ti] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[ci][s], xf[ti][s],
                                                                            acc[ci][ti], 0, 0, 0);
        }
    };

    const int nk = (p.K + kBK - 1) / kBK;
    gload(0);
    sstore(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const bool more = kt + 1 < nk;
        if (more) gload(kt + 1);
        compute(kt & 1);
        if (more) sstore((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue -------------------------------------------------------------------------
    constexpr int shift = Shift<WB, AB>::value;
#pragma unroll
    for (int ci = 0; ci < NC; ++ci) {
        const int cb = c0 + wave_c * WC + ci * 32 + 16 * g;
        float sc[16], bs[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int c = cb + r;
            bool ok = c < p.Nout;
            float sw = ok ? p.s_w[p.s_w_per_channel ? c : 0] : 1.0f;
            sc[r] = p.s_x * sw;
            bs[r] = (ok && p.bias) ? p.bias[c] : 0.0f;
        }
#pragma unroll
        for (int ti = 0; ti < NTK; ++ti) {
            const int m = t0 + wave_t * WT + ti * 32 + li;
            epilogue_block(p, acc[ci][ti], shift, m, cb, sc, bs);
        }
    }
}

template <int WB, int AB, int TC, int TT, int WAVES_C, int WAVES_T>
hipError_t launch(const GemmParams &p, hipStream_t stream) {
    const int n_ct = (p.Nout + TC - 1) / TC;
    const int n_tt = (p.M + TT - 1) / TT;
    const int64_t blocks = (int64_t)n_ct * n_tt;
    hipLaunchKernelGGL((gemm_kernel<WB, AB, TC, TT, WAVES_C, WAVES_T>), dim3((unsigned)blocks),
                       dim3(WAVES_C * WAVES_T * 64), 0, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t gemm_launch(const GemmParams &p, int wb, int ab, hipStream_t stream) {
    if (wb == 4 && ab == 4) return launch<4, 4, 128, 128, 2, 2>(p, stream);
    if (wb == 2 && ab == 4) return launch<2, 4, 128, 128, 2, 2>(p, stream);
    if (wb == 8 && ab == 8) return launch<8, 8, 128, 128, 2, 2>(p, stream);
    return hipErrorInvalidValue;
}

}  // namespace vitq
