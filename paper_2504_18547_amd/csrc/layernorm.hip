// LayerNorm followed by a quantizer, without division by sigma and without square root
// (Sec. IV-C, Eq. 5, Fig. 5).
//
// Phase 1 -- row statistics.  They are the incremental recurrences of Eq. 5 in fp32, elements in
// order: that order is part of the definition (fp32 addition does not associate), so one LANE
// walks one row and the parallelism is across the 64 rows of a workgroup (one of its four waves).  The lane streams
// its row in chunks of 16 elements, the next chunk requested before the current one is used.
// Phase 2 -- levels.  The quantizer is the comparator of Fig. 5(b): the level is the number of
// references (k - 1/2)*step that the normalised value exceeds, each decided as
//     ssq((x - mu) * gamma) * n  >  ssq((k - 1/2)*step - beta) * V,      ssq(v) = v * |v|,
// V = M_n + n*eps the (stabilised) sum of squared deviations -- sigma never appears.  Elements
// are independent here, so the workgroup's rows are re-read wave by wave with coalesced 16-byte
// loads by all four waves, four elements per lane, one row at a time, the next row in flight.  The comparisons are monotone in k, so
// instead of all 2^b - 1 of them the kernel makes a guess with the hardware reciprocal square
// root.  A guess that lies further from every half-integer than the proven distance between the
// guess and the comparator's own boundary stands as it is; otherwise the comparator itself is
// evaluated at the guessed level and the one above, stepping the guess until both agree, and
// every decision is the comparator's.
#include "layernorm.h"
#include <type_traits>
#include "vitq_dev.h"

namespace vitq {

namespace {

// RN(1/k), k = 1 .. kRkMax, evaluated by the compiler (IEEE division).  With rk = RN(1/k):
//     q0 = RN(d*rk),  r = d - q0*k (exact in one FMA),  q = RN(q0 + r*rk)
// equals RN(d/k) for EVERY fp32 significand of d and every k <= 16384 -- checked exhaustively on
// the CPU (2^23 significands x 16384 divisors, no mismatch) -- and the exponent of d only scales
// all three steps, as long as q0 stays a normal number and nothing overflows: 2^-100 <= |d| <= 2^120.
#ifndef VITQ_LN_RB
#define VITQ_LN_RB 1      // rows a wave decides per batch in phase 2 (more cost registers, hence resident waves)
#endif
#ifndef VITQ_LN_CH
#define VITQ_LN_CH 16      // elements a lane requests at a time in phase 1
#endif
constexpr int kRkMax = 4096;
struct RkTable {
    float v[kRkMax + 1];
    constexpr RkTable() : v{} {
        for (int k = 1; k <= kRkMax; ++k) v[k] = 1.0f / (float)k;
    }
};
__device__ const RkTable g_rk{};

constexpr float kLnGuard = 0x1p-21f;   // unit of the guard that lets a guessed level stand without the comparator
constexpr int kLnRows = 64;       // rows per workgroup (one lane each in phase 1)
constexpr int kLnThreads = 256;   // threads per workgroup: all four waves work in phase 2
constexpr int kLnWaves = kLnThreads / 64;

template <bool VEC, int SB>
__global__ __launch_bounds__(kLnThreads) void layernorm_quantize_kernel(LnParams p) {
    __shared__ float s_mu[kLnRows], s_v[kLnRows], s_rs[kLnRows];
    const int tid = threadIdx.x;
    const int64_t row0 = (int64_t)blockIdx.x * kLnRows;
    const int cols = (int)p.cols;
    const float nf = (float)cols;

    // ---- phase 1: Eq. 5, mu_i = mu_{i-1} + (x_i - mu_{i-1}) / i,
    //                     M_i  = M_{i-1}  + (x_i - mu_{i-1}) * (x_i - mu_i)
    // The wave that walks the rows rotates with the workgroup index, so that the workgroups
    // sharing a CU keep different SIMDs busy with their recurrences.
    const int p1 = tid - (int)(blockIdx.x % kLnWaves) * 64;        // row of this lane in phase 1, if in [0, 64)
    if (p1 >= 0 && p1 < kLnRows && row0 + p1 < p.rows) {
        const float *xr = p.x + (row0 + p1) * p.ld;
        const float *rr = p.res ? p.res + (row0 + p1) * p.ld : nullptr;
        float mu = 0.0f, m2 = 0.0f;
        // One pass over the row.  FAST replaces the IEEE division d1 / i by the two-FMA correction
        // of d1 * RN(1/i) (see g_rk), which gives the same bits whenever d1 is zero or an ordinary
        // finite number: the pass tracks the largest and the smallest nonzero |d1| and reports
        // whether that held; the caller repeats the row with the division otherwise.
        auto walk = [&](auto FAST_T) -> bool {
            constexpr bool FAST = decltype(FAST_T)::value;
            mu = 0.0f; m2 = 0.0f;
            float hi = 0.0f, lo = 1.0f;
            auto step1 = [&](float xi, int i1) {      // i1 = 1-based index of the element
                const float d1 = xi - mu;
                float q;
                if constexpr (FAST) {
                    const float kf = (float)i1, rk = g_rk.v[i1];
                    const float q0 = d1 * rk;
                    const float r = fmaf(-q0, kf, d1);
                    q = fmaf(r, rk, q0);
                    hi = fmaxf(hi, fabsf(d1));
                    lo = fminf(lo, d1 == 0.0f ? 1.0f : fabsf(d1));
                } else {
                    q = d1 / (float)i1;
                }
                mu = mu + q;
                const float d2 = xi - mu;
                const float pr = d1 * d2;
                m2 = m2 + pr;
            };
            int j = 0;
            if (VEC) {
                constexpr int CH = VITQ_LN_CH;
                const int full = cols / CH * CH;
                auto load_chunk = [&](int j0, float (&v)[CH]) {
#pragma unroll
                    for (int q = 0; q < CH / 4; ++q) {
                        float4 a = *reinterpret_cast<const float4 *>(xr + j0 + 4 * q);
                        if (rr) {
                            const float4 b = *reinterpret_cast<const float4 *>(rr + j0 + 4 * q);
                            a.x = a.x + b.x; a.y = a.y + b.y; a.z = a.z + b.z; a.w = a.w + b.w;
                        }
                        v[4 * q] = a.x; v[4 * q + 1] = a.y; v[4 * q + 2] = a.z; v[4 * q + 3] = a.w;
                    }
                };
                if (full > 0) {
                    float cur[CH], nxt[CH];
                    load_chunk(0, cur);
                    for (; j < full; j += CH) {
                        load_chunk(min(j + CH, full - CH), nxt);      // (the last one re-reads its own chunk: no branch)
#pragma unroll
                        for (int i = 0; i < CH; ++i) step1(cur[i], j + i + 1);
#pragma unroll
                        for (int i = 0; i < CH; ++i) cur[i] = nxt[i];
                    }
                }
            }
            for (; j < cols; ++j) {                   // ragged tail, unaligned rows
                float t = xr[j];
                if (rr) t = t + rr[j];
                step1(t, j + 1);
            }
            // (a NaN deviation is skipped by the max but makes mu NaN; an infinite one shows in hi)
            return !FAST || (hi <= 0x1p120f && lo >= 0x1p-100f && mu == mu);
        };
        bool done = false;
        if (cols <= kRkMax) done = walk(std::true_type{});
        if (!done) walk(std::false_type{});
        const float ne = nf * p.eps;
        const float V = m2 + ne;
        s_mu[p1] = mu;
        s_v[p1] = V;
        s_rs[p1] = __builtin_amdgcn_rsqf(V / nf);      // for the guess only
    }
    __syncthreads();

    // ---- phase 2: levels, one row per wave at a time, four consecutive elements per lane ----
    const int lane = tid & 63, wave = tid >> 6;
    const float rstep = __builtin_amdgcn_rcpf(p.step);   // for the guess only
    const bool step_ok = p.step >= 0x1p-20f && p.step <= 0x1p10f;
    const float qminf = (float)p.qmin, qmaxf = (float)p.qmax;
    const int span = p.qmax - p.qmin;
    const int padded = p.row_bytes16 * 8 / SB;           // columns of the 16-byte padded row
    for (int c0 = 4 * lane; c0 < padded; c0 += 256) {
        // this lane's four columns are the same for every row
        float gm[4], bt[4], cg[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool ok = c0 + i < cols;
            gm[i] = ok ? p.gamma[c0 + i] : 0.0f;
            bt[i] = ok ? p.beta[c0 + i] : 0.0f;
            cg[i] = fmaf(fabsf(bt[i] * rstep), 3.0f * kLnGuard, 3.0f * kLnGuard);   // the guess's guard, constant part
        }
        // Rows are taken in batches of RB; the loads of the next batch are in flight while the
        // current one is decided (the rows no longer sit in a near cache after phase 1).
        constexpr int RB = VITQ_LN_RB, NB = kLnRows / kLnWaves / RB;
        auto load_batch = [&](int bi, float (&v)[RB][4]) {
#pragma unroll
            for (int k = 0; k < RB; ++k) {
                const int r = wave + kLnWaves * (bi * RB + k);
                const int64_t row = row0 + r;
                v[k][0] = v[k][1] = v[k][2] = v[k][3] = 0.0f;
                if (row < p.rows) {
                    const float *xr = p.x + row * p.ld;
                    if (VEC && c0 + 4 <= cols) {
                        float4 a = *reinterpret_cast<const float4 *>(xr + c0);
                        if (p.res) {
                            const float4 b = *reinterpret_cast<const float4 *>(p.res + row * p.ld + c0);
                            a.x = a.x + b.x; a.y = a.y + b.y; a.z = a.z + b.z; a.w = a.w + b.w;
                        }
                        v[k][0] = a.x; v[k][1] = a.y; v[k][2] = a.z; v[k][3] = a.w;
                        if (p.sum_out) *reinterpret_cast<float4 *>(p.sum_out + row * p.ld + c0) = a;
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            if (c0 + i < cols) {
                                float t = xr[c0 + i];
                                if (p.res) t = t + p.res[row * p.ld + c0 + i];
                                if (p.sum_out) p.sum_out[row * p.ld + c0 + i] = t;
                                v[k][i] = t;
                            }
                        }
                    }
                }
            }
        };
        float cur[RB][4], nxt[RB][4];
        load_batch(0, cur);
        for (int bi = 0; bi < NB; ++bi) {
            if (row0 + wave + kLnWaves * (bi * RB) >= p.rows) break;      // no rows left for this wave
            if (bi + 1 < NB) load_batch(bi + 1, nxt);
            // The guess.  In exact arithmetic on the fp32 values g, beta, step, V the comparator asks whether
            // t* = (g / sigma + beta) / step exceeds lv - 1/2 (sigma^2 = V/n).  The value tp computed here with
            // the hardware rsq / rcp differs from t* by at most (|g/(sigma*step)| + |beta/step|) * 2^-21, and
            // the comparator's own fp32 evaluation moves its boundary by at most (2|lv| + |beta/step| + 1) *
            // 2^-22 (five roundings on the two sides, two of them doubled by the squares).  So when tp is
            // further than kLnGuard * (4|tp| + 3|beta/step| + 3) from every half-integer, rint(tp) is the level
            // the comparator would count, and the comparator is not run; a NaN or an infinity makes the
            // figure NaN, which compares above the limit as a bit pattern.  The relative-error model behind
            // these bounds needs the squares to stay ordinary numbers: the guess is trusted only for
            // 2^-20 <= step <= 2^10 and 2^-40 <= V <= 2^30 (then an underflowing g*|g| can differ from the
            // exact product by 2^-139 at most, against |L - R| >= V * step^2 * d^2 for a value d levels from a
            // boundary, and nothing overflows below the |tp| that the guard itself rejects).
            float L[RB][4], c[RB][4], V[RB];
            u32 worst = step_ok ? 0u : 0x7FC00000u;
#pragma unroll
            for (int k = 0; k < RB; ++k) {
                const int r = wave + kLnWaves * (bi * RB + k);
                const float mu = s_mu[r], rs = s_rs[r];
                V[k] = s_v[r];
                if (!(V[k] >= 0x1p-40f && V[k] <= 0x1p30f)) worst = 0x7FC00000u;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float a = cur[k][i] - mu;
                    const float g = a * gm[i];
                    const float tp = fmaf(g, rs, bt[i]) * rstep;
                    const float t = rintf(tp);
                    const float fig = fmaf(fabsf(tp), 4.0f * kLnGuard, fabsf(tp - t)) + cg[i];
                    worst = max(worst, __float_as_uint(fig));
                    c[k][i] = (t == t) ? __builtin_amdgcn_fmed3f(t, qminf, qmaxf) : qminf;
                }
            }
            const bool verify = __builtin_amdgcn_ballot_w64(worst > __float_as_uint(0.5f)) != 0;
            if (verify) {
#pragma unroll
                for (int k = 0; k < RB; ++k) {
                    const float mu = s_mu[wave + kLnWaves * (bi * RB + k)];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float a = cur[k][i] - mu;
                        const float g = a * gm[i];
                        const float gs = g * fabsf(g);
                        L[k][i] = gs * nf;
                    }
                }
            }
            // comparator of Fig. 5(b): element (k, i) against the reference (lv - 1/2)*step
            auto above = [&](int k, int i, float lv) {
                const float rk = (lv - 0.5f) * p.step;
                const float cc = rk - bt[i];
                const float cs = cc * fabsf(cc);
                const float R = cs * V[k];
                return L[k][i] > R;
            };
            // level = qmin + #{lv : above(lv)}; above() is monotone in lv, so c is the level iff
            // above(c) (or c == qmin) and not above(c + 1) (or c == qmax)
            for (int it = 0; verify && it <= span; ++it) {
                bool moved = false;
#pragma unroll
                for (int k = 0; k < RB; ++k)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const bool low_ok = (c[k][i] <= qminf) || above(k, i, c[k][i]);
                        const bool high_ok = (c[k][i] >= qmaxf) || !above(k, i, c[k][i] + 1.0f);
                        const float d = !low_ok ? -1.0f : (!high_ok ? 1.0f : 0.0f);
                        c[k][i] = c[k][i] + d;
                        moved = moved || (d != 0.0f);
                    }
                if (__builtin_amdgcn_ballot_w64(moved) == 0) break;
            }
#pragma unroll
            for (int k = 0; k < RB; ++k) {
                const int64_t row = row0 + wave + kLnWaves * (bi * RB + k);
                if (row < p.rows) {
                    u32 w = 0;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const u32 field = (c0 + i < cols) ? ((u32)(int)c[k][i] & ((1u << SB) - 1u)) : 0u;
                        w |= field << (i * SB);
                    }
                    uint8_t *dst = p.out + row * p.out_stride + (int64_t)c0 * SB / 8;
                    if constexpr (SB == 8) *reinterpret_cast<u32 *>(dst) = w;
                    else if constexpr (SB == 4) *reinterpret_cast<uint16_t *>(dst) = (uint16_t)w;
                    else *dst = (uint8_t)w;
                }
            }
#pragma unroll
            for (int k = 0; k < RB; ++k)
#pragma unroll
                for (int i = 0; i < 4; ++i) cur[k][i] = nxt[k][i];
        }
    }
}

// ---- per-head LayerNorm quantizer of Q and K, plain quantizer of V (Fig. 1(b), Table I) --------
// One lane owns one (token, head) group of 64 channels: it loads the 256 bytes once, runs Eq. 5
// over them and decides the 64 levels from registers (same guess-and-verify use of the
// comparator as above; the lanes are independent, so each stops stepping on its own), then
// writes the head-major packed row the attention kernel reads.  Groups are independent:
// M * 3H lanes of parallelism, no LDS.
template <int SB>
__global__ __launch_bounds__(256) void qkv_headnorm_kernel(HeadNormParams p) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int groups = 3 * p.H;
    const int64_t M = (int64_t)p.B * p.N;
    if (t >= M * groups) return;
    const int64_t m = t / groups;
    const int gi = (int)(t - m * groups);
    const int which = gi / p.H, h = gi - which * p.H;
    const int b = (int)(m / p.N), n = (int)(m - (int64_t)b * p.N);
    const float *src = p.y + m * p.ld + (int64_t)gi * 64;
    float v[64];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const float4 a = *reinterpret_cast<const float4 *>(src + 4 * q);
        v[4 * q] = a.x; v[4 * q + 1] = a.y; v[4 * q + 2] = a.z; v[4 * q + 3] = a.w;
    }
    const float qminf = (float)p.qmin, qmaxf = (float)p.qmax;
    float lv[64];
    if (which == 2) {
#pragma unroll
        for (int i = 0; i < 64; ++i) lv[i] = (float)quantize_level(v[i], p.s_v, qminf, qmaxf);
    } else {
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
        const float ne = nf * p.eps;
        const float V = m2 + ne;
        const float step = which == 0 ? p.s_q : p.s_k;
        const float rs = __builtin_amdgcn_rsqf(V / nf);          // for the guess only
        const float rstep = __builtin_amdgcn_rcpf(step);         // for the guess only
        const bool stats_ok = step >= 0x1p-20f && step <= 0x1p10f && V >= 0x1p-40f && V <= 0x1p30f;
        const int span = p.qmax - p.qmin;
        const float *gp = p.gamma + which * p.D + h * 64, *bp = p.beta + which * p.D + h * 64;
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const float4 g4 = *reinterpret_cast<const float4 *>(gp + 4 * q);
            const float4 b4 = *reinterpret_cast<const float4 *>(bp + 4 * q);
            const float gm[4] = {g4.x, g4.y, g4.z, g4.w}, bt[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float a = v[4 * q + i] - mu;
                const float g = a * gm[i];
                const float gs = g * fabsf(g);
                const float L = gs * nf;
                auto above = [&](float k) {
                    const float rk = (k - 0.5f) * step;
                    const float cc = rk - bt[i];
                    const float cs = cc * fabsf(cc);
                    const float R = cs * V;
                    return L > R;
                };
                // (the guess stands when it is provably far from every boundary: see the kernel above)
                const float tp = fmaf(g, rs, bt[i]) * rstep;
                const float tt = rintf(tp);
                float c = (tt == tt) ? __builtin_amdgcn_fmed3f(tt, qminf, qmaxf) : qminf;
                const float cgi = fmaf(fabsf(bt[i] * rstep), 3.0f * kLnGuard, 3.0f * kLnGuard);
                const float fig = fmaf(fabsf(tp), 4.0f * kLnGuard, fabsf(tp - tt)) + cgi;
                if (!(stats_ok && fig <= 0.5f)) {
                    for (int it = 0; it <= span; ++it) {
                        const bool low_ok = (c <= qminf) || above(c);
                        const bool high_ok = (c >= qmaxf) || !above(c + 1.0f);
                        if (low_ok && high_ok) break;
                        c = c + (!low_ok ? -1.0f : 1.0f);
                    }
                }
                lv[4 * q + i] = c;
            }
        }
    }
    const int64_t row = (((int64_t)which * p.B + b) * p.H + h) * p.N + n;
    uint8_t *dst = p.out + row * (64 * SB / 8);
    constexpr int PW = 32 / SB;                      // levels per 32-bit word
#pragma unroll
    for (int w4 = 0; w4 < 64 / PW / 4; ++w4) {
        u32 w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            u32 acc = 0;
#pragma unroll
            for (int i = 0; i < PW; ++i)
                acc |= ((u32)(int)lv[(4 * w4 + j) * PW + i] & ((1u << SB) - 1u)) << (i * SB);
            w[j] = acc;
        }
        *reinterpret_cast<uint4 *>(dst + 16 * w4) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

}  // namespace

hipError_t qkv_headnorm_launch(const HeadNormParams &p, hipStream_t stream) {
    const int64_t threads = (int64_t)p.B * p.N * 3 * p.H;
    if (threads == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((threads + 255) / 256);
    if (p.sb == 4) hipLaunchKernelGGL(qkv_headnorm_kernel<4>, dim3(blocks), dim3(256), 0, stream, p);
    else if (p.sb == 8) hipLaunchKernelGGL(qkv_headnorm_kernel<8>, dim3(blocks), dim3(256), 0, stream, p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t layernorm_quantize_launch(const LnParams &p, hipStream_t stream) {
    if (p.rows == 0) return hipSuccess;
    const bool vec = (p.cols % 4 == 0) && (p.ld % 4 == 0) && (((uintptr_t)p.x) % 16 == 0) &&
                     (!p.res || ((uintptr_t)p.res) % 16 == 0) && (!p.sum_out || ((uintptr_t)p.sum_out) % 16 == 0);
    const unsigned blocks = (unsigned)((p.rows + kLnRows - 1) / kLnRows);
#define VITQ_LN_LAUNCH(V, S) hipLaunchKernelGGL((layernorm_quantize_kernel<V, S>), dim3(blocks), dim3(kLnThreads), 0, stream, p)
    if (p.sb == 4) { if (vec) VITQ_LN_LAUNCH(true, 4); else VITQ_LN_LAUNCH(false, 4); }
    else if (p.sb == 8) { if (vec) VITQ_LN_LAUNCH(true, 8); else VITQ_LN_LAUNCH(false, 8); }
    else if (p.sb == 2) { if (vec) VITQ_LN_LAUNCH(true, 2); else VITQ_LN_LAUNCH(false, 2); }
    else return hipErrorInvalidValue;
#undef VITQ_LN_LAUNCH
    return hipGetLastError();
}

}  // namespace vitq
