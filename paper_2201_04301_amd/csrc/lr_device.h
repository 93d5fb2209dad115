// Device helpers shared by the logistic-regression kernels (paper Sec. II-A: the minibatch
// gradient of the logistic loss): wave reductions and the two residuals of a row.
#pragma once
#include "gcada_internal.h"

namespace gcada {

constexpr int kWave = 64;

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// Sum over the 64 lanes through the data-parallel-primitive lane moves (a few cycles each, where
// a shuffle through the LDS crossbar takes a hundred): lanes ^1, ^2, mirror within 8, mirror
// within 16, then the four rows' totals in ascending order.  Every lane gets the total.
__device__ __forceinline__ double dpp_move(double v, int ctrl_is)
{
    // ctrl_is: 0 = quad_perm [1,0,3,2], 1 = quad_perm [2,3,0,1], 2 = row_half_mirror, 3 = row_mirror
    const long long b = __double_as_longlong(v);
    int lo = (int)(b & 0xffffffffll), hi = (int)(b >> 32);
    switch (ctrl_is) {
    case 0: lo = __builtin_amdgcn_update_dpp(0, lo, 0xB1, 0xF, 0xF, true); hi = __builtin_amdgcn_update_dpp(0, hi, 0xB1, 0xF, 0xF, true); break;
    case 1: lo = __builtin_amdgcn_update_dpp(0, lo, 0x4E, 0xF, 0xF, true); hi = __builtin_amdgcn_update_dpp(0, hi, 0x4E, 0xF, 0xF, true); break;
    case 2: lo = __builtin_amdgcn_update_dpp(0, lo, 0x141, 0xF, 0xF, true); hi = __builtin_amdgcn_update_dpp(0, hi, 0x141, 0xF, 0xF, true); break;
    default: lo = __builtin_amdgcn_update_dpp(0, lo, 0x140, 0xF, 0xF, true); hi = __builtin_amdgcn_update_dpp(0, hi, 0x140, 0xF, 0xF, true); break;
    }
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
__device__ __forceinline__ double lane_value(double v, int l)
{
    const long long b = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_readlane((int)(b & 0xffffffffll), l);
    const int hi = __builtin_amdgcn_readlane((int)(b >> 32), l);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
__device__ __forceinline__ double wave_total(double v)
{
    v += dpp_move(v, 0);
    v += dpp_move(v, 1);
    v += dpp_move(v, 2);
    v += dpp_move(v, 3);
    return ((lane_value(v, 0) + lane_value(v, 16)) + lane_value(v, 32)) + lane_value(v, 48);
}

// ---- sums over the 16 lanes of a row through data-parallel-primitive moves only ----
// A shuffle goes through the LDS crossbar (a hundred cycles, more while other waves stream tiles
// through LDS); a DPP move is part of the add that uses it.  Within a row of 16 lanes four moves
// are exclusive-ors of the lane number: with 8 (rotate by 8), 7 (mirror within 8), 2 and 1 (quad
// permutations); together they reach all 16 lanes.
template <int STEP>
__device__ __forceinline__ float row_xor(float v)
{
    static_assert(STEP >= 0 && STEP < 4, "four moves");
    constexpr int ctrl = STEP == 0 ? 0x128       // row_ror:8          lane ^ 8
                       : STEP == 1 ? 0x141       // row_half_mirror    lane ^ 7
                       : STEP == 2 ? 0x4E        // quad_perm [2,3,0,1] lane ^ 2
                                   : 0xB1;       // quad_perm [1,0,3,2] lane ^ 1
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, 0xF, 0xF, true));
}

// v[0..N) per lane -> sums over the 16 lanes of the lane's row, N <= 32.  Each halving step
// exchanges half of the remaining values with the partner lane (bit 8, 4, 2, 1 of the lane number
// says which half a lane keeps: the upper one if the bit is set); once one value is left the
// remaining moves add the partner's.  Afterwards v[0..max(1, N/16)) holds the row's sums of the
// values row_butterfly_first<N>(lane) + j, in every lane (each value max(1, 16/N) times per row).
template <int N, int STEP = 0>
struct RowButterfly {
    static __device__ __forceinline__ void run(float (&v)[N], int lane)
    {
        if constexpr (STEP < 4) {
            if constexpr (N > 1) {
                const bool up = (lane & (8 >> STEP)) != 0;
                float w[N / 2];
#pragma unroll
                for (int i = 0; i < N / 2; ++i) {
                    const float send = up ? v[i] : v[i + N / 2];
                    const float keep = up ? v[i + N / 2] : v[i];
                    w[i] = keep + row_xor<STEP>(send);
                }
                RowButterfly<N / 2, STEP + 1>::run(w, lane);
#pragma unroll
                for (int i = 0; i < ((N >> (4 - STEP)) > 1 ? (N >> (4 - STEP)) : 1); ++i) v[i] = w[i];
            } else {
                v[0] += row_xor<STEP>(v[0]);
                RowButterfly<1, STEP + 1>::run(v, lane);
            }
        }
    }
};
template <int N>
__device__ __forceinline__ int row_butterfly_first(int lane)
{
    int e = 0, n = N;
#pragma unroll
    for (int step = 0; step < 4 && n > 1; ++step, n >>= 1)
        if (lane & (8 >> step)) e += n / 2;
    return e;
}
// Sum over the 16 lanes of the row, every lane gets it.
__device__ __forceinline__ float row_total(float v)
{
    v += row_xor<3>(v);
    v += row_xor<2>(v);
    v += row_xor<1>(v);
    v += row_xor<0>(v);
    return v;
}

// The logistic residuals below sit on the critical path of every logistic kernel (in the team
// kernel one wave forms them for each tile while eight others wait at the next barrier), so they
// are built from the hardware's exp2 / log2 / reciprocal instructions (1 ulp each) with the
// corrections that keep every result within a few ulp, instead of the library routines, whose
// dependent instruction chains are five to ten times longer.

// 1 / d for 1 <= d <= 2: hardware reciprocal and one Newton step.
__device__ __forceinline__ float recip_1to2(float d)
{
    const float r = __builtin_amdgcn_rcpf(d);
    return fmaf(fmaf(-d, r, 1.0f), r, r);
}

__device__ __forceinline__ float sigmoidf_(float t)
{
    const float e = exp_nonpos(-fabsf(t));
    const float s = recip_1to2(1.0f + e);
    return t >= 0 ? s : e * s;
}

// e^t - 1 for |t| < 0.5: t + t^2 (1/2! + t/3! + ... + t^7/9!); the first term left out is
// below 6e-10 |t|.
__device__ __forceinline__ float expm1_small(float t)
{
    float p = 0x1.71de3ap-19f;            // 1/9!
    p = fmaf(p, t, 0x1.a01a02p-16f);      // 1/8!
    p = fmaf(p, t, 0x1.a01a02p-13f);      // 1/7!
    p = fmaf(p, t, 0x1.6c16c2p-10f);      // 1/6!
    p = fmaf(p, t, 0x1.111112p-7f);       // 1/5!
    p = fmaf(p, t, 0x1.555556p-5f);       // 1/4!
    p = fmaf(p, t, 0x1.555556p-3f);       // 1/3!
    p = fmaf(p, t, 0.5f);
    return fmaf(t * t, p, t);
}

// log(1 + e) for 0 <= e <= 1.  Below 2^-12 the series e - e^2/2 (the next term is under 2e-8 e);
// above it the hardware logarithm of the rounded sum, whose absolute error (6e-8) is then below
// 3e-4 of the result -- this value only enters the reported loss, a sum over the minibatch.
__device__ __forceinline__ float log1p_unit(float e)
{
    const float series = fmaf(-0.5f * e, e, e);
    const float viaLog = 0x1.62e43p-1f * __builtin_amdgcn_logf(1.0f + e);
    return e < 0x1p-12f ? series : viaLog;
}

// r = residual at theta^k, dr = r - (residual at theta_stale), from z = x.theta^k and
// dz = x.(theta^k - theta_stale).
// Logistic loss log(1 + exp(-y z)), y = +-1: the difference of the two sigmoids is formed
// without cancellation.  Quadratic error loss 0.5 (z - y)^2 (the linear-regression model of the
// paper's experiment, Sec. VI): r = z - y, and the difference of the residuals is dz itself.
__device__ __forceinline__ void residuals(bool quadratic, float z, float dz, float y, float& r, float& dr,
                                          float& loss)
{
    if (quadratic) {
        r = z - y;
        dr = dz;
        loss = 0.5f * r * r;
        return;
    }
    const float a = -y * z;
    const float sa = sigmoidf_(a);
    r = -y * sa;
    const float t = y * dz;              // (-y z~) - (-y z)
    const float b = a + t;
    float dsig;                          // sigma(a) - sigma(b)
    const bool small = fabsf(t) < 0.5f;
    const float sb = sigmoidf_(small ? -b : b);
    if (small)
        dsig = -sa * sb * expm1_small(t);
    else
        dsig = sa - sb;
    dr = -y * dsig;
    loss = fmaxf(a, 0.0f) + log1p_unit(exp_nonpos(-fabsf(a)));
}

}  // namespace gcada
