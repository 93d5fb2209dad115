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

// v[0..N) per lane -> every lane l ends with the sum over all 64 lanes of v[l >> (6 - log2 N)].
// Each of the log2(N) halving steps exchanges half of the remaining values with lane ^ S.
template <int N, int S>
struct Butterfly {
    static __device__ __forceinline__ void run(float (&v)[N], int lane)
    {
        if constexpr (S >= 1) {
            if constexpr (N > 1) {
                const bool up = (lane & S) != 0;
                float w[N / 2];
#pragma unroll
                for (int i = 0; i < N / 2; ++i) {
                    const float send = up ? v[i] : v[i + N / 2];
                    const float keep = up ? v[i + N / 2] : v[i];
                    w[i] = keep + __shfl_xor(send, S, kWave);
                }
                Butterfly<N / 2, S / 2>::run(w, lane);
                v[0] = w[0];
            } else {
                v[0] += __shfl_xor(v[0], S, kWave);
                Butterfly<1, S / 2>::run(v, lane);
            }
        }
    }
};

__device__ __forceinline__ float sigmoidf_(float t)
{
    const float e = expf(-fabsf(t));
    const float s = 1.0f / (1.0f + e);
    return t >= 0 ? s : e * s;
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
    if (fabsf(t) < 0.5f)
        dsig = -sa * sigmoidf_(-b) * expm1f(t);
    else
        dsig = sa - sigmoidf_(b);
    dr = -y * dsig;
    loss = fmaxf(a, 0.0f) + log1pf(expf(-fabsf(a)));
}

}  // namespace gcada
