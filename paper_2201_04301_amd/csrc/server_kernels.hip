// Server side of the iteration: selection (a2), masked innovation sum (a3), AMSGrad-style
// update and history (a4).  Paper: Eq. (9) and Algorithm 1 for the rule and the ages, Sec. IV
// for the aggregate, Eq. (8a)-(8c) for the update.
#include "gcada_internal.h"

namespace gcada {

namespace {

constexpr int kWave = 64;

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// Sum n doubles with a whole block in a fixed order (deterministic): thread t takes
// elements t, t+B, ...; then a tree over waves.  Result valid on thread 0.
template <int B>
__device__ double block_sum_strided(const double* __restrict__ v, int n, double* s_tmp)
{
    double a = 0;
    for (int i = threadIdx.x; i < n; i += B) a += v[i];
    a = wave_sum(a);
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    __syncthreads();
    if (lane == 0) s_tmp[wave] = a;
    __syncthreads();
    double t = 0;
    if (threadIdx.x == 0)
        for (int w = 0; w < B / kWave; ++w) t += s_tmp[w];
    return t;
}

constexpr int kSelBlock = 256;

// One block.  stat_g <- sum of its partials; rhs <- (c/D) * sum of the history ring;
// mask_g <- stat_g > rhs  or  tau_g >= D  or  rhs == 0;  ages updated;  loss assembled.
__global__ __launch_bounds__(kSelBlock) void select_kernel(
    Hyper hy, const double* __restrict__ part_stat, int n_stat, const double* __restrict__ part_loss,
    int n_loss_total, const double* __restrict__ nring, int32_t* __restrict__ tau,
    double* __restrict__ stat, uint8_t* __restrict__ mask, Ctl* __restrict__ ctl,
    uint8_t* __restrict__ mask_out, float* __restrict__ loss_out)
{
    __shared__ double s_tmp[kSelBlock / kWave];
    __shared__ double s_rhs;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;

    if (threadIdx.x == 0) {
        double hsum = 0;
        for (int j = 0; j < hy.D; ++j) hsum += nring[j];
        s_rhs = hy.c / (double)hy.D * hsum;
    }
    const double lsum = block_sum_strided<kSelBlock>(part_loss, n_loss_total, s_tmp);
    __syncthreads();
    const double rhs = s_rhs;
    if (threadIdx.x == 0) {
        const double loss =
            lsum / ((double)hy.G * (double)hy.mu) + 0.5 * (double)hy.l2 * ctl->theta_sq;
        ctl->rhs = rhs;
        ctl->loss = loss;
        if (loss_out) *loss_out = (float)loss;
    }
    // one wave per group, groups dealt round-robin to the waves
    for (int g = wave; g < hy.G; g += kSelBlock / kWave) {
        double a = 0;
        const double* v = part_stat + (int64_t)g * n_stat;
        for (int i = lane; i < n_stat; i += kWave) a += v[i];
        a = wave_sum(a);
        if (lane == 0) {
            const int t = tau[g];
            const bool sel = (a > rhs) || (t >= hy.D) || (rhs == 0.0);
            stat[g] = a;
            mask[g] = sel ? 1 : 0;
            if (mask_out) mask_out[g] = sel ? 1 : 0;
            tau[g] = sel ? 1 : t + 1;
        }
    }
}

constexpr int kUpdBlock = 256;

template <int VW>
__device__ __forceinline__ void load_vec(const float* __restrict__ p, float (&v)[VW])
{
    if constexpr (VW == 4) {
        const float4 t = *(const float4*)p;
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
        v[0] = *p;
    }
}

template <int VW>
__device__ __forceinline__ void store_vec(float* __restrict__ p, const float (&v)[VW])
{
    if constexpr (VW == 4) {
        *(float4*)p = make_float4(v[0], v[1], v[2], v[3]);
    } else {
        *p = v[0];
    }
}

// grid: ceil(p / (256*VW)) blocks.  Thread owns VW consecutive parameters.
//   agg  += sum over selected g (ascending) of grad_g - last_g;  last_g <- grad_g
//   h, vhat, theta^{k+1} by Eq. (8a)-(8c);  theta^{k+1} goes to ring slot (k+1) mod (D+1)
//   per-block partials of ||alpha h / sqrt(eps+vhat)||^2 and ||theta^{k+1}||^2;
//   the block that finishes last adds them up in a fixed order, stores the history entry at
//   index k mod D and advances k.
template <int VW>
__global__ __launch_bounds__(kUpdBlock) void server_update_kernel(
    Hyper hy, const uint8_t* __restrict__ mask, const float* __restrict__ grad,
    float* __restrict__ last, float* __restrict__ agg, float* __restrict__ h,
    float* __restrict__ vhat, float* __restrict__ ring, double* __restrict__ nring,
    double* part_sq, Ctl* ctl)
{
    __shared__ double s_a[kUpdBlock / kWave], s_b[kUpdBlock / kWave];
    __shared__ bool s_last;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const long long k = ctl->k;
    const int nslot = hy.D + 1;
    const float* __restrict__ th = ring + (int64_t)(k % nslot) * hy.pstride;
    float* __restrict__ tn = ring + (int64_t)((k + 1) % nslot) * hy.pstride;
    const float b1 = (float)hy.beta1, b2 = (float)hy.beta2, al = (float)hy.alpha,
                ep = (float)hy.eps;
    const float ob1 = (float)(1.0 - hy.beta1), ob2 = (float)(1.0 - hy.beta2);

    const int64_t j0 = ((int64_t)blockIdx.x * kUpdBlock + threadIdx.x) * VW;
    double sq = 0, tsq = 0;
    if (j0 < hy.p) {
        float a[VW], hv[VW], vv[VW], tv[VW], nv[VW];
        load_vec<VW>(agg + j0, a);
        for (int g = 0; g < hy.G; ++g) {
            if (!mask[g]) continue;
            const int64_t o = (int64_t)g * hy.p + j0;
            float gg[VW], ll[VW];
            load_vec<VW>(grad + o, gg);
            load_vec<VW>(last + o, ll);
#pragma unroll
            for (int q = 0; q < VW; ++q) a[q] += gg[q] - ll[q];
            store_vec<VW>(last + o, gg);
        }
        load_vec<VW>(h + j0, hv);
        load_vec<VW>(vhat + j0, vv);
        load_vec<VW>(th + j0, tv);
#pragma unroll
        for (int q = 0; q < VW; ++q) {
            hv[q] = b1 * hv[q] + ob1 * a[q];
            const float v = b2 * vv[q] + ob2 * a[q] * a[q];
            vv[q] = fmaxf(vv[q], v);
            const float step = al * hv[q] / sqrtf(ep + vv[q]);
            nv[q] = tv[q] - step;
            sq += (double)step * (double)step;
            tsq += (double)nv[q] * (double)nv[q];
        }
        store_vec<VW>(agg + j0, a);
        store_vec<VW>(h + j0, hv);
        store_vec<VW>(vhat + j0, vv);
        store_vec<VW>(tn + j0, nv);
    }
    sq = wave_sum(sq);
    tsq = wave_sum(tsq);
    if (lane == 0) { s_a[wave] = sq; s_b[wave] = tsq; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double x = 0, y = 0;
        for (int w = 0; w < kUpdBlock / kWave; ++w) { x += s_a[w]; y += s_b[w]; }
        part_sq[2 * (int64_t)blockIdx.x] = x;
        part_sq[2 * (int64_t)blockIdx.x + 1] = y;
        __threadfence();                                    // publish the partials device-wide
        const unsigned int done = atomicAdd(&ctl->cnt_b, 1u);
        s_last = (done == gridDim.x - 1);
    }
    __syncthreads();
    if (s_last) {
        __threadfence();                                    // see every block's partials
        double x = 0, y = 0;
        for (int i = threadIdx.x; i < (int)gridDim.x; i += kUpdBlock) {
            x += part_sq[2 * (int64_t)i];
            y += part_sq[2 * (int64_t)i + 1];
        }
        x = wave_sum(x);
        y = wave_sum(y);
        __syncthreads();
        if (lane == 0) { s_a[wave] = x; s_b[wave] = y; }
        __syncthreads();
        if (threadIdx.x == 0) {
            double xs = 0, ys = 0;
            for (int w = 0; w < kUpdBlock / kWave; ++w) { xs += s_a[w]; ys += s_b[w]; }
            nring[k % hy.D] = xs;
            ctl->theta_sq = ys;
            ctl->k = k + 1;
            ctl->cnt_b = 0;
        }
    }
}

// ||theta^k||^2 of the current slot (one block).
__global__ __launch_bounds__(256) void theta_sq_kernel(Hyper hy, const float* __restrict__ ring,
                                                        Ctl* __restrict__ ctl)
{
    __shared__ double s_tmp[256 / kWave];
    const float* th = ring + (int64_t)(ctl->k % (hy.D + 1)) * hy.pstride;
    double a = 0;
    for (int64_t i = threadIdx.x; i < hy.p; i += 256) a += (double)th[i] * (double)th[i];
    a = wave_sum(a);
    if (threadIdx.x % kWave == 0) s_tmp[threadIdx.x / kWave] = a;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0;
        for (int w = 0; w < 256 / kWave; ++w) t += s_tmp[w];
        ctl->theta_sq = t;
    }
}

}  // namespace

hipError_t select_plan(gcada_ctx* c)
{
    const int64_t per_block = kUpdBlock * 4;
    c->n_epi_blocks = (int32_t)((c->hy.p + per_block - 1) / per_block);
    // the scalar update path (p % 4 != 0) needs 4x the blocks
    if (c->hy.p % 4) c->n_epi_blocks = (int32_t)((c->hy.p + kUpdBlock - 1) / kUpdBlock);
    return hipSuccess;
}

hipError_t select_groups(gcada_ctx* c, uint8_t* mask_out, float* loss_out, hipStream_t s)
{
    select_kernel<<<1, kSelBlock, 0, s>>>(c->hy, c->part_stat, c->n_stat_used, c->part_loss,
                                          c->n_loss_part * c->hy.G, c->nring, c->tau, c->stat,
                                          c->mask, c->ctl, mask_out, loss_out);
    return hipGetLastError();
}

hipError_t server_update(gcada_ctx* c, hipStream_t s)
{
    if (c->hy.p % 4 == 0)
        server_update_kernel<4><<<c->n_epi_blocks, kUpdBlock, 0, s>>>(
            c->hy, c->mask, c->grad, c->last, c->agg, c->h, c->vhat, c->ring, c->nring,
            c->part_sq, c->ctl);
    else
        server_update_kernel<1><<<c->n_epi_blocks, kUpdBlock, 0, s>>>(
            c->hy, c->mask, c->grad, c->last, c->agg, c->h, c->vhat, c->ring, c->nring,
            c->part_sq, c->ctl);
    return hipGetLastError();
}

hipError_t refresh_theta_sq(gcada_ctx* c, hipStream_t s)
{
    theta_sq_kernel<<<1, 256, 0, s>>>(c->hy, c->ring, c->ctl);
    return hipGetLastError();
}

}  // namespace gcada
