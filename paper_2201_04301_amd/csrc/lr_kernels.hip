// Logistic-regression gradients at two iterates on the same minibatch (step a1 of the
// iteration; minibatch gradient = gradient of the sum of per-sample losses, paper Sec. II-A).
//
// For group g with minibatch rows x_i, labels y_i in {-1,+1}:
//   z_i  = x_i . theta^k            dz_i = x_i . (theta^k - theta_stale_g)
//   r_i  = -y_i sigmoid(-y_i z_i)   (residual at theta^k)
//   dr_i = r_i - r~_i               (difference to the residual at theta_stale_g, computed
//                                    from dz_i without cancellation)
//   grad_g = sum_i r_i x_i + mu*l2*theta^k
//   s_g    = sum_i dr_i x_i + mu*l2*(theta^k - theta_stale_g)     stat_g = ||s_g||^2
// The forward kernel streams the rows once for the two dot products, the backward kernel
// streams them again (column slabs) for the two weighted row sums.
#include "lr_device.h"

namespace gcada {

namespace {

// Row id of sample i of group g at iteration k.
__device__ __forceinline__ int64_t row_of(const int32_t* idx, int g, int i, int mu, long long k,
                                          int64_t rows)
{
    if (idx) return (int64_t)idx[(int64_t)g * mu + i];
    return (int64_t)(((unsigned long long)k * (unsigned long long)mu + (unsigned long long)i) %
                     (unsigned long long)rows);
}

constexpr int kFwdWaves = 4;   // waves per block
constexpr int kFwdRows = 4;    // rows per wave

// grid: (blocks_per_group, G); block: kFwdWaves * 64
template <bool VEC>
__global__ __launch_bounds__(kFwdWaves* kWave) void lr_forward(
    const ShardDesc* __restrict__ shards, const int32_t* __restrict__ idx,
    const float* __restrict__ ring, const int32_t* __restrict__ tau, const Ctl* __restrict__ ctl,
    Hyper hy, float* __restrict__ res, double* __restrict__ part_loss)
{
    const int g = blockIdx.y;
    if (hy.sel && !hy.sel[g]) {                  // unselected group: no gradient, no loss
        if (threadIdx.x == 0) part_loss[(int64_t)g * gridDim.x + blockIdx.x] = 0;
        return;
    }
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int d = (int)hy.p, mu = hy.mu;
    const long long k = hy.k;
    const int cur = hy.cur;
    const int old = stale_slot_of(hy, tau[g]);
    const float* __restrict__ th = ring + (int64_t)cur * hy.pstride;
    const float* __restrict__ ts = ring + (int64_t)old * hy.pstride;
    const ShardDesc sh = shards[g];
    const float* __restrict__ X = (const float*)sh.X;
    const float* __restrict__ Y = (const float*)sh.y;

    const int i0 = (blockIdx.x * kFwdWaves + wave) * kFwdRows;
    const float* xr[kFwdRows];
    float yv[kFwdRows];
    bool ok[kFwdRows];
#pragma unroll
    for (int r = 0; r < kFwdRows; ++r) {
        ok[r] = i0 + r < mu;
        const int64_t row = ok[r] ? row_of(idx, g, i0 + r, mu, k, sh.rows) : 0;
        xr[r] = X + row * sh.ld;
        yv[r] = ok[r] ? global_load(Y + row) : 1.0f;
    }
    float z[kFwdRows] = {}, dz[kFwdRows] = {};
    if (VEC) {
        for (int j = lane * 4; j < d; j += kWave * 4) {
            const float4 t = *(const float4*)(th + j);
            const float4 u = *(const float4*)(ts + j);
            const float4 dl = make_float4(t.x - u.x, t.y - u.y, t.z - u.z, t.w - u.w);
#pragma unroll
            for (int r = 0; r < kFwdRows; ++r) {
                if (!ok[r]) continue;
                const float4 x = global_load4(xr[r] + j);
                z[r] += x.x * t.x + x.y * t.y + x.z * t.z + x.w * t.w;
                dz[r] += x.x * dl.x + x.y * dl.y + x.z * dl.z + x.w * dl.w;
            }
        }
    } else {
        for (int j = lane; j < d; j += kWave) {
            const float t = th[j], dl = t - ts[j];
#pragma unroll
            for (int r = 0; r < kFwdRows; ++r) {
                if (!ok[r]) continue;
                const float x = global_load(xr[r] + j);
                z[r] += x * t;
                dz[r] += x * dl;
            }
        }
    }
    double lsum = 0;
#pragma unroll
    for (int r = 0; r < kFwdRows; ++r) {
        const float zz = wave_sum(z[r]), dd = wave_sum(dz[r]);
        if (ok[r] && lane == 0) {
            float rr, dr, ls;
            residuals(hy.quadratic != 0, zz, dd, yv[r], rr, dr, ls);
            float2* out = (float2*)res + ((int64_t)g * mu + i0 + r);
            *out = make_float2(rr, dr);
            lsum += (double)ls;
        }
    }
    __shared__ double sl[kFwdWaves];
    if (lane == 0) sl[wave] = lsum;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0;
        for (int w = 0; w < kFwdWaves; ++w) t += sl[w];
        part_loss[(int64_t)g * gridDim.x + blockIdx.x] = t;
    }
}

constexpr int kBwdWaves = 8;          // waves per block, rows are dealt round-robin to waves
constexpr int kBwdCols = kWave * 4;   // columns per block (VEC) -- one float4 per lane

// grid: (column slabs, G); block: kBwdWaves * 64; dynamic LDS: mu float2 (residual pairs)
template <bool VEC>
__global__ __launch_bounds__(kBwdWaves* kWave) void lr_backward(
    const ShardDesc* __restrict__ shards, const int32_t* __restrict__ idx,
    const float* __restrict__ ring, const int32_t* __restrict__ tau, const Ctl* __restrict__ ctl,
    Hyper hy, const float* __restrict__ res, float* __restrict__ gbuf, const int32_t* __restrict__ which,
    double* __restrict__ part_stat)
{
    extern __shared__ float2 s_res[];                       // mu entries
    __shared__ float4 s_acc[2][kBwdWaves][kWave];           // cross-wave reduction

    const int g = blockIdx.y;
    if (hy.sel && !hy.sel[g]) return;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int d = (int)hy.p, mu = hy.mu;
    const long long k = hy.k;
    const ShardDesc sh = shards[g];
    const float* __restrict__ X = (const float*)sh.X;

    for (int i = threadIdx.x; i < mu; i += blockDim.x)
        s_res[i] = ((const float2*)res)[(int64_t)g * mu + i];
    __syncthreads();

    constexpr int CW = VEC ? 4 : 1;                          // columns per lane
    const int j = blockIdx.x * (kWave * CW) + lane * CW;
    float4 ag = make_float4(0, 0, 0, 0), as = make_float4(0, 0, 0, 0);
    if (j < d) {
        int i = wave;
        // four rows in flight per wave
        for (; i + 3 * kBwdWaves < mu; i += 4 * kBwdWaves) {
            float4 x[4];
            float2 w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int ii = i + u * kBwdWaves;
                const int64_t row = row_of(idx, g, ii, mu, k, sh.rows);
                if (VEC) x[u] = global_load4(X + row * sh.ld + j);
                else x[u] = make_float4(global_load(X + row * sh.ld + j), 0, 0, 0);
                w[u] = s_res[ii];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                ag.x += w[u].x * x[u].x; ag.y += w[u].x * x[u].y;
                ag.z += w[u].x * x[u].z; ag.w += w[u].x * x[u].w;
                as.x += w[u].y * x[u].x; as.y += w[u].y * x[u].y;
                as.z += w[u].y * x[u].z; as.w += w[u].y * x[u].w;
            }
        }
        for (; i < mu; i += kBwdWaves) {
            const int64_t row = row_of(idx, g, i, mu, k, sh.rows);
            float4 x;
            if (VEC) x = global_load4(X + row * sh.ld + j);
            else x = make_float4(global_load(X + row * sh.ld + j), 0, 0, 0);
            const float2 w = s_res[i];
            ag.x += w.x * x.x; ag.y += w.x * x.y; ag.z += w.x * x.z; ag.w += w.x * x.w;
            as.x += w.y * x.x; as.y += w.y * x.y; as.z += w.y * x.z; as.w += w.y * x.w;
        }
    }
    s_acc[0][wave][lane] = ag;
    s_acc[1][wave][lane] = as;
    __syncthreads();
    double sq = 0;
    if (wave == 0) {
        if (j < d) {
            float4 tg = s_acc[0][0][lane], tsn = s_acc[1][0][lane];
            for (int w = 1; w < kBwdWaves; ++w) {
                const float4 a = s_acc[0][w][lane], b = s_acc[1][w][lane];
                tg.x += a.x; tg.y += a.y; tg.z += a.z; tg.w += a.w;
                tsn.x += b.x; tsn.y += b.y; tsn.z += b.z; tsn.w += b.w;
            }
            const int cur = hy.cur;
            const int old = stale_slot_of(hy, tau[g]);
            const float* th = ring + (int64_t)cur * hy.pstride;
            const float* ts = ring + (int64_t)old * hy.pstride;
            const float ml = (float)mu * hy.l2;
            float gv[4] = {tg.x, tg.y, tg.z, tg.w}, sv[4] = {tsn.x, tsn.y, tsn.z, tsn.w};
#pragma unroll
            for (int q = 0; q < CW; ++q) {
                if (j + q < d) {
                    if (hy.l2 != 0.0f) {
                        const float t = th[j + q];
                        gv[q] += ml * t;
                        sv[q] += ml * (t - ts[j + q]);
                    }
                    fresh_row(gbuf, which, hy, g)[j + q] = gv[q];
                    sq += (double)sv[q] * (double)sv[q];
                }
            }
        }
        sq = wave_sum(sq);
        if (lane == 0) part_stat[(int64_t)g * gridDim.x + blockIdx.x] = sq;
    }
}

}  // namespace

hipError_t lr_plan(gcada_ctx* c)
{
    const int mu = c->hy.mu;
    const int d = (int)c->hy.p;
    c->n_loss_part_lr = (mu + kFwdWaves * kFwdRows - 1) / (kFwdWaves * kFwdRows);   // per group
    c->n_loss_part = c->n_loss_part_lr;
    c->n_stat_part = (d + kWave - 1) / kWave;        // per group, worst case (scalar path)
    hipError_t e;
    if ((e = hipMalloc(&c->res, sizeof(float) * 2 * (size_t)c->hy.G * mu)) != hipSuccess) return e;
    return hipSuccess;
}

static bool lr_vec_ok(const gcada_ctx* c)
{
    if (c->hy.p % 4) return false;
    for (const auto& s : c->shards)
        if ((s.ld % 4) || ((uintptr_t)s.X % 16)) return false;
    return true;
}

hipError_t lr_gradients(gcada_ctx* c, const int32_t* idx, hipStream_t s)
{
    if (lr_tile_applies(c)) return lr_tile_gradients(c, idx, s);
    if (lr_team_applies(c)) return lr_team_gradients(c, idx, s);
    c->n_loss_used = c->n_loss_part_lr * c->hy.G;
    const Hyper& hy = c->hy;
    const bool vec = lr_vec_ok(c);
    const int d = (int)hy.p;
    dim3 gf(c->n_loss_part_lr, hy.G), bf(kFwdWaves * kWave);
    if (vec) {
        lr_forward<true><<<gf, bf, 0, s>>>(c->d_shards, idx, c->ring, c->tau, c->ctl, hy, c->res,
                                            c->part_loss);
        c->n_stat_used = (d + kBwdCols - 1) / kBwdCols;
        dim3 gb(c->n_stat_used, hy.G), bb(kBwdWaves * kWave);
        lr_backward<true><<<gb, bb, sizeof(float2) * hy.mu, s>>>(
            c->d_shards, idx, c->ring, c->tau, c->ctl, hy, c->res, c->gbuf, c->which, c->part_stat);
    } else {
        lr_forward<false><<<gf, bf, 0, s>>>(c->d_shards, idx, c->ring, c->tau, c->ctl, hy, c->res,
                                             c->part_loss);
        c->n_stat_used = (d + kWave - 1) / kWave;
        dim3 gb(c->n_stat_used, hy.G), bb(kBwdWaves * kWave);
        lr_backward<false><<<gb, bb, sizeof(float2) * hy.mu, s>>>(
            c->d_shards, idx, c->ring, c->tau, c->ctl, hy, c->res, c->gbuf, c->which, c->part_stat);
    }
    return hipGetLastError();
}

}  // namespace gcada
