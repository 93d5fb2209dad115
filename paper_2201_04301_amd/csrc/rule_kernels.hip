// The selection rule as the paper states it for the parameter server (Sec. IV, the condition
// with L_g; Algorithm 1): group g is selected when
//     L_g^2 ||theta^k - theta^{k - tau_g}||^2  >  (c/D) sum_{d<=D} ||theta^{k+1-d} - theta^{k-d}||^2
// or its age has reached D.  The decision needs no gradient, so it is taken BEFORE the gradient
// stage, and only the selected groups evaluate a gradient -- one, at theta^k.
// Also here: the smoothness constants L_g of the linear models by power iteration on the shard.
#include "gcada_internal.h"

namespace gcada {

namespace {

constexpr int kWave = 64;
constexpr int kBlock = 256;

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// block sum in a fixed order; result valid on thread 0
__device__ __forceinline__ double block_sum(double a, double* s_tmp)
{
    a = wave_sum(a);
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    __syncthreads();
    if (lane == 0) s_tmp[wave] = a;
    __syncthreads();
    double t = 0;
    if (threadIdx.x == 0)
        for (int w = 0; w < kBlock / kWave; ++w) t += s_tmp[w];
    return t;
}

// One block: distances, threshold, left sides, mask.  stat <- the left sides.
__device__ __forceinline__ void rule_select_block(
    const Hyper& hy, const double* __restrict__ part_dist, int nb, const double* __restrict__ L,
    const double* __restrict__ nring, const int32_t* __restrict__ tau, double* __restrict__ stat,
    uint8_t* __restrict__ mask, Ctl* __restrict__ ctl, uint8_t* __restrict__ mask_out,
    unsigned long long present)
{
    __shared__ double s_dist[64];            // D <= 64 is checked on the host
    __shared__ double s_rhs;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    for (int t = wave; t < hy.D; t += kBlock / kWave) {
        double a = 0;
        if ((present >> t) & 1ull)           // (an age no group has: nobody computed its distance)
            for (int i = lane; i < nb; i += kWave) a += part_dist[(int64_t)t * nb + i];
        a = wave_sum(a);
        if (lane == 0) s_dist[t] = a;
    }
    if (wave == 0) {
        double v = 0;
        for (int j = lane; j < hy.D; j += kWave) v += nring[j];
        v = wave_sum(v);
        if (lane == 0) s_rhs = hy.c / (double)hy.D * v;
    }
    __syncthreads();
    const double rhs = s_rhs;
    for (int g = threadIdx.x; g < hy.G; g += kBlock) {
        const int t = tau[g];                                   // 1 <= t <= D
        const double lhs = L[g] * L[g] * s_dist[t - 1];
        const bool sel = (lhs > rhs) || (t >= hy.D) || (rhs == 0.0);
        stat[g] = lhs;
        mask[g] = sel ? 1 : 0;
        if (mask_out) mask_out[g] = sel ? 1 : 0;
    }
    if (threadIdx.x == 0) ctl->rhs = rhs;
}

// Partial squared distances of theta^k to the older iterates of the ring that some group's age
// points at (groups that uploaded together share their age: often a few of the D distances are
// needed, and each costs a pass over two iterates), and -- by the block that finishes last -- the
// selection.
// grid: (nb, D); part[t][b] = sum over the block's slab of (theta^k - theta^{k-1-t})^2.
__global__ __launch_bounds__(kBlock) void rule_dist_select_kernel(
    Hyper hy, const float* __restrict__ ring, double* __restrict__ part, const double* __restrict__ L,
    const double* __restrict__ nring, const int32_t* __restrict__ tau, double* __restrict__ stat,
    uint8_t* __restrict__ mask, Ctl* __restrict__ ctl, uint8_t* __restrict__ mask_out)
{
    __shared__ double s_tmp[kBlock / kWave];
    __shared__ bool s_last;
    __shared__ unsigned long long s_present;
    const int t = blockIdx.y + 1;                               // age
    // the ages in use, bit age-1 (every block forms the same set)
    if (threadIdx.x == 0) s_present = 0;
    __syncthreads();
    {
        unsigned long long m = 0;
        for (int g = threadIdx.x; g < hy.G; g += kBlock) m |= 1ull << (tau[g] - 1);
        if (m) atomicOr(&s_present, m);
    }
    __syncthreads();
    const unsigned long long present = s_present;
    if (!((present >> (t - 1)) & 1ull)) return;
    int slot = hy.cur - t;
    if (slot < 0) slot += hy.D + 1;
    const float* a = ring + (int64_t)hy.cur * hy.pstride;
    const float* b = ring + (int64_t)slot * hy.pstride;
    double acc = 0;
    for (int64_t j = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * 4; j < hy.pstride;
         j += (int64_t)gridDim.x * kBlock * 4) {
        const float4 x = *(const float4*)(a + j), y = *(const float4*)(b + j);
        const double d0 = (double)x.x - (double)y.x, d1 = (double)x.y - (double)y.y;
        const double d2 = (double)x.z - (double)y.z, d3 = (double)x.w - (double)y.w;
        acc += d0 * d0 + d1 * d1 + d2 * d2 + d3 * d3;
    }
    const double tot = block_sum(acc, s_tmp);
    if (threadIdx.x == 0) {
        part[(int64_t)blockIdx.y * gridDim.x + blockIdx.x] = tot;
        __threadfence();                                        // publish the partial device-wide
        const unsigned total = gridDim.x * (unsigned)__popcll(present);
        s_last = atomicAdd(&ctl->cnt_a, 1u) == total - 1;
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();                                            // see every block's partial
    rule_select_block(hy, part, (int)gridDim.x, L, nring, tau, stat, mask, ctl, mask_out, present);
    if (threadIdx.x == 0) ctl->cnt_a = 0;
}

// One block, after the gradient stage: mean loss over the samples that were evaluated (the
// unselected groups left zero partials), 0 when no group was selected.
__global__ __launch_bounds__(kBlock) void rule_loss_kernel(Hyper hy, const double* __restrict__ part_loss,
                                                           int n_loss_total, const uint8_t* __restrict__ mask,
                                                           Ctl* __restrict__ ctl, float* __restrict__ loss_out)
{
    __shared__ double s_tmp[kBlock / kWave];
    double a = 0;
    for (int i = threadIdx.x; i < n_loss_total; i += kBlock) a += part_loss[i];
    const double lsum = block_sum(a, s_tmp);
    double n = 0;
    for (int g = threadIdx.x; g < hy.G; g += kBlock) n += mask[g] ? 1.0 : 0.0;
    const double nsel = block_sum(n, s_tmp);
    if (threadIdx.x == 0) {
        const double loss = nsel > 0 ? lsum / (nsel * (double)hy.mu) + 0.5 * (double)hy.l2 * ctl->theta_sq : 0.0;
        ctl->loss = loss;
        if (loss_out) *loss_out = (float)loss;
    }
}

// ---- power iteration on X^T X of one shard (linear models) ----------------------------------
// t_i = x_i . v for a chunk of rows: one wave per row.  grid: ceil(rows / 4), block 256.
__global__ __launch_bounds__(kBlock) void pi_forward_kernel(const float* __restrict__ X, int64_t rows, int64_t ld,
                                                            int d, const double* __restrict__ v,
                                                            double* __restrict__ t)
{
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int64_t i = (int64_t)blockIdx.x * (kBlock / kWave) + wave;
    if (i >= rows) return;
    const float* x = X + i * ld;
    double a = 0;
    for (int j = lane; j < d; j += kWave) a += (double)x[j] * v[j];
    a = wave_sum(a);
    if (lane == 0) t[i] = a;
}

// w_part[chunk][j] = sum over the chunk's rows of t_i X[i][j].  grid: (ceil(d / 256), chunks).
__global__ __launch_bounds__(kBlock) void pi_backward_kernel(const float* __restrict__ X, int64_t rows, int64_t ld,
                                                             int d, const double* __restrict__ t,
                                                             int64_t rows_per_chunk, double* __restrict__ w_part)
{
    const int j = blockIdx.x * kBlock + threadIdx.x;
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_chunk;
    const int64_t r1 = r0 + rows_per_chunk < rows ? r0 + rows_per_chunk : rows;
    if (j >= d) return;
    double a = 0;
    for (int64_t i = r0; i < r1; ++i) a += t[i] * (double)X[i * ld + j];
    w_part[(int64_t)blockIdx.y * d + j] = a;
}

// w = sum of the chunk partials (fixed order); partial ||w||^2 per block.  grid: ceil(d / 256).
__global__ __launch_bounds__(kBlock) void pi_reduce_kernel(const double* __restrict__ w_part, int chunks, int d,
                                                           double* __restrict__ w, double* __restrict__ part_sq)
{
    __shared__ double s_tmp[kBlock / kWave];
    const int j = blockIdx.x * kBlock + threadIdx.x;
    double a = 0;
    if (j < d) {
        for (int c = 0; c < chunks; ++c) a += w_part[(int64_t)c * d + j];
        w[j] = a;
    }
    const double sq = block_sum(a * a, s_tmp);
    if (threadIdx.x == 0) part_sq[blockIdx.x] = sq;
}

// One block: norm = sqrt(sum of the partials); v <- w / norm; norms[it] <- norm.
__global__ __launch_bounds__(kBlock) void pi_normalize_kernel(const double* __restrict__ w, const double* __restrict__ part_sq,
                                                              int nparts, int d, double* __restrict__ v,
                                                              double* __restrict__ norm_out)
{
    __shared__ double s_tmp[kBlock / kWave];
    __shared__ double s_norm;
    double a = 0;
    for (int i = threadIdx.x; i < nparts; i += kBlock) a += part_sq[i];
    const double tot = block_sum(a, s_tmp);
    if (threadIdx.x == 0) {
        s_norm = sqrt(tot);
        *norm_out = s_norm;
    }
    __syncthreads();
    const double inv = s_norm > 0 ? 1.0 / s_norm : 0.0;
    for (int j = threadIdx.x; j < d; j += kBlock) v[j] = w[j] * inv;
}

// Per-worker minibatches (Sec. IV, Algorithm 1): the minibatch of group g is that of its fastest
// worker, argmin_m T_m^k (ties: lowest m).  grid: G blocks; out[g][i] = idx_workers[g][m*][i].
__global__ __launch_bounds__(kBlock) void pick_fastest_kernel(int M_G, int mu, const int32_t* __restrict__ idx_workers,
                                                              const double* __restrict__ delays,
                                                              int32_t* __restrict__ out, int32_t* __restrict__ worker_out)
{
    const int g = blockIdx.x;
    int best = 0;
    double tb = delays[(int64_t)g * M_G];
    for (int m = 1; m < M_G; ++m) {
        const double t = delays[(int64_t)g * M_G + m];
        if (t < tb) { tb = t; best = m; }
    }
    const int32_t* src = idx_workers + ((int64_t)g * M_G + best) * mu;
    for (int i = threadIdx.x; i < mu; i += kBlock) out[(int64_t)g * mu + i] = src[i];
    if (worker_out && threadIdx.x == 0) worker_out[g] = best;
}

}  // namespace

hipError_t pick_fastest_workers(gcada_ctx* c, const int32_t* idx_workers, const double* delays,
                                int32_t* worker_out, hipStream_t s)
{
    pick_fastest_kernel<<<c->hy.G, kBlock, 0, s>>>(c->M_G, c->hy.mu, idx_workers, delays, c->idx_eff, worker_out);
    return hipGetLastError();
}

// Selection under the server-side rule; enqueued before the gradient stage.
hipError_t rule_select(gcada_ctx* c, uint8_t* mask_out, hipStream_t s)
{
    const int nb = c->rule_nb;
    rule_dist_select_kernel<<<dim3(nb, c->hy.D), kBlock, 0, s>>>(c->hy, c->ring, c->rule_part, c->rule_L, c->nring,
                                                                 c->tau, c->stat, c->mask, c->ctl, mask_out);
    return hipGetLastError();
}

hipError_t rule_loss(gcada_ctx* c, float* loss_out, hipStream_t s)
{
    rule_loss_kernel<<<1, kBlock, 0, s>>>(c->hy, c->part_loss, c->n_loss_used, c->mask, c->ctl, loss_out);
    return hipGetLastError();
}

hipError_t rule_plan(gcada_ctx* c)
{
    // (the server-side rule itself is limited to D <= 64 -- one bit per age, checked by
    // gcada_set_rule; the buffers below are needed by every context)
    hipError_t es = rule_static_scratch(&c->static_scratch);
    if (es != hipSuccess) return es;
    const int64_t per_block = (int64_t)kBlock * 4;
    // (every block ends with an atomic on one counter: a few hundred blocks per distance, not thousands)
    c->rule_nb = (int)std::min<int64_t>((c->hy.pstride + per_block - 1) / per_block, 256);
    hipError_t e;
    if ((e = hipMalloc(&c->rule_part, sizeof(double) * (size_t)c->rule_nb * c->hy.D)) != hipSuccess) return e;
    if ((e = hipMalloc(&c->rule_L, sizeof(double) * (size_t)c->hy.G)) != hipSuccess) return e;
    if ((e = hipMalloc(&c->idx_eff, sizeof(int32_t) * (size_t)c->hy.G * c->hy.mu)) != hipSuccess) return e;
    return hipMemset(c->rule_L, 0, sizeof(double) * (size_t)c->hy.G);
}

void rule_free(gcada_ctx* c)
{
    if (c->rule_part) (void)hipFree(c->rule_part);
    if (c->rule_L) (void)hipFree(c->rule_L);
    if (c->idx_eff) (void)hipFree(c->idx_eff);
    c->idx_eff = nullptr;
    c->rule_part = nullptr;
    c->rule_L = nullptr;
}

// ---- scratch of one power iteration --------------------------------------------------------
// v, w: d doubles; t: rows doubles; wp: chunks x d; psq: one per 256 columns; norm: 1.
struct PiLayout {
    int d, chunks, nbd;
    int64_t rows, rpc;
    size_t off_v, off_t, off_w, off_wp, off_psq, off_norm, total;    // in doubles
};

static PiLayout pi_layout(const gcada_ctx* c, int g)
{
    PiLayout L{};
    const ShardDesc& sh = c->shards[g];
    L.d = (int)c->hy.p;
    L.rows = sh.rows;
    L.chunks = (int)std::min<int64_t>(256, (L.rows + 63) / 64);
    L.rpc = (L.rows + L.chunks - 1) / L.chunks;
    L.nbd = (L.d + kBlock - 1) / kBlock;
    auto up = [](size_t n) { return (n + 31) / 32 * 32; };          // 256-byte pieces
    size_t o = 0;
    L.off_v = o; o += up((size_t)L.d);
    L.off_t = o; o += up((size_t)L.rows);
    L.off_w = o; o += up((size_t)L.d);
    L.off_wp = o; o += up((size_t)L.chunks * L.d);
    L.off_psq = o; o += up((size_t)L.nbd);
    L.off_norm = o; o += 32;
    L.total = o;
    return L;
}

// The `iters` rounds of the power iteration on shard g, all in `base` (L.total doubles), start
// vector already in place; the last round leaves ||X^T X v|| in base[off_norm].
static hipError_t pi_rounds(const gcada_ctx* c, int g, int iters, const PiLayout& L, double* base, hipStream_t s)
{
    const ShardDesc& sh = c->shards[g];
    const float* X = (const float*)sh.X;
    double *v = base + L.off_v, *t = base + L.off_t, *w = base + L.off_w, *wp = base + L.off_wp;
    double *psq = base + L.off_psq, *norm = base + L.off_norm;
    for (int it = 0; it < iters; ++it) {
        pi_forward_kernel<<<(unsigned)((L.rows + 3) / 4), kBlock, 0, s>>>(X, L.rows, sh.ld, L.d, v, t);
        pi_backward_kernel<<<dim3(L.nbd, L.chunks), kBlock, 0, s>>>(X, L.rows, sh.ld, L.d, t, L.rpc, wp);
        pi_reduce_kernel<<<L.nbd, kBlock, 0, s>>>(wp, L.chunks, L.d, w, psq);
        pi_normalize_kernel<<<1, kBlock, 0, s>>>(w, psq, L.nbd, L.d, v, norm);
    }
    return hipGetLastError();
}

// Start vector of the power iteration: a fixed pattern with a component along every coordinate,
// of unit length.
static double pi_start_value(int j) { return 1.0 + 0.5 * ((j * 2654435761u >> 16) & 0xff) / 255.0; }

// Largest eigenvalue of X^T X of shard g by `iters` steps of power iteration from a fixed start
// vector.  Synchronises the stream.  lambda_out on the host.
hipError_t rule_power_iteration(gcada_ctx* c, int g, int iters, double* lambda_out, hipStream_t s)
{
    const PiLayout L = pi_layout(c, g);
    double* base = nullptr;
    hipError_t e = hipMalloc(&base, 8 * L.total);
    if (e != hipSuccess) return e;
    auto done = [&](hipError_t r) { (void)hipFree(base); return r; };
    std::vector<double> h0(L.d);
    double n2 = 0;
    for (int j = 0; j < L.d; ++j) { h0[j] = pi_start_value(j); n2 += h0[j] * h0[j]; }
    for (int j = 0; j < L.d; ++j) h0[j] /= std::sqrt(n2);
    if ((e = hipMemcpyAsync(base + L.off_v, h0.data(), 8 * (size_t)L.d, hipMemcpyHostToDevice, s)) != hipSuccess) return done(e);
    if ((e = pi_rounds(c, g, iters, L, base, s)) != hipSuccess) return done(e);
    double lam = 0;
    if ((e = hipMemcpyAsync(&lam, base + L.off_norm, 8, hipMemcpyDeviceToHost, s)) != hipSuccess) return done(e);
    if ((e = hipStreamSynchronize(s)) != hipSuccess) return done(e);
    *lambda_out = lam;                  // ||X^T X v|| with ||v|| = 1 converges to lambda_max
    return done(hipSuccess);
}

// ---- the same with no allocation at all ----------------------------------------------------
// Scratch of the power iteration in a static device array (every device the library runs on
// holds its own copy until the process ends).  In host code the array's NAME is not a device
// address; hipGetSymbolAddress gives the address of the current device's copy, and only that
// pointer is ever handed to a kernel.
constexpr size_t kStaticScratchDoubles = (size_t)2 << 20;            // 16 MiB
static __device__ __align__(256) double scratch[kStaticScratchDoubles];

constexpr int kMaxDevices = 64;
static double* g_scratch_ptr[kMaxDevices];                            // per device, resolved once

size_t rule_static_scratch_doubles() { return kStaticScratchDoubles; }

size_t rule_power_iteration_scratch_doubles(const gcada_ctx* c, int g) { return pi_layout(c, g).total; }

// Address of the current device's copy of the array (resolved at the first call on that device).
hipError_t rule_static_scratch(double** ptr)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[dev]) {
        double* p = nullptr;
        e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

// One thread: the start vector in the host routine's arithmetic (same operations in the same
// order, no fused multiply-adds), so both routes start from the same bits.
__global__ void pi_start_kernel(int d, double* __restrict__ v)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    double n2 = 0;
    for (int j = 0; j < d; ++j) {
        const double h = __dadd_rn(1.0, __ddiv_rn(__dmul_rn(0.5, (double)((j * 2654435761u >> 16) & 0xff)), 255.0));
        v[j] = h;
        n2 = __dadd_rn(n2, __dmul_rn(h, h));
    }
    const double nrm = __dsqrt_rn(n2);
    for (int j = 0; j < d; ++j) v[j] = __ddiv_rn(v[j], nrm);
}

// L_g = kappa * lambda / rows + l2, as the host routine forms it.
__global__ void pi_finish_kernel(const double* __restrict__ norm, double kappa, double rows, double l2,
                                 double* __restrict__ out)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) *out = __dadd_rn(__ddiv_rn(__dmul_rn(kappa, *norm), rows), l2);
}

// All groups' constants, one after the other in the static array, result written on the device in
// stream order.  No allocation, no synchronisation, no host copy.
hipError_t rule_smoothness_static(gcada_ctx* c, int iters, double* L_out_dev, hipStream_t s)
{
    double* base = c->static_scratch;
    if (!base) return hipErrorInvalidValue;
    const double kappa = c->dims.model == GCADA_LINREG ? 1.0 : 0.25;
    for (int g = 0; g < c->hy.G; ++g) {
        const PiLayout L = pi_layout(c, g);
        if (L.total > kStaticScratchDoubles) return hipErrorInvalidValue;      // (the caller has checked)
        pi_start_kernel<<<1, 64, 0, s>>>(L.d, base + L.off_v);
        hipError_t e = pi_rounds(c, g, iters, L, base, s);
        if (e != hipSuccess) return e;
        pi_finish_kernel<<<1, 64, 0, s>>>(base + L.off_norm, kappa, (double)c->shards[g].rows, (double)c->dims.l2,
                                          L_out_dev + g);
    }
    return hipGetLastError();
}

}  // namespace gcada
