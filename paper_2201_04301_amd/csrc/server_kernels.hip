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

// Selection (step a2) by one wave per group: stat_g <- sum of its partials (fixed order);
// mask_g <- stat_g > rhs  or  tau_g >= D  or  rhs == 0.
__device__ __forceinline__ void select_groups_block(const Hyper& hy, const double* __restrict__ part_stat,
                                                    int n_stat, const int32_t* __restrict__ tau,
                                                    double rhs, uint8_t* s_mask, double* stat_out,
                                                    uint8_t* mask_a, uint8_t* mask_b, int nwaves)
{
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    for (int g = wave; g < hy.G; g += nwaves) {
        double a = 0;
        const double* v = part_stat + (int64_t)g * n_stat;
        for (int i = lane; i < n_stat; i += kWave) a += v[i];
        a = wave_sum(a);
        if (lane == 0) {
            const bool sel = (a > rhs) || (tau[g] >= hy.D) || (rhs == 0.0);
            s_mask[g] = sel ? 1 : 0;
            if (stat_out) stat_out[g] = a;
            if (mask_a) mask_a[g] = sel ? 1 : 0;
            if (mask_b) mask_b[g] = sel ? 1 : 0;
        }
    }
}

// grid: G blocks.  Adds one group's partial statistics in a fixed order (thread-strided, then a
// tree) so that the server kernel finds a single number per group.
__global__ __launch_bounds__(kSelBlock) void stat_reduce_kernel(const double* __restrict__ part_stat,
                                                               int n_stat, double* __restrict__ out)
{
    __shared__ double s_tmp[kSelBlock / kWave];
    const double t = block_sum_strided<kSelBlock>(part_stat + (int64_t)blockIdx.x * n_stat, n_stat, s_tmp);
    if (threadIdx.x == 0) out[blockIdx.x] = t;
}

// One block, used when the partial statistics are too many for every update block to re-add.
// Writes stat, mask, rhs, loss and the caller's outputs; the ages are advanced by the update.
__global__ __launch_bounds__(kSelBlock) void select_kernel(
    Hyper hy, const double* __restrict__ part_stat, int n_stat, const double* __restrict__ part_loss,
    int n_loss_total, const double* __restrict__ nring, const int32_t* __restrict__ tau,
    double* __restrict__ stat, uint8_t* __restrict__ mask, Ctl* __restrict__ ctl,
    uint8_t* __restrict__ mask_out, float* __restrict__ loss_out)
{
    __shared__ double s_tmp[kSelBlock / kWave];
    __shared__ double s_rhs;
    extern __shared__ uint8_t s_mask[];
    // one partial per group (they were added up beforehand): a thread per group, its loads
    // issued before the threshold and the loss are formed
    const bool direct = n_stat == 1;
    double my_stat = 0;
    int my_tau = 0;
    if (direct && (int)threadIdx.x < hy.G) {
        my_stat = part_stat[threadIdx.x];
        my_tau = tau[threadIdx.x];
    }
    if (threadIdx.x < kWave) {
        const double r = history_threshold(hy, nring);
        if (threadIdx.x == 0) s_rhs = r;
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
    if (direct && hy.G <= kSelBlock) {
        if ((int)threadIdx.x < hy.G) {
            const int g = threadIdx.x;
            const bool sel = (my_stat > rhs) || (my_tau >= hy.D) || (rhs == 0.0);
            stat[g] = my_stat;
            mask[g] = sel ? 1 : 0;
            if (mask_out) mask_out[g] = sel ? 1 : 0;
        }
        return;
    }
    select_groups_block(hy, part_stat, n_stat, tau, rhs, s_mask, stat, mask, mask_out,
                        kSelBlock / kWave);
}

// Statistic sums and selection in one launch, one block per group (lazy gradient store): the
// group's partials are added in the order of stat_reduce_kernel, the threshold is formed by every
// block from the D history entries, block 0 also forms the loss.  Writes what select_kernel
// writes, for its group.
__global__ __launch_bounds__(kSelBlock) void stat_select_kernel(
    Hyper hy, const double* __restrict__ part_stat, int n_stat, const double* __restrict__ part_loss,
    int n_loss_total, const double* __restrict__ nring, const int32_t* __restrict__ tau,
    double* __restrict__ stat, uint8_t* __restrict__ mask, Ctl* __restrict__ ctl,
    uint8_t* __restrict__ mask_out, float* __restrict__ loss_out,
    const uint8_t* __restrict__ stored, uint8_t* __restrict__ redo, uint8_t* __restrict__ hot)
{
    __shared__ double s_tmp[kSelBlock / kWave];
    __shared__ double s_rhs;
    const int g = blockIdx.x;
    int my_tau = 0;
    uint8_t my_stored = 0;
    if (threadIdx.x == 0) { my_tau = tau[g]; my_stored = stored[g]; }
    if (threadIdx.x < kWave) {
        const double r = history_threshold(hy, nring);
        if (threadIdx.x == 0) s_rhs = r;
    }
    const double t = block_sum_strided<kSelBlock>(part_stat + (int64_t)g * n_stat, n_stat, s_tmp);
    double lsum = 0;
    if (g == 0) lsum = block_sum_strided<kSelBlock>(part_loss, n_loss_total, s_tmp);
    __syncthreads();
    if (threadIdx.x == 0) {
        const double rhs = s_rhs;
        const bool sel = (t > rhs) || (my_tau >= hy.D) || (rhs == 0.0);
        stat[g] = t;
        mask[g] = sel ? 1 : 0;
        if (mask_out) mask_out[g] = sel ? 1 : 0;
        redo[g] = sel && !my_stored ? 1 : 0;
        hot[g] = t > rhs ? 1 : 0;
        if (g == 0) {
            const double loss =
                lsum / ((double)hy.G * (double)hy.mu) + 0.5 * (double)hy.l2 * ctl->theta_sq;
            ctl->rhs = rhs;
            ctl->loss = loss;
            if (loss_out) *loss_out = (float)loss;
        }
    }
}

// The store flags of the lazy gradient store, on their own (after a change of state; a step
// sets the flags of the next one in its last launch).  One wave.
__global__ __launch_bounds__(kWave) void lazy_flags_kernel(Hyper hy, const double* __restrict__ nring,
                                                          const int32_t* __restrict__ tau,
                                                          const uint8_t* __restrict__ hot,
                                                          uint8_t* __restrict__ store_now)
{
    store_flags_wave(hy, nring, tau, hot, store_now);
}

constexpr int kUpdBlock = 1024;

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

// gradient rows are read once per step: streaming loads
template <int VW>
__device__ __forceinline__ void load_vec_stream(const float* __restrict__ p, float (&v)[VW])
{
    if constexpr (VW == 4) {
        const float4 t = global_load4_stream(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
        v[0] = __builtin_nontemporal_load(p);
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

struct ServerArgs {
    Hyper hy;
    const double* part_stat;   // SELECT: [G][n_stat]
    int n_stat;
    const double* part_loss;   // SELECT: n_loss_total entries
    int n_loss_total;
    double* stat;
    uint8_t* mask;             // written (SELECT) or read (!SELECT)
    uint8_t* mask_out;
    float* loss_out;
    const float* gbuf;         // 2 halves x G rows x pstride
    int32_t* which;            // G: half holding the last uploaded gradient (flipped on upload)
    float* agg;
    float* h;
    float* vhat;
    float* ring;
    double* nring;
    int32_t* tau;
    double* part_sq;
    Ctl* ctl;
};

// grid: ceil(p / (B*VW)) blocks of B threads.  Thread owns VW consecutive parameters.
//   SELECT: every block first derives the selection mask from the partial statistics (same
//           fixed order everywhere, so all blocks agree); block 0 publishes it with the loss.
//   a3: agg += sum over selected g (ascending) of grad_g - last_g;  last_g <- grad_g
//   a4: h, vhat, theta^{k+1} by Eq. (8a)-(8c);  theta^{k+1} goes to ring slot (k+1) mod (D+1)
//   per-block partials of ||alpha h / sqrt(eps+vhat)||^2 and ||theta^{k+1}||^2;
//   the block that finishes last (the only block, when the grid has one) adds them up in a
//   fixed order, stores the history entry at index k mod D and advances the ages (Algorithm 1).
// The kernel is a chain of dependent memory round trips, so every load that does not depend on
// the mask is issued at the top, and the loads of the selected groups go out four groups at a
// time.  dynamic LDS: G bytes (mask) + G ints (selected list) + G doubles (statistics).
template <int B, int VW, bool SELECT>
__global__ __launch_bounds__(B) void server_step_kernel(ServerArgs a)
{
    __shared__ double s_a[B / kWave], s_b[B / kWave];
    __shared__ double s_rhs;
    __shared__ int s_nsel;
    __shared__ bool s_last;
    extern __shared__ double s_dyn[];
    const Hyper& hy = a.hy;
    double* s_stat = s_dyn;                                   // G
    int* s_sel = (int*)(s_dyn + hy.G);                        // G
    int* s_which = s_sel + hy.G;                              // G
    uint8_t* s_mask = (uint8_t*)(s_which + hy.G);             // G
    Ctl* ctl = a.ctl;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    constexpr int NW = B / kWave;
    const float* __restrict__ th = a.ring + (int64_t)hy.cur * hy.pstride;
    float* __restrict__ tn = a.ring + (int64_t)hy.nxt * hy.pstride;

    // a block walks over slabs of B * VW parameters: blockIdx.x, blockIdx.x + gridDim.x, ...
    int64_t j0 = ((int64_t)blockIdx.x * B + threadIdx.x) * VW;
    const int64_t jstep = (int64_t)gridDim.x * B * VW;
    bool active = j0 < hy.pstride;            // pads stay zero: their step is alpha*0/sqrt(eps)
    float ac[VW] = {}, hv[VW] = {}, vv[VW] = {}, tv[VW] = {}, nv[VW];
    if (active) {
        load_vec<VW>(a.agg + j0, ac);
        load_vec<VW>(a.h + j0, hv);
        load_vec<VW>(a.vhat + j0, vv);
        load_vec<VW>(th + j0, tv);
    }
    const bool pub = SELECT && blockIdx.x == 0;
    int my_tau = 0;
    if ((int)threadIdx.x < hy.G) my_tau = a.tau[threadIdx.x];      // groups beyond B are read below
    for (int g = threadIdx.x; g < hy.G; g += B) s_which[g] = a.which[g];
    if constexpr (SELECT) {
        // statistics: one wave per group, partials added in lane-strided order then butterfly
        for (int g = wave; g < hy.G; g += NW) {
            double t = 0;
            const double* v = a.part_stat + (int64_t)g * a.n_stat;
            for (int i = lane; i < a.n_stat; i += kWave) t += v[i];
            t = wave_sum(t);
            if (lane == 0) s_stat[g] = t;
        }
        double lpart = 0;
        if (pub)
            for (int i = threadIdx.x; i < a.n_loss_total; i += B) lpart += a.part_loss[i];
        if (wave == 0) {
            const double r = history_threshold(hy, a.nring);
            if (lane == 0) s_rhs = r;
        }
        if (pub) {
            lpart = wave_sum(lpart);
            if (lane == 0) s_a[wave] = lpart;
        }
        __syncthreads();
        const double rhs = s_rhs;
        for (int g = threadIdx.x; g < hy.G; g += B) {
            const int t = g < B ? my_tau : a.tau[g];
            const double st = s_stat[g];
            const bool sel = (st > rhs) || (t >= hy.D) || (rhs == 0.0);
            s_mask[g] = sel ? 1 : 0;
            if (pub) {
                a.stat[g] = st;
                a.mask[g] = sel ? 1 : 0;
                if (a.mask_out) a.mask_out[g] = sel ? 1 : 0;
            }
        }
        if (pub && threadIdx.x == 0) {
            double lsum = 0;
            for (int w = 0; w < NW; ++w) lsum += s_a[w];
            const double loss =
                lsum / ((double)hy.G * (double)hy.mu) + 0.5 * (double)hy.l2 * ctl->theta_sq;
            ctl->rhs = rhs;
            ctl->loss = loss;
            if (a.loss_out) *a.loss_out = (float)loss;
        }
    } else {
        for (int g = threadIdx.x; g < hy.G; g += B) s_mask[g] = a.mask[g];
    }
    __syncthreads();
    // ascending list of the selected groups (wave 0, 64 groups per ballot)
    if (wave == 0) {
        int n = 0;
        for (int g0 = 0; g0 < hy.G; g0 += kWave) {
            const int g = g0 + lane;
            const bool sel = g < hy.G && s_mask[g];
            const unsigned long long bal = __ballot(sel);
            if (sel) s_sel[n + __popcll(bal & ((1ull << lane) - 1ull))] = g;
            n += __popcll(bal);
        }
        if (lane == 0) s_nsel = n;
    }
    __syncthreads();
    const int nsel = s_nsel;

    const float b1 = (float)hy.beta1, b2 = (float)hy.beta2, al = (float)hy.alpha,
                ep = (float)hy.eps;
    const float ob1 = (float)(1.0 - hy.beta1), ob2 = (float)(1.0 - hy.beta2);
    double sq = 0, tsq = 0;
    while (active) {
        // innovation of a selected group: its fresh row minus the row it uploaded last; nothing
        // is copied -- the finishing block flips which[g] instead
        int i = 0;
        for (; i + 4 <= nsel; i += 4) {              // four groups' loads in flight, added in order
            float gg[4][VW], ll[4][VW];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int g = s_sel[i + e], wl = s_which[g];
                load_vec_stream<VW>(a.gbuf + ((int64_t)(1 - wl) * hy.G + g) * hy.pstride + j0, gg[e]);
                load_vec_stream<VW>(a.gbuf + ((int64_t)wl * hy.G + g) * hy.pstride + j0, ll[e]);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int q = 0; q < VW; ++q) ac[q] += gg[e][q] - ll[e][q];
        }
        for (; i < nsel; ++i) {
            const int g = s_sel[i], wl = s_which[g];
            float gg[VW], ll[VW];
            load_vec_stream<VW>(a.gbuf + ((int64_t)(1 - wl) * hy.G + g) * hy.pstride + j0, gg);
            load_vec_stream<VW>(a.gbuf + ((int64_t)wl * hy.G + g) * hy.pstride + j0, ll);
#pragma unroll
            for (int q = 0; q < VW; ++q) ac[q] += gg[q] - ll[q];
        }
#pragma unroll
        for (int q = 0; q < VW; ++q) {
            // explicit fused multiply-adds: the rounding must not depend on how the compiler
            // contracts the expression in one instantiation of this kernel or another
            hv[q] = fmaf(b1, hv[q], ob1 * ac[q]);
            const float v = fmaf(b2, vv[q], ob2 * ac[q] * ac[q]);
            vv[q] = fmaxf(vv[q], v);
            const float step = al * hv[q] / sqrtf(ep + vv[q]);
            nv[q] = tv[q] - step;
            sq += (double)step * (double)step;
            tsq += (double)nv[q] * (double)nv[q];
        }
        store_vec<VW>(a.agg + j0, ac);
        store_vec<VW>(a.h + j0, hv);
        store_vec<VW>(a.vhat + j0, vv);
        store_vec<VW>(tn + j0, nv);
        j0 += jstep;
        active = j0 < hy.pstride;
        if (active) {
            load_vec<VW>(a.agg + j0, ac);
            load_vec<VW>(a.h + j0, hv);
            load_vec<VW>(a.vhat + j0, vv);
            load_vec<VW>(th + j0, tv);
        }
    }
    sq = wave_sum(sq);
    tsq = wave_sum(tsq);
    __syncthreads();
    if (lane == 0) { s_a[wave] = sq; s_b[wave] = tsq; }
    __syncthreads();
    double xs = 0, ys = 0;
    if (gridDim.x == 1) {
        if (threadIdx.x == 0)
            for (int w = 0; w < NW; ++w) { xs += s_a[w]; ys += s_b[w]; }
    } else {
        if (threadIdx.x == 0) {
            double x = 0, y = 0;
            for (int w = 0; w < NW; ++w) { x += s_a[w]; y += s_b[w]; }
            a.part_sq[2 * (int64_t)blockIdx.x] = x;
            a.part_sq[2 * (int64_t)blockIdx.x + 1] = y;
            __threadfence();                                // publish the partials device-wide
            const unsigned int done = atomicAdd(&ctl->cnt_b, 1u);
            s_last = (done == gridDim.x - 1);
        }
        __syncthreads();
        if (!s_last) return;
        __threadfence();                                    // see every block's partials
        double x = 0, y = 0;
        for (int i = threadIdx.x; i < (int)gridDim.x; i += B) {
            x += a.part_sq[2 * (int64_t)i];
            y += a.part_sq[2 * (int64_t)i + 1];
        }
        x = wave_sum(x);
        y = wave_sum(y);
        __syncthreads();
        if (lane == 0) { s_a[wave] = x; s_b[wave] = y; }
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int w = 0; w < NW; ++w) { xs += s_a[w]; ys += s_b[w]; }
            ctl->cnt_b = 0;
        }
    }
    if (threadIdx.x == 0) {
        a.nring[hy.kmodD] = xs;
        ctl->theta_sq = ys;
    }
    // every block has used the old ages by now
    for (int g = threadIdx.x; g < hy.G; g += B) {
        const int t = g < B ? my_tau : a.tau[g];
        a.tau[g] = s_mask[g] ? 1 : t + 1;
        if (s_mask[g]) a.which[g] = 1 - s_which[g];          // the fresh row becomes the stored one
    }
}

// ||theta^k||^2 of the current slot.  grid: any number of blocks <= the entries of part (one
// partial each, fixed slab order); the block that finishes last adds them up in a fixed order.
__global__ __launch_bounds__(256) void theta_sq_kernel(Hyper hy, const float* __restrict__ ring,
                                                        double* __restrict__ part, Ctl* __restrict__ ctl)
{
    __shared__ double s_tmp[256 / kWave];
    __shared__ bool s_last;
    const float* th = ring + (int64_t)hy.cur * hy.pstride;
    double a = 0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < hy.p; i += (int64_t)gridDim.x * 256)
        a += (double)th[i] * (double)th[i];
    a = wave_sum(a);
    if (threadIdx.x % kWave == 0) s_tmp[threadIdx.x / kWave] = a;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0;
        for (int w = 0; w < 256 / kWave; ++w) t += s_tmp[w];
        if (gridDim.x == 1) {
            ctl->theta_sq = t;
            s_last = false;
        } else {
            part[blockIdx.x] = t;
            __threadfence();
            s_last = atomicAdd(&ctl->cnt_c, 1u) == gridDim.x - 1;
        }
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    double t = 0;
    for (int i = threadIdx.x; i < (int)gridDim.x; i += 256) t += part[i];
    t = wave_sum(t);
    __syncthreads();
    if (threadIdx.x % kWave == 0) s_tmp[threadIdx.x / kWave] = t;
    __syncthreads();
    if (threadIdx.x == 0) {
        double u = 0;
        for (int w = 0; w < 256 / kWave; ++w) u += s_tmp[w];
        ctl->theta_sq = u;
        ctl->cnt_c = 0;
    }
}

}  // namespace

constexpr int kBigBlock = 1024;

hipError_t select_plan(gcada_ctx* c)
{
    // every per-parameter vector is padded to pstride (a multiple of 64): always four per thread.
    // At most one block per compute unit (its 68 registers per thread let only one 1024-thread
    // block be resident there anyway): each block prepares the selection once, walks over its
    // slabs of the parameter vector and ends with a device-wide fence -- about 4 + 11 us that a
    // second round of blocks would pay again (4.2 M parameters, no upload: 46 -> 35 us).
    const int64_t per_block = (int64_t)kUpdBlock * 4;
    const int64_t slabs = (c->hy.pstride + per_block - 1) / per_block;
    hipDeviceProp_t prop;
    hipError_t e = hipGetDeviceProperties(&prop, c->device);
    if (e != hipSuccess) return e;
    c->n_epi_blocks = (int32_t)std::min<int64_t>(slabs, (int64_t)prop.multiProcessorCount);
    return hipSuccess;
}

template <int B, int VW>
static void launch_server(bool self_select, int blocks, size_t lds, hipStream_t s, const ServerArgs& a)
{
    if (self_select) server_step_kernel<B, VW, true><<<blocks, B, lds, s>>>(a);
    else server_step_kernel<B, VW, false><<<blocks, B, lds, s>>>(a);
}

// Selection + masked innovation sum + server update + history for one iteration.
hipError_t server_step(gcada_ctx* c, uint8_t* mask_out, float* loss_out, bool preselected, hipStream_t s)
{
    const size_t lds = ((size_t)c->hy.G * 17 + 15) / 16 * 16;   // a double, two ints, a byte per group
    ServerArgs a{};
    a.hy = c->hy; a.part_stat = c->part_stat; a.n_stat = c->n_stat_used;
    a.part_loss = c->part_loss; a.n_loss_total = c->n_loss_used;
    a.stat = c->stat; a.mask = c->mask; a.mask_out = mask_out; a.loss_out = loss_out;
    a.gbuf = c->gbuf; a.which = c->which; a.agg = c->agg; a.h = c->h; a.vhat = c->vhat;
    a.ring = c->ring; a.nring = c->nring; a.tau = c->tau; a.part_sq = c->part_sq; a.ctl = c->ctl;
    if (!preselected && c->n_stat_used > 16) {
        // many partials per group (MLP weight-gradient tiles): add them up with one block per group
        stat_reduce_kernel<<<c->hy.G, kSelBlock, 0, s>>>(c->part_stat, c->n_stat_used, c->stat_sum);
        a.part_stat = c->stat_sum;
        a.n_stat = 1;
    }
    // every update block re-adds the (remaining) partial statistics when that is cheap
    const bool self_select = !preselected && (int64_t)c->hy.G * a.n_stat + c->n_loss_used <= 4096;
    if (!self_select && !preselected)
        select_kernel<<<1, kSelBlock, ((size_t)c->hy.G + 15) / 16 * 16, s>>>(
            c->hy, a.part_stat, a.n_stat, c->part_loss, c->n_loss_used, c->nring, c->tau,
            c->stat, c->mask, c->ctl, mask_out, loss_out);
    if (c->hy.pstride <= (int64_t)kBigBlock * 4)
        // the whole parameter vector fits one block: no cross-block hand-over at the end
        launch_server<kBigBlock, 4>(self_select, 1, lds, s, a);
    else
        launch_server<kUpdBlock, 4>(self_select, c->n_epi_blocks, lds, s, a);
    return hipGetLastError();
}

hipError_t lazy_flags(gcada_ctx* c, hipStream_t s)
{
    lazy_flags_kernel<<<1, kWave, 0, s>>>(c->hy, c->nring, c->tau, c->hot, c->store_now);
    return hipGetLastError();
}

// Selection alone (statistic sums, threshold, mask, loss), for a step whose gradient stage wrote
// only the fresh gradients of c->store_now: also marks in c->redo the selected groups whose
// gradient is still to be written.  server_step(..., preselected = true, ...) follows.
hipError_t server_select(gcada_ctx* c, uint8_t* mask_out, float* loss_out, hipStream_t s)
{
    stat_select_kernel<<<c->hy.G, kSelBlock, 0, s>>>(
        c->hy, c->part_stat, c->n_stat_used, c->part_loss, c->n_loss_used, c->nring, c->tau, c->stat,
        c->mask, c->ctl, mask_out, loss_out, c->store_now, c->redo, c->hot);
    return hipGetLastError();
}

hipError_t refresh_theta_sq(gcada_ctx* c, hipStream_t s)
{
    // one block per 8K parameters, at most as many as there are partial slots
    const int blocks = (int)std::max<int64_t>(1, std::min<int64_t>(2 * (int64_t)c->n_epi_blocks, (c->hy.p + 8191) / 8192));
    theta_sq_kernel<<<blocks, 256, 0, s>>>(c->hy, c->ring, c->part_sq, c->ctl);
    return hipGetLastError();
}

}  // namespace gcada
