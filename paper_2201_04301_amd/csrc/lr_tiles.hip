// Single-pass logistic-regression gradients for d <= 4096 (step a1; paper Sec. II-A).
//
// Each workgroup (1024 threads) keeps a tile of R whole rows in registers -- 16 rows x 4 columns
// per thread, the 16 waves arranged WR (rows) x WC (columns) with 256*WC = d.  Because the tile
// holds complete rows, the two dot products per row (with theta^k and with theta^k - theta_stale)
// finish inside the workgroup; the residuals follow, and the two weighted row sums over the
// tile's rows are formed straight from the registers.  The minibatch is therefore read from
// HBM exactly once and no workgroup ever waits for another.  Tiles of one group leave partial
// column sums; a second, small kernel adds them in a fixed order (deterministic), writes the
// group's gradient and the partial squared norms of the gradient difference.
#include "lr_device.h"

namespace gcada {

namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / kWave;     // 16
constexpr int kTR = 16;                      // tile rows per thread

struct TileArgs {
    Hyper hy;
    const ShardDesc* shards;
    const int32_t* idx;
    const float* ring;
    const int32_t* tau;
    float* part_g;        // [G][RB][d] partial sums of r_i x_i over the tile's rows
    float* part_s;        // [G][RB][d] partial sums of dr_i x_i
    double* part_loss;    // [G][RB]
    int RB;               // row blocks (tiles) per group
};

// grid: G * RB workgroups, one tile each.
template <int WC>
__global__ __launch_bounds__(kThreads) void lr_tile_kernel(TileArgs a)
{
    constexpr int WR = kWaves / WC;
    constexpr int R = kTR * WR;

    __shared__ int s_row[R];
    __shared__ float s_dot[WC][R * 2];
    __shared__ float2 s_res[R];
    __shared__ float4 s_acc[WR > 1 ? 2 : 1][WR > 1 ? kWaves : 1][kWave];
    __shared__ double s_red[kWaves];

    const Hyper& hy = a.hy;
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int wr = wave / WC, wc = wave % WC;
    const int g = blockIdx.x / a.RB, rb = blockIdx.x % a.RB;
    if (hy.sel && !hy.sel[g]) {                  // unselected group: no gradient, no loss
        if (tid == 0) a.part_loss[blockIdx.x] = 0;
        return;
    }
    const int mu = hy.mu;
    const long long k = hy.k;
    const ShardDesc sh = a.shards[g];
    const float* __restrict__ X = (const float*)sh.X;

    // row ids first: the tile's loads depend on nothing else
    int my_row = 0;
    if (tid < R) {
        const int i = rb * R + tid;
        if (a.idx) {
            my_row = a.idx[(int64_t)g * mu + i];
        } else {
            // cyclic window: (k * mu + i) mod rows, kept in 64-bit products of reduced factors
            const unsigned long long n = (unsigned long long)sh.rows;
            my_row = (int)((((unsigned long long)k % n) * ((unsigned long long)mu % n) +
                            (unsigned long long)i) % n);
        }
        s_row[tid] = my_row;
    }
    const int col = wc * 256 + lane * 4;
    __syncthreads();

    // the tile: all 16 loads of a thread are in flight at once
    float4 x[kTR];
#pragma unroll
    for (int u = 0; u < kTR; ++u) {
        // the row id is the same for the whole wave: keep it in a scalar register
        const int64_t row = __builtin_amdgcn_readfirstlane(s_row[wr * kTR + u]);
        x[u] = global_load4(X + row * sh.ld + col);
    }
    // while the tile streams in: labels, the two iterates
    float my_y = 1.0f;
    if (tid < R) my_y = global_load((const float*)sh.y + my_row);
    const float* __restrict__ th = a.ring + (int64_t)hy.cur * hy.pstride;
    const int old = stale_slot_of(hy, a.tau[g]);
    const float* __restrict__ ts = a.ring + (int64_t)old * hy.pstride;
    const float4 th4 = *(const float4*)(th + col);
    const float4 u4 = *(const float4*)(ts + col);
    const float4 dl4 = make_float4(th4.x - u4.x, th4.y - u4.y, th4.z - u4.z, th4.w - u4.w);
    // partial dot products of the wave's 256 columns, four rows at a time
#pragma unroll
    for (int qt = 0; qt < 4; ++qt) {
        float v[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float4 q = x[qt * 4 + i];
            v[2 * i] = q.x * th4.x + q.y * th4.y + q.z * th4.z + q.w * th4.w;
            v[2 * i + 1] = q.x * dl4.x + q.y * dl4.y + q.z * dl4.z + q.w * dl4.w;
        }
        Butterfly<8, 32>::run(v, lane);              // lane holds value (lane >> 3)
        if ((lane & 7) == 0) s_dot[wc][(wr * kTR + qt * 4) * 2 + (lane >> 3)] = v[0];
    }
    __syncthreads();
    double lsum = 0;
    if (tid < R) {
        float z = 0, dz = 0;
#pragma unroll
        for (int w = 0; w < WC; ++w) {               // fixed order over the column waves
            z += s_dot[w][2 * tid];
            dz += s_dot[w][2 * tid + 1];
        }
        float r, dr, ls;
        residuals(hy.quadratic != 0, z, dz, my_y, r, dr, ls);
        s_res[tid] = make_float2(r, dr);
        lsum = (double)ls;
    }
    lsum = wave_sum(lsum);
    if (lane == 0) s_red[wave] = lsum;
    __syncthreads();
    if (tid == 0) {
        double t = 0;
        for (int w = 0; w < (R + kWave - 1) / kWave; ++w) t += s_red[w];
        a.part_loss[blockIdx.x] = t;
    }
    // weighted row sums of the tile, from the registers
    float4 ag = make_float4(0, 0, 0, 0), as = make_float4(0, 0, 0, 0);
#pragma unroll
    for (int u = 0; u < kTR; ++u) {
        const float2 w = s_res[wr * kTR + u];
        ag.x += w.x * x[u].x; ag.y += w.x * x[u].y; ag.z += w.x * x[u].z; ag.w += w.x * x[u].w;
        as.x += w.y * x[u].x; as.y += w.y * x[u].y; as.z += w.y * x[u].z; as.w += w.y * x[u].w;
    }
    if constexpr (WR > 1) {
        s_acc[0][wave][lane] = ag;
        s_acc[1][wave][lane] = as;
        __syncthreads();
        if (wr == 0) {
#pragma unroll
            for (int w = 1; w < WR; ++w) {
                const float4 p = s_acc[0][w * WC + wc][lane], q = s_acc[1][w * WC + wc][lane];
                ag.x += p.x; ag.y += p.y; ag.z += p.z; ag.w += p.w;
                as.x += q.x; as.y += q.y; as.z += q.z; as.w += q.w;
            }
        }
    }
    if (wr == 0) {
        const int64_t o = (int64_t)blockIdx.x * hy.p + col;
        *(float4*)(a.part_g + o) = ag;
        *(float4*)(a.part_s + o) = as;
    }
}

constexpr int kRedBlock = 256;

// grid: (ceil(d/4 / 256), G).  Adds the RB tile partials of a group in a fixed order, adds the
// l2 terms, writes the group's gradient and one partial squared norm per block.
__global__ __launch_bounds__(kRedBlock) void lr_tile_reduce(
    Hyper hy, const float* __restrict__ part_g, const float* __restrict__ part_s, int RB,
    const float* __restrict__ ring, const int32_t* __restrict__ tau, float* __restrict__ gbuf,
    const int32_t* __restrict__ which,
    double* __restrict__ part_stat)
{
    __shared__ double s_red[kRedBlock / kWave];
    const int g = blockIdx.y;
    if (hy.sel && !hy.sel[g]) return;
    const int64_t j = ((int64_t)blockIdx.x * kRedBlock + threadIdx.x) * 4;
    double sq = 0;
    if (j < hy.p) {
        const float* pg = part_g + (int64_t)g * RB * hy.p + j;
        const float* ps = part_s + (int64_t)g * RB * hy.p + j;
        float4 t = make_float4(0, 0, 0, 0), u = t;
        if (hy.l2 != 0.0f) {
            t = *(const float4*)(ring + (int64_t)hy.cur * hy.pstride + j);
            const int old = stale_slot_of(hy, tau[g]);
            u = *(const float4*)(ring + (int64_t)old * hy.pstride + j);
        }
        float4 ag = make_float4(0, 0, 0, 0), as = ag;
        int rb = 0;
        for (; rb + 8 <= RB; rb += 8) {          // eight tiles' loads in flight, added in order
            float4 p[8], q[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                p[e] = *(const float4*)(pg + (int64_t)(rb + e) * hy.p);
                q[e] = *(const float4*)(ps + (int64_t)(rb + e) * hy.p);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                ag.x += p[e].x; ag.y += p[e].y; ag.z += p[e].z; ag.w += p[e].w;
                as.x += q[e].x; as.y += q[e].y; as.z += q[e].z; as.w += q[e].w;
            }
        }
        for (; rb < RB; ++rb) {
            const float4 p = *(const float4*)(pg + (int64_t)rb * hy.p);
            const float4 q = *(const float4*)(ps + (int64_t)rb * hy.p);
            ag.x += p.x; ag.y += p.y; ag.z += p.z; ag.w += p.w;
            as.x += q.x; as.y += q.y; as.z += q.z; as.w += q.w;
        }
        if (hy.l2 != 0.0f) {
            const float ml = (float)hy.mu * hy.l2;
            ag.x += ml * t.x; ag.y += ml * t.y; ag.z += ml * t.z; ag.w += ml * t.w;
            as.x += ml * (t.x - u.x); as.y += ml * (t.y - u.y);
            as.z += ml * (t.z - u.z); as.w += ml * (t.w - u.w);
        }
        *(float4*)(fresh_row(gbuf, which, hy, g) + j) = ag;
        sq = (double)as.x * as.x + (double)as.y * as.y + (double)as.z * as.z + (double)as.w * as.w;
    }
    sq = wave_sum(sq);
    if (threadIdx.x % kWave == 0) s_red[threadIdx.x / kWave] = sq;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0;
        for (int w = 0; w < kRedBlock / kWave; ++w) t += s_red[w];
        part_stat[(int64_t)g * gridDim.x + blockIdx.x] = t;
    }
}

}  // namespace

struct LrTilePlan {
    int WC = 0;           // 0: not applicable
    int R = 0, RB = 0, n_stat = 0;
    float* part_g = nullptr;
    float* part_s = nullptr;
};

// Decide whether the single-pass kernel applies (d in {256, 512, ..., 4096} so that a tile holds
// whole rows; mu a multiple of the tile's rows) and size its scratch.
hipError_t lr_tile_plan(gcada_ctx* c)
{
    auto* pl = new LrTilePlan();
    c->lr_tiles = pl;
    const int d = (int)c->hy.p, mu = c->hy.mu, G = c->hy.G;
    int WC = 0;
    for (int w : {1, 2, 4, 8, 16})
        if (d == 256 * w) WC = w;
    if (!WC) return hipSuccess;
    const int R = kTR * (kWaves / WC);
    if (mu % R) return hipSuccess;
    pl->R = R;
    pl->RB = mu / R;
    pl->n_stat = (d / 4 + kRedBlock - 1) / kRedBlock;
    const size_t n = (size_t)G * pl->RB * d;
    hipError_t e;
    if ((e = hipMalloc(&pl->part_g, n * sizeof(float))) != hipSuccess) return e;
    if ((e = hipMalloc(&pl->part_s, n * sizeof(float))) != hipSuccess) return e;
    pl->WC = WC;
    c->n_loss_part = std::max(c->n_loss_part, pl->RB);
    c->n_stat_part = std::max(c->n_stat_part, pl->n_stat);
    return hipSuccess;
}

void lr_tile_free(gcada_ctx* c)
{
    if (!c->lr_tiles) return;
    if (c->lr_tiles->part_g) (void)hipFree(c->lr_tiles->part_g);
    if (c->lr_tiles->part_s) (void)hipFree(c->lr_tiles->part_s);
    delete c->lr_tiles;
    c->lr_tiles = nullptr;
}

bool lr_tile_applies(const gcada_ctx* c)
{
    if (!c->allow_single_pass || !c->lr_tiles || c->lr_tiles->WC == 0) return false;
    for (const auto& s : c->shards)
        if ((s.ld % 4) || ((uintptr_t)s.X % 16)) return false;
    return true;
}

hipError_t lr_tile_gradients(gcada_ctx* c, const int32_t* idx, hipStream_t s)
{
    const LrTilePlan* pl = c->lr_tiles;
    TileArgs a{};
    a.hy = c->hy; a.shards = c->d_shards; a.idx = idx; a.ring = c->ring; a.tau = c->tau;
    a.part_g = pl->part_g; a.part_s = pl->part_s; a.part_loss = c->part_loss;
    a.RB = pl->RB;
    const int grid = c->hy.G * pl->RB;
    switch (pl->WC) {
    case 1: lr_tile_kernel<1><<<grid, kThreads, 0, s>>>(a); break;
    case 2: lr_tile_kernel<2><<<grid, kThreads, 0, s>>>(a); break;
    case 4: lr_tile_kernel<4><<<grid, kThreads, 0, s>>>(a); break;
    case 8: lr_tile_kernel<8><<<grid, kThreads, 0, s>>>(a); break;
    default: lr_tile_kernel<16><<<grid, kThreads, 0, s>>>(a); break;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (c->dominant_only) return hipSuccess;      // benchmark diagnostic: the tile kernel alone
    dim3 gr(pl->n_stat, c->hy.G);
    lr_tile_reduce<<<gr, kRedBlock, 0, s>>>(c->hy, pl->part_g, pl->part_s, pl->RB, c->ring, c->tau,
                                             c->gbuf, c->which, c->part_stat);
    c->n_stat_used = pl->n_stat;
    c->n_loss_used = c->hy.G * pl->RB;
    return hipGetLastError();
}

}  // namespace gcada
