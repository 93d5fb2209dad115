// Single-pass logistic-regression gradients for d <= 4096 (step a1; paper Sec. II-A).
//
// Each workgroup (1024 threads) keeps a tile of R whole rows in registers -- 16 rows x 4 columns
// per thread, the 16 waves arranged WR (rows) x WC (columns) with 256*WC >= d (WC the smallest
// power of two that covers the row; lanes past d idle).  Because the tile
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

// What a tile needs from the step BEFORE it when that step's finish runs in the same launch
// (lr_tile_step_kernel): the new iterate and each group's stale slot arrive as tagged words that
// the finishing workgroups of the launch publish.
struct StepLink {
    const unsigned long long* xtheta;   // [p] {tag, bits of theta^{k}_j}: the iterate this tile is evaluated at
    const unsigned long long* xsel;     // [G] {tag, ring slot of the group's stale iterate}
    unsigned tag;
    WaitPolicy wait;
    Ctl* ctl;
};

template <int WC>
struct TileShared {
    static constexpr int WR = kWaves / WC;
    static constexpr int R = kTR * WR;
    int s_row[R];
    float s_dot[WC][R * 2];
    float2 s_res[R];
    float4 s_acc[WR > 1 ? 2 : 1][WR > 1 ? kWaves : 1][kWave];
    double s_red[kWaves];
};

// Row ids of the tile into LDS (one barrier).  Returns this thread's own row id and validity
// (tid < R only).
template <int WC>
__device__ __forceinline__ void tile_rows(const TileArgs& a, TileShared<WC>& sm, const ShardDesc& sh, int g, int rb,
                                          int& my_row, bool& my_valid)
{
    constexpr int R = TileShared<WC>::R;
    const Hyper& hy = a.hy;
    const int tid = threadIdx.x;
    const int mu = hy.mu;
    const long long k = hy.k;
    // row ids first: the tile's loads depend on nothing else
    // (the last tile of a group may reach past the minibatch: such rows load nothing and weigh 0)
    my_row = 0;
    my_valid = false;
    if (tid < R) {
        const int i = rb * R + tid;
        my_valid = i < mu;
        if (!my_valid) {
            my_row = 0;
        } else if (a.idx) {
            my_row = a.idx[(int64_t)g * mu + i];
        } else {
            // cyclic window: (k * mu + i) mod rows, kept in 64-bit products of reduced factors
            const unsigned long long n = (unsigned long long)sh.rows;
            my_row = (int)((((unsigned long long)k % n) * ((unsigned long long)mu % n) +
                            (unsigned long long)i) % n);
        }
        sm.s_row[tid] = my_valid ? my_row : -1;
    }
    __syncthreads();
}

// The tile: all 16 loads of a thread are in flight at once.
template <int WC>
__device__ __forceinline__ void tile_issue(const TileArgs& a, const TileShared<WC>& sm, const ShardDesc& sh,
                                           float4 (&x)[kTR])
{
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int wr = wave / WC, wc = wave % WC;
    const int col = wc * 256 + lane * 4;
    const bool col_ok = col < (int)a.hy.p;       // d is a multiple of 4; the last column wave may be partly idle
    const float* __restrict__ X = (const float*)sh.X;
#pragma unroll
    for (int u = 0; u < kTR; ++u) {
        // the row id is the same for the whole wave: keep it in a scalar register
        const int64_t row = __builtin_amdgcn_readfirstlane(sm.s_row[wr * kTR + u]);
        x[u] = col_ok && row >= 0 ? global_load4_stream(X + row * sh.ld + col) : make_float4(0, 0, 0, 0);
    }
}

// Dot products, residuals, weighted row sums, tile partials.  link == nullptr: the iterate and the
// stale slot are read from the ring and the ages (the step before has completed); otherwise they
// are polled from the words the finishing workgroups of this launch publish.
template <int WC>
__device__ __forceinline__ void tile_finish(const TileArgs& a, TileShared<WC>& sm, const ShardDesc& sh, int g, int rb,
                                            int my_row, bool my_valid, float4 (&x)[kTR], const StepLink* link)
{
    constexpr int WR = TileShared<WC>::WR;
    constexpr int R = TileShared<WC>::R;
    const Hyper& hy = a.hy;
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int wr = wave / WC, wc = wave % WC;
    const int col = wc * 256 + lane * 4;
    const bool col_ok = col < (int)hy.p;
    const int tile = g * a.RB + rb;
    // while the tile streams in: labels, the two iterates
    float my_y = 1.0f;
    if (tid < R) my_y = global_load((const float*)sh.y + my_row);
    float4 th4 = make_float4(0, 0, 0, 0), u4 = th4;
    if (link == nullptr) {
        const float* __restrict__ th = a.ring + (int64_t)hy.cur * hy.pstride;
        const int old = stale_slot_of(hy, a.tau[g]);
        const float* __restrict__ ts = a.ring + (int64_t)old * hy.pstride;
        if (col_ok) {
            th4 = *(const float4*)(th + col);
            u4 = *(const float4*)(ts + col);
        }
    } else {
        // (these loads return after the tile's own, which were issued before them: by then the
        // words have normally arrived; the wait is bounded)
        unsigned long long w[4] = {0, 0, 0, 0}, ws = 0;
        unsigned spins = 0;
        for (;;) {
            bool ok = true;
            if (col_ok) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    w[e] = __hip_atomic_load(link->xtheta + col + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                    ok = ok && (unsigned)(w[e] >> 32) == link->tag + link->wait.tag_skew;
                }
            }
            ws = __hip_atomic_load(link->xsel + g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            ok = ok && (unsigned)(ws >> 32) == link->tag + link->wait.tag_skew;
            if (__all(ok)) break;
            if (++spins > link->wait.limit) {        // never in a healthy launch: report, do not hang
                if (lane == 0) raise_device_error(link->ctl, 4u);
                break;
            }
        }
        const int old = (int)(unsigned)(ws & 0xffffffffull) % (hy.D + 1);     // (in range even after a give-up)
        if (col_ok) {
            th4 = make_float4(__uint_as_float((unsigned)w[0]), __uint_as_float((unsigned)w[1]),
                              __uint_as_float((unsigned)w[2]), __uint_as_float((unsigned)w[3]));
            u4 = *(const float4*)(a.ring + (int64_t)old * hy.pstride + col);
        }
    }
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
        // sums over the 16 lanes of a row through DPP moves, then over the four rows
        RowButterfly<8>::run(v, lane);
        v[0] += __shfl_xor(v[0], 16, kWave);
        v[0] += __shfl_xor(v[0], 32, kWave);
        if (lane < 16 && (lane & 1) == 0)
            sm.s_dot[wc][(wr * kTR + qt * 4) * 2 + row_butterfly_first<8>(lane)] = v[0];
    }
    __syncthreads();
    double lsum = 0;
    if (tid < R) {
        float z = 0, dz = 0;
#pragma unroll
        for (int w = 0; w < WC; ++w) {               // fixed order over the column waves
            z += sm.s_dot[w][2 * tid];
            dz += sm.s_dot[w][2 * tid + 1];
        }
        float r, dr, ls;
        residuals(hy.quadratic != 0, z, dz, my_y, r, dr, ls);
        if (!my_valid) r = dr = ls = 0.0f;
        sm.s_res[tid] = make_float2(r, dr);
        lsum = (double)ls;
    }
    __syncthreads();
    // the tile's loss sum is nobody's input here: the waves that hold rows add it up while the
    // others go on (R is a multiple of 64 or smaller than 64, so such a wave is all rows or wave 0)
    if (wave < (R + kWave - 1) / kWave) {
        lsum = wave_total(lsum);
        if (lane == 0) sm.s_red[wave] = lsum;
    }
    // weighted row sums of the tile, from the registers
    float4 ag = make_float4(0, 0, 0, 0), as = make_float4(0, 0, 0, 0);
#pragma unroll
    for (int u = 0; u < kTR; ++u) {
        const float2 w = sm.s_res[wr * kTR + u];
        ag.x += w.x * x[u].x; ag.y += w.x * x[u].y; ag.z += w.x * x[u].z; ag.w += w.x * x[u].w;
        as.x += w.y * x[u].x; as.y += w.y * x[u].y; as.z += w.y * x[u].z; as.w += w.y * x[u].w;
    }
    if constexpr (WR > 1) {
        sm.s_acc[0][wave][lane] = ag;
        sm.s_acc[1][wave][lane] = as;
        __syncthreads();
        if (wr == 0) {
#pragma unroll
            for (int w = 1; w < WR; ++w) {
                const float4 p = sm.s_acc[0][w * WC + wc][lane], q = sm.s_acc[1][w * WC + wc][lane];
                ag.x += p.x; ag.y += p.y; ag.z += p.z; ag.w += p.w;
                as.x += q.x; as.y += q.y; as.z += q.z; as.w += q.w;
            }
        }
    }
    if constexpr (R > kWave) {
        __syncthreads();
        if (tid == 0) {
            double t = 0;
            for (int w = 0; w < R / kWave; ++w) t += sm.s_red[w];
            a.part_loss[tile] = t;
        }
    } else {
        if (tid == 0) a.part_loss[tile] = lsum;
    }
    if (wr == 0) {
        if (rb == 0 && hy.l2 != 0.0f) {
            // the l2 terms mu*lambda*theta^k and mu*lambda*(theta^k - theta_stale) ride on the
            // group's first tile: both iterates are in registers here, and whoever adds the
            // tiles up needs neither them nor the group's age (explicit fused multiply-adds)
            const float ml = (float)hy.mu * hy.l2;
            ag.x = fmaf(ml, th4.x, ag.x); ag.y = fmaf(ml, th4.y, ag.y);
            ag.z = fmaf(ml, th4.z, ag.z); ag.w = fmaf(ml, th4.w, ag.w);
            as.x = fmaf(ml, dl4.x, as.x); as.y = fmaf(ml, dl4.y, as.y);
            as.z = fmaf(ml, dl4.z, as.z); as.w = fmaf(ml, dl4.w, as.w);
        }
        if (col_ok) {
            const int64_t o = (int64_t)tile * hy.p + col;
            *(float4*)(a.part_g + o) = ag;
            *(float4*)(a.part_s + o) = as;
        }
    }
}

// grid: G * RB workgroups, one tile each.
template <int WC>
__global__ __launch_bounds__(kThreads) void lr_tile_kernel(TileArgs a)
{
    __shared__ TileShared<WC> sm;
    const int g = blockIdx.x / a.RB, rb = blockIdx.x % a.RB;
    if (a.hy.sel && !a.hy.sel[g]) {              // unselected group: no gradient, no loss
        if (threadIdx.x == 0) a.part_loss[blockIdx.x] = 0;
        return;
    }
    const ShardDesc sh = a.shards[g];
    int my_row;
    bool my_valid;
    float4 x[kTR];
    tile_rows<WC>(a, sm, sh, g, rb, my_row, my_valid);
    tile_issue<WC>(a, sm, sh, x);
    tile_finish<WC>(a, sm, sh, g, rb, my_row, my_valid, x, nullptr);
}

constexpr int kRedBlock = 256;

// grid: (ceil(d/4 / 256), G).  Adds the RB tile partials of a group in a fixed order (the l2
// terms are part of the first tile's), writes the group's gradient and one partial squared norm
// per block.
__global__ __launch_bounds__(kRedBlock) void lr_tile_reduce(
    Hyper hy, const float* __restrict__ part_g, const float* __restrict__ part_s, int RB,
    float* __restrict__ gbuf, const int32_t* __restrict__ which, double* __restrict__ part_stat)
{
    __shared__ double s_red[kRedBlock / kWave];
    const int g = blockIdx.y;
    if (hy.sel && !hy.sel[g]) return;
    const int64_t j = ((int64_t)blockIdx.x * kRedBlock + threadIdx.x) * 4;
    double sq = 0;
    if (j < hy.p) {
        const float* pg = part_g + (int64_t)g * RB * hy.p + j;
        const float* ps = part_s + (int64_t)g * RB * hy.p + j;
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


// ---- fused finish: tile reduce + selection (a2) + masked innovation sum (a3) + update (a4) ----
//
// The three small steps after the tile kernel are a chain of short memory round trips; as
// separate launches each also pays a launch, a drain and cold first loads.  Here one launch does
// them all.  A block owns 4*CL columns of EVERY group: it adds the tile partials of its columns
// (same order as lr_tile_reduce), writes the fresh gradients, keeps the innovations
// grad_g - last_g in LDS and publishes one partial squared norm per group.  The statistic of
// Eq. (9) needs all columns, so the blocks meet once: each publishes its partials as tagged words
// and polls (bounded) those of the others; the grid has at most 64 blocks, one per compute unit
// at most, so all blocks are resident.  Every block then derives the same mask,
// and updates its columns by Eq. (8a)-(8c); the block that finishes last closes the history
// entry, as in the stand-alone server kernel.
constexpr int kFinGroups = 16;            // group lanes of a block
constexpr int kFinMaxG = 64;              // innovations kept in LDS: kFinMaxG x 4*CL floats

struct FinishArgs {
    Hyper hy;
    const float* part_g;
    const float* part_s;
    int RB;
    const double* part_loss;
    int n_loss_total;
    unsigned long long* xstat;   // [G][gridDim.x] tagged doubles: partial squared norms
    unsigned long long* xsq;     // [gridDim.x][2] tagged doubles: ||step||^2, ||theta^{k+1}||^2
    unsigned tag;                // of this launch (never 0, never that of a recent launch)
    WaitPolicy wait;             // bound of the polls; tag_skew != 0 only in the test of the give-up path
    // the two sums of the PREVIOUS launch are still per block (nobody waits for them at the end
    // of a launch): this launch adds them up, uses them and stores them
    const unsigned long long* xsq_prev;
    unsigned tag_prev;
    int fold_prev;               // 0: history and ||theta^k||^2 are already complete
    int pre;                     // 1: server-side rule (Sec. IV): the mask was decided before the
                                 //    gradients (a.mask, a.stat, Ctl::rhs are inputs); only the
                                 //    selected groups left tile partials; no statistic, no exchange
    int prev_kmodD;              // history index the previous launch's ||step||^2 belongs to
    // when the tiles of the NEXT step run in the same launch (lr_tile_step_kernel): the new iterate
    // and the groups' stale slots also go out as tagged words (null otherwise)
    unsigned long long* xtheta;  // [p] {tag, bits of theta^{k+1}_j}
    unsigned long long* xsel;    // [G] {tag, ring slot of theta^{(k+1) - tau_g^{k+1}}}
    double* stat;
    uint8_t* mask;
    uint8_t* mask_out;
    float* loss_out;
    float* gbuf;
    int32_t* which;
    float* agg;
    float* h;
    float* vhat;
    float* ring;
    double* nring;
    int32_t* tau;
    Ctl* ctl;
};

// A double that one block hands to the others travels as two tagged 64-bit words
// {tag, low half} and {tag, high half}, written and read with relaxed atomics that go past the
// per-XCD L2s: a reader polls the words themselves and needs no fence or separate flag; a word
// of an earlier launch carries an older tag.
__device__ __forceinline__ void tagged_store(unsigned long long* slot, double v, unsigned tag)
{
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    __hip_atomic_store(slot, ((unsigned long long)tag << 32) | (b & 0xffffffffull), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_SYSTEM);
    __hip_atomic_store(slot + 1, ((unsigned long long)tag << 32) | (b >> 32), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_SYSTEM);
}
__device__ __forceinline__ void tagged_issue(const unsigned long long* slot, unsigned long long& lo,
                                             unsigned long long& hi)
{
    lo = __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    hi = __hip_atomic_load(slot + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}
__device__ __forceinline__ bool tagged_check(unsigned long long lo, unsigned long long hi, unsigned tag, double& v)
{
    v = __longlong_as_double((long long)((hi << 32) | (lo & 0xffffffffull)));
    return (unsigned)(lo >> 32) == tag && (unsigned)(hi >> 32) == tag;
}
__device__ __forceinline__ bool tagged_load(const unsigned long long* slot, unsigned tag, double& v)
{
    const unsigned long long lo = __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    const unsigned long long hi = __hip_atomic_load(slot + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    v = __longlong_as_double((long long)((hi << 32) | (lo & 0xffffffffull)));
    return (unsigned)(lo >> 32) == tag && (unsigned)(hi >> 32) == tag;
}

// The work of one finishing block: CL * 16 threads (tid = 0 .. CL*16-1; thread = (group lane gl,
// column lane cl)), block blk of S.  Two workgroup barriers; a caller whose workgroup has more
// threads lets the others execute two barriers of their own.  NFLY: tile partials whose loads are
// in flight together (they are added in the same order whatever it is).  NCH: 16 * NCH >= G.
template <int CL, int NFLY, int NCH>
__device__ __forceinline__ void finish_body(const FinishArgs& a, const int tid, const int blk, const int S)
{
    constexpr int B = CL * kFinGroups, NW = B / kWave;
    __shared__ float4 s_delta[kFinMaxG][CL];
    __shared__ double s_ps[kFinMaxG], s_stat[kFinMaxG];
    __shared__ int s_which[kFinMaxG], s_tau[kFinMaxG];
    __shared__ double s_red[NW];
    __shared__ double s_rhs;

    const Hyper& hy = a.hy;
    Ctl* ctl = a.ctl;
    const int wave = tid / kWave, lane = tid % kWave;
    const int gl = tid / CL, cl = tid % CL;
    const int G = hy.G;
    const int64_t j = ((int64_t)blk * CL + cl) * 4;
    const bool jok = j < hy.p;                   // the last block's columns may end early (p % 4 == 0)
    const float* __restrict__ th = a.ring + (int64_t)hy.cur * hy.pstride;
    float* __restrict__ tn = a.ring + (int64_t)hy.nxt * hy.pstride;

    // NCH: passes over the groups (G <= 16 * NCH <= kFinMaxG)
    static_assert(4 * CL <= kWave, "the updating threads must sit in wave 0");

    // 1. The way to the statistic first -- the other blocks wait for it: tile partials of the
    //    block's columns, added in lr_tile_reduce's order (the l2 terms are part of the first
    //    tile's); partial squared norm.
    // (the ages and halves go to LDS for later; their loads are not waited for before the tile
    // loads are out)
    int my_which = 0, my_tau = 0;
    if (tid < G) { my_which = a.which[tid]; my_tau = a.tau[tid]; }
    bool pre_sel = false;                        // server-side rule: lane g of every wave holds mask[g]
    if (a.pre && lane < G) pre_sel = a.mask[lane] != 0;
    const unsigned long long pre_bits = __ballot(pre_sel);
    const int RB = a.RB;
    float4 agk[NCH];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
        const int g = ch * kFinGroups + gl;
        double sq = 0;
        agk[ch] = make_float4(0, 0, 0, 0);
        if (g < G && jok && (!a.pre || ((pre_bits >> g) & 1ull))) {
            const float* pg = a.part_g + (int64_t)g * RB * hy.p + j;
            const float* ps = a.part_s + (int64_t)g * RB * hy.p + j;
            float4 ag = make_float4(0, 0, 0, 0), as = ag;
            int rb = 0;
            if (NFLY >= 16 && RB >= 16) {            // sixteen tiles' loads in flight, added in order
                float4 p[16], q[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    p[e] = *(const float4*)(pg + (int64_t)e * hy.p);
                    q[e] = *(const float4*)(ps + (int64_t)e * hy.p);
                }
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    ag.x += p[e].x; ag.y += p[e].y; ag.z += p[e].z; ag.w += p[e].w;
                    as.x += q[e].x; as.y += q[e].y; as.z += q[e].z; as.w += q[e].w;
                }
                rb = 16;
            }
            for (; NFLY >= 8 && rb + 8 <= RB; rb += 8) {   // eight tiles' loads in flight, added in order
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
            for (; rb + 4 <= RB; rb += 4) {          // four tiles' loads in flight, added in order
                float4 p[4], q[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    p[e] = *(const float4*)(pg + (int64_t)(rb + e) * hy.p);
                    q[e] = *(const float4*)(ps + (int64_t)(rb + e) * hy.p);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
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
            agk[ch] = ag;
            sq = (double)as.x * as.x + (double)as.y * as.y + (double)as.z * as.z + (double)as.w * as.w;
        }
        // the CL column lanes of a group lane are neighbours within a row of 16 lanes: DPP moves
        // (lanes ^1, ^2, mirror within 8, mirror within 16), a fixed order
        static_assert(CL == 1 || CL == 2 || CL == 4 || CL == 8 || CL == 16, "column lanes of a group lane");
        if constexpr (CL >= 2) sq += dpp_move(sq, 0);
        if constexpr (CL >= 4) sq += dpp_move(sq, 1);
        if constexpr (CL >= 8) sq += dpp_move(sq, 2);
        if constexpr (CL >= 16) sq += dpp_move(sq, 3);
        if (g < G && cl == 0) s_ps[g] = sq;
    }
    if (tid < G) { s_which[tid] = my_which; s_tau[tid] = my_tau; }
    for (int g = tid + B; g < G; g += B) { s_which[g] = a.which[g]; s_tau[g] = a.tau[g]; }
    __syncthreads();
    if (!a.pre)
        for (int g = tid; g < G; g += B) tagged_store(a.xstat + 2 * ((int64_t)g * S + blk), s_ps[g], a.tag);

    // 2. While the partials travel: everything else this block needs.  The update (a3, a4) of
    //    its 4*CL columns is done by the first 4*CL threads, one column each (a short instruction
    //    stream per lane instead of a long one on a few lanes).
    const int64_t jc = (int64_t)blk * 4 * CL + tid;
    const bool upd = tid < 4 * CL && jc < hy.p;
    float ac = 0, hv = 0, vv = 0, tv = 0;
    if (upd) {
        ac = a.agg[jc];
        hv = a.h[jc];
        vv = a.vhat[jc];
        tv = th[jc];
    }
    // (only loads here, nothing that waits for one: sums over more than one element per thread
    // are finished after the exchange)
    double lpart = 0, hist = 0, theta_sq = 0, psq = 0, ptsq = 0;
    unsigned long long plo[2] = {0, 0}, phi[2] = {0, 0};
    if (blk == 0 && tid < a.n_loss_total) lpart = a.part_loss[tid];
    if (wave == 0) {
        if (a.fold_prev) {
            // lane i: block i's sums of the previous launch (complete: that launch has ended)
            if (lane < S) {
                tagged_issue(a.xsq_prev + 4 * (int64_t)lane, plo[0], phi[0]);
                tagged_issue(a.xsq_prev + 4 * (int64_t)lane + 2, plo[1], phi[1]);
            }
        } else if (blk == 0) {
            theta_sq = ctl->theta_sq;
        }
        if (lane < hy.D && !(a.fold_prev && lane == a.prev_kmodD)) hist = a.nring[lane];
    }
    // both halves of each group's gradient rows are asked for now and the stored one is picked
    // when they are used, after the wait below, so no load waits for another
    float4 h0k[NCH], h1k[NCH];
    int wlk[NCH];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
        const int g = ch * kFinGroups + gl;
        h0k[ch] = h1k[ch] = make_float4(0, 0, 0, 0);
        wlk[ch] = 0;
        if (g < G && jok && (!a.pre || ((pre_bits >> g) & 1ull))) {
            wlk[ch] = s_which[g];      // read before this block published: block 0 may flip it now
            h0k[ch] = *(const float4*)(a.gbuf + (int64_t)g * hy.pstride + j);
            h1k[ch] = *(const float4*)(a.gbuf + ((int64_t)G + g) * hy.pstride + j);
        }
    }

    // a2: lane i collects block i's partial of four groups at a time (polling the tagged words
    // is the wait); every block adds the same numbers in the same order and so reaches the same
    // statistics and mask
    bool first = true;
    for (int g0 = wave; g0 < (a.pre ? 0 : G); g0 += 4 * NW) {
        double v[4] = {0, 0, 0, 0};
        bool got[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) got[e] = lane >= S || g0 + e * NW >= G;
        unsigned spins = 0;
        for (;;) {
            unsigned long long lo[4], hi[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (!got[e]) tagged_issue(a.xstat + 2 * ((int64_t)(g0 + e * NW) * S + lane), lo[e], hi[e]);
            if (first) {
                // while the first answers travel (loads return in order, so this waits only for
                // the older ones): the threshold of Eq. (9); wave 0 always gets here (G >= 1)
                first = false;
                if (wave == 0) {
                    for (int i = lane + kWave; i < hy.D; i += kWave)
                        if (!(a.fold_prev && i == a.prev_kmodD)) hist += a.nring[i];
                    if (a.fold_prev) {
                        bool prev_ok = true;
                        if (lane < S) {
                            prev_ok = tagged_check(plo[0], phi[0], a.tag_prev, psq);
                            prev_ok = tagged_check(plo[1], phi[1], a.tag_prev, ptsq) && prev_ok;
                        }
                        if (!__all(prev_ok) && lane == 0) raise_device_error(ctl, 2u);
                        psq = wave_total(psq);
                        ptsq = wave_total(ptsq);
                        if (blk == 0 && lane == 0) {
                            a.nring[a.prev_kmodD] = psq;         // no block reads this entry in this launch
                            ctl->theta_sq = ptsq;
                        }
                        theta_sq = ptsq;
                        // the entry takes its place in the lane-strided order of the history sum
                        if (lane == a.prev_kmodD % kWave) hist += psq;
                    }
                    hist = wave_total(hist);
                    if (lane == 0) s_rhs = hy.c / (double)hy.D * hist;
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (!got[e]) got[e] = tagged_check(lo[e], hi[e], a.tag + a.wait.tag_skew, v[e]);
            if (__all(got[0] && got[1] && got[2] && got[3])) break;
            if (++spins > a.wait.limit) {            // never in a healthy launch: report, do not hang
                if (lane == 0) raise_device_error(ctl, 1u);
                break;
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const double t = wave_total(v[e]);
            if (lane == 0 && g0 + e * NW < G) s_stat[g0 + e * NW] = t;
        }
    }
    const bool pub = blk == 0;
    if (pub) {
        for (int i = tid + B; i < a.n_loss_total; i += B) lpart += a.part_loss[i];
        lpart = wave_total(lpart);
        if (lane == 0) s_red[wave] = lpart;
    }
    // fresh gradients out, innovations grad_g - last_g into LDS
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
        const int g = ch * kFinGroups + gl;
        if (g < G && jok && (!a.pre || ((pre_bits >> g) & 1ull))) {
            const float4 ag = agk[ch];
            const float4 last4 = wlk[ch] ? h1k[ch] : h0k[ch];
            *(float4*)(a.gbuf + ((int64_t)(1 - wlk[ch]) * G + g) * hy.pstride + j) = ag;
            s_delta[g][cl] = make_float4(ag.x - last4.x, ag.y - last4.y, ag.z - last4.z, ag.w - last4.w);
        }
    }
    __syncthreads();
    const double rhs = a.pre ? 0.0 : s_rhs;
    // the decision of Eq. (9): lane g of every wave takes it for group g; the ballot is the mask
    bool sel = false;
    if (lane < G && !a.pre) sel = (s_stat[lane] > rhs) || (s_tau[lane] >= hy.D) || (rhs == 0.0);
    const unsigned long long selbits = a.pre ? pre_bits : __ballot(sel);
    if (a.pre) sel = pre_sel;
    if (pub && wave == 0) {
        // every block copied the ages and the halves to its LDS before it published its partials
        // (server-side rule: no block waits for another, so they are updated by the block that
        // finishes last, below)
        if (lane < G) {
            const int t = s_tau[lane];
            if (!a.pre) {
                a.stat[lane] = s_stat[lane];
                a.mask[lane] = sel ? 1 : 0;
                if (a.mask_out) a.mask_out[lane] = sel ? 1 : 0;
            }
            if (!a.pre) {
                a.tau[lane] = sel ? 1 : t + 1;
                if (sel) a.which[lane] = 1 - s_which[lane];
                // where the group's stale iterate sits in the next step: theta^k after an upload
                // (age 1 then), the slot it had otherwise
                if (a.xsel)
                    __hip_atomic_store(a.xsel + lane,
                                       ((unsigned long long)a.tag << 32) | (unsigned)(sel ? hy.cur : stale_slot_of(hy, t)),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            }
        }
        if (lane == 0) {
            double lsum = 0;
            for (int w = 0; w < NW; ++w) lsum += s_red[w];
            double loss;
            if (a.pre) {
                // mean over the samples that were evaluated (the unselected groups left zero
                // partials), 0 when no group was selected
                const double nsel = (double)__popcll(selbits);
                loss = nsel > 0 ? lsum / (nsel * (double)hy.mu) + 0.5 * (double)hy.l2 * theta_sq : 0.0;
            } else {
                loss = lsum / ((double)G * (double)hy.mu) + 0.5 * (double)hy.l2 * theta_sq;
                ctl->rhs = rhs;
            }
            ctl->loss = loss;
            if (a.loss_out) *a.loss_out = (float)loss;
        }
    }
    if (wave != 0) return;

    // a3 + a4: the innovations of the selected groups in ascending order (the LDS reads of eight
    // groups go out together; a select, not a branch, keeps or skips each), then Eq. (8a)-(8c)
    double sq = 0, tsq = 0;
    if (upd) {
        const float* s_df = (const float*)s_delta;          // [g][4*CL] as plain floats
        for (int g0 = 0; g0 < G; g0 += 8) {
            float d[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) d[e] = s_df[min(g0 + e, G - 1) * (4 * CL) + tid];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const bool on = g0 + e < G && ((selbits >> (g0 + e)) & 1ull);
                ac = on ? ac + d[e] : ac;
            }
        }
        const float b1 = (float)hy.beta1, b2 = (float)hy.beta2, al = (float)hy.alpha, ep = (float)hy.eps;
        const float ob1 = (float)(1.0 - hy.beta1), ob2 = (float)(1.0 - hy.beta2);
        hv = fmaf(b1, hv, ob1 * ac);
        const float v = fmaf(b2, vv, ob2 * ac * ac);
        vv = fmaxf(vv, v);
        const float step = al * hv / sqrtf(ep + vv);
        const float nv = tv - step;
        sq = (double)step * (double)step;
        tsq = (double)nv * (double)nv;
        a.agg[jc] = ac;
        a.h[jc] = hv;
        a.vhat[jc] = vv;
        tn[jc] = nv;
        if (a.xtheta)
            __hip_atomic_store(a.xtheta + jc, ((unsigned long long)a.tag << 32) | __float_as_uint(nv), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_SYSTEM);
    }
    // ||step||^2 and ||theta^{k+1}||^2 stay per block: the next launch (or lr_tile_close_kernel)
    // adds them up, so no block waits for the others here
    sq = wave_total(sq);
    tsq = wave_total(tsq);
    unsigned done = 0;
    if (lane == 0) {
        tagged_store(a.xsq + 4 * (int64_t)blk, sq, a.tag);
        tagged_store(a.xsq + 4 * (int64_t)blk + 2, tsq, a.tag);
        if (a.pre) done = __hip_atomic_fetch_add(&ctl->cnt_b, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (!a.pre) return;
    // server-side rule: the next kernel in the stream (the selection) reads the history, so the
    // block that counts itself last collects the per-block sums now (lane i: block i's)
    done = __builtin_amdgcn_readfirstlane(done);
    if (done != (unsigned)S - 1) return;
    double x = 0, y = 0;
    bool gx = lane >= S, gy = gx;
    unsigned spins = 0;
    for (;;) {
        if (!gx) gx = tagged_load(a.xsq + 4 * (int64_t)lane, a.tag, x);
        if (!gy) gy = tagged_load(a.xsq + 4 * (int64_t)lane + 2, a.tag, y);
        if (__all(gx && gy)) break;
        if (++spins > a.wait.limit) {
            if (lane == 0) raise_device_error(ctl, 1u);
            break;
        }
    }
    x = wave_total(x);
    y = wave_total(y);
    if (lane < G) {
        // every block has read the ages and the halves by now
        a.tau[lane] = pre_sel ? 1 : s_tau[lane] + 1;
        if (pre_sel) a.which[lane] = 1 - s_which[lane];
    }
    if (lane == 0) {
        a.nring[hy.kmodD] = x;
        ctl->theta_sq = y;
        __hip_atomic_store(&ctl->cnt_b, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// grid: d / (4*CL) blocks of CL * 16 threads.
template <int CL>
__global__ __launch_bounds__(CL * kFinGroups) void lr_tile_finish_kernel(FinishArgs a)
{
    finish_body<CL, 16, kFinMaxG / kFinGroups>(a, threadIdx.x, blockIdx.x, gridDim.x);
}

// ---- one launch per step: the finish of step k-1 at the head of the tiles of step k -------------
//
// The rows a step reads depend on its row ids only, never on the iterate; what depends on the
// iterate -- the dot products -- comes after the rows have arrived.  So the finish of the step
// before (a chain of short memory round trips on a few workgroups) can run while all workgroups
// wait for their rows: every workgroup requests its tile at once, except the first S, in which
// four waves run the pending finish first (a wave's loads return in order, so a wave with tile
// loads in flight could not get through that chain); the new iterate and the groups' stale
// slots go out as tagged words, and every workgroup picks them up where it needs them.  All
// workgroups of the grid are resident (checked on the host).
template <int WC, int NCH>
__global__ __launch_bounds__(kThreads) void lr_tile_step_kernel(TileArgs a, FinishArgs f, int S)
{
    __shared__ TileShared<WC> sm;
    constexpr int kFinThreads = 16 * kFinGroups;
    const int tid = threadIdx.x;
    const int g = blockIdx.x / a.RB, rb = blockIdx.x % a.RB;
    const ShardDesc sh = a.shards[g];
    const bool fin_block = (int)blockIdx.x < S;
    const bool fin_thread = fin_block && tid < kFinThreads;
    int my_row;
    bool my_valid;
    float4 x[kTR];
    tile_rows<WC>(a, sm, sh, g, rb, my_row, my_valid);
    // (a finishing workgroup requests its tile after the finish: the tile's registers and the
    // finish's do not fit a thread together; its 256 KB arrive while the others still stream)
    if (fin_block) {
        if (fin_thread) {
            finish_body<16, 8, NCH>(f, tid, blockIdx.x, S);
        } else {
            __syncthreads();
            __syncthreads();
        }
    }
    tile_issue<WC>(a, sm, sh, x);
    StepLink link{f.xtheta, f.xsel, f.tag, f.wait, f.ctl};
    tile_finish<WC>(a, sm, sh, g, rb, my_row, my_valid, x, &link);
}

// One wave: completes what the last fused finish left per block -- the history entry
// ||theta^{k+1} - theta^k||^2 (Eq. (9)) and ||theta^{k+1}||^2 -- in the order the next fused launch
// would have used.
__global__ __launch_bounds__(kWave) void lr_tile_close_kernel(const unsigned long long* xsq, unsigned tag,
                                                              int S, int kmodD, double* nring, Ctl* ctl)
{
    const int lane = threadIdx.x;
    double x = 0, y = 0;
    bool ok = true;
    if (lane < S) {
        ok = tagged_load(xsq + 4 * (int64_t)lane, tag, x);
        ok = tagged_load(xsq + 4 * (int64_t)lane + 2, tag, y) && ok;
    }
    if (!__all(ok) && lane == 0) raise_device_error(ctl, 2u);
    x = wave_total(x);
    y = wave_total(y);
    if (lane == 0) {
        nring[kmodD] = x;
        ctl->theta_sq = y;
    }
}

}  // namespace

struct LrTilePlan {
    int WC = 0;           // 0: not applicable
    int R = 0, RB = 0, n_stat = 0;
    float* part_g = nullptr;
    float* part_s = nullptr;
    int fin_CL = 0;       // column lanes of a block of the fused finish; 0: not applicable
    int fin_S = 0;        // its blocks
    unsigned long long* fin_x = nullptr;   // tagged words: [G][S][2] statistics, then 2 x [S][4] sums
    unsigned fin_launches = 0;
    bool fin_pending = false;   // the last fused finish left its two sums per block
    int fin_pending_kmodD = 0;
    unsigned fin_pending_tag = 0;
    hipStream_t fin_stream = nullptr;
    // one launch per step (lr_tile_step_kernel): a second set of tile partials (a step's tiles are
    // written while the finish of the step before reads its own), the words that carry the new
    // iterate and the stale slots, and the step whose finish is still to run
    float* part_g2 = nullptr;
    float* part_s2 = nullptr;
    unsigned long long* xtheta = nullptr;
    unsigned long long* xsel = nullptr;
    bool step_ok = false;       // the shape allows it
    bool step_pending = false;
    Hyper pend_hy{};
    int pend_parity = 0;
    uint8_t* pend_mask_out = nullptr;
    float* pend_loss_out = nullptr;
    hipStream_t pend_stream = nullptr;
};

// The step kernel for a row width (WC column waves) and a group count (NCH passes of 16 groups).
typedef void (*StepKernel)(TileArgs, FinishArgs, int);
template <int WC>
static StepKernel step_kernel_for(int G)
{
    if (G <= kFinGroups) return lr_tile_step_kernel<WC, 1>;
    if (G <= 2 * kFinGroups) return lr_tile_step_kernel<WC, 2>;
    return lr_tile_step_kernel<WC, kFinMaxG / kFinGroups>;
}
static StepKernel step_kernel(int WC, int G)
{
    switch (WC) {
    case 1: return step_kernel_for<1>(G);
    case 2: return step_kernel_for<2>(G);
    case 4: return step_kernel_for<4>(G);
    case 8: return step_kernel_for<8>(G);
    default: return step_kernel_for<16>(G);
    }
}
static hipError_t step_kernel_fits(int WC, int G, int grid, int cus, bool* ok)
{
    int per_cu = 0;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)step_kernel(WC, G), kThreads, 0);
    if (e != hipSuccess) return e;
    *ok = per_cu >= 1 && grid <= cus;            // one workgroup per compute unit: all resident
    return hipSuccess;
}

// Decide whether the single-pass kernel applies (d <= 4096, a multiple of 4, so that a tile holds
// whole rows; lanes past the row's end idle, the last tile of a group may be partly empty) and
// size its scratch.
hipError_t lr_tile_plan(gcada_ctx* c)
{
    auto* pl = new LrTilePlan();
    c->lr_tiles = pl;
    const int d = (int)c->hy.p, mu = c->hy.mu, G = c->hy.G;
    int WC = 0;
    for (int w : {16, 8, 4, 2, 1})
        if (d <= 256 * w) WC = w;
    if (!WC || d % 4 != 0) return hipSuccess;                  // rows that are no whole float4s: other kernels
    const int R = kTR * (kWaves / WC);
    pl->R = R;
    pl->RB = (mu + R - 1) / R;                   // the last tile of a group may be partly empty
    pl->n_stat = (d / 4 + kRedBlock - 1) / kRedBlock;
    const size_t n = (size_t)G * pl->RB * d;
    hipError_t e;
    if ((e = hipMalloc(&pl->part_g, n * sizeof(float))) != hipSuccess) return e;
    if ((e = hipMalloc(&pl->part_s, n * sizeof(float))) != hipSuccess) return e;
    pl->WC = WC;
    c->n_loss_part = std::max(c->n_loss_part, pl->RB);
    c->n_stat_part = std::max(c->n_stat_part, pl->n_stat);
    // fused finish: all of its blocks must be resident at once (they wait for each other)
    hipDeviceProp_t prop;
    if ((e = hipGetDeviceProperties(&prop, c->device)) != hipSuccess) return e;
    if (G <= kFinMaxG) {
        const int CL = 16;
        const int S = (d + 4 * CL - 1) / (4 * CL);
        if (S <= prop.multiProcessorCount && S <= kWave) {
            const size_t words = (size_t)2 * G * S + (size_t)8 * S;
            if ((e = hipMalloc(&pl->fin_x, words * 8)) != hipSuccess) return e;
            if ((e = hipMemset(pl->fin_x, 0, words * 8)) != hipSuccess) return e;    // tag 0: never used
            pl->fin_CL = CL;
            pl->fin_S = S;
            // one launch per step: the grid must hold the S finishing blocks and be resident at once
            const int grid = G * pl->RB;
            bool fits = false;
            if (grid >= S && (e = step_kernel_fits(WC, G, grid, prop.multiProcessorCount, &fits)) != hipSuccess) return e;
            if (fits) {
                if ((e = hipMalloc(&pl->part_g2, n * sizeof(float))) != hipSuccess) return e;
                if ((e = hipMalloc(&pl->part_s2, n * sizeof(float))) != hipSuccess) return e;
                const size_t w2 = (size_t)c->hy.pstride + kFinMaxG;
                if ((e = hipMalloc(&pl->xtheta, w2 * 8)) != hipSuccess) return e;
                if ((e = hipMemset(pl->xtheta, 0, w2 * 8)) != hipSuccess) return e;       // tag 0: never used
                pl->xsel = pl->xtheta + c->hy.pstride;
                c->n_loss_part = std::max(c->n_loss_part, 2 * pl->RB);                    // two sets of loss partials
                pl->step_ok = true;
            }
        }
    }
    return hipSuccess;
}

void lr_tile_free(gcada_ctx* c)
{
    if (!c->lr_tiles) return;
    if (c->lr_tiles->part_g) (void)hipFree(c->lr_tiles->part_g);
    if (c->lr_tiles->part_s) (void)hipFree(c->lr_tiles->part_s);
    if (c->lr_tiles->fin_x) (void)hipFree(c->lr_tiles->fin_x);
    if (c->lr_tiles->part_g2) (void)hipFree(c->lr_tiles->part_g2);
    if (c->lr_tiles->part_s2) (void)hipFree(c->lr_tiles->part_s2);
    if (c->lr_tiles->xtheta) (void)hipFree(c->lr_tiles->xtheta);
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
    c->n_loss_used = c->hy.G * pl->RB;
    if (c->lr_fused_finish) return hipSuccess;    // lr_tile_finish adds the partials itself
    dim3 gr(pl->n_stat, c->hy.G);
    lr_tile_reduce<<<gr, kRedBlock, 0, s>>>(c->hy, pl->part_g, pl->part_s, pl->RB, c->gbuf, c->which,
                                             c->part_stat);
    c->n_stat_used = pl->n_stat;
    return hipGetLastError();
}

// Both rules: the default one (the mask comes from the gradients of this step) and the
// server-side one (the mask is an input).
bool lr_tile_finish_applies(const gcada_ctx* c)
{
    return c->allow_fused_finish && lr_tile_applies(c) && c->lr_tiles->fin_CL != 0;
}

// Arguments of the finish of the step `hy` describes, over the given tile partials; advances the
// launch counter (tags, the two sum buffers in turn) and the history bookkeeping.
static hipError_t finish_args(gcada_ctx* c, const Hyper& hy, const float* part_g, const float* part_s,
                              const double* part_loss, uint8_t* mask_out, float* loss_out, bool preselected,
                              hipStream_t s, FinishArgs& a)
{
    LrTilePlan* pl = c->lr_tiles;
    a = FinishArgs{};
    a.hy = hy; a.part_g = part_g; a.part_s = part_s; a.RB = pl->RB;
    a.part_loss = part_loss; a.n_loss_total = hy.G * pl->RB;
    unsigned long long* sums = pl->fin_x + (size_t)2 * hy.G * pl->fin_S;
    const unsigned n = pl->fin_launches++;
    a.xstat = pl->fin_x;
    a.xsq = sums + (size_t)(n & 1u) * 4 * pl->fin_S;            // two buffers in turn: the other one
    a.xsq_prev = sums + (size_t)((n & 1u) ^ 1u) * 4 * pl->fin_S;   // is read while this one is written
    // tags 1 .. 2^32-1 in turn: a slot only ever holds the tag of an earlier launch
    a.tag = n % 0xffffffffu + 1u;
    a.wait = c->wait_policy();
    a.pre = preselected ? 1 : 0;
    if (preselected && pl->fin_pending) return hipErrorInvalidValue;   // the caller completes the history first
    a.fold_prev = pl->fin_pending ? 1 : 0;
    a.tag_prev = pl->fin_pending_tag;
    a.prev_kmodD = pl->fin_pending_kmodD;
    pl->fin_pending = !preselected;          // the server-side variant closes its history entry itself
    pl->fin_pending_kmodD = hy.kmodD;
    pl->fin_pending_tag = a.tag;
    pl->fin_stream = s;
    a.stat = c->stat; a.mask = c->mask; a.mask_out = mask_out; a.loss_out = loss_out;
    a.gbuf = c->gbuf; a.which = c->which; a.agg = c->agg; a.h = c->h; a.vhat = c->vhat;
    a.ring = c->ring; a.nring = c->nring; a.tau = c->tau; a.ctl = c->ctl;
    // every buffer the kernel dereferences unconditionally (mask_out and loss_out may be null)
    for (const void* q : {(const void*)a.part_g, (const void*)a.part_s, (const void*)a.part_loss,
                          (const void*)a.xstat, (const void*)a.xsq, (const void*)a.xsq_prev,
                          (const void*)a.stat, (const void*)a.mask, (const void*)a.gbuf,
                          (const void*)a.which, (const void*)a.agg, (const void*)a.h,
                          (const void*)a.vhat, (const void*)a.ring, (const void*)a.nring,
                          (const void*)a.tau, (const void*)a.ctl})
        if (!q) return hipErrorInvalidValue;
    if ((int64_t)pl->fin_S * pl->fin_CL * 4 < hy.p || hy.p % 4 != 0) return hipErrorInvalidValue;
    return hipSuccess;
}

// Tile reduce + selection + masked innovation sum + server update in one launch; replaces
// lr_tile_reduce and server_step after lr_tile_gradients.
hipError_t lr_tile_finish(gcada_ctx* c, uint8_t* mask_out, float* loss_out, bool preselected, hipStream_t s)
{
    LrTilePlan* pl = c->lr_tiles;
    if (c->n_loss_used != c->hy.G * pl->RB) return hipErrorInvalidValue;
    FinishArgs a;
    hipError_t e = finish_args(c, c->hy, pl->part_g, pl->part_s, c->part_loss, mask_out, loss_out, preselected, s, a);
    if (e != hipSuccess) return e;
    lr_tile_finish_kernel<16><<<pl->fin_S, 16 * kFinGroups, 0, s>>>(a);
    return hipGetLastError();
}

// ---- one launch per step ----------------------------------------------------------------------
bool lr_tile_step_applies(const gcada_ctx* c)
{
    return c->allow_deferred_finish && c->rule == GCADA_RULE_GRADIENT_DIFFERENCE && lr_tile_finish_applies(c) &&
           c->lr_tiles->step_ok;
}

bool lr_tile_step_pending(const gcada_ctx* c) { return c->lr_tiles && c->lr_tiles->step_pending; }

// Step c->hy.k: its tiles, and -- in the same launch -- the finish of the step before, if that is
// still to run.  The finish of THIS step runs with the next call (or lr_tile_flush): mask_out and
// loss_out are written then.
hipError_t lr_tile_step(gcada_ctx* c, const int32_t* idx, uint8_t* mask_out, float* loss_out, hipStream_t s)
{
    LrTilePlan* pl = c->lr_tiles;
    const int parity = (int)(c->hy.k & 1);
    const int grid = c->hy.G * pl->RB;
    TileArgs a{};
    a.hy = c->hy; a.shards = c->d_shards; a.idx = idx; a.ring = c->ring; a.tau = c->tau;
    a.part_g = parity ? pl->part_g2 : pl->part_g;
    a.part_s = parity ? pl->part_s2 : pl->part_s;
    a.part_loss = c->part_loss + (size_t)parity * grid;
    a.RB = pl->RB;
    if (!pl->step_pending) {
        // nothing to finish: the state is complete, the plain tile kernel reads it
        switch (pl->WC) {
        case 1: lr_tile_kernel<1><<<grid, kThreads, 0, s>>>(a); break;
        case 2: lr_tile_kernel<2><<<grid, kThreads, 0, s>>>(a); break;
        case 4: lr_tile_kernel<4><<<grid, kThreads, 0, s>>>(a); break;
        case 8: lr_tile_kernel<8><<<grid, kThreads, 0, s>>>(a); break;
        default: lr_tile_kernel<16><<<grid, kThreads, 0, s>>>(a); break;
        }
    } else {
        const int pp = pl->pend_parity;
        FinishArgs f;
        hipError_t e = finish_args(c, pl->pend_hy, pp ? pl->part_g2 : pl->part_g, pp ? pl->part_s2 : pl->part_s,
                                   c->part_loss + (size_t)pp * grid, pl->pend_mask_out, pl->pend_loss_out, false, s, f);
        if (e != hipSuccess) return e;
        f.xtheta = pl->xtheta;
        f.xsel = pl->xsel;
        if (pp == parity || !f.xtheta || grid < pl->fin_S) return hipErrorInvalidValue;
        step_kernel(pl->WC, c->hy.G)<<<grid, kThreads, 0, s>>>(a, f, pl->fin_S);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    pl->step_pending = true;
    pl->pend_hy = c->hy;
    pl->pend_parity = parity;
    pl->pend_mask_out = mask_out;
    pl->pend_loss_out = loss_out;
    pl->pend_stream = s;
    return hipSuccess;
}

// Run the finish that is still to come (on `s`, or on the stream of its step when use_step_stream).
hipError_t lr_tile_flush(gcada_ctx* c, hipStream_t s, bool use_step_stream)
{
    LrTilePlan* pl = c->lr_tiles;
    if (!pl || !pl->step_pending) return hipSuccess;
    if (use_step_stream) s = pl->pend_stream;
    const int pp = pl->pend_parity;
    const int grid = pl->pend_hy.G * pl->RB;
    FinishArgs f;
    hipError_t e = finish_args(c, pl->pend_hy, pp ? pl->part_g2 : pl->part_g, pp ? pl->part_s2 : pl->part_s,
                               c->part_loss + (size_t)pp * grid, pl->pend_mask_out, pl->pend_loss_out, false, s, f);
    if (e != hipSuccess) return e;
    pl->step_pending = false;
    lr_tile_finish_kernel<16><<<pl->fin_S, 16 * kFinGroups, 0, s>>>(f);
    return hipGetLastError();
}

// Complete the history entry and ||theta||^2 of the last fused finish, if they are still per
// block: before anything other than the next fused finish reads them.  On the stream of that
// step when `s` is null.
hipError_t lr_tile_close(gcada_ctx* c, hipStream_t s, bool use_step_stream)
{
    LrTilePlan* pl = c->lr_tiles;
    if (!pl || !pl->fin_pending) return hipSuccess;
    const unsigned n = pl->fin_launches - 1;
    const unsigned long long* sums = pl->fin_x + (size_t)2 * c->hy.G * pl->fin_S + (size_t)(n & 1u) * 4 * pl->fin_S;
    lr_tile_close_kernel<<<1, kWave, 0, use_step_stream ? pl->fin_stream : s>>>(
        sums, pl->fin_pending_tag, pl->fin_S, pl->fin_pending_kmodD, c->nring, c->ctl);
    pl->fin_pending = false;
    return hipGetLastError();
}

// The state was replaced from outside: nothing of the last fused finish is pending any more.
void lr_tile_forget(gcada_ctx* c)
{
    if (c->lr_tiles) {
        c->lr_tiles->fin_pending = false;
        c->lr_tiles->step_pending = false;       // (its mask and loss are never written)
    }
}

}  // namespace gcada
