// Single-pass logistic-regression gradients for wide rows (d a multiple of 4096, d >= 8192):
// step a1 for shapes whose rows do not fit one workgroup's registers (paper Sec. II-A).
//
// A TEAM of TS = d/4096 workgroups shares the rows of a tile: member m keeps columns
// [4096 m, 4096 (m+1)) of R = 4 rows in registers (two float4 per row and thread).  Every member
// forms its partial dot products and publishes them (64 bytes) in a small exchange buffer; TWO
// TILES LATER it collects the partials of all members, forms the residuals and adds the tile's
// contribution to its 4096 columns of the two weighted row sums straight from the registers.
// Four register tiles are live per thread (loading / multiplied / waiting / added), so the
// exchange latency hides behind two tiles of loads and the minibatch is read from HBM exactly
// once.  A member owns its columns for all rows of a group: the column sums never leave
// registers until the group is finished, and no partial sums are written.
//
// Exchange protocol (no read-modify-write atomics, no fences): a partial is eight 8-byte pairs
// {value, tag}; tag = sequence number of the tile, so a pair is valid exactly when its tag
// matches.  Pairs are written and read with system-scope cache policy (sc0 sc1), i.e. past the
// non-coherent L2 of the 8 XCDs.  Four slots per team: a member that publishes tile t has seen
// every member's tile t-2, and a member that has published tile t-2 has already consumed tile
// t-4, whose slot tile t takes.  Every wait is bounded; when a bound is hit the kernel raises
// Ctl::error and runs to its end without waiting again.
//
// One workgroup barrier per tile: wave 0 forms the residuals of tile t-2 before the barrier of
// stage t and publishes the partials of tile t after it; the two small LDS arrays involved are
// double-buffered by the parity of t.
#include "lr_device.h"

namespace gcada {

namespace {

constexpr int kThreads = 512;
constexpr int kWaves = 8;
constexpr int kV = 2;                    // float4 per row and thread, 256 columns apart
constexpr int kR = 4;                    // rows per tile
constexpr int kSlab = 4096;              // columns per member
constexpr int kSlots = 4;
constexpr int kTiles = 4;                // register tiles per thread
constexpr int kPartial = 2 * kR;         // values a member publishes per tile
constexpr int kSlotBytes = kPartial * 8; // per member and slot
constexpr unsigned kPollLimit = 1u << 16;
constexpr int kCoherent = 17;            // buffer cache policy: sc0 | sc1

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

struct TeamArgs {
    Hyper hy;
    const ShardDesc* shards;
    const int32_t* idx;
    const float* ring;
    const int32_t* tau;
    Ctl* ctl;
    void* xch;               // [NT][kSlots][TS][kPartial] pairs {value, tag}
    float* gbuf;
    const int32_t* which;
    double* part_stat;       // [G][TS]
    double* part_loss;       // [G]
    int TS, NT;
    unsigned tag_base;       // tags of this launch are tag_base + tile sequence number
};

// workgroup id -> (team, member).  Consecutive workgroup ids go to different XCDs (id mod 8); a
// team is made of ids congruent mod 8 when it fits, so that its exchange stays near one L2.
__device__ __forceinline__ void team_of(int wg, int TS, int nWG, int& team, int& m)
{
    const int per_xcd = nWG / 8;
    if (nWG % 8 == 0 && per_xcd % TS == 0) {
        const int xcd = wg % 8, slot = wg / 8;
        team = xcd * (per_xcd / TS) + slot / TS;
        m = slot % TS;
    } else {
        team = wg / TS;
        m = wg % TS;
    }
}

// Per-thread state of one group's pass that the stages share.
struct TeamRegs {
    float4 xb[kTiles][kR][kV];   // register tiles; tile t lives in xb[t % kTiles]
    float yl[kTiles];            // labels of the tile's rows (wave 0, lanes < kR)
    float4 th4[kV], dl4[kV];     // theta^k and theta^k - theta_stale at this thread's columns
    float4 ag[kV], as[kV];       // column sums of r_i x_i and dr_i x_i
    int rows_nxt[kR];            // row ids of the tile that is loaded next (wave-uniform)
    double lacc;                 // loss (wave 0, lanes < kR)
};

// One pipeline stage; J = t mod 4 is a compile-time constant so that every tile index is static.
//   tile t+1 starts loading, tile t is multiplied and published, tile t-2 gets its residuals
//   and is added.  seq0 = sequence number of the group's tile 0.
template <int J>
__device__ __forceinline__ void team_stage(const TeamArgs& a, TeamRegs& R, const ShardDesc& sh,
                                           __amdgpu_buffer_rsrc_t xr, int t, int ntile, int g, int m,
                                           int col, unsigned seq0, unsigned cyc_base, bool& gave_up,
                                           float (&s_dot)[2][kWaves][kPartial], float2 (&s_res)[2][kR])
{
    constexpr int JN = (J + 1) % kTiles, JC = J, JA = (J + 2) % kTiles;   // loading, current, added
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const bool have_load = t + 1 < ntile, have_cur = t < ntile, have_add = t >= 2;
    const bool poller = wave == 0 && lane < a.TS * kR;
    typedef const int32_t __attribute__((address_space(4))) const_i32;

    // the poll goes out before this stage's tile loads, so it also comes back before them; the
    // partials it reads were published two stages ago
    u32x4 pol = {0u, 0u, 0u, 0u};
    const int poll_off = (int)((seq0 + (unsigned)t - 2u) % kSlots) * a.TS * kSlotBytes + lane * 16;
    if (have_add && poller) pol = __builtin_amdgcn_raw_buffer_load_b128(xr, poll_off, 0, kCoherent);

    if (have_load) {
        if (wave == 0 && lane < kR) {
            int myrow = R.rows_nxt[0];
#pragma unroll
            for (int u = 1; u < kR; ++u) myrow = lane == u ? R.rows_nxt[u] : myrow;
            R.yl[JN] = global_load((const float*)sh.y + myrow);
        }
#pragma unroll
        for (int u = 0; u < kR; ++u) {
            const float* xrow = (const float*)sh.X + (int64_t)R.rows_nxt[u] * sh.ld + col;
#pragma unroll
            for (int q = 0; q < kV; ++q) R.xb[JN][u][q] = global_load4(xrow + 256 * q);
        }
    }
    // row ids of tile t+2 through scalar loads (constant address space, uniform address): they
    // are counted apart from the vector loads, so fetching them never waits for a tile in flight
#pragma unroll
    for (int u = 0; u < kR; ++u) {
        int rr = 0;
        if (t + 2 < ntile) {
            if (a.idx) rr = ((const_i32*)(uintptr_t)a.idx)[(int64_t)g * a.hy.mu + (t + 2) * kR + u];
            else rr = (int)((cyc_base + (unsigned)((t + 2) * kR + u)) % (unsigned)sh.rows);
        }
        R.rows_nxt[u] = __builtin_amdgcn_readfirstlane(rr);
    }

    // wave 0: residuals of tile t-2 from all members' partials
    if (have_add && wave == 0) {
        const unsigned want = a.tag_base + seq0 + (unsigned)t - 2u;
        unsigned spins = 0;
        bool ok = !poller || (pol.y == want && pol.w == want);
        while (!gave_up && !__all(ok)) {
            if (poller && !ok) {
                pol = __builtin_amdgcn_raw_buffer_load_b128(xr, poll_off, 0, kCoherent);
                ok = pol.y == want && pol.w == want;
            }
            if (++spins > kPollLimit) {
                if (lane == 0)
                    __hip_atomic_fetch_or(&a.ctl->error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                gave_up = true;
            }
        }
        // lane l holds member l/4's partial (z, dz) of row l%4: add the members in a fixed tree
        float z = poller ? __uint_as_float(pol.x) : 0.0f;
        float dz = poller ? __uint_as_float(pol.z) : 0.0f;
#pragma unroll
        for (int o = kR; o < kWave; o <<= 1) {
            z += __shfl_xor(z, o, kWave);
            dz += __shfl_xor(dz, o, kWave);
        }
        if (lane < kR) {
            float r, dr, ls;
            residuals(z, dz, R.yl[JA], r, dr, ls);
            s_res[t & 1][lane] = make_float2(r, dr);
            R.lacc += (double)ls;
        }
    }

    if (have_cur) {
        float v[kPartial];
#pragma unroll
        for (int u = 0; u < kR; ++u) {
            float s0 = 0.0f, s1 = 0.0f;
#pragma unroll
            for (int q = 0; q < kV; ++q) {
                const float4 x4 = R.xb[JC][u][q];
                s0 += x4.x * R.th4[q].x + x4.y * R.th4[q].y + x4.z * R.th4[q].z + x4.w * R.th4[q].w;
                s1 += x4.x * R.dl4[q].x + x4.y * R.dl4[q].y + x4.z * R.dl4[q].z + x4.w * R.dl4[q].w;
            }
            v[2 * u] = s0;
            v[2 * u + 1] = s1;
        }
        Butterfly<kPartial, 32>::run(v, lane);       // lanes 8e hold value e
        if ((lane & 7) == 0) s_dot[t & 1][wave][lane >> 3] = v[0];
    }
    __syncthreads();

    if (have_cur && wave == 0) {
        // member partial: lane l adds value l%8 over the waves in a fixed tree, lanes < 8 publish
        float w = s_dot[t & 1][lane >> 3][lane & 7];
#pragma unroll
        for (int o = 8; o < kWave; o <<= 1) w += __shfl_xor(w, o, kWave);
        if (lane < kPartial) {
            const unsigned seq = seq0 + (unsigned)t;
            const u32x2 pr = {__float_as_uint(w), a.tag_base + seq};
            __builtin_amdgcn_raw_buffer_store_b64(pr, xr, ((int)(seq % kSlots) * a.TS + m) * kSlotBytes + lane * 8,
                                                  0, kCoherent);
        }
    }
    if (have_add) {
#pragma unroll
        for (int u = 0; u < kR; ++u) {
            const float2 w2 = s_res[t & 1][u];
#pragma unroll
            for (int q = 0; q < kV; ++q) {
                const float4 x4 = R.xb[JA][u][q];
                R.ag[q].x += w2.x * x4.x; R.ag[q].y += w2.x * x4.y; R.ag[q].z += w2.x * x4.z; R.ag[q].w += w2.x * x4.w;
                R.as[q].x += w2.y * x4.x; R.as[q].y += w2.y * x4.y; R.as[q].z += w2.y * x4.z; R.as[q].w += w2.y * x4.w;
            }
        }
    }
}

// grid: NT * TS workgroups of 512 threads, all resident at once (checked on the host).
__global__ __launch_bounds__(kThreads) void lr_team_kernel(TeamArgs a)
{
    __shared__ float s_dot[2][kWaves][kPartial];  // per-wave partial dots, by parity of the tile
    __shared__ float2 s_res[2][kR];               // residuals (r, dr), by parity of the stage
    __shared__ double s_red[kWaves];

    const Hyper& hy = a.hy;
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    int team, m;
    team_of(blockIdx.x, a.TS, a.NT * a.TS, team, m);
    const int mu = hy.mu;
    const int col = m * kSlab + wave * (256 * kV) + lane * 4;    // and col + 256
    const int ntile = mu / kR;
    __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(
        (char*)a.xch + (int64_t)team * kSlots * a.TS * kSlotBytes, 0, kSlots * a.TS * kSlotBytes, 0x00020000);
    unsigned seq0 = 0;                           // sequence number of the group's first tile
    bool gave_up = false;                        // wave 0: a bounded wait was exhausted
    typedef const int32_t __attribute__((address_space(4))) const_i32;

    TeamRegs R;
#pragma unroll
    for (int q = 0; q < kV; ++q)
        R.th4[q] = *(const float4*)(a.ring + (int64_t)hy.cur * hy.pstride + col + 256 * q);
#pragma unroll
    for (int j = 0; j < kTiles; ++j) R.yl[j] = 1.0f;

    for (int g = team; g < hy.G; g += a.NT, seq0 += (unsigned)ntile) {
        const ShardDesc sh = a.shards[g];
        {
            const float* stale = a.ring + (int64_t)stale_slot_of(hy, a.tau[g]) * hy.pstride + col;
#pragma unroll
            for (int q = 0; q < kV; ++q) {
                const float4 u4 = *(const float4*)(stale + 256 * q);
                R.dl4[q] = make_float4(R.th4[q].x - u4.x, R.th4[q].y - u4.y, R.th4[q].z - u4.z, R.th4[q].w - u4.w);
                R.ag[q] = make_float4(0, 0, 0, 0);
                R.as[q] = make_float4(0, 0, 0, 0);
            }
        }
        R.lacc = 0;
        // cyclic window: first row of this step's window, (k * mu) mod rows, in 32 bits
        const unsigned cyc_base = (unsigned)((((unsigned long long)hy.k % (unsigned long long)sh.rows) *
                                              ((unsigned long long)mu % (unsigned long long)sh.rows)) %
                                             (unsigned long long)sh.rows);
        // prologue: tile 0 starts loading, row ids of tile 1
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
            for (int u = 0; u < kR; ++u) {
                int rr = 0;
                if (pass < ntile) {
                    if (a.idx) rr = ((const_i32*)(uintptr_t)a.idx)[(int64_t)g * mu + pass * kR + u];
                    else rr = (int)((cyc_base + (unsigned)(pass * kR + u)) % (unsigned)sh.rows);
                }
                R.rows_nxt[u] = __builtin_amdgcn_readfirstlane(rr);
            }
            if (pass == 0) {
                if (wave == 0 && lane < kR) {
                    int myrow = R.rows_nxt[0];
#pragma unroll
                    for (int u = 1; u < kR; ++u) myrow = lane == u ? R.rows_nxt[u] : myrow;
                    R.yl[0] = global_load((const float*)sh.y + myrow);
                }
#pragma unroll
                for (int u = 0; u < kR; ++u) {
                    const float* xrow = (const float*)sh.X + (int64_t)R.rows_nxt[u] * sh.ld + col;
#pragma unroll
                    for (int q = 0; q < kV; ++q) R.xb[0][u][q] = global_load4(xrow + 256 * q);
                }
            }
        }
        // stages 0 .. ntile+1 (the last two only drain)
        const int last = ntile + 1;
        for (int t = 0; t <= last; t += kTiles) {
            team_stage<0>(a, R, sh, xr, t, ntile, g, m, col, seq0, cyc_base, gave_up, s_dot, s_res);
            if (t + 1 > last) break;
            team_stage<1>(a, R, sh, xr, t + 1, ntile, g, m, col, seq0, cyc_base, gave_up, s_dot, s_res);
            if (t + 2 > last) break;
            team_stage<2>(a, R, sh, xr, t + 2, ntile, g, m, col, seq0, cyc_base, gave_up, s_dot, s_res);
            if (t + 3 > last) break;
            team_stage<3>(a, R, sh, xr, t + 3, ntile, g, m, col, seq0, cyc_base, gave_up, s_dot, s_res);
        }

        // the group is finished: this member's 4096 columns of the gradient and of s_g
        double sq = 0;
        float* out = fresh_row(a.gbuf, a.which, hy, g) + col;
#pragma unroll
        for (int q = 0; q < kV; ++q) {
            if (hy.l2 != 0.0f) {
                const float ml = (float)mu * hy.l2;
                R.ag[q].x += ml * R.th4[q].x; R.ag[q].y += ml * R.th4[q].y; R.ag[q].z += ml * R.th4[q].z; R.ag[q].w += ml * R.th4[q].w;
                R.as[q].x += ml * R.dl4[q].x; R.as[q].y += ml * R.dl4[q].y; R.as[q].z += ml * R.dl4[q].z; R.as[q].w += ml * R.dl4[q].w;
            }
            *(float4*)(out + 256 * q) = R.ag[q];
            sq += (double)R.as[q].x * R.as[q].x + (double)R.as[q].y * R.as[q].y + (double)R.as[q].z * R.as[q].z +
                  (double)R.as[q].w * R.as[q].w;
        }
        sq = wave_sum(sq);
        __syncthreads();
        if (lane == 0) s_red[wave] = sq;
        __syncthreads();
        if (tid == 0) {
            double tsum = 0;
            for (int wv = 0; wv < kWaves; ++wv) tsum += s_red[wv];
            a.part_stat[(int64_t)g * a.TS + m] = tsum;
        }
        if (m == 0 && wave == 0) {
            double l = lane < kR ? R.lacc : 0.0;
            l = wave_sum(l);
            if (lane == 0) a.part_loss[g] = l;
        }
        __syncthreads();
    }
}

}  // namespace

struct LrTeamPlan {
    int TS = 0, NT = 0;      // TS = 0: not applicable
    void* xch = nullptr;
};

// Decide whether the team kernel applies (d a multiple of 4096 and at least 8192, mu a multiple
// of the tile's rows, a whole number of teams fits the device with every workgroup resident).
hipError_t lr_team_plan(gcada_ctx* c)
{
    auto* pl = new LrTeamPlan();
    c->lr_team = pl;
    const int d = (int)c->hy.p, mu = c->hy.mu;
    if (d % kSlab || d < 2 * kSlab || mu % kR) return hipSuccess;
    const int TS = d / kSlab;
    if (TS * kR > kWave) return hipSuccess;          // one wave polls all members' partials
    hipDeviceProp_t prop;
    hipError_t e = hipGetDeviceProperties(&prop, c->device);
    if (e != hipSuccess) return e;
    int per_cu = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)lr_team_kernel, kThreads, 0);
    if (e != hipSuccess) return e;
    const int cap = per_cu > 0 ? prop.multiProcessorCount : 0;     // one workgroup per CU
    const int NT = cap / TS;
    if (NT < 1) return hipSuccess;
    const size_t n = (size_t)NT * kSlots * TS * kSlotBytes;
    if ((e = hipMalloc(&pl->xch, n)) != hipSuccess) return e;
    if ((e = hipMemset(pl->xch, 0, n)) != hipSuccess) return e;
    pl->TS = TS;
    pl->NT = NT;
    c->n_stat_part = std::max(c->n_stat_part, TS);
    c->n_loss_part = std::max(c->n_loss_part, 1);
    return hipSuccess;
}

void lr_team_free(gcada_ctx* c)
{
    if (!c->lr_team) return;
    if (c->lr_team->xch) (void)hipFree(c->lr_team->xch);
    delete c->lr_team;
    c->lr_team = nullptr;
}

bool lr_team_applies(const gcada_ctx* c)
{
    if (!c->allow_single_pass || !c->lr_team || c->lr_team->TS == 0) return false;
    for (const auto& s : c->shards)
        if ((s.ld % 4) || ((uintptr_t)s.X % 16)) return false;
    return true;
}

hipError_t lr_team_reset(gcada_ctx* c)
{
    if (!c->lr_team || c->lr_team->TS == 0) return hipSuccess;
    const size_t n = (size_t)c->lr_team->NT * kSlots * c->lr_team->TS * kSlotBytes;
    c->team_launches = 0;
    return hipMemset(c->lr_team->xch, 0, n);
}

hipError_t lr_team_gradients(gcada_ctx* c, const int32_t* idx, hipStream_t s)
{
    const LrTeamPlan* pl = c->lr_team;
    TeamArgs a{};
    a.hy = c->hy; a.shards = c->d_shards; a.idx = idx; a.ring = c->ring; a.tau = c->tau;
    a.ctl = c->ctl; a.xch = pl->xch; a.gbuf = c->gbuf; a.which = c->which;
    a.part_stat = c->part_stat; a.part_loss = c->part_loss;
    a.TS = pl->TS; a.NT = pl->NT;
    // tags never repeat within the four-slot window: 2^20 tiles per launch at most, and the
    // launch counter advances the base (wrap-around after 4096 launches lands on tags long gone)
    const unsigned tiles = (unsigned)((c->hy.G + pl->NT - 1) / pl->NT) * (unsigned)(c->hy.mu / kR);
    a.tag_base = (unsigned)((c->team_launches++ % 4095u) + 1u) << 20;
    if (tiles >= (1u << 20)) return hipErrorInvalidValue;
    lr_team_kernel<<<pl->NT * pl->TS, kThreads, 0, s>>>(a);
    c->n_stat_used = pl->TS;
    c->n_loss_used = c->hy.G;
    return hipGetLastError();
}

}  // namespace gcada
