// Single-pass logistic-regression gradients for wide rows (d a multiple of 4096, d >= 8192):
// step a1 for shapes whose rows do not fit one workgroup's registers (paper Sec. II-A).
//
// A TEAM of TS = d/4096 workgroups shares the rows of a tile: member m keeps columns
// [4096 m, 4096 (m+1)) of R = 4 rows in registers (two float4 per row and thread).  Every member
// forms its partial dot products, publishes them (48 bytes) in a small exchange buffer and, ONE
// TILE LATER, collects the partials of all members, forms the residuals and adds the tile's
// contribution to its 4096 columns of the two weighted row sums straight from the registers.
// Three register tiles are in flight per thread (being loaded / multiplied / waiting for the
// residuals), so the exchange latency hides behind the next tile's load and the minibatch is
// read from HBM exactly once.  A member owns its columns for all rows of a group: the column
// sums never leave registers until the group is finished, and no partial sums are written.
//
// Exchange protocol (no read-modify-write atomics, no fences): a partial is three 16-byte chunks
// {value, value, value, tag}; tag = sequence number of the tile, so a chunk is valid exactly when
// its tag matches.  Chunks are written and read with system-scope cache policy (sc0 sc1), i.e.
// past the non-coherent L2 of the 8 XCDs.  Four slots per team: a slot is reused only after every
// member has consumed it (a member publishes tile t+3 only after all members published t+1,
// which they do after consuming t-1).  Every wait is bounded; when a bound is hit the kernel
// raises Ctl::error and runs to its end without waiting again.
#include "gcada_internal.h"

namespace gcada {

namespace {

constexpr int kWave = 64;
constexpr int kThreads = 512;
constexpr int kWaves = 8;
constexpr int kV = 2;                    // float4 per row and thread, 256 columns apart
constexpr int kR = 4;                    // rows per tile
constexpr int kSlab = 4096;              // columns per member
constexpr int kSlots = 4;
constexpr int kChunks = 3;               // 16-byte chunks per partial (8 floats + tags)
constexpr unsigned kPollLimit = 1u << 16;
constexpr int kCoherent = 17;            // buffer cache policy: sc0 | sc1

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

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

__device__ __forceinline__ float sigmoidf_(float t)
{
    const float e = expf(-fabsf(t));
    const float s = 1.0f / (1.0f + e);
    return t >= 0 ? s : e * s;
}

// r = residual at theta^k, dr = r - (residual at theta_stale), from z = x.theta^k and
// dz = x.(theta^k - theta_stale), the difference of the sigmoids formed without cancellation.
__device__ __forceinline__ void residuals(float z, float dz, float y, float& r, float& dr, float& loss)
{
    const float a = -y * z;
    const float sa = sigmoidf_(a);
    r = -y * sa;
    const float t = y * dz;
    const float b = a + t;
    float dsig;
    if (fabsf(t) < 0.5f)
        dsig = -sa * sigmoidf_(-b) * expm1f(t);
    else
        dsig = sa - sigmoidf_(b);
    dr = -y * dsig;
    loss = fmaxf(a, 0.0f) + log1pf(expf(-fabsf(a)));
}

struct TeamArgs {
    Hyper hy;
    const ShardDesc* shards;
    const int32_t* idx;
    const float* ring;
    const int32_t* tau;
    Ctl* ctl;
    u32x4* xch;              // [NT][kSlots][TS][kChunks]
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

// grid: NT * TS workgroups of 512 threads, all resident at once (checked on the host).
__global__ __launch_bounds__(kThreads) void lr_team_kernel(TeamArgs a)
{
    __shared__ float s_dot[kWaves][2 * kR];     // per-wave partial dots of the current tile
    __shared__ float s_x[kWave / kChunks][2 * kR];   // the members' partials of the previous tile
    __shared__ float2 s_res[kR];
    __shared__ double s_red[kWaves];

    const Hyper& hy = a.hy;
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    int team, m;
    team_of(blockIdx.x, a.TS, a.NT * a.TS, team, m);
    const int mu = hy.mu;
    const int col = m * kSlab + wave * (256 * kV) + lane * 4;    // and col + 256
    float4 th4[kV];
#pragma unroll
    for (int q = 0; q < kV; ++q) th4[q] = *(const float4*)(a.ring + (int64_t)hy.cur * hy.pstride + col + 256 * q);
    const int ntile = mu / kR;
    __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(a.xch + (int64_t)team * kSlots * a.TS * kChunks), 0, kSlots * a.TS * kChunks * 16, 0x00020000);
    unsigned seq = 0;                            // tile sequence number within this launch
    bool gave_up = false;                        // wave 0: a bounded wait was exhausted
    // row ids come through scalar loads (constant address space, uniform address): they are
    // tracked separately from the vector loads of the tiles, so fetching them never waits for a
    // tile in flight
    typedef const int32_t __attribute__((address_space(4))) const_i32;
    const_i32* idxc = (const_i32*)(uintptr_t)a.idx;

    for (int g = team; g < hy.G; g += a.NT) {
        const ShardDesc sh = a.shards[g];
        const float* __restrict__ X = (const float*)sh.X;
        const float* __restrict__ Y = (const float*)sh.y;
        float4 dl4[kV], ag[kV], as[kV];
        {
            const float* stale = a.ring + (int64_t)stale_slot_of(hy, a.tau[g]) * hy.pstride + col;
#pragma unroll
            for (int q = 0; q < kV; ++q) {
                const float4 u4 = *(const float4*)(stale + 256 * q);
                dl4[q] = make_float4(th4[q].x - u4.x, th4[q].y - u4.y, th4[q].z - u4.z, th4[q].w - u4.w);
                ag[q] = make_float4(0, 0, 0, 0);
                as[q] = make_float4(0, 0, 0, 0);
            }
        }
        double lacc = 0;                         // member 0, lanes < kR of wave 0
        float4 xb0[kR][kV], xb1[kR][kV], xb2[kR][kV];   // the three register tiles
        int rows_nxt[kR];                        // row ids of the tile after the next one
        float y0 = 1.0f, y1 = 1.0f, y2 = 1.0f;   // labels of the rows in xb0..xb2 (wave 0, lanes < kR)
        // cyclic window: first row of this step's window, (k * mu) mod rows, in 32 bits
        const unsigned cyc_base = (unsigned)((((unsigned long long)hy.k % (unsigned long long)sh.rows) *
                                              ((unsigned long long)mu % (unsigned long long)sh.rows)) %
                                             (unsigned long long)sh.rows);

        // row ids are fetched one tile ahead of the loads that use them
#define GCADA_FETCH_ROWS(T)                                                                          \
    _Pragma("unroll") for (int u = 0; u < kR; ++u) {                                                 \
        int rr = 0;                                                                                  \
        if ((T) < ntile) {                                                                           \
            if (a.idx) rr = idxc[(int64_t)g * mu + (T) * kR + u];                                    \
            else rr = (int)((cyc_base + (unsigned)((T) * kR + u)) % (unsigned)sh.rows);              \
        }                                                                                            \
        rows_nxt[u] = __builtin_amdgcn_readfirstlane(rr);                                                                          \
    }
#define GCADA_LOAD_TILE(XB, YB)                                                          \
    if (wave == 0 && lane < kR) {                                                        \
        int myrow = rows_nxt[0];                                                         \
        _Pragma("unroll") for (int u = 1; u < kR; ++u) myrow = lane == u ? rows_nxt[u] : myrow; \
        YB = global_load(Y + myrow);                                                                 \
    }                                                                                    \
    _Pragma("unroll") for (int u = 0; u < kR; ++u) {                                     \
        const float* xrow = X + (int64_t)rows_nxt[u] * sh.ld + col;                      \
        _Pragma("unroll") for (int q = 0; q < kV; ++q) XB[u][q] = global_load4(xrow + 256 * q); \
    }

        // One pipeline stage: tile t is multiplied and published (from XC), tile t+1 starts
        // loading (into XN), tile t-1 gets its residuals and is added (from XP).
#define GCADA_STAGE(XP, XC, XN, YP, YN)                                                                     \
    {                                                                                               \
        const bool have_cur = t < ntile, have_prev = t >= 1;                                        \
        u32x4 pol = {0u, 0u, 0u, 0u};                                                               \
        const int pslot = (int)((seq + kSlots - 1) % kSlots);                                       \
        const bool poller = wave == 0 && lane < a.TS * kChunks;                                     \
        if (have_prev && poller)   /* issued before this iteration's tile loads: returns first */  \
            pol = __builtin_amdgcn_raw_buffer_load_b128(xr, (pslot * a.TS * kChunks + lane) * 16, 0, kCoherent); \
        if (t + 1 < ntile) { GCADA_LOAD_TILE(XN, YN) }                                              \
        GCADA_FETCH_ROWS(t + 2)                                                                     \
        if (have_cur) {                                                                             \
            float v[2 * kR];                                                                        \
            _Pragma("unroll") for (int u = 0; u < kR; ++u) {                                        \
                float s0 = 0.0f, s1 = 0.0f;                                                         \
                _Pragma("unroll") for (int q = 0; q < kV; ++q) {                                    \
                    const float4 x4 = XC[u][q];                                                     \
                    s0 += x4.x * th4[q].x + x4.y * th4[q].y + x4.z * th4[q].z + x4.w * th4[q].w;    \
                    s1 += x4.x * dl4[q].x + x4.y * dl4[q].y + x4.z * dl4[q].z + x4.w * dl4[q].w;    \
                }                                                                                   \
                v[2 * u] = s0;                                                                      \
                v[2 * u + 1] = s1;                                                                  \
            }                                                                                       \
            _Pragma("unroll") for (int e = 0; e < 2 * kR; ++e) v[e] = wave_sum(v[e]);               \
            if (lane == 0) {                                                                        \
                _Pragma("unroll") for (int e = 0; e < 2 * kR; ++e) s_dot[wave][e] = v[e];           \
            }                                                                                       \
        }                                                                                           \
        __syncthreads();                                                                            \
        if (have_cur && wave == 0 && lane < kChunks) {                                              \
            /* member partial: the 16 waves added in a fixed order; chunk `lane` of 3 */           \
            float w[3] = {0.0f, 0.0f, 0.0f};                                                        \
            _Pragma("unroll") for (int q = 0; q < 3; ++q) {                                         \
                const int e = lane * 3 + q;                                                         \
                if (e < 2 * kR) {                                                                   \
                    float tsum = 0.0f;                                                              \
                    for (int wv = 0; wv < kWaves; ++wv) tsum += s_dot[wv][e];                       \
                    w[q] = tsum;                                                                    \
                }                                                                                   \
            }                                                                                       \
            u32x4 ch = {__float_as_uint(w[0]), __float_as_uint(w[1]), __float_as_uint(w[2]),        \
                        a.tag_base + seq};                                                          \
            const int cslot = (int)(seq % kSlots);                                                  \
            __builtin_amdgcn_raw_buffer_store_b128(ch, xr, ((cslot * a.TS + m) * kChunks + lane) * 16, 0, kCoherent); \
        }                                                                                           \
        if (have_prev) {                                                                            \
            if (wave == 0) {                                                                        \
                const unsigned want = a.tag_base + seq - 1;                                         \
                unsigned spins = 0;                                                                 \
                bool ok = !poller || pol.w == want;                                                 \
                while (!gave_up && !__all(ok)) {                                                    \
                    if (poller && !ok) {                                                            \
                        pol = __builtin_amdgcn_raw_buffer_load_b128(xr, (pslot * a.TS * kChunks + lane) * 16, 0, kCoherent); \
                        ok = pol.w == want;                                                         \
                    }                                                                               \
                    if (++spins > kPollLimit) {                                                     \
                        if (lane == 0)                                                              \
                            __hip_atomic_fetch_or(&a.ctl->error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); \
                        gave_up = true;                                                             \
                    }                                                                               \
                }                                                                                   \
                if (poller) {                                                                       \
                    const int mem = lane / kChunks, c3 = (lane % kChunks) * 3;                      \
                    s_x[mem][c3] = __uint_as_float(pol.x);                                          \
                    if (c3 + 1 < 2 * kR) s_x[mem][c3 + 1] = __uint_as_float(pol.y);                 \
                    if (c3 + 2 < 2 * kR) s_x[mem][c3 + 2] = __uint_as_float(pol.z);                 \
                }                                                                                   \
                __builtin_amdgcn_wave_barrier();                                                    \
                if (lane < kR) {                                                                    \
                    float z = 0.0f, dz = 0.0f;                                                      \
                    for (int mm = 0; mm < a.TS; ++mm) { z += s_x[mm][2 * lane]; dz += s_x[mm][2 * lane + 1]; } \
                    float r, dr, ls;                                                                \
                    residuals(z, dz, YP, r, dr, ls);                                                \
                    s_res[lane] = make_float2(r, dr);                                               \
                    lacc += (double)ls;                                                             \
                }                                                                                   \
            }                                                                                       \
        }                                                                                           \
        __syncthreads();                                                                            \
        if (have_prev) {                                                                            \
            _Pragma("unroll") for (int u = 0; u < kR; ++u) {                                        \
                const float2 w2 = s_res[u];                                                         \
                _Pragma("unroll") for (int q = 0; q < kV; ++q) {                                    \
                    const float4 x4 = XP[u][q];                                                     \
                    ag[q].x += w2.x * x4.x; ag[q].y += w2.x * x4.y; ag[q].z += w2.x * x4.z; ag[q].w += w2.x * x4.w; \
                    as[q].x += w2.y * x4.x; as[q].y += w2.y * x4.y; as[q].z += w2.y * x4.z; as[q].w += w2.y * x4.w; \
                }                                                                                   \
            }                                                                                       \
        }                                                                                           \
        if (have_cur) ++seq;                                                                        \
        ++t;                                                                                        \
    }

        // prologue: rows of tiles 0 and 1, loads of tile 0
        GCADA_FETCH_ROWS(0)
        GCADA_LOAD_TILE(xb0, y0)
        GCADA_FETCH_ROWS(1)
        int t = 0;
        while (t <= ntile) {
            GCADA_STAGE(xb2, xb0, xb1, y2, y1)
            if (t > ntile) break;
            GCADA_STAGE(xb0, xb1, xb2, y0, y2)
            if (t > ntile) break;
            GCADA_STAGE(xb1, xb2, xb0, y1, y0)
        }
#undef GCADA_STAGE
#undef GCADA_LOAD_TILE
#undef GCADA_FETCH_ROWS

        // the group is finished: this member's 4096 columns of the gradient and of s_g
        double sq = 0;
        float* out = fresh_row(a.gbuf, a.which, hy, g) + col;
#pragma unroll
        for (int q = 0; q < kV; ++q) {
            if (hy.l2 != 0.0f) {
                const float ml = (float)mu * hy.l2;
                ag[q].x += ml * th4[q].x; ag[q].y += ml * th4[q].y; ag[q].z += ml * th4[q].z; ag[q].w += ml * th4[q].w;
                as[q].x += ml * dl4[q].x; as[q].y += ml * dl4[q].y; as[q].z += ml * dl4[q].z; as[q].w += ml * dl4[q].w;
            }
            *(float4*)(out + 256 * q) = ag[q];
            sq += (double)as[q].x * as[q].x + (double)as[q].y * as[q].y + (double)as[q].z * as[q].z +
                  (double)as[q].w * as[q].w;
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
            lacc = wave_sum(lacc);       // lanes >= kR hold 0
            if (lane == 0) a.part_loss[g] = lacc;
        }
        __syncthreads();
    }
}

}  // namespace

struct LrTeamPlan {
    int TS = 0, NT = 0;      // TS = 0: not applicable
    u32x4* xch = nullptr;
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
    if (TS * kChunks > kWave) return hipSuccess;     // one wave polls all members' chunks
    hipDeviceProp_t prop;
    hipError_t e = hipGetDeviceProperties(&prop, c->device);
    if (e != hipSuccess) return e;
    int per_cu = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)lr_team_kernel, kThreads, 0);
    if (e != hipSuccess) return e;
    const int cap = per_cu > 0 ? prop.multiProcessorCount : 0;     // one workgroup per CU
    const int NT = cap / TS;
    if (NT < 1) return hipSuccess;
    const size_t n = (size_t)NT * kSlots * TS * kChunks;
    if ((e = hipMalloc(&pl->xch, n * sizeof(u32x4))) != hipSuccess) return e;
    if ((e = hipMemset(pl->xch, 0, n * sizeof(u32x4))) != hipSuccess) return e;
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
    const size_t n = (size_t)c->lr_team->NT * kSlots * c->lr_team->TS * kChunks;
    c->team_launches = 0;
    return hipMemset(c->lr_team->xch, 0, n * sizeof(u32x4));
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
