// Single-pass logistic-regression gradients for wide rows (d > 4096, a multiple of 4):
// step a1 for shapes whose rows do not fit one workgroup's registers (paper Sec. II-A).
//
// A TEAM of TS = ceil(d/4096) workgroups shares the rows of a tile: member m owns columns
// [4096 m, 4096 (m+1)) (the last member those that exist) of R = 4 rows (two float4 per row
// and thread).  Every member forms its
// partial dot products and publishes them (64 bytes) in a small exchange buffer; TWO TILES LATER
// it collects the partials of all members, forms the residuals and adds the tile's contribution
// to its 4096 columns of the two weighted row sums.  While a tile waits for its residuals it is
// parked in LDS (each thread keeps its own 128 bytes per tile there -- LDS as private spill
// space, no synchronisation needed), so the registers hold the tile being multiplied plus the
// TWO tiles whose loads are in flight.  The minibatch is read from HBM exactly once.  A member
// owns its columns for all rows of a group: the column sums never leave registers until the
// group is finished, and no partial sums are written.
//
// Exchange protocol (no read-modify-write atomics, no fences): a partial is eight 8-byte pairs
// {value, tag}; tag = sequence number of the tile, so a pair is valid exactly when its tag
// matches.  Pairs are written and read as relaxed 64-bit atomics at system scope, i.e. past the
// non-coherent L2 of the 8 XCDs.  Four slots per team: a member that publishes tile t has seen
// every member's tile t-2, and a member that has published tile t-2 has already consumed tile
// t-4, whose slot tile t takes.  Every wait is bounded; when a bound is hit the kernel raises
// Ctl::error and runs to its end without waiting again.
//
// Eight DATA waves stream the tiles; two more waves do the exchange and load no tiles (a wave's
// loads return in order, so a poll behind tile loads would wait for them): the PUBLISHER wave adds
// the data waves' partial dots of tile t after the barrier of stage t and publishes them; the
// EXCHANGE wave requests the members' words of tile t-1 before the barrier of stage t, forms the
// residuals after it, and the data waves use them after the barrier of stage t+1.  One workgroup
// barrier per tile; the small LDS arrays involved are double-buffered by the parity of t.  All
// sums over lanes go through DPP moves (no LDS crossbar: it is busy with the parked tiles).
#include "lr_device.h"

namespace gcada {

namespace {

constexpr int kDataWaves = 8;
constexpr int kDataThreads = kDataWaves * 64;
constexpr int kThreads = kDataThreads + 128;  // plus the exchange wave and the publisher wave
constexpr int kV = 2;                    // float4 per row and thread, 256 columns apart
constexpr int kR = 4;                    // rows per tile
constexpr int kSlab = 4096;              // columns per member
constexpr int kSlots = 4;
constexpr int kRegTiles = 3;             // register tiles per thread: multiplied + two loading
constexpr int kPartial = 2 * kR;         // values a member publishes per tile
constexpr int kSlotBytes = kPartial * 8; // per member and slot
constexpr int kParkBytes = 2 * kR * kV * kDataThreads * 16;   // two parked tiles: 131072
// lane layouts: the publisher wave adds the waves' partial dots as (value, data wave) =
// (lane / 8, lane % 8), the exchange wave the members' partials as (row, member) = (lane / 16, lane % 16)
static_assert(kR == 4 && kPartial == 8 && kDataWaves == 8, "lane layouts of the two exchange waves");

// A pair {value, tag} of the exchange buffer travels as one 64-bit word.  Relaxed atomic
// accesses at system scope: the hardware goes past the non-coherent L2s (sc0 sc1), and the
// compiler neither merges nor hoists them -- a plain load in a polling loop would be read once.
__device__ __forceinline__ unsigned long long pair_load(const unsigned long long* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}
__device__ __forceinline__ void pair_store(unsigned long long* p, float value, unsigned tag)
{
    __hip_atomic_store(p, ((unsigned long long)tag << 32) | __float_as_uint(value), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_SYSTEM);
}
__device__ __forceinline__ float pair_value(unsigned long long w) { return __uint_as_float((unsigned)w); }
__device__ __forceinline__ unsigned pair_tag(unsigned long long w) { return (unsigned)(w >> 32); }

struct TeamArgs {
    Hyper hy;
    const ShardDesc* shards;
    const int32_t* idx;
    const float* ring;
    const int32_t* tau;
    Ctl* ctl;
    unsigned long long* xch; // [NT][kSlots][TS][kPartial] pairs {value, tag}
    float* gbuf;
    const int32_t* which;
    double* part_stat;       // [G][TS]
    double* part_loss;       // [G]
    int TS, NT;
    unsigned tag_base;       // tags of this launch are tag_base + tile sequence number
    WaitPolicy wait;         // bound of the polls; tag_skew != 0 only in the test of the give-up path
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

// Per-thread state of a data wave.
struct TeamRegs {
    float4 xb[kRegTiles][kR][kV];   // register tiles; tile n lives in xb[n % 3]
    float4 th4[kV], dl4[kV];        // theta^k and theta^k - theta_stale at this thread's columns
    float4 ag[kV], as[kV];          // column sums of r_i x_i and dr_i x_i
};

// Wave-uniform bookkeeping.  The team's tiles form ONE sequence n = 0 .. ntot-1 over all groups
// the team works on (group ordinal n / ntile), so the loads never pause between groups.
struct TeamSeq {
    int ntile, ntot;                // tiles per group, tiles of this team in this launch
    // the tile that is requested next (n+2 in stage n)
    int rows_nxt[kR];
    const float* x_nxt;
    int64_t ld_nxt;
    // where the row-id fetch stands (tile n+3 in stage n)
    int gF, tF;
    // tile n (multiplied) and tile n-2 (added): group and tile within the group
    int gC, tC, gA, tA;
};

struct TeamLds {
    float4 s_dot[2][kDataWaves][kPartial];  // per-wave partial dots (one per 16-lane row), by parity of the tile
    float2 s_res[2][kR];                    // residuals (r, dr), by parity of the stage
    double s_red[kDataWaves];
};

// The team's next group after g: g + NT, g + 2 NT, ... -- under the server-side rule only groups
// whose mask is set (the others evaluate nothing).  Returns a value >= G when there is none.
__device__ __forceinline__ int team_next_group(const Hyper& hy, int g, int NT)
{
    do g += NT; while (g < hy.G && hy.sel && !hy.sel[g]);
    return g;
}

// Describe the tile after the one S.gF/S.tF point at -- row ids through scalar loads (constant
// address space, uniform address): they are counted apart from the vector loads, so fetching
// them never waits for a tile in flight.  Past the end of the sequence the last tile is
// described again (it is requested, never used).
__device__ __forceinline__ void team_fetch(const TeamArgs& a, TeamSeq& S, int nF, int NT)
{
    typedef const int32_t __attribute__((address_space(4))) const_i32;
    typedef const ShardDesc __attribute__((address_space(4))) const_shard;
    if (nF < S.ntot && nF > 0) {
        if (++S.tF == S.ntile) { S.tF = 0; S.gF = team_next_group(a.hy, S.gF, NT); }
    }
    const_shard* sh = (const_shard*)(uintptr_t)a.shards + S.gF;
    // (every data wave runs this once per tile, between two tiles' worth of arithmetic: it is kept
    // to a handful of scalar instructions -- the kernel is bound by how fast a wave gets through
    // its instructions, not by memory.  The modulo arithmetic of the cyclic window in particular
    // stays out of the path that has row ids.)
    if (a.idx) {
        const_i32* ids = (const_i32*)(uintptr_t)a.idx + (int64_t)S.gF * a.hy.mu;
        const int i0 = S.tF * kR, last = a.hy.mu - 1;
#pragma unroll
        for (int u = 0; u < kR; ++u) {
            // the last tile of a group may reach past the minibatch: such a row repeats the last
            // one (it is loaded, its residuals are zero)
            S.rows_nxt[u] = __builtin_amdgcn_readfirstlane(ids[min(i0 + u, last)]);
        }
    } else {
        const unsigned rows = (unsigned)sh->rows;
        // cyclic window: first row of this step's window, (k * mu) mod rows, in 32 bits
        const unsigned cyc_base = (unsigned)((((unsigned long long)a.hy.k % rows) *
                                              ((unsigned long long)a.hy.mu % rows)) % rows);
#pragma unroll
        for (int u = 0; u < kR; ++u) {
            const int i = min(S.tF * kR + u, a.hy.mu - 1);
            S.rows_nxt[u] = __builtin_amdgcn_readfirstlane((int)((cyc_base + (unsigned)i) % rows));
        }
    }
    S.x_nxt = (const float*)sh->X;
    S.ld_nxt = sh->ld;
}

// A data thread's two column quadruples.  The last member of a team may own fewer than 4096
// columns (d is a multiple of 4, not necessarily of 4096): a quadruple past the row's end is
// switched off -- it loads an in-range stand-in (its products meet zeros of theta), and its sums
// are neither stored nor counted.
struct TeamCols {
    int c[kV];
    bool ok[kV];
};

// Request the tile described in S into register tile JL.
template <int JL>
__device__ __forceinline__ void team_load_tile(TeamRegs& R, const TeamSeq& S, const TeamCols& C)
{
#pragma unroll
    for (int u = 0; u < kR; ++u) {
        const float* xrow = S.x_nxt + (int64_t)S.rows_nxt[u] * S.ld_nxt;
#pragma unroll
        for (int q = 0; q < kV; ++q) R.xb[JL][u][q] = global_load4_stream(xrow + C.c[q]);
    }
}

// A position in the team's tile sequence: group and tile within the group.
struct TeamCursor {
    int g, t;
};
// Move the cursor on to tile nF of the sequence (one step per stage); past the end of the sequence
// it stays on the last tile.
__device__ __forceinline__ void team_cursor_advance(const TeamArgs& a, TeamCursor& c, int ntile, int ntot, int nF)
{
    if (nF < ntot && nF > 0) {
        if (++c.t == ntile) { c.t = 0; c.g = team_next_group(a.hy, c.g, a.NT); }
    }
}
// Row id of row `prow` of the tile the cursor points at (a load when ids are given), and the label
// of a row of a group's shard; for the exchange wave, one row per 16 lanes.
__device__ __forceinline__ int team_row_id(const TeamArgs& a, const TeamCursor& c, int prow)
{
    typedef const ShardDesc __attribute__((address_space(4))) const_shard;
    const int i = min(c.t * kR + prow, a.hy.mu - 1);     // a row past the minibatch repeats the last one
    if (a.idx) return global_load(a.idx + (int64_t)c.g * a.hy.mu + i);
    const_shard* sh = (const_shard*)(uintptr_t)a.shards + c.g;
    const unsigned rows = (unsigned)sh->rows;
    const unsigned cyc_base = (unsigned)((((unsigned long long)a.hy.k % rows) *
                                          ((unsigned long long)a.hy.mu % rows)) % rows);
    return (int)((cyc_base + (unsigned)i) % rows);
}
__device__ __forceinline__ float team_label(const TeamArgs& a, int g, int row)
{
    typedef const ShardDesc __attribute__((address_space(4))) const_shard;
    const_shard* sh = (const_shard*)(uintptr_t)a.shards + g;
    return global_load((const float*)sh->y + row);
}

// theta^k - theta_stale of group g at this thread's columns
__device__ __forceinline__ void team_delta(const TeamArgs& a, const TeamRegs& R, int g, const TeamCols& C,
                                           float4 (&dl)[kV])
{
    const float* stale = a.ring + (int64_t)stale_slot_of(a.hy, a.tau[g]) * a.hy.pstride;
#pragma unroll
    for (int q = 0; q < kV; ++q) {
        const float4 u4 = *(const float4*)(stale + C.c[q]);
        dl[q] = C.ok[q] ? make_float4(R.th4[q].x - u4.x, R.th4[q].y - u4.y, R.th4[q].z - u4.z, R.th4[q].w - u4.w)
                        : make_float4(0, 0, 0, 0);
    }
}

// One pipeline stage of a DATA wave; J = n mod 3 is a compile-time constant so that every
// register tile index is static, and every stage requests a tile, so that the number of loads
// in flight at every wait is known statically (otherwise the compiler has to wait for all of
// them, including the tiles that were only just requested).  Tile n+2 starts loading, tile n is
// multiplied and parked, tile n-2 is added from where it was parked.
template <int J>
__device__ __forceinline__ void team_data_stage(const TeamArgs& a, TeamRegs& R, TeamSeq& S, int n, int m,
                                                const TeamCols& C, TeamLds& L, float4* park)
{
    constexpr int JL = (J + 2) % kRegTiles;      // the register tile that is loaded in this stage
    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const bool have_cur = n < S.ntot, have_add = n >= 2 && n - 2 < S.ntot;

    team_load_tile<JL>(R, S, C);
    team_fetch(a, S, n + 3, a.NT);

    if (have_cur) {
        if (S.tC == 0) team_delta(a, R, S.gC, C, R.dl4);         // first tile of a group
        float v[kPartial];
#pragma unroll
        for (int u = 0; u < kR; ++u) {
            float s0 = 0.0f, s1 = 0.0f;
#pragma unroll
            for (int q = 0; q < kV; ++q) {
                const float4 x4 = R.xb[J][u][q];
                s0 += x4.x * R.th4[q].x + x4.y * R.th4[q].y + x4.z * R.th4[q].z + x4.w * R.th4[q].w;
                s1 += x4.x * R.dl4[q].x + x4.y * R.dl4[q].y + x4.z * R.dl4[q].z + x4.w * R.dl4[q].w;
            }
            v[2 * u] = s0;
            v[2 * u + 1] = s1;
        }
        RowButterfly<kPartial>::run(v, lane);        // sums over the 16 lanes of a row, no LDS traffic
        if ((lane & 1) == 0)
            ((float*)&L.s_dot[n & 1][wave][row_butterfly_first<kPartial>(lane)])[lane >> 4] = v[0];
    }
    __syncthreads();

    // this thread's slots of the parking area for tiles of this parity
    float4* mine = park + (n & 1) * (kR * kV * kDataThreads) + tid;
    if (have_add) {
#pragma unroll
        for (int u = 0; u < kR; ++u) {
            const float2 w2 = L.s_res[n & 1][u];
#pragma unroll
            for (int q = 0; q < kV; ++q) {
                const float4 x4 = mine[(u * kV + q) * kDataThreads];
                R.ag[q].x += w2.x * x4.x; R.ag[q].y += w2.x * x4.y; R.ag[q].z += w2.x * x4.z; R.ag[q].w += w2.x * x4.w;
                R.as[q].x += w2.y * x4.x; R.as[q].y += w2.y * x4.y; R.as[q].z += w2.y * x4.z; R.as[q].w += w2.y * x4.w;
            }
        }
    }
    if (have_cur) {
#pragma unroll
        for (int u = 0; u < kR; ++u)
#pragma unroll
            for (int q = 0; q < kV; ++q) mine[(u * kV + q) * kDataThreads] = R.xb[J][u][q];
        if (++S.tC == S.ntile) { S.tC = 0; S.gC = team_next_group(a.hy, S.gC, a.NT); }
    }

    if (have_add) {
        if (S.tA == S.ntile - 1) {
            // group S.gA is finished: this member's 4096 columns of the gradient and of s_g
            const int g = S.gA;
            double sq = 0;
            float* out = fresh_row(a.gbuf, a.which, a.hy, g);
            float4 dlo[kV];
            if (a.hy.l2 != 0.0f) team_delta(a, R, g, C, dlo);
#pragma unroll
            for (int q = 0; q < kV; ++q) {
                if (a.hy.l2 != 0.0f) {
                    const float ml = (float)a.hy.mu * a.hy.l2;
                    R.ag[q].x += ml * R.th4[q].x; R.ag[q].y += ml * R.th4[q].y; R.ag[q].z += ml * R.th4[q].z; R.ag[q].w += ml * R.th4[q].w;
                    R.as[q].x += ml * dlo[q].x; R.as[q].y += ml * dlo[q].y; R.as[q].z += ml * dlo[q].z; R.as[q].w += ml * dlo[q].w;
                }
                if (C.ok[q]) {
                    *(float4*)(out + C.c[q]) = R.ag[q];
                    sq += (double)R.as[q].x * R.as[q].x + (double)R.as[q].y * R.as[q].y +
                          (double)R.as[q].z * R.as[q].z + (double)R.as[q].w * R.as[q].w;
                }
                R.ag[q] = make_float4(0, 0, 0, 0);
                R.as[q] = make_float4(0, 0, 0, 0);
            }
            sq = wave_sum(sq);
            if (lane == 0) L.s_red[wave] = sq;
            __syncthreads();                     // the exchange and publisher waves join this barrier as well
            if (tid == 0) {
                double tsum = 0;
                for (int wv = 0; wv < kDataWaves; ++wv) tsum += L.s_red[wv];
                a.part_stat[(int64_t)g * a.TS + m] = tsum;
            }
            S.tA = 0;
            S.gA = team_next_group(a.hy, S.gA, a.NT);
        } else {
            ++S.tA;
        }
    }
}

// What the exchange wave carries from one stage to the next.
struct TeamCtl {
    // per lane, for its row (lane / 16) of a tile, in rings indexed by tile mod 3: at the start of
    // stage n the labels of tiles n-1, n, n+1 and the row ids of tiles n+2, n+3, n+4
    float y[kRegTiles];
    int id[kRegTiles];
    TeamCursor c2, c5;            // tiles n+2 (whose labels are requested in stage n) and n+5 (row ids)
    int gR, tR;                   // group and tile-in-group of the tile whose residuals are formed next
    int gA, tA;                   // the same for the tile the data waves add in this stage (n-2)
    bool gave_up;                 // a bounded wait was exhausted
    double lacc, lacc_prev;       // loss sums: of the group whose residuals are being formed, of the one before
};

// Two waves besides the data waves, neither of which loads tiles (a wave's loads return in order:
// a poll behind tile loads would wait for them).
//
// The EXCHANGE wave collects: in stage n it requests the other members' words of tile n-1 (every
// member published them right after its barrier of stage n-1) as soon as it is done with stage
// n-1, joins the barrier of stage n, and then forms the residuals of tile n-1, which the data
// waves use after the barrier of stage n+1.  The round trip to the words (well over a
// microsecond while the tiles stream) thus runs while the wave waits at the barrier, and nothing
// the wave does in front of a barrier waits for a load.  Its other loads -- the label of its row
// of tile n+2 and the row id of tile n+5, three stages ahead of their use each -- are requested
// AFTER the words have arrived and are older than the next stage's polls, so waiting for those
// polls never waits for anything else.  It stores nothing to global memory inside the loop: a
// wave with a store in flight cannot tell which of its loads have returned.
//
// The PUBLISHER wave adds the data waves' partial dots of tile n after the barrier of stage n and
// publishes them; it only ever stores.
template <int J>
__device__ __forceinline__ void team_exchange_stage(const TeamArgs& a, unsigned long long* xt, int n, int m,
                                                    int ntile, int ntot, TeamCtl& K, TeamLds& L)
{
    constexpr int JR = (J + 2) % kRegTiles;                   // ring slot of tiles n-1 and n+2
    const int lane = threadIdx.x % kWave;
    const bool have_add = n >= 2 && n - 2 < ntot;
    const bool have_res = n >= 1 && n - 1 < ntot;             // tile n-1 exists
    const int prow = lane >> 4, pmem = lane & 15;             // the (row, member) whose pairs this lane polls
    const bool poller = pmem < a.TS;

    // lane l requests member l%16's pairs (z, dz) of row l/16 of tile n-1: slot (n-1) mod 4
    const unsigned long long* mine =
        xt + (int)(((unsigned)n + 3u) % kSlots) * a.TS * kPartial + pmem * kPartial + prow * 2;
    unsigned long long pz = 0, pdz = 0;
    if (poller && have_res) {
        pz = pair_load(mine);
        pdz = pair_load(mine + 1);
    }
    __syncthreads();

    if (have_res) {
        const unsigned want = a.tag_base + a.wait.tag_skew + (unsigned)n - 1u;
        bool ok = !poller || (pair_tag(pz) == want && pair_tag(pdz) == want);
        unsigned spins = 0;
        while (!K.gave_up && !__all(ok)) {       // a member's words were not there yet: ask again
            if (poller && !ok) {
                pz = pair_load(mine);
                pdz = pair_load(mine + 1);
                ok = pair_tag(pz) == want && pair_tag(pdz) == want;
            }
            if (++spins > a.wait.limit) {
                if (lane == 0) raise_device_error(a.ctl, 1u);
                K.gave_up = true;
            }
        }
        // lane l holds member l%16's partial (z, dz) of row l/16: add the members of a row in a
        // fixed tree; every lane of the row gets the sums and forms the row's residuals
        const float z = row_total(poller ? pair_value(pz) : 0.0f);
        const float dz = row_total(poller ? pair_value(pdz) : 0.0f);
        if (K.tR == 0) { K.lacc_prev = K.lacc; K.lacc = 0; }         // a new group begins
        float r, dr, ls;
        residuals(a.hy.quadratic != 0, z, dz, K.y[JR], r, dr, ls);
        if (K.tR * kR + prow >= a.hy.mu) r = dr = ls = 0.0f;          // row past the minibatch
        if (pmem == 0) {
            L.s_res[(n + 1) & 1][prow] = make_float2(r, dr);
            K.lacc += (double)ls;
        }
        if (++K.tR == ntile) { K.tR = 0; K.gR = team_next_group(a.hy, K.gR, a.NT); }
    }
    // the label of tile n+2 (its row id came three stages ago) and the row id of tile n+5 take the
    // ring slots that tile n-1 has just left
    K.y[JR] = team_label(a, K.c2.g, K.id[JR]);
    K.id[JR] = team_row_id(a, K.c5, prow);
    team_cursor_advance(a, K.c2, ntile, ntot, n + 3);
    team_cursor_advance(a, K.c5, ntile, ntot, n + 6);

    if (have_add) {
        if (K.tA == ntile - 1) {
            __syncthreads();                     // the data waves' barrier at the end of a group
            // tile n-2 closed group K.gA; if there is a tile n-1 it opened the next group
            double l = pmem == 0 ? (have_res ? K.lacc_prev : K.lacc) : 0.0;
            l = wave_sum(l);
            if (m == 0 && lane == 0) a.part_loss[K.gA] = l;
            K.tA = 0;
            K.gA = team_next_group(a.hy, K.gA, a.NT);
        } else {
            ++K.tA;
        }
    }
}

// One stage of the PUBLISHER wave; tA counts the tiles of the group the data waves are adding.
__device__ __forceinline__ void team_publish_stage(const TeamArgs& a, unsigned long long* xt, int n, int m,
                                                   int ntile, int ntot, int& tA, TeamLds& L)
{
    const int lane = threadIdx.x % kWave;
    __syncthreads();
    if (n < ntot) {
        // member partial: lane l adds value l/8 of data wave l%8 (its four row sums), then the
        // eight waves in a fixed tree (lanes ^1, ^2, ^7)
        const float4 q = L.s_dot[n & 1][lane & 7][lane >> 3];
        float w = ((q.x + q.y) + q.z) + q.w;
        w += row_xor<3>(w);
        w += row_xor<2>(w);
        w += row_xor<1>(w);
        if ((lane & 7) == 0)
            pair_store(xt + ((n % kSlots) * a.TS + m) * kPartial + (lane >> 3), w, a.tag_base + (unsigned)n);
    }
    if (n >= 2 && n - 2 < ntot) {
        if (tA == ntile - 1) {
            __syncthreads();                     // the data waves' barrier at the end of a group
            tA = 0;
        } else {
            ++tA;
        }
    }
}

// grid: NT * TS workgroups of 640 threads (eight data waves, the exchange wave and the publisher
// wave), all resident
// at once (checked on the host); dynamic LDS: kParkBytes.
__global__ __launch_bounds__(kThreads) void lr_team_kernel(TeamArgs a)
{
    extern __shared__ float4 park[];
    __shared__ TeamLds L;

    const Hyper& hy = a.hy;
    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);   // uniform: the role branch is scalar
    int team, m;
    team_of(blockIdx.x, a.TS, a.NT * a.TS, team, m);
    if (team >= hy.G) return;                    // the whole team leaves: nobody waits for it

    // stages 0 .. ntot+1 (the last two only drain), three at a time; stages past the end do
    // nothing but request the last tile again
    const int ntile = (hy.mu + kR - 1) / kR;
    // the team's groups: team, team + NT, ... -- under the server-side rule the selected ones only
    // (an unselected group contributes a zero loss partial and nothing else)
    int g_first = -1, ngroups = 0;
    for (int g = team; g < hy.G; g += a.NT) {
        if (!hy.sel || hy.sel[g]) {
            if (g_first < 0) g_first = g;
            ++ngroups;
        } else if (m == 0 && tid == 0) {
            a.part_loss[g] = 0;
        }
    }
    if (ngroups == 0) return;                    // the whole team leaves
    const int ntot = ngroups * ntile;
    const int nstage = ntot + 2;

    unsigned long long* xt = a.xch + (int64_t)team * kSlots * a.TS * kPartial;   // the team's slots
    if (wave == kDataWaves) {
        // ---- exchange wave ----
        const int prow = lane >> 4;
        TeamCtl K;
        K.gave_up = false; K.lacc = K.lacc_prev = 0;
        K.gR = K.gA = g_first; K.tR = K.tA = 0;
        // labels of tiles 0 and 1, row ids of tiles 2, 3 and 4 (ring slots by tile mod 3)
        TeamCursor c = {g_first, 0};
        K.y[0] = team_label(a, c.g, team_row_id(a, c, prow));
        team_cursor_advance(a, c, ntile, ntot, 1);
        K.y[1] = team_label(a, c.g, team_row_id(a, c, prow));
        team_cursor_advance(a, c, ntile, ntot, 2);
        K.c2 = c;
        K.y[2] = 1.0f;
        K.id[2] = team_row_id(a, c, prow);
        team_cursor_advance(a, c, ntile, ntot, 3);
        K.id[0] = team_row_id(a, c, prow);
        team_cursor_advance(a, c, ntile, ntot, 4);
        K.id[1] = team_row_id(a, c, prow);
        team_cursor_advance(a, c, ntile, ntot, 5);
        K.c5 = c;
        for (int n = 0; n < nstage; n += kRegTiles) {
            team_exchange_stage<0>(a, xt, n, m, ntile, ntot, K, L);
            team_exchange_stage<1>(a, xt, n + 1, m, ntile, ntot, K, L);
            team_exchange_stage<2>(a, xt, n + 2, m, ntile, ntot, K, L);
        }
    } else if (wave == kDataWaves + 1) {
        // ---- publisher wave ----
        int tA = 0;
        for (int n = 0; n < nstage; n += kRegTiles) {
            team_publish_stage(a, xt, n, m, ntile, ntot, tA, L);
            team_publish_stage(a, xt, n + 1, m, ntile, ntot, tA, L);
            team_publish_stage(a, xt, n + 2, m, ntile, ntot, tA, L);
        }
    } else {
        // ---- data waves ----
        TeamSeq S;
        S.ntile = ntile; S.ntot = ntot;
        S.gF = S.gC = S.gA = g_first;
        S.tF = S.tC = S.tA = 0;
        TeamCols C;
#pragma unroll
        for (int q = 0; q < kV; ++q) {
            const int col = m * kSlab + wave * (256 * kV) + lane * 4 + 256 * q;
            C.ok[q] = col < (int)hy.p;
            C.c[q] = C.ok[q] ? col : lane * 4;           // stand-in: a column every row has
        }
        TeamRegs R;
#pragma unroll
        for (int q = 0; q < kV; ++q) {
            R.th4[q] = C.ok[q] ? *(const float4*)(a.ring + (int64_t)hy.cur * hy.pstride + C.c[q])
                               : make_float4(0, 0, 0, 0);
            R.ag[q] = make_float4(0, 0, 0, 0);
            R.as[q] = make_float4(0, 0, 0, 0);
            R.dl4[q] = make_float4(0, 0, 0, 0);
        }
        // prologue: tiles 0 and 1 start loading (there are at least two), tile 2 is described
        team_fetch(a, S, 0, a.NT);
        team_load_tile<0>(R, S, C);
        team_fetch(a, S, 1, a.NT);
        team_load_tile<1>(R, S, C);
        team_fetch(a, S, 2, a.NT);
        for (int n = 0; n < nstage; n += kRegTiles) {
            team_data_stage<0>(a, R, S, n, m, C, L, park);
            team_data_stage<1>(a, R, S, n + 1, m, C, L, park);
            team_data_stage<2>(a, R, S, n + 2, m, C, L, park);
        }
    }
}

}  // namespace

struct LrTeamPlan {
    int TS = 0, NT = 0;      // TS = 0: not applicable
    unsigned long long* xch = nullptr;
};

// Decide whether the team kernel applies (d a multiple of 4 above 4096, at least two tiles of
// rows per group -- the last one may be partly empty --, a whole team fits the device with every
// workgroup resident).
hipError_t lr_team_plan(gcada_ctx* c)
{
    auto* pl = new LrTeamPlan();
    c->lr_team = pl;
    const int d = (int)c->hy.p, mu = c->hy.mu;
    if (d % 4 || d <= kSlab || mu <= kR) return hipSuccess;      // at least two tiles per group
    const int TS = (d + kSlab - 1) / kSlab;      // the last member may own fewer columns
    if (TS * kR > kWave) return hipSuccess;          // one wave polls all members' partials
    hipDeviceProp_t prop;
    hipError_t e = hipGetDeviceProperties(&prop, c->device);
    if (e != hipSuccess) return e;
    int per_cu = 0;
    e = hipFuncSetAttribute((const void*)lr_team_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kParkBytes);
    if (e != hipSuccess) return e;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)lr_team_kernel, kThreads, kParkBytes);
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
    const unsigned tiles = (unsigned)((c->hy.G + pl->NT - 1) / pl->NT) * (unsigned)((c->hy.mu + kR - 1) / kR);
    a.tag_base = (unsigned)((c->team_launches++ % 4095u) + 1u) << 20;
    a.wait = c->wait_policy();
    if (tiles >= (1u << 20)) return hipErrorInvalidValue;
    lr_team_kernel<<<pl->NT * pl->TS, kThreads, kParkBytes, s>>>(a);
    c->n_stat_used = pl->TS;
    c->n_loss_used = c->hy.G;
    return hipGetLastError();
}

}  // namespace gcada
