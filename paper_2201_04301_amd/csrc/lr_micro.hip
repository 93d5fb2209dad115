// Small linear models (d <= 256): the whole iteration -- steps a1 to a4 -- in ONE launch.
//
// With a few thousand numbers per group the iteration is a chain of memory round trips and
// launches, not a bandwidth problem: three or four separate kernels cost a launch, a drain and a
// set of cold first loads each, and the host cannot even enqueue them as fast as they run.
// Here one workgroup per group computes the group's two gradients (paper Sec. II-A; a wave takes
// whole rows, so a dot product never leaves the wave), its statistic of Eq. (9) and its
// innovation grad_g - last_g, and hands statistic, loss and innovation to workgroup 0 as tagged
// 64-bit words (relaxed atomics that go past the per-XCD L2s; the reader polls the words
// themselves, so there is no fence and no flag).  Workgroup 0 collects them (bounded wait; the
// grid has at most 64 workgroups, all resident), selects (Eq. (9), Algorithm 1), sums the
// innovations of the selected groups in ascending order and updates by Eq. (8a)-(8c).
#include "lr_device.h"

namespace gcada {

namespace {

constexpr int kMicroThreads = 256;
constexpr int kMicroWaves = kMicroThreads / kWave;     // 4
constexpr int kMicroMaxG = 64;
constexpr int kMicroMaxD = 256;
constexpr int kMicroMaxRows = 128;                     // minibatch rows per group
constexpr int kMicroMaxWords = 1024;                   // G * (d + 4): what workgroup 0 collects
constexpr int kMicroRowsInFlight = 8;                  // rows a wave has in flight

struct MicroArgs {
    Hyper hy;
    const ShardDesc* shards;
    const int32_t* idx;
    unsigned long long* xw;      // [G][d + 4] tagged words: statistic (2), loss sum (2), innovation (d)
    unsigned tag;                // of this launch (never 0, never that of a recent launch)
    WaitPolicy wait;             // bound of the polls; tag_skew != 0 only in the test of the give-up path
    int dry;                     // 1: timing run, workgroup 0 collects but changes no state
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

__device__ __forceinline__ float dpp_move_f(float v, int which_move)
{
    const int b = __float_as_int(v);
    int r;
    switch (which_move) {
    case 0: r = __builtin_amdgcn_update_dpp(0, b, 0xB1, 0xF, 0xF, true); break;    // quad_perm [1,0,3,2]
    case 1: r = __builtin_amdgcn_update_dpp(0, b, 0x4E, 0xF, 0xF, true); break;    // quad_perm [2,3,0,1]
    case 2: r = __builtin_amdgcn_update_dpp(0, b, 0x141, 0xF, 0xF, true); break;   // row_half_mirror
    default: r = __builtin_amdgcn_update_dpp(0, b, 0x140, 0xF, 0xF, true); break;  // row_mirror
    }
    return __int_as_float(r);
}
// Sum over the 64 lanes in a fixed order; every lane gets the total (see wave_total).
__device__ __forceinline__ float wave_total_f(float v)
{
    v += dpp_move_f(v, 0);
    v += dpp_move_f(v, 1);
    v += dpp_move_f(v, 2);
    v += dpp_move_f(v, 3);
    const int b = __float_as_int(v);
    return ((__int_as_float(__builtin_amdgcn_readlane(b, 0)) + __int_as_float(__builtin_amdgcn_readlane(b, 16))) +
            __int_as_float(__builtin_amdgcn_readlane(b, 32))) + __int_as_float(__builtin_amdgcn_readlane(b, 48));
}

__device__ __forceinline__ void word_store(unsigned long long* p, unsigned value, unsigned tag)
{
    __hip_atomic_store(p, ((unsigned long long)tag << 32) | value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}
__device__ __forceinline__ void double_store(unsigned long long* p, double v, unsigned tag)
{
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    word_store(p, (unsigned)(b & 0xffffffffull), tag);
    word_store(p + 1, (unsigned)(b >> 32), tag);
}

// grid: G workgroups of 256 threads.  A lane owns columns 4*lane .. 4*lane+3 (lanes beyond d/4
// carry zeros); wave w of a workgroup takes rows w, w+4, ... of the group's minibatch.
__global__ __launch_bounds__(kMicroThreads) void lr_micro_kernel(MicroArgs a)
{
    __shared__ float4 s_acc[2][kMicroWaves][kWave];
    __shared__ double s_loss[kMicroWaves];
    __shared__ float s_delta[kMicroMaxWords];          // workgroup 0: [G][d]
    __shared__ double s_stat[kMicroMaxG], s_lsum[kMicroMaxG];
    __shared__ unsigned s_half[kMicroMaxG][4];         // halves of the two doubles of a group
    __shared__ int s_tau[kMicroMaxG], s_which[kMicroMaxG];
    __shared__ double s_red[2][kMicroWaves];
    __shared__ double s_rhs;

    const Hyper& hy = a.hy;
    Ctl* ctl = a.ctl;
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int g = blockIdx.x, G = hy.G, d = (int)hy.p, mu = hy.mu;
    const bool col = 4 * lane < d;                      // d is a multiple of 4
    const ShardDesc sh = a.shards[g];
    const float* __restrict__ X = (const float*)sh.X;
    const float* __restrict__ Y = (const float*)sh.y;
    const int my_tau = a.tau[g], my_which = a.which[g];
    const float* __restrict__ th = a.ring + (int64_t)hy.cur * hy.pstride;
    const float* __restrict__ ts = a.ring + (int64_t)stale_slot_of(hy, my_tau) * hy.pstride;
    float4 t4 = make_float4(0, 0, 0, 0), u4 = t4, last4 = t4;
    if (col) {
        t4 = *(const float4*)(th + 4 * lane);
        u4 = *(const float4*)(ts + 4 * lane);
        last4 = *(const float4*)(a.gbuf + ((int64_t)my_which * G + g) * hy.pstride + 4 * lane);
    }
    const float4 dl4 = make_float4(t4.x - u4.x, t4.y - u4.y, t4.z - u4.z, t4.w - u4.w);

    // a1: the wave's rows, kMicroRowsInFlight at a time
    float4 ag = make_float4(0, 0, 0, 0), as = ag;
    double lsum = 0;
    for (int i0 = wave; i0 < mu; i0 += kMicroWaves * kMicroRowsInFlight) {
        float4 x[kMicroRowsInFlight];
        float y[kMicroRowsInFlight];
#pragma unroll
        for (int u = 0; u < kMicroRowsInFlight; ++u) {
            const int i = i0 + u * kMicroWaves;
            x[u] = make_float4(0, 0, 0, 0);
            y[u] = 1.0f;
            if (i < mu) {
                int64_t row;
                if (a.idx) row = a.idx[(int64_t)g * mu + i];
                else row = (int64_t)(((unsigned long long)hy.k * (unsigned long long)mu + (unsigned long long)i) %
                                     (unsigned long long)sh.rows);
                if (col) x[u] = global_load4(X + row * sh.ld + 4 * lane);
                y[u] = global_load(Y + row);
            }
        }
#pragma unroll
        for (int u = 0; u < kMicroRowsInFlight; ++u) {
            const int i = i0 + u * kMicroWaves;
            if (i < mu) {                                // the same for the whole wave
                const float z = wave_total_f(x[u].x * t4.x + x[u].y * t4.y + x[u].z * t4.z + x[u].w * t4.w);
                const float dz = wave_total_f(x[u].x * dl4.x + x[u].y * dl4.y + x[u].z * dl4.z + x[u].w * dl4.w);
                float r, dr, ls;
                residuals(hy.quadratic != 0, z, dz, y[u], r, dr, ls);
                ag.x += r * x[u].x; ag.y += r * x[u].y; ag.z += r * x[u].z; ag.w += r * x[u].w;
                as.x += dr * x[u].x; as.y += dr * x[u].y; as.z += dr * x[u].z; as.w += dr * x[u].w;
                lsum += (double)ls;
            }
        }
    }
    s_acc[0][wave][lane] = ag;
    s_acc[1][wave][lane] = as;
    if (lane == 0) s_loss[wave] = lsum;
    __syncthreads();
    if (wave == 0) {
        // the group's gradient, statistic and innovation
        float4 tg = s_acc[0][0][lane], tsn = s_acc[1][0][lane];
        double lg = s_loss[0];
#pragma unroll
        for (int w = 1; w < kMicroWaves; ++w) {
            const float4 p = s_acc[0][w][lane], q = s_acc[1][w][lane];
            tg.x += p.x; tg.y += p.y; tg.z += p.z; tg.w += p.w;
            tsn.x += q.x; tsn.y += q.y; tsn.z += q.z; tsn.w += q.w;
            lg += s_loss[w];
        }
        if (hy.l2 != 0.0f) {
            const float ml = (float)mu * hy.l2;
            tg.x = fmaf(ml, t4.x, tg.x); tg.y = fmaf(ml, t4.y, tg.y);
            tg.z = fmaf(ml, t4.z, tg.z); tg.w = fmaf(ml, t4.w, tg.w);
            tsn.x = fmaf(ml, dl4.x, tsn.x); tsn.y = fmaf(ml, dl4.y, tsn.y);
            tsn.z = fmaf(ml, dl4.z, tsn.z); tsn.w = fmaf(ml, dl4.w, tsn.w);
        }
        double sq = 0;
        unsigned long long* mine = a.xw + (int64_t)g * (d + 4);
        if (col) {
            sq = (double)tsn.x * tsn.x + (double)tsn.y * tsn.y + (double)tsn.z * tsn.z + (double)tsn.w * tsn.w;
            word_store(mine + 4 + 4 * lane + 0, __float_as_uint(tg.x - last4.x), a.tag);
            word_store(mine + 4 + 4 * lane + 1, __float_as_uint(tg.y - last4.y), a.tag);
            word_store(mine + 4 + 4 * lane + 2, __float_as_uint(tg.z - last4.z), a.tag);
            word_store(mine + 4 + 4 * lane + 3, __float_as_uint(tg.w - last4.w), a.tag);
            if (!a.dry) *(float4*)(a.gbuf + ((int64_t)(1 - my_which) * G + g) * hy.pstride + 4 * lane) = tg;
        }
        sq = wave_total(sq);
        if (lane == 0) {
            double_store(mine, sq, a.tag);
            double_store(mine + 2, lg, a.tag);
        }
    }
    if (g != 0) return;

    // ---- workgroup 0: collect, select (a2), sum the innovations (a3), update (a4) ----
    // loads that wait for nobody first
    const bool upd = tid < d;
    float ac = 0, hv = 0, vv = 0, tv = 0;
    if (upd) {
        ac = a.agg[tid];
        hv = a.h[tid];
        vv = a.vhat[tid];
        tv = th[tid];
    }
    double hist = 0;
    if (wave == 0 && lane < hy.D) hist = a.nring[lane];
    const double theta_sq = ctl->theta_sq;
    for (int q = tid; q < G; q += kMicroThreads) { s_tau[q] = a.tau[q]; s_which[q] = a.which[q]; }
    // thread t collects words t, t + 256, ... of the G * (d + 4) published ones
    const int per = d + 4, total = G * per;
    unsigned val[kMicroMaxWords / kMicroThreads];
    bool got[kMicroMaxWords / kMicroThreads];
#pragma unroll
    for (int e = 0; e < kMicroMaxWords / kMicroThreads; ++e) {
        got[e] = tid + e * kMicroThreads >= total;
        val[e] = 0;
    }
    unsigned spins = 0;
    for (;;) {
        bool all = true;
#pragma unroll
        for (int e = 0; e < kMicroMaxWords / kMicroThreads; ++e) {
            if (!got[e]) {
                const unsigned long long w = __hip_atomic_load(a.xw + tid + e * kMicroThreads, __ATOMIC_RELAXED,
                                                               __HIP_MEMORY_SCOPE_SYSTEM);
                if ((unsigned)(w >> 32) == a.tag + a.wait.tag_skew) {
                    got[e] = true;
                    val[e] = (unsigned)w;
                }
            }
            all = all && got[e];
        }
        if (__syncthreads_and(all)) break;
        if (++spins > a.wait.limit) {                  // never in a healthy launch: report, do not hang
            if (tid == 0) raise_device_error(ctl, 1u);
            break;
        }
    }
#pragma unroll
    for (int e = 0; e < kMicroMaxWords / kMicroThreads; ++e) {
        const int w = tid + e * kMicroThreads;
        if (w < total) {
            const int gg = w / per, o = w % per;
            if (o < 4) s_half[gg][o] = val[e];
            else s_delta[gg * d + (o - 4)] = __uint_as_float(val[e]);
        }
    }
    if (wave == 0) {
        hist = wave_total(hist);                         // D <= 64: one history entry per lane
        if (lane == 0) s_rhs = hy.c / (double)hy.D * hist;
    }
    __syncthreads();
    for (int q = tid; q < G; q += kMicroThreads) {
        s_stat[q] = __longlong_as_double((long long)(((unsigned long long)s_half[q][1] << 32) | s_half[q][0]));
        s_lsum[q] = __longlong_as_double((long long)(((unsigned long long)s_half[q][3] << 32) | s_half[q][2]));
    }
    __syncthreads();
    const double rhs = s_rhs;
    bool sel = false;
    if (lane < G) sel = (s_stat[lane] > rhs) || (s_tau[lane] >= hy.D) || (rhs == 0.0);
    const unsigned long long selbits = __ballot(sel);          // G <= 64: lane g of every wave decides for g
    if (wave == 0 && !a.dry) {
        // every workgroup read its age and its half before it published
        if (lane < G) {
            a.stat[lane] = s_stat[lane];
            a.mask[lane] = sel ? 1 : 0;
            if (a.mask_out) a.mask_out[lane] = sel ? 1 : 0;
            a.tau[lane] = sel ? 1 : s_tau[lane] + 1;
            if (sel) a.which[lane] = 1 - s_which[lane];
        }
        if (lane == 0) {
            double lsum_all = 0;
            for (int q = 0; q < G; ++q) lsum_all += s_lsum[q];
            const double loss = lsum_all / ((double)G * (double)mu) + 0.5 * (double)hy.l2 * theta_sq;
            ctl->rhs = rhs;
            ctl->loss = loss;
            if (a.loss_out) *a.loss_out = (float)loss;
        }
    }
    double sq = 0, tsq = 0;
    if (upd) {
        for (int q = 0; q < G; ++q) {
            const bool on = (selbits >> q) & 1ull;
            const float dq = s_delta[q * d + tid];
            ac = on ? ac + dq : ac;
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
        if (!a.dry) {
            a.agg[tid] = ac;
            a.h[tid] = hv;
            a.vhat[tid] = vv;
            (a.ring + (int64_t)hy.nxt * hy.pstride)[tid] = nv;
        }
    }
    sq = wave_total(sq);
    tsq = wave_total(tsq);
    if (lane == 0) { s_red[0][wave] = sq; s_red[1][wave] = tsq; }
    __syncthreads();
    if (tid == 0 && !a.dry) {
        double x = 0, y = 0;
        for (int w = 0; w < kMicroWaves; ++w) { x += s_red[0][w]; y += s_red[1][w]; }
        a.nring[hy.kmodD] = x;
        ctl->theta_sq = y;
    }
}

}  // namespace

struct LrMicroPlan {
    bool ok = false;
    unsigned long long* xw = nullptr;
    unsigned launches = 0;
};

hipError_t lr_micro_plan(gcada_ctx* c)
{
    auto* pl = new LrMicroPlan();
    c->lr_micro = pl;
    const int d = (int)c->hy.p, G = c->hy.G;
    hipDeviceProp_t prop;
    hipError_t e = hipGetDeviceProperties(&prop, c->device);
    if (e != hipSuccess) return e;
    // one workgroup walks through all rows of a group: only worth it for short minibatches
    if (d % 4 != 0 || d > kMicroMaxD || G > kMicroMaxG || G > prop.multiProcessorCount ||
        (int64_t)G * (d + 4) > kMicroMaxWords || c->hy.D > kWave || c->hy.mu > kMicroMaxRows)
        return hipSuccess;
    const size_t words = (size_t)G * (d + 4);
    if ((e = hipMalloc(&pl->xw, words * 8)) != hipSuccess) return e;
    if ((e = hipMemset(pl->xw, 0, words * 8)) != hipSuccess) return e;      // tag 0: never used
    pl->ok = true;
    return hipSuccess;
}

void lr_micro_free(gcada_ctx* c)
{
    if (!c->lr_micro) return;
    if (c->lr_micro->xw) (void)hipFree(c->lr_micro->xw);
    delete c->lr_micro;
    c->lr_micro = nullptr;
}

// Shapes the one-launch path serves, with the default rule (the server-side rule selects before
// the gradients and goes through the general kernels).
bool lr_micro_applies(const gcada_ctx* c)
{
    if (!c->allow_single_pass || !c->allow_fused_finish || !c->lr_micro || !c->lr_micro->ok) return false;
    if (c->hy.sel != nullptr) return false;
    for (const auto& s : c->shards)
        if ((s.ld % 4) || ((uintptr_t)s.X % 16)) return false;
    return true;
}

// The whole iteration (dry: a timing run that changes no state).
hipError_t lr_micro_step(gcada_ctx* c, const int32_t* idx, uint8_t* mask_out, float* loss_out, bool dry,
                         hipStream_t s)
{
    LrMicroPlan* pl = c->lr_micro;
    MicroArgs a{};
    a.hy = c->hy; a.shards = c->d_shards; a.idx = idx; a.xw = pl->xw;
    // tags 1 .. 2^32-1 in turn: a slot only ever holds the tag of an earlier launch
    a.tag = pl->launches++ % 0xffffffffu + 1u;
    a.wait = c->wait_policy();
    a.dry = dry ? 1 : 0;
    a.stat = c->stat; a.mask = c->mask; a.mask_out = mask_out; a.loss_out = loss_out;
    a.gbuf = c->gbuf; a.which = c->which; a.agg = c->agg; a.h = c->h; a.vhat = c->vhat;
    a.ring = c->ring; a.nring = c->nring; a.tau = c->tau; a.ctl = c->ctl;
    for (const void* q : {(const void*)a.shards, (const void*)a.xw, (const void*)a.stat, (const void*)a.mask,
                          (const void*)a.gbuf, (const void*)a.which, (const void*)a.agg, (const void*)a.h,
                          (const void*)a.vhat, (const void*)a.ring, (const void*)a.nring, (const void*)a.tau,
                          (const void*)a.ctl})
        if (!q) return hipErrorInvalidValue;
    lr_micro_kernel<<<c->hy.G, kMicroThreads, 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace gcada
