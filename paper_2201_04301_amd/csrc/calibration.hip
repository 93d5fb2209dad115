// Benchmark diagnostic: what a plain contiguous read of device memory reaches on this machine.
// The HBM-bound gradient kernels (step a1 of the iteration: one read of the minibatch rows) are
// held against the published peak; this figure says how much of that peak any read gets here.
#include <algorithm>

#include "gcada_internal.h"

namespace gcada {

namespace {

typedef float cal_f32x4 __attribute__((ext_vector_type(4)));

// Every block walks chunks of blockDim.x * U consecutive 16-byte words, grid-strided; U loads per
// thread are in flight at once.  The sum keeps the loads alive; it is never stored in practice.
template <int U, bool NT>
__global__ void stream_read_kernel(const cal_f32x4* __restrict__ p, size_t n16, float* __restrict__ sink)
{
    const size_t chunk = (size_t)blockDim.x * U;
    const size_t nchunks = n16 / chunk;
    cal_f32x4 acc = {0, 0, 0, 0};
    for (size_t c = blockIdx.x; c < nchunks; c += gridDim.x) {
        const cal_f32x4* q = p + c * chunk + threadIdx.x;
        cal_f32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const auto* g = (const __attribute__((address_space(1))) cal_f32x4*)(q + (size_t)u * blockDim.x);
            v[u] = NT ? __builtin_nontemporal_load(g) : *g;       // non-temporal: streams past the caches
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc += v[u];
    }
    if (acc.x + acc.y + acc.z + acc.w == 12345.678f) *sink = acc.x;     // (never true for the buffers used)
}

template <int U, bool NT>
hipError_t time_shape(const void* buf, size_t bytes, int blocks, int threads, int reps, float* sink, hipStream_t s,
                      hipEvent_t e0, hipEvent_t e1, double* gbps)
{
    const size_t n16 = bytes / 16;
    stream_read_kernel<U, NT><<<blocks, threads, 0, s>>>((const cal_f32x4*)buf, n16, sink);     // warm-up
    hipError_t e = hipEventRecord(e0, s);
    for (int r = 0; r < reps && e == hipSuccess; ++r) {
        stream_read_kernel<U, NT><<<blocks, threads, 0, s>>>((const cal_f32x4*)buf, n16, sink);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e != hipSuccess) return e;
    // bytes actually read: whole chunks only
    const size_t chunk = (size_t)threads * U * 16;
    const double read = (double)(bytes / chunk * chunk);
    *gbps = read * reps / ((double)ms * 1e-3) / 1e9;
    return hipSuccess;
}


// The same for the access pattern of the wide-row gradient kernel (lr_team_kernel): the minibatch
// rows of every group, gathered by their ids from the groups' shards, each row cut into pieces of
// 4096 columns (16 KB) that go to the members of a team of workgroups, four rows per tile, three
// tiles in flight per workgroup, one workgroup barrier per tile -- but no arithmetic and no
// exchange.  What this kernel reaches is what that access pattern allows on this machine.
struct GatherReadArgs {
    const ShardDesc* shards;
    const int32_t* idx;      // [G][mu] row ids
    int G, mu, TS;           // TS = d / 4096 members per team
    float* sink;
};
constexpr int kGatherThreads = 512, kGatherRows = 4, kGatherDepth = 3, kGatherSlab = 4096;

__global__ __launch_bounds__(kGatherThreads) void gather_read_kernel(GatherReadArgs a)
{
    typedef const ShardDesc __attribute__((address_space(4))) const_shard;
    typedef const int32_t __attribute__((address_space(4))) const_i32;
    const int wg = blockIdx.x, nWG = gridDim.x;
    // teams made of workgroup ids congruent mod 8 (one XCD), as in the gradient kernel
    const int per_xcd = nWG / 8, xcd = wg % 8, slot = wg / 8;
    const int team = xcd * (per_xcd / a.TS) + slot / a.TS, m = slot % a.TS;
    const int teams = nWG / a.TS;
    const int ntile = a.G * a.mu / kGatherRows / teams;          // tiles of this team (exact: checked on the host)
    const int q0 = team * ntile * kGatherRows;
    const_i32* ids = (const_i32*)(uintptr_t)a.idx;
    cal_f32x4 buf[kGatherDepth][kGatherRows][2];
    cal_f32x4 acc = {0, 0, 0, 0};
    auto issue = [&](int j, cal_f32x4 (&b)[kGatherRows][2]) {
#pragma unroll
        for (int r = 0; r < kGatherRows; ++r) {
            const int q = q0 + j * kGatherRows + r;              // < G * mu
            const_shard* sh = (const_shard*)(uintptr_t)a.shards + q / a.mu;
            const int row = __builtin_amdgcn_readfirstlane(ids[q]);
            const float* x = (const float*)sh->X + (int64_t)row * sh->ld + m * kGatherSlab;
#pragma unroll
            for (int v = 0; v < 2; ++v)
                b[r][v] = __builtin_nontemporal_load(
                    (const __attribute__((address_space(1))) cal_f32x4*)x + threadIdx.x + v * kGatherThreads);
        }
    };
#pragma unroll
    for (int s = 0; s < kGatherDepth; ++s)
        if (s < ntile) issue(s, buf[s]);
    for (int j = 0; j < ntile; j += kGatherDepth) {
#pragma unroll
        for (int s = 0; s < kGatherDepth; ++s) {
            if (j + s < ntile) {
#pragma unroll
                for (int r = 0; r < kGatherRows; ++r) acc += buf[s][r][0] + buf[s][r][1];
            }
            __syncthreads();
            if (j + s + kGatherDepth < ntile) issue(j + s + kGatherDepth, buf[s]);
        }
    }
    if (acc.x + acc.y + acc.z + acc.w == 12345.678f) *a.sink = acc.x;     // (keeps the loads alive)
}

}  // namespace

hipError_t hbm_read_calibration(const void* buf, size_t bytes, int reps, hipStream_t s, double* best_gbps,
                                double* best_plain_gbps)
{
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e != hipSuccess) return e;
    if ((e = hipEventCreate(&e1)) != hipSuccess) { (void)hipEventDestroy(e0); return e; }
    float* sink = nullptr;
    if ((e = hipMalloc(&sink, sizeof(float))) != hipSuccess) {
        (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
        return e;
    }
    int dev = 0, cus = 256;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) cus = prop.multiProcessorCount;
    double best = 0, best_plain = 0;
    for (int threads : {256, 512, 1024})
        for (int per_cu : {1, 2, 4, 16}) {
            double g8 = 0, g16 = 0, n8 = 0, n16 = 0;
            if ((e = time_shape<8, false>(buf, bytes, cus * per_cu, threads, reps, sink, s, e0, e1, &g8)) != hipSuccess) break;
            if ((e = time_shape<16, false>(buf, bytes, cus * per_cu, threads, reps, sink, s, e0, e1, &g16)) != hipSuccess) break;
            if ((e = time_shape<8, true>(buf, bytes, cus * per_cu, threads, reps, sink, s, e0, e1, &n8)) != hipSuccess) break;
            if ((e = time_shape<16, true>(buf, bytes, cus * per_cu, threads, reps, sink, s, e0, e1, &n16)) != hipSuccess) break;
            best_plain = std::max(best_plain, std::max(g8, g16));
            best = std::max(best, std::max(std::max(g8, g16), std::max(n8, n16)));
        }
    (void)hipFree(sink);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return e;
    *best_gbps = best;
    if (best_plain_gbps) *best_plain_gbps = best_plain;
    return hipSuccess;
}

// Gathered read of the context's shards in the wide-row kernel's pattern; `reps` launches on
// distinct minibatches (idx + r * idx_stride) between two events.  The caller has checked the shape.
hipError_t gather_read_calibration(gcada_ctx* c, const int32_t* idx, int64_t idx_stride, int reps, hipStream_t s,
                                   double* gbps)
{
    const int d = (int)c->hy.p, TS = d / kGatherSlab;
    hipDeviceProp_t prop;
    hipError_t e = hipGetDeviceProperties(&prop, c->device);
    if (e != hipSuccess) return e;
    const int nWG = prop.multiProcessorCount / 8 * 8;
    if (nWG < 8 || (nWG / 8) % TS || ((int64_t)c->hy.G * c->hy.mu / kGatherRows) % (nWG / TS)) return hipErrorInvalidValue;
    hipEvent_t e0, e1;
    if ((e = hipEventCreate(&e0)) != hipSuccess) return e;
    if ((e = hipEventCreate(&e1)) != hipSuccess) { (void)hipEventDestroy(e0); return e; }
    float* sink = nullptr;
    if ((e = hipMalloc(&sink, sizeof(float))) != hipSuccess) {
        (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
        return e;
    }
    GatherReadArgs a{c->d_shards, idx, c->hy.G, c->hy.mu, TS, sink};
    gather_read_kernel<<<nWG, kGatherThreads, 0, s>>>(a);                  // warm-up
    e = hipEventRecord(e0, s);
    for (int r = 0; r < reps && e == hipSuccess; ++r) {
        a.idx = idx + (int64_t)r * idx_stride;
        gather_read_kernel<<<nWG, kGatherThreads, 0, s>>>(a);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipFree(sink);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return e;
    *gbps = (double)c->hy.G * c->hy.mu * d * 4.0 * reps / ((double)ms * 1e-3) / 1e9;
    return hipSuccess;
}

}  // namespace gcada
