// Internal declarations shared by the translation units of libgcada (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "gcada.h"

namespace gcada {

// One group's data shard as the kernels see it.
struct ShardDesc {
    const void* X;   // rows x ld, fp32 or bf16
    const void* y;   // rows: fp32 +-1 (logistic) or int32 class (MLP)
    int64_t rows;
    int64_t ld;
};

// Device-resident control block: everything a step decides stays on the device.
struct Ctl {
    double rhs;             // threshold of the last step
    double loss;            // loss of the last step
    double theta_sq;        // ||theta^k||^2 (for the l2 term of the loss)
    unsigned int cnt_a;     // "last block done" counters, reset by the block that finishes
    unsigned int cnt_b;
    unsigned int cnt_c;
    unsigned int error;     // sticky device-side error flag (0 = none)
    unsigned int* host_flag;   // pinned host word that mirrors `error` (the host reads it without a
                               // device call); null: no mirror
};

// A bounded wait between workgroups gave up (or a hand-over was found incomplete): the results
// of this step are not valid.  Sticky on the device, and mirrored to the host.
__device__ __forceinline__ void raise_device_error(Ctl* ctl, unsigned bits)
{
    __hip_atomic_fetch_or(&ctl->error, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned int* hf = ctl->host_flag;
    if (hf) __hip_atomic_store(hf, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// How long a kernel polls for another workgroup's words before it gives up, and -- for the test
// of that path -- a tag offset that makes the wait look for words nobody publishes.
struct WaitPolicy {
    unsigned limit;         // polls
    unsigned tag_skew;      // added to the tag a wait looks for (0 in every real launch)
};
constexpr unsigned kDefaultPollLimit = 1u << 16;

// Scalars every kernel needs, passed by value.
struct Hyper {
    long long k;            // iteration index of this launch (the host counts the iterations)
    int32_t cur;            // ring slot of theta^k      = k mod (D+1)
    int32_t nxt;            // ring slot of theta^{k+1}  = (k+1) mod (D+1)
    int32_t kmodD;          // history index of this iteration = k mod D
    int32_t G, D, mu;
    int64_t p, pstride;     // parameters; floats between ring slots
    float l2;
    int32_t quadratic;      // linear models: 1 = quadratic error loss, 0 = logistic loss
    const uint8_t* sel;     // server-side rule (Sec. IV): the mask decided BEFORE the gradients; a
                            // group with 0 evaluates nothing, the others evaluate one gradient at
                            // theta^k only.  Null (default rule): every group, both iterates.
    double c, alpha, beta1, beta2, eps;
};

// Ring slot of group g's stale iterate theta^{k - tau_g}; 1 <= tau_g <= D < number of slots.
__host__ __device__ inline int stale_slot_of(const Hyper& hy, int tau_g)
{
    const int s = hy.cur - tau_g;
    return s < 0 ? s + hy.D + 1 : s;
}

// Row of gbuf the fresh gradient of group g is written to in this step (the half that does not
// hold the gradient the group uploaded last); an upload then only flips which[g].
__device__ inline float* fresh_row(float* gbuf, const int32_t* which, const Hyper& hy, int g)
{
    return gbuf + ((int64_t)(1 - which[g]) * hy.G + g) * hy.pstride;
}

// Loads through pointers that were themselves read from memory (the shard table): the compiler
// cannot tell their address space and would fall back to flat accesses, whose completion is
// counted together with LDS and scalar traffic.  These helpers state that the data is global.
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 global_load4(const float* p)
{
    const f32x4 v = *(const __attribute__((address_space(1))) f32x4*)p;
    return make_float4(v.x, v.y, v.z, v.w);
}
// The same for data that is read exactly once (the minibatch rows; gradient rows in the server
// step): a non-temporal load, which streams past the caches instead of displacing what is reused.
// On this machine a plain contiguous read reaches about 6.3 TB/s with ordinary loads and about
// 7.2 TB/s with these.
__device__ __forceinline__ float4 global_load4_stream(const float* p)
{
    const f32x4 v = __builtin_nontemporal_load((const __attribute__((address_space(1))) f32x4*)p);
    return make_float4(v.x, v.y, v.z, v.w);
}
template <typename T>
__device__ __forceinline__ T global_load(const T* p)
{
    return *(const __attribute__((address_space(1))) T*)p;
}

// e^x for x <= 0.  The product x log2(e) is split into its rounded value and the rounding error,
// so the result keeps its relative accuracy for large |x| too.
__device__ __forceinline__ float exp_nonpos(float x)
{
    const float l2e_hi = 0x1.715476p+0f, l2e_lo = 0x1.4ae0cp-26f;    // log2(e) = hi + lo
    const float h = x * l2e_hi;
    const float l = fmaf(x, l2e_hi, -h) + x * l2e_lo;
    const float e = __builtin_amdgcn_exp2f(h);
    return fmaf(e, l * 0x1.62e43p-1f, e);                             // 2^(h+l) = 2^h (1 + l ln 2)
}

// Right side of Eq. (9) with c_d = c/D.  Called by one whole wave (64 lanes): the D history
// entries are loaded in parallel and added in the butterfly's fixed order.
__device__ __forceinline__ double history_threshold(const Hyper& hy, const double* __restrict__ nring)
{
    const int lane = threadIdx.x % 64;
    double v = 0;
    for (int j = lane; j < hy.D; j += 64) v += nring[j];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return hy.c / (double)hy.D * v;
}

// Lazy gradient store: before the gradient kernels run, the groups whose selection does not
// depend on the statistic are known -- age D reached, or an all-zero history (threshold 0, every
// group is selected).  Those write their fresh gradient during the gradient stage, and so do the
// groups whose statistic exceeded the threshold in the previous step (`hot`: a guess that spares
// most recomputation while many groups still upload in every step; a wrong guess costs a store
// or a recomputation, never a different result).  A group that is selected without having
// written its gradient gets it from a second, short launch.  Called by one whole wave.
__device__ __forceinline__ void store_flags_wave(const Hyper& hy, const double* __restrict__ nring,
                                                 const int32_t* __restrict__ tau,
                                                 const uint8_t* __restrict__ hot,
                                                 uint8_t* __restrict__ store_now)
{
    const double rhs = history_threshold(hy, nring);
    for (int g = threadIdx.x % 64; g < hy.G; g += 64)
        store_now[g] = (tau[g] >= hy.D) || (rhs == 0.0) || hot[g] ? 1 : 0;
}

struct MlpWork;       // MLP activations and compute copies (mlp_kernels.hip)
struct LrTilePlan;    // single-pass logistic path, rows that fit one workgroup (lr_tiles.hip)
struct LrTeamPlan;    // single-pass logistic path, wide rows shared by a team (lr_team.hip)
struct LrMicroPlan;   // small linear models: the whole iteration in one launch (lr_micro.hip)

}  // namespace gcada

struct gcada_ctx {
    // what the next launch's waits do (see WaitPolicy); reset after every step
    gcada::WaitPolicy wait_policy() const
    {
        return expire_next_wait ? gcada::WaitPolicy{64u, 0x40000000u} : gcada::WaitPolicy{gcada::kDefaultPollLimit, 0u};
    }
    gcada_dims dims{};
    gcada::Hyper hy{};
    int32_t M_G = 1;
    int device = 0;
    int64_t k = 0;                 // iterations done; copied into Hyper::k before every launch
    bool theta_set = false;
    std::vector<gcada::ShardDesc> shards;   // host copy
    std::vector<uint8_t> shard_set;

    // device state
    gcada::ShardDesc* d_shards = nullptr;
    float* ring = nullptr;         // (D+1) x pstride : last D+1 iterates
    float* h = nullptr;
    float* vhat = nullptr;
    float* agg = nullptr;
    float* gbuf = nullptr;         // 2 halves x G rows x pstride: gradients (see which)
    int32_t* which = nullptr;      // G: half of gbuf that holds group g's last uploaded gradient;
                                   //    the fresh gradient of a step is written to the other half
    int32_t* tau = nullptr;        // G
    double* nring = nullptr;       // D
    double* stat = nullptr;        // G
    uint8_t* mask = nullptr;       // G
    gcada::Ctl* ctl = nullptr;

    // scratch
    float* res = nullptr;          // logistic: G x mu x 2 (residual at theta^k, residual difference)
    double* part_loss = nullptr;   // per-block partial loss sums
    double* part_stat = nullptr;   // G x n_stat_part partial squared norms
    double* stat_sum = nullptr;    // G: the partials of a group added up (when they are many)
    double* part_sq = nullptr;     // epilogue partials: 2 per block (||step||^2, ||theta_new||^2)
    int32_t n_loss_part = 0;   // allocated partial loss sums per group
    int32_t n_loss_part_lr = 0;   // blocks per group of the general logistic forward kernel
    int32_t n_stat_part = 0;   // allocated partial squared norms per group
    int32_t n_stat_used = 0;   // partials per group the last gradient launch wrote
    int32_t n_loss_used = 0;   // partial loss sums (all groups) the last gradient launch wrote
    int32_t n_epi_blocks = 0;

    gcada::MlpWork* mlp = nullptr;
    gcada::LrTilePlan* lr_tiles = nullptr;
    gcada::LrTeamPlan* lr_team = nullptr;
    gcada::LrMicroPlan* lr_micro = nullptr;
    unsigned team_launches = 0;    // advances the exchange tags of the team kernel
    // server-side rule (Sec. IV): 0 = gradient-difference statistic, 1 = L_g^2 ||theta^k - theta_stale||^2
    int32_t rule = 0;
    double* rule_L = nullptr;      // G smoothness constants (device)
    double* rule_part = nullptr;   // D x rule_nb partial squared distances
    int32_t rule_nb = 0;
    bool rule_L_set = false;
    int32_t* idx_eff = nullptr;    // G x mu: minibatch ids of the groups' fastest workers
    // lazy gradient store (MLP): the gradient stage writes only the fresh gradients of store_now,
    // a second launch those of redo (selected by the statistic afterwards)
    bool lazy_store = false;
    bool flags_valid = false;    // store_now holds the flags of the step to come (set by the last launch of a step)
    uint8_t* store_now = nullptr;  // G
    uint8_t* redo = nullptr;       // G
    uint8_t* hot = nullptr;        // G: the statistic exceeded the threshold in the previous step
    bool allow_gram = true;        // first-layer statistic through Gram matrices when it pays (bf16 MLP)
    bool allow_single_pass = true;
    bool allow_fused_finish = true;
    bool allow_deferred_finish = false;   // whole-row logistic path: one launch per step (finish of step k-1 with the tiles of step k)
    bool lr_fused_finish = false;  // this step: lr_tile_finish replaces lr_tile_reduce + server_step

    unsigned int* err_mirror = nullptr;   // pinned host word the kernels' give-up paths write to
    bool poisoned = false;         // a launch failed part-way through a step: set_theta / set_state first
    bool expire_next_wait = false; // diagnostic: the next step's waits look for words nobody publishes
    double* static_scratch = nullptr;     // this device's copy of the library's static scratch array

    bool dominant_only = false;    // benchmark diagnostic: launch only the dominant gradient kernel(s)
    std::string stage_name;

    std::string err;
};

namespace gcada {

// Each returns hipSuccess or the launch error.  All work is enqueued on `s`.
hipError_t lr_plan(gcada_ctx* c);                      // sizes scratch (create time)
hipError_t lr_gradients(gcada_ctx* c, const int32_t* idx, hipStream_t s);

// single-pass logistic gradients with whole-row register tiles (lr_tiles.hip)
hipError_t lr_tile_plan(gcada_ctx* c);
void lr_tile_free(gcada_ctx* c);
bool lr_tile_applies(const gcada_ctx* c);
hipError_t lr_tile_gradients(gcada_ctx* c, const int32_t* idx, hipStream_t s);
// tile reduce + selection + innovation sum + server update in one launch (preselected: the
// server-side rule has decided the mask before the gradient stage)
bool lr_tile_finish_applies(const gcada_ctx* c);
hipError_t lr_tile_finish(gcada_ctx* c, uint8_t* mask_out, float* loss_out, bool preselected, hipStream_t s);
// the fused finish leaves the last history entry and ||theta||^2 per block; lr_tile_close adds
// them up (on `s`, or on the stream of that step) before anyone else reads them
hipError_t lr_tile_close(gcada_ctx* c, hipStream_t s, bool use_step_stream);
void lr_tile_forget(gcada_ctx* c);
// one launch per step: the finish of a step runs at the head of the next step's tile launch
bool lr_tile_step_applies(const gcada_ctx* c);
bool lr_tile_step_pending(const gcada_ctx* c);
hipError_t lr_tile_step(gcada_ctx* c, const int32_t* idx, uint8_t* mask_out, float* loss_out, hipStream_t s);
hipError_t lr_tile_flush(gcada_ctx* c, hipStream_t s, bool use_step_stream);

// single-pass logistic gradients for wide rows: teams of workgroups share a tile (lr_team.hip)
hipError_t lr_team_plan(gcada_ctx* c);
void lr_team_free(gcada_ctx* c);
bool lr_team_applies(const gcada_ctx* c);
hipError_t lr_team_reset(gcada_ctx* c);       // clear the exchange buffer
hipError_t lr_team_gradients(gcada_ctx* c, const int32_t* idx, hipStream_t s);

// small linear models (d <= 256): gradients, selection and update in one launch (lr_micro.hip)
hipError_t lr_micro_plan(gcada_ctx* c);
void lr_micro_free(gcada_ctx* c);
bool lr_micro_applies(const gcada_ctx* c);
hipError_t lr_micro_step(gcada_ctx* c, const int32_t* idx, uint8_t* mask_out, float* loss_out, bool dry,
                         hipStream_t s);

hipError_t mlp_plan(gcada_ctx* c);
void mlp_free(gcada_ctx* c);
hipError_t mlp_gradients(gcada_ctx* c, const int32_t* idx, hipStream_t s);
hipError_t mlp_refresh_weights(gcada_ctx* c, hipStream_t s);   // compute copies of all ring slots
// ... of one slot; flags: the same launch also sets the store flags of the step that follows
hipError_t mlp_refresh_slot(gcada_ctx* c, int slot, bool flags, hipStream_t s);

hipError_t select_plan(gcada_ctx* c);
// selection (a2) + masked innovation sum (a3) + server update and history (a4); advances
// Ctl::k and the ages; writes mask_out / loss_out
// preselected: the mask (and rhs, loss) were already decided by the server-side rule
hipError_t server_step(gcada_ctx* c, uint8_t* mask_out, float* loss_out, bool preselected, hipStream_t s);
hipError_t server_select(gcada_ctx* c, uint8_t* mask_out, float* loss_out, hipStream_t s);
hipError_t lazy_flags(gcada_ctx* c, hipStream_t s);
hipError_t mlp_store_selected(gcada_ctx* c, hipStream_t s);
bool mlp_gram_active(const gcada_ctx* c);

// server-side rule of Sec. IV (rule_kernels.hip)
hipError_t rule_plan(gcada_ctx* c);
void rule_free(gcada_ctx* c);
hipError_t rule_select(gcada_ctx* c, uint8_t* mask_out, hipStream_t s);
hipError_t rule_loss(gcada_ctx* c, float* loss_out, hipStream_t s);
hipError_t rule_power_iteration(gcada_ctx* c, int g, int iters, double* lambda_out, hipStream_t s);
// the same without any allocation: scratch in the library's static device array, result on the device
hipError_t rule_static_scratch(double** ptr);                  // this device's copy of the array
size_t rule_static_scratch_doubles();
size_t rule_power_iteration_scratch_doubles(const gcada_ctx* c, int g);
hipError_t rule_smoothness_static(gcada_ctx* c, int iters, double* L_out_dev, hipStream_t s);
// per-worker minibatches: idx_eff <- ids of each group's fastest worker
hipError_t pick_fastest_workers(gcada_ctx* c, const int32_t* idx_workers, const double* delays,
                                int32_t* worker_out, hipStream_t s);
// plain contiguous read of `bytes` of device memory, best of a few launch shapes, in GB/s (calibration.hip)
hipError_t hbm_read_calibration(const void* buf, size_t bytes, int reps, hipStream_t s, double* best_gbps,
                                double* best_plain_gbps);
hipError_t gather_read_calibration(gcada_ctx* c, const int32_t* idx, int64_t idx_stride, int reps, hipStream_t s,
                                   double* gbps);
// ||theta^k||^2 of the current slot -> Ctl::theta_sq (after set_theta / set_state)
hipError_t refresh_theta_sq(gcada_ctx* c, hipStream_t s);

}  // namespace gcada
