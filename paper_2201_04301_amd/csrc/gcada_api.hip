// C-ABI of libgcada: context management, argument checks, state transfer, and the order of the
// kernels that make one iteration (Algorithm 1 of the paper, all groups at once).
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>

#include "gcada_internal.h"

using gcada::Ctl;
using gcada::ShardDesc;

namespace {

thread_local std::string g_create_err;

int fail(gcada_ctx* c, int code, const std::string& msg)
{
    if (c) c->err = msg; else g_create_err = msg;
    return code;
}

int fail_hip(gcada_ctx* c, hipError_t e, const char* what)
{
    std::string m = std::string(what) + ": " + hipGetErrorString(e);
    (void)hipGetLastError();   // clear the sticky launch error
    return fail(c, e == hipErrorOutOfMemory ? GCADA_ENOMEM : GCADA_EDEVICE, m);
}

#define HIP_TRY(ctx, call)                                             \
    do {                                                               \
        hipError_t e__ = (call);                                       \
        if (e__ != hipSuccess) return fail_hip(ctx, e__, #call);       \
    } while (0)

template <typename T>
hipError_t dalloc(T** p, size_t n)
{
    hipError_t e = hipMalloc((void**)p, std::max<size_t>(n, 1) * sizeof(T));
    if (e == hipSuccess) e = hipMemset(*p, 0, std::max<size_t>(n, 1) * sizeof(T));
    return e;
}

const char* kWaitFailed =
    "a wait or a hand-over between workgroups inside a kernel of an earlier step failed; the state is not valid: "
    "call gcada_set_theta or gcada_set_state";

// A bounded wait inside a kernel gave up: the results of that step are not valid.  (After a
// device synchronisation: reads the device's own flag.)
int check_device_flag(gcada_ctx* c)
{
    Ctl z{};
    hipError_t e = hipMemcpy(&z, c->ctl, sizeof(z), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail_hip(c, e, "read control block");
    if (z.error != 0 || (c->err_mirror && *(volatile unsigned int*)c->err_mirror != 0))
        return fail(c, GCADA_EDEVICE, kWaitFailed);
    return GCADA_OK;
}

// The same without touching the device: the kernels' give-up paths also write a pinned host word.
// It shows the failures of the steps that have FINISHED on the device by now.
int check_host_mirror(gcada_ctx* c)
{
    if (c->err_mirror && *(volatile unsigned int*)c->err_mirror != 0) return fail(c, GCADA_EDEVICE, kWaitFailed);
    return GCADA_OK;
}

// Fresh control block (no error, counters 0) that points at the host mirror.
hipError_t reset_control_block(gcada_ctx* c)
{
    Ctl z{};
    z.host_flag = c->err_mirror;
    if (c->err_mirror) *(volatile unsigned int*)c->err_mirror = 0;
    return hipMemcpy(c->ctl, &z, sizeof(z), hipMemcpyHostToDevice);
}

int64_t param_count(const gcada_dims& d)
{
    if (d.model != GCADA_MLP) return d.widths[0];
    int64_t p = 0;
    for (int l = 1; l < d.n_widths; ++l)
        p += (int64_t)d.widths[l] * d.widths[l - 1] + d.widths[l];
    return p;
}

void free_all(gcada_ctx* c)
{
    if (!c) return;
    gcada::mlp_free(c);
    gcada::lr_tile_free(c);
    gcada::lr_micro_free(c);
    gcada::lr_team_free(c);
    gcada::rule_free(c);
    void* ptrs[] = {c->d_shards, c->ring, c->h, c->vhat, c->agg, c->gbuf, c->which, c->tau,
                    c->nring, c->stat, c->mask, c->ctl, c->res, c->part_loss, c->part_stat, c->stat_sum,
                    c->part_sq, c->store_now, c->redo, c->hot};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    if (c->err_mirror) (void)hipHostFree(c->err_mirror);
    c->err_mirror = nullptr;
}

}  // namespace

extern "C" {

const char* gcada_version(void) { return "gcada-gfx950 0.1"; }

const char* gcada_last_error(const gcada_ctx* ctx)
{
    return ctx ? ctx->err.c_str() : g_create_err.c_str();
}

int gcada_create(const gcada_dims* dims, int32_t G, int32_t M_G, int32_t D, double c,
                 double alpha, double beta1, double beta2, double eps, gcada_ctx** out)
try {
    if (!dims || !out) return fail(nullptr, GCADA_EINVAL, "dims and out must not be NULL");
    if (dims->model != GCADA_LOGREG && dims->model != GCADA_MLP && dims->model != GCADA_LINREG)
        return fail(nullptr, GCADA_EINVAL, "dims.model must be GCADA_LOGREG, GCADA_MLP or GCADA_LINREG");
    if (dims->dtype != GCADA_F32 && dims->dtype != GCADA_BF16)
        return fail(nullptr, GCADA_EINVAL, "dims.dtype must be GCADA_F32 or GCADA_BF16");
    if (dims->model != GCADA_MLP && (dims->n_widths != 1 || dims->dtype != GCADA_F32))
        return fail(nullptr, GCADA_EINVAL, "logistic regression takes one width and fp32 data");
    if (dims->model == GCADA_MLP && (dims->n_widths < 2 || dims->n_widths > GCADA_MAX_WIDTHS))
        return fail(nullptr, GCADA_EINVAL, "MLP takes 2..8 layer widths");
    for (int l = 0; l < dims->n_widths; ++l)
        if (dims->widths[l] < 1)
            return fail(nullptr, GCADA_EINVAL, "every width must be >= 1");
    if (dims->model == GCADA_MLP && dims->widths[dims->n_widths - 1] > 128)
        return fail(nullptr, GCADA_EINVAL, "MLP output width (classes) must be <= 128");
    if (dims->batch < 1 || dims->batch > 4096)
        return fail(nullptr, GCADA_EINVAL, "dims.batch (mu) must be in [1, 4096]");
    if (!(dims->l2 >= 0.0f) || (dims->dtype == GCADA_BF16 && dims->l2 != 0.0f))
        return fail(nullptr, GCADA_EINVAL, "dims.l2 must be >= 0 (and 0 for bf16)");
    if (G < 1 || G > 4096) return fail(nullptr, GCADA_EINVAL, "G must be in [1, 4096]");
    if (M_G < 1) return fail(nullptr, GCADA_EINVAL, "M_G must be >= 1");
    if (D < 1 || D > 1024) return fail(nullptr, GCADA_EINVAL, "D must be in [1, 1024]");
    if (!(c >= 0.0)) return fail(nullptr, GCADA_EINVAL, "c must be >= 0");
    if (!(alpha > 0.0)) return fail(nullptr, GCADA_EINVAL, "alpha must be > 0");
    if (!(beta1 >= 0.0 && beta1 < 1.0 && beta2 >= 0.0 && beta2 < 1.0))
        return fail(nullptr, GCADA_EINVAL, "beta1, beta2 must be in [0, 1)");
    if (!(eps > 0.0)) return fail(nullptr, GCADA_EINVAL, "eps must be > 0");

    gcada_ctx* x = new (std::nothrow) gcada_ctx();
    if (!x) return fail(nullptr, GCADA_ENOMEM, "host allocation failed");
    x->dims = *dims;
    x->M_G = M_G;
    gcada::Hyper& hy = x->hy;
    hy.G = G; hy.D = D; hy.mu = dims->batch;
    hy.p = param_count(*dims);
    hy.pstride = (hy.p + 63) / 64 * 64;
    hy.l2 = dims->l2;
    hy.quadratic = dims->model == GCADA_LINREG ? 1 : 0;
    hy.c = c; hy.alpha = alpha; hy.beta1 = beta1; hy.beta2 = beta2; hy.eps = eps;
    x->shards.assign(G, ShardDesc{nullptr, nullptr, 0, 0});
    x->shard_set.assign(G, 0);

    auto bail = [&](hipError_t e, const char* what) {
        int rc = fail_hip(nullptr, e, what);
        free_all(x);
        delete x;
        return rc;
    };
    hipError_t e;
    if ((e = hipGetDevice(&x->device)) != hipSuccess) return bail(e, "hipGetDevice");
    const size_t p = (size_t)hy.pstride, Gp = (size_t)G * p;   // every vector padded to pstride
    if ((e = dalloc(&x->d_shards, (size_t)G)) != hipSuccess) return bail(e, "alloc shards");
    if ((e = dalloc(&x->ring, (size_t)(D + 1) * hy.pstride)) != hipSuccess) return bail(e, "alloc iterates");
    if ((e = dalloc(&x->h, p)) != hipSuccess) return bail(e, "alloc h");
    if ((e = dalloc(&x->vhat, p)) != hipSuccess) return bail(e, "alloc vhat");
    if ((e = dalloc(&x->agg, p)) != hipSuccess) return bail(e, "alloc aggregate");
    if ((e = dalloc(&x->gbuf, 2 * Gp)) != hipSuccess) return bail(e, "alloc gradients");
    if ((e = dalloc(&x->which, (size_t)G)) != hipSuccess) return bail(e, "alloc gradient index");
    if ((e = dalloc(&x->tau, (size_t)G)) != hipSuccess) return bail(e, "alloc ages");
    if ((e = dalloc(&x->nring, (size_t)D)) != hipSuccess) return bail(e, "alloc history");
    if ((e = dalloc(&x->stat, (size_t)G)) != hipSuccess) return bail(e, "alloc stat");
    if ((e = dalloc(&x->mask, (size_t)G)) != hipSuccess) return bail(e, "alloc mask");
    if ((e = dalloc(&x->stat_sum, (size_t)G)) != hipSuccess) return bail(e, "alloc stat sums");
    if ((e = dalloc(&x->store_now, (size_t)G)) != hipSuccess) return bail(e, "alloc store flags");
    if ((e = dalloc(&x->redo, (size_t)G)) != hipSuccess) return bail(e, "alloc store flags");
    if ((e = dalloc(&x->hot, (size_t)G)) != hipSuccess) return bail(e, "alloc store flags");
    // an MLP whose fresh gradients (G rows of p floats per step) are a large write stores them lazily
    x->lazy_store = dims->model == GCADA_MLP && Gp * sizeof(float) >= ((size_t)64 << 20);
    if ((e = dalloc(&x->ctl, 1)) != hipSuccess) return bail(e, "alloc control block");
    if ((e = hipHostMalloc((void**)&x->err_mirror, sizeof(unsigned int), hipHostMallocDefault)) != hipSuccess)
        return bail(e, "alloc error mirror");
    if ((e = reset_control_block(x)) != hipSuccess) return bail(e, "control block");

    e = dims->model != GCADA_MLP ? gcada::lr_plan(x) : gcada::mlp_plan(x);
    if (e != hipSuccess) return bail(e, "model plan");
    if ((e = gcada::select_plan(x)) != hipSuccess) return bail(e, "server plan");
    if ((e = gcada::rule_plan(x)) != hipSuccess) return bail(e, "selection rule plan");
    if (dims->model != GCADA_MLP && (e = gcada::lr_tile_plan(x)) != hipSuccess)
        return bail(e, "single-pass logistic plan");
    if (dims->model != GCADA_MLP && (e = gcada::lr_team_plan(x)) != hipSuccess)
        return bail(e, "team logistic plan");
    if (dims->model != GCADA_MLP && (e = gcada::lr_micro_plan(x)) != hipSuccess)
        return bail(e, "one-launch logistic plan");
    if ((e = dalloc(&x->part_loss, (size_t)G * x->n_loss_part)) != hipSuccess) return bail(e, "alloc scratch");
    if ((e = dalloc(&x->part_stat, (size_t)G * x->n_stat_part)) != hipSuccess) return bail(e, "alloc scratch");
    if ((e = dalloc(&x->part_sq, (size_t)2 * x->n_epi_blocks)) != hipSuccess) return bail(e, "alloc scratch");
    if ((e = hipDeviceSynchronize()) != hipSuccess) return bail(e, "hipDeviceSynchronize");
    *out = x;
    return GCADA_OK;
} catch (...) {
    return fail(nullptr, GCADA_ENOMEM, "unexpected exception in gcada_create");
}

void gcada_destroy(gcada_ctx* ctx)
{
    if (!ctx) return;
    (void)hipDeviceSynchronize();
    free_all(ctx);
    delete ctx;
}

int gcada_set_shard(gcada_ctx* ctx, int32_t g, const void* X, const void* y, int64_t rows,
                    int64_t ld)
try {
    if (!ctx) return GCADA_EINVAL;
    if (g < 0 || g >= ctx->hy.G) return fail(ctx, GCADA_EINVAL, "set_shard: g out of range");
    if (!X || !y) return fail(ctx, GCADA_EINVAL, "set_shard: X and y must not be NULL");
    if (rows < 1) return fail(ctx, GCADA_EINVAL, "set_shard: rows must be >= 1");
    if (ld < ctx->dims.widths[0]) return fail(ctx, GCADA_EINVAL, "set_shard: ld < widths[0]");
    const int esz = ctx->dims.dtype == GCADA_BF16 ? 2 : 4;
    if ((uintptr_t)X % esz || (uintptr_t)y % 4)
        return fail(ctx, GCADA_EINVAL, "set_shard: misaligned pointer");
    ShardDesc s{X, y, rows, ld};
    HIP_TRY(ctx, hipMemcpy(ctx->d_shards + g, &s, sizeof(s), hipMemcpyHostToDevice));
    ctx->shards[g] = s;
    ctx->shard_set[g] = 1;
    return GCADA_OK;
} catch (...) {
    return fail(ctx, GCADA_ENOMEM, "unexpected exception in gcada_set_shard");
}

// Copy the host's iteration count and the ring indices derived from it into the kernel arguments.
static void set_iteration(gcada_ctx* ctx)
{
    gcada::Hyper& hy = ctx->hy;
    hy.k = ctx->k;
    hy.cur = (int32_t)(ctx->k % (hy.D + 1));
    hy.nxt = (int32_t)((ctx->k + 1) % (hy.D + 1));
    hy.kmodD = (int32_t)(ctx->k % hy.D);
}

// Fill every ring slot with theta0, zero the rest, ages = D.
static int reset_run(gcada_ctx* ctx, const float* theta0_any)
{
    const gcada::Hyper& hy = ctx->hy;
    const size_t p = (size_t)hy.pstride, Gp = (size_t)hy.G * p;
    for (int s = 0; s <= hy.D; ++s)
        HIP_TRY(ctx, hipMemcpy(ctx->ring + (size_t)s * hy.pstride, theta0_any,
                               (size_t)hy.p * sizeof(float), hipMemcpyDefault));
    HIP_TRY(ctx, hipMemset(ctx->h, 0, p * 4));
    HIP_TRY(ctx, hipMemset(ctx->vhat, 0, p * 4));
    HIP_TRY(ctx, hipMemset(ctx->agg, 0, p * 4));
    HIP_TRY(ctx, hipMemset(ctx->gbuf, 0, 2 * Gp * 4));
    HIP_TRY(ctx, hipMemset(ctx->which, 0, (size_t)hy.G * 4));
    HIP_TRY(ctx, hipMemset(ctx->nring, 0, (size_t)hy.D * 8));
    HIP_TRY(ctx, hipMemset(ctx->stat, 0, (size_t)hy.G * 8));
    HIP_TRY(ctx, hipMemset(ctx->mask, 0, (size_t)hy.G));
    std::vector<int32_t> tau(hy.G, hy.D);
    HIP_TRY(ctx, hipMemcpy(ctx->tau, tau.data(), (size_t)hy.G * 4, hipMemcpyHostToDevice));
    HIP_TRY(ctx, reset_control_block(ctx));
    ctx->k = 0;
    return GCADA_OK;
}

static int after_state_change(gcada_ctx* ctx)
{
    ctx->poisoned = false;
    ctx->expire_next_wait = false;
    set_iteration(ctx);
    gcada::lr_tile_forget(ctx);
    ctx->flags_valid = false;
    HIP_TRY(ctx, hipMemset(ctx->hot, 0, (size_t)ctx->hy.G));
    if (ctx->dims.model != GCADA_MLP) HIP_TRY(ctx, gcada::lr_team_reset(ctx));
    HIP_TRY(ctx, gcada::refresh_theta_sq(ctx, nullptr));
    if (ctx->dims.model == GCADA_MLP) HIP_TRY(ctx, gcada::mlp_refresh_weights(ctx, nullptr));
    HIP_TRY(ctx, hipDeviceSynchronize());
    return GCADA_OK;
}

int gcada_set_theta(gcada_ctx* ctx, const float* theta0)
try {
    if (!ctx) return GCADA_EINVAL;
    if (!theta0) return fail(ctx, GCADA_EINVAL, "set_theta: theta0 must not be NULL");
    int rc = reset_run(ctx, theta0);
    if (rc != GCADA_OK) return rc;
    rc = after_state_change(ctx);
    if (rc != GCADA_OK) return rc;
    ctx->theta_set = true;
    return GCADA_OK;
} catch (...) {
    return fail(ctx, GCADA_ENOMEM, "unexpected exception in gcada_set_theta");
}

static int step_launches(gcada_ctx* ctx, const int32_t* idx, uint8_t* mask_out, float* loss_out, hipStream_t s);

int gcada_step(gcada_ctx* ctx, const int32_t* idx, uint8_t* mask_out, float* loss_out,
               void* stream)
{
    if (!ctx) return GCADA_EINVAL;
    if (!ctx->theta_set) return fail(ctx, GCADA_ESTATE, "step: gcada_set_theta has not been called");
    for (int g = 0; g < ctx->hy.G; ++g)
        if (!ctx->shard_set[g]) return fail(ctx, GCADA_ESTATE, "step: a group has no shard");
    if (ctx->poisoned)
        return fail(ctx, GCADA_ESTATE, "step: a launch of an earlier step failed part-way; the state is not valid: "
                                       "call gcada_set_theta or gcada_set_state");
    // a wait that gave up inside a kernel of an earlier step (one that has finished by now)
    if (int rc = check_host_mirror(ctx)) return rc;
    const int64_t k0 = ctx->k;
    const int rc = step_launches(ctx, idx, mask_out, loss_out, (hipStream_t)stream);
    ctx->expire_next_wait = false;
    // some kernels of the step may be in the stream already: the device state is then neither that
    // of step k nor of step k+1
    if (rc != GCADA_OK && rc != GCADA_ESTATE) { ctx->poisoned = true; ctx->k = k0; }
    return rc;
}

// The launches of one iteration, in order.
static int step_launches(gcada_ctx* ctx, const int32_t* idx, uint8_t* mask_out, float* loss_out, hipStream_t s)
{
    set_iteration(ctx);
    hipError_t e;
    const bool server_rule = ctx->rule == GCADA_RULE_SERVER;
    ctx->hy.sel = server_rule ? ctx->mask : nullptr;
    // whole-row logistic path with one launch per step: the finish of a step runs at the head of
    // the next step's launch; any other path first lets a finish that is still to come run
    const bool deferred = ctx->dims.model != GCADA_MLP && !gcada::lr_micro_applies(ctx) && gcada::lr_tile_step_applies(ctx);
    if (!deferred && (e = gcada::lr_tile_flush(ctx, s, false)) != hipSuccess) return fail_hip(ctx, e, "finish kernel");
    if (deferred) {
        ctx->lr_fused_finish = true;
        if ((e = gcada::lr_tile_step(ctx, idx, mask_out, loss_out, s)) != hipSuccess) return fail_hip(ctx, e, "step kernel");
        ctx->k += 1;
        return GCADA_OK;
    }
    if (ctx->dims.model != GCADA_MLP && gcada::lr_micro_applies(ctx)) {
        // small linear model: the whole iteration is one launch
        ctx->lr_fused_finish = false;
        if ((e = gcada::lr_tile_close(ctx, s, false)) != hipSuccess) return fail_hip(ctx, e, "history kernel");
        if ((e = gcada::lr_micro_step(ctx, idx, mask_out, loss_out, false, s)) != hipSuccess)
            return fail_hip(ctx, e, "one-launch kernel");
        ctx->k += 1;
        return GCADA_OK;
    }
    ctx->lr_fused_finish = ctx->dims.model != GCADA_MLP && gcada::lr_tile_finish_applies(ctx);
    // the selection kernel of the server-side rule and every kernel but the fused finish read the
    // complete history
    if ((!ctx->lr_fused_finish || server_rule) && (e = gcada::lr_tile_close(ctx, s, false)) != hipSuccess)
        return fail_hip(ctx, e, "history kernel");
    if (server_rule) {
        // Sec. IV / Algorithm 1: the server decides first, from the iterates alone; the gradient
        // kernels then skip the unselected groups and the stale iterate
        if (!ctx->rule_L_set) return fail(ctx, GCADA_ESTATE, "step: the server-side rule needs the constants L_g");
        if ((e = gcada::rule_select(ctx, mask_out, s)) != hipSuccess) return fail_hip(ctx, e, "selection kernels");
        ctx->hy.sel = ctx->mask;
    } else {
        ctx->hy.sel = nullptr;
    }
    // lazy gradient store: the gradient stage writes the fresh gradients of the groups that are
    // selected whatever the statistic says; the selection then names the others to be written
    const bool lazy = ctx->dims.model == GCADA_MLP && ctx->lazy_store && !server_rule;
    if (lazy && !ctx->flags_valid && (e = gcada::lazy_flags(ctx, s)) != hipSuccess)
        return fail_hip(ctx, e, "store flag kernel");
    e = ctx->dims.model != GCADA_MLP ? gcada::lr_gradients(ctx, idx, s) : gcada::mlp_gradients(ctx, idx, s);
    if (e != hipSuccess) return fail_hip(ctx, e, "gradient kernels");
    if (server_rule && !ctx->lr_fused_finish && (e = gcada::rule_loss(ctx, loss_out, s)) != hipSuccess)
        return fail_hip(ctx, e, "loss kernel");
    if (lazy) {
        if ((e = gcada::server_select(ctx, mask_out, loss_out, s)) != hipSuccess)
            return fail_hip(ctx, e, "selection kernels");
        if ((e = gcada::mlp_store_selected(ctx, s)) != hipSuccess)
            return fail_hip(ctx, e, "gradient store kernels");
    }
    e = ctx->lr_fused_finish ? gcada::lr_tile_finish(ctx, mask_out, loss_out, server_rule, s)
                             : gcada::server_step(ctx, mask_out, loss_out, server_rule || lazy, s);
    if (e != hipSuccess) return fail_hip(ctx, e, "server kernels");
    if (ctx->dims.model == GCADA_MLP) {
        // compute copies (padded, transposed, bf16) of the new iterate's hidden-layer weights; the
        // same launch sets the store flags of the next step from the ages and history just written
        e = gcada::mlp_refresh_slot(ctx, (int)((ctx->k + 1) % (ctx->hy.D + 1)), ctx->lazy_store, s);
        if (e != hipSuccess) return fail_hip(ctx, e, "weight copy kernel");
        ctx->flags_valid = ctx->lazy_store;
    }
    ctx->k += 1;
    return GCADA_OK;
}

int gcada_step_workers(gcada_ctx* ctx, const int32_t* idx_workers, const double* delays,
                       int32_t* worker_out, uint8_t* mask_out, float* loss_out, void* stream)
{
    if (!ctx) return GCADA_EINVAL;
    if (!idx_workers || !delays)
        return fail(ctx, GCADA_EINVAL, "step_workers: idx_workers and delays must not be NULL");
    hipError_t e = gcada::pick_fastest_workers(ctx, idx_workers, delays, worker_out, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "fastest-worker kernel");
    return gcada_step(ctx, ctx->idx_eff, mask_out, loss_out, stream);
}

int gcada_state(gcada_ctx* ctx, gcada_state_view* out)
{
    if (!ctx) return GCADA_EINVAL;
    if (!out) return fail(ctx, GCADA_EINVAL, "state: out must not be NULL");
    if (int rc = check_host_mirror(ctx)) return rc;
    if (hipError_t e = gcada::lr_tile_flush(ctx, nullptr, true); e != hipSuccess)
        return fail_hip(ctx, e, "finish kernel");
    if (hipError_t e = gcada::lr_tile_close(ctx, nullptr, true); e != hipSuccess)
        return fail_hip(ctx, e, "history kernel");
    gcada_state_view v{};
    v.p = ctx->hy.p; v.G = ctx->hy.G; v.D = ctx->hy.D; v.M_G = ctx->M_G;
    v.k = ctx->k;
    v.slot_stride = ctx->hy.pstride;
    v.grad_stride = ctx->hy.pstride;
    v.cur_slot = (int32_t)(ctx->k % (ctx->hy.D + 1));
    v.theta_ring = ctx->ring; v.h = ctx->h; v.vhat = ctx->vhat; v.agg = ctx->agg;
    v.gbuf = ctx->gbuf; v.which = ctx->which; v.tau = ctx->tau; v.dtheta_sq = ctx->nring;
    v.stat = ctx->stat; v.rhs = &ctx->ctl->rhs; v.mask = ctx->mask; v.loss = &ctx->ctl->loss;
    *out = v;
    return GCADA_OK;
}

int gcada_get_state(gcada_ctx* ctx, gcada_state_host* out)
try {
    if (!ctx) return GCADA_EINVAL;
    if (!out) return fail(ctx, GCADA_EINVAL, "get_state: out must not be NULL");
    const gcada::Hyper& hy = ctx->hy;
    const size_t p = (size_t)hy.p;
    const int nslot = hy.D + 1;
    HIP_TRY(ctx, gcada::lr_tile_flush(ctx, nullptr, true));
    HIP_TRY(ctx, gcada::lr_tile_close(ctx, nullptr, true));
    HIP_TRY(ctx, hipDeviceSynchronize());
    if (int rc = check_device_flag(ctx)) return rc;
    std::vector<int32_t> tau(hy.G);
    HIP_TRY(ctx, hipMemcpy(tau.data(), ctx->tau, (size_t)hy.G * 4, hipMemcpyDeviceToHost));
    const int cur = (int)(ctx->k % nslot);
    if (out->theta)
        HIP_TRY(ctx, hipMemcpy(out->theta, ctx->ring + (size_t)cur * hy.pstride, p * 4, hipMemcpyDeviceToHost));
    if (out->h) HIP_TRY(ctx, hipMemcpy(out->h, ctx->h, p * 4, hipMemcpyDeviceToHost));
    if (out->vhat) HIP_TRY(ctx, hipMemcpy(out->vhat, ctx->vhat, p * 4, hipMemcpyDeviceToHost));
    if (out->agg) HIP_TRY(ctx, hipMemcpy(out->agg, ctx->agg, p * 4, hipMemcpyDeviceToHost));
    if (out->theta_stale)
        for (int g = 0; g < hy.G; ++g) {
            const int slot = (int)(((ctx->k - tau[g]) % nslot + nslot) % nslot);
            HIP_TRY(ctx, hipMemcpy(out->theta_stale + (size_t)g * p, ctx->ring + (size_t)slot * hy.pstride,
                                   p * 4, hipMemcpyDeviceToHost));
        }
    if (out->last) {
        std::vector<int32_t> wh(hy.G);
        HIP_TRY(ctx, hipMemcpy(wh.data(), ctx->which, (size_t)hy.G * 4, hipMemcpyDeviceToHost));
        for (int g = 0; g < hy.G; ++g)
            HIP_TRY(ctx, hipMemcpy(out->last + (size_t)g * p,
                                   ctx->gbuf + ((size_t)wh[g] * hy.G + g) * hy.pstride, p * 4,
                                   hipMemcpyDeviceToHost));
    }
    if (out->tau) std::memcpy(out->tau, tau.data(), (size_t)hy.G * 4);
    if (out->dtheta_sq)
        HIP_TRY(ctx, hipMemcpy(out->dtheta_sq, ctx->nring, (size_t)hy.D * 8, hipMemcpyDeviceToHost));
    out->k = ctx->k;
    return GCADA_OK;
} catch (...) {
    return fail(ctx, GCADA_ENOMEM, "unexpected exception in gcada_get_state");
}

int gcada_set_state(gcada_ctx* ctx, const gcada_state_host* in)
try {
    if (!ctx) return GCADA_EINVAL;
    if (!in || !in->theta || !in->h || !in->vhat || !in->agg || !in->theta_stale || !in->last ||
        !in->tau || !in->dtheta_sq)
        return fail(ctx, GCADA_EINVAL, "set_state: every buffer must be given");
    const gcada::Hyper& hy = ctx->hy;
    if (in->k < 0) return fail(ctx, GCADA_EINVAL, "set_state: k must be >= 0");
    for (int g = 0; g < hy.G; ++g)
        if (in->tau[g] < 1 || in->tau[g] > hy.D)
            return fail(ctx, GCADA_EINVAL, "set_state: tau out of [1, D]");
    const size_t p = (size_t)hy.p;
    const int nslot = hy.D + 1;
    HIP_TRY(ctx, hipDeviceSynchronize());
    const int cur = (int)(in->k % nslot);
    // unreferenced slots get the current iterate (they are never read before being rewritten)
    for (int s = 0; s < nslot; ++s)
        HIP_TRY(ctx, hipMemcpy(ctx->ring + (size_t)s * hy.pstride, in->theta, p * 4, hipMemcpyHostToDevice));
    std::vector<uint8_t> filled(nslot, 0);
    for (int g = 0; g < hy.G; ++g) {
        const int slot = (int)(((in->k - in->tau[g]) % nslot + nslot) % nslot);
        if (filled[slot] || slot == cur) continue;
        HIP_TRY(ctx, hipMemcpy(ctx->ring + (size_t)slot * hy.pstride, in->theta_stale + (size_t)g * p,
                               p * 4, hipMemcpyHostToDevice));
        filled[slot] = 1;
    }
    HIP_TRY(ctx, hipMemcpy(ctx->h, in->h, p * 4, hipMemcpyHostToDevice));
    HIP_TRY(ctx, hipMemcpy(ctx->vhat, in->vhat, p * 4, hipMemcpyHostToDevice));
    HIP_TRY(ctx, hipMemcpy(ctx->agg, in->agg, p * 4, hipMemcpyHostToDevice));
    // stored gradients go to half 0 of gbuf
    HIP_TRY(ctx, hipMemset(ctx->which, 0, (size_t)hy.G * 4));
    HIP_TRY(ctx, hipMemcpy2D(ctx->gbuf, (size_t)hy.pstride * 4, in->last, p * 4, p * 4, hy.G,
                             hipMemcpyHostToDevice));
    HIP_TRY(ctx, hipMemcpy(ctx->tau, in->tau, (size_t)hy.G * 4, hipMemcpyHostToDevice));
    HIP_TRY(ctx, hipMemcpy(ctx->nring, in->dtheta_sq, (size_t)hy.D * 8, hipMemcpyHostToDevice));
    HIP_TRY(ctx, reset_control_block(ctx));
    ctx->k = in->k;
    int rc = after_state_change(ctx);
    if (rc != GCADA_OK) return rc;
    ctx->theta_set = true;
    return GCADA_OK;
} catch (...) {
    return fail(ctx, GCADA_ENOMEM, "unexpected exception in gcada_set_state");
}

int gcada_set_option(gcada_ctx* ctx, int32_t option, int32_t value)
{
    if (!ctx) return GCADA_EINVAL;
    // (a finish that is still to come runs under the options its step was issued with)
    if (option != GCADA_OPT_EXPIRE_NEXT_WAIT)
        if (hipError_t e = gcada::lr_tile_flush(ctx, nullptr, true); e != hipSuccess) return fail_hip(ctx, e, "finish kernel");
    if (option == GCADA_OPT_DEFERRED_FINISH) {
        ctx->allow_deferred_finish = value != 0;
        return GCADA_OK;
    }
    if (option == GCADA_OPT_SINGLE_PASS_LOGREG) {
        ctx->allow_single_pass = value != 0;
        return GCADA_OK;
    }
    if (option == GCADA_OPT_FUSED_FINISH) {
        ctx->allow_fused_finish = value != 0;
        return GCADA_OK;
    }
    if (option == GCADA_OPT_GRAM_STATISTIC) {
        ctx->allow_gram = value != 0;
        return GCADA_OK;
    }
    if (option == GCADA_OPT_LAZY_GRADIENT_STORE) {
        ctx->lazy_store = value != 0 && ctx->dims.model == GCADA_MLP;
        ctx->flags_valid = false;
        return GCADA_OK;
    }
    if (option == GCADA_OPT_EXPIRE_NEXT_WAIT) {
        ctx->expire_next_wait = value != 0;
        return GCADA_OK;
    }
    return fail(ctx, GCADA_EINVAL, "set_option: unknown option");
}

int gcada_set_rule(gcada_ctx* ctx, int32_t rule, const double* L)
{
    if (!ctx) return GCADA_EINVAL;
    if (hipError_t e = gcada::lr_tile_flush(ctx, nullptr, true); e != hipSuccess) return fail_hip(ctx, e, "finish kernel");
    if (rule != GCADA_RULE_GRADIENT_DIFFERENCE && rule != GCADA_RULE_SERVER)
        return fail(ctx, GCADA_EINVAL, "set_rule: unknown rule");
    if (L) {
        for (int g = 0; g < ctx->hy.G; ++g)
            if (!(L[g] >= 0.0) || !std::isfinite(L[g]))
                return fail(ctx, GCADA_EINVAL, "set_rule: every L_g must be finite and >= 0");
        hipError_t e = hipMemcpy(ctx->rule_L, L, sizeof(double) * (size_t)ctx->hy.G, hipMemcpyHostToDevice);
        if (e != hipSuccess) return fail_hip(ctx, e, "set_rule: copy of L");
        ctx->rule_L_set = true;
    }
    if (rule == GCADA_RULE_SERVER && !ctx->rule_L_set)
        return fail(ctx, GCADA_EINVAL, "set_rule: the server-side rule needs the constants L_g");
    if (rule == GCADA_RULE_SERVER && ctx->hy.D > 64)
        return fail(ctx, GCADA_EINVAL, "set_rule: the server-side rule supports D <= 64");
    ctx->rule = rule;
    return GCADA_OK;
}

int gcada_estimate_smoothness(gcada_ctx* ctx, int32_t iters, double* L_out, void* stream)
try {
    if (!ctx) return GCADA_EINVAL;
    if (!L_out || iters < 1) return fail(ctx, GCADA_EINVAL, "estimate_smoothness: L_out must not be NULL, iters >= 1");
    if (ctx->dims.model == GCADA_MLP)
        return fail(ctx, GCADA_EINVAL, "estimate_smoothness: linear models only (pass L_g to gcada_set_rule for an MLP)");
    for (int g = 0; g < ctx->hy.G; ++g)
        if (!ctx->shard_set[g]) return fail(ctx, GCADA_ESTATE, "estimate_smoothness: a group has no shard");
    // smoothness constant of the group's local function, the average loss over its shard
    // (Sec. IV): kappa * lambda_max(X^T X) / rows + lambda, kappa = 1/4 logistic, 1 quadratic
    const double kappa = ctx->dims.model == GCADA_LINREG ? 1.0 : 0.25;
    for (int g = 0; g < ctx->hy.G; ++g) {
        double lam = 0;
        hipError_t e = gcada::rule_power_iteration(ctx, g, iters, &lam, (hipStream_t)stream);
        if (e != hipSuccess) return fail_hip(ctx, e, "estimate_smoothness: power iteration");
        L_out[g] = kappa * lam / (double)ctx->shards[g].rows + (double)ctx->dims.l2;
    }
    return GCADA_OK;
} catch (...) {
    return fail(ctx, GCADA_ENOMEM, "unexpected exception in gcada_estimate_smoothness");
}

int gcada_estimate_smoothness_static(gcada_ctx* ctx, int32_t iters, double* L_out, void* stream)
{
    if (!ctx) return GCADA_EINVAL;
    if (!L_out || iters < 1)
        return fail(ctx, GCADA_EINVAL, "estimate_smoothness_static: L_out must not be NULL, iters >= 1");
    if (ctx->dims.model == GCADA_MLP)
        return fail(ctx, GCADA_EINVAL, "estimate_smoothness_static: linear models only");
    for (int g = 0; g < ctx->hy.G; ++g)
        if (!ctx->shard_set[g]) return fail(ctx, GCADA_ESTATE, "estimate_smoothness_static: a group has no shard");
    if (!ctx->static_scratch)
        return fail(ctx, GCADA_EDEVICE, "estimate_smoothness_static: the static scratch array was not resolved on this device");
    for (int g = 0; g < ctx->hy.G; ++g)
        if (gcada::rule_power_iteration_scratch_doubles(ctx, g) > gcada::rule_static_scratch_doubles()) {
            char msg[200];
            std::snprintf(msg, sizeof(msg),
                          "estimate_smoothness_static: shard %d needs %zu doubles of scratch, the static array holds %zu "
                          "(use gcada_estimate_smoothness)", g, gcada::rule_power_iteration_scratch_doubles(ctx, g),
                          gcada::rule_static_scratch_doubles());
            return fail(ctx, GCADA_EINVAL, msg);
        }
    hipError_t e = gcada::rule_smoothness_static(ctx, iters, L_out, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "estimate_smoothness_static: power iteration");
    return GCADA_OK;
}

const char* gcada_timed_stage(gcada_ctx* ctx)
{
    if (!ctx) return "";
    if (ctx->dims.model == GCADA_MLP)
        ctx->stage_name = gcada::mlp_gram_active(ctx)
            ? "mlp gradient stage (mlp_gemm forward/backward/weight-gradient, bias; first-layer statistic from Gram "
              "matrices, first-layer weight gradients after the selection for uploading groups only: fewer flops executed "
              "than the algorithmic count)"
            : "mlp gradient stage (gather, mlp_gemm forward/backward/weight-gradient, bias)";
    else if (ctx->rule != GCADA_RULE_SERVER && gcada::lr_micro_applies(ctx)) ctx->stage_name = "lr_micro_kernel (the whole iteration)";
    else if (gcada::lr_tile_applies(ctx)) ctx->stage_name = "lr_tile_kernel";
    else if (gcada::lr_team_applies(ctx)) ctx->stage_name = "lr_team_kernel";
    else ctx->stage_name = "lr_forward+lr_backward";
    return ctx->stage_name.c_str();
}

int gcada_time_gradient_stage(gcada_ctx* ctx, const int32_t* idx, int64_t idx_stride, int32_t reps,
                              void* stream, double* ms_per_rep)
try {
    if (!ctx) return GCADA_EINVAL;
    if (reps < 1 || !ms_per_rep) return fail(ctx, GCADA_EINVAL, "time_gradient_stage: reps >= 1 and an output are required");
    if (!ctx->theta_set) return fail(ctx, GCADA_ESTATE, "time_gradient_stage: gcada_set_theta has not been called");
    for (int g = 0; g < ctx->hy.G; ++g)
        if (!ctx->shard_set[g]) return fail(ctx, GCADA_ESTATE, "time_gradient_stage: a group has no shard");
    hipStream_t s = (hipStream_t)stream;
    if (hipError_t ef = gcada::lr_tile_flush(ctx, s, false); ef != hipSuccess) return fail_hip(ctx, ef, "finish kernel");
    set_iteration(ctx);
    hipEvent_t e0, e1;
    HIP_TRY(ctx, hipEventCreate(&e0));
    if (hipError_t ee = hipEventCreate(&e1); ee != hipSuccess) {
        (void)hipEventDestroy(e0);
        return fail_hip(ctx, ee, "hipEventCreate");
    }
    ctx->dominant_only = true;
    hipError_t e = hipSuccess;
    if (ctx->dims.model == GCADA_MLP && ctx->lazy_store && ctx->rule != GCADA_RULE_SERVER)
        e = gcada::lazy_flags(ctx, s);       // the stage stores what a step at this state would
    if (e == hipSuccess) e = hipEventRecord(e0, s);
    for (int r = 0; r < reps && e == hipSuccess; ++r)
    {
        const int32_t* ir = idx ? idx + (int64_t)r * idx_stride : nullptr;
        if (ctx->dims.model != GCADA_MLP && ctx->rule != GCADA_RULE_SERVER && gcada::lr_micro_applies(ctx))
            e = gcada::lr_micro_step(ctx, ir, nullptr, nullptr, true, s);      // changes no state
        else
            e = ctx->dims.model != GCADA_MLP ? gcada::lr_gradients(ctx, ir, s)
                                             : gcada::mlp_gradients(ctx, ir, s);
    }
    ctx->dominant_only = false;
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return fail_hip(ctx, e, "time_gradient_stage");
    *ms_per_rep = (double)ms / reps;
    return GCADA_OK;
} catch (...) {
    return fail(ctx, GCADA_ENOMEM, "unexpected exception in gcada_time_gradient_stage");
}

int gcada_hbm_read_calibration(const void* buf, int64_t bytes, int32_t reps, void* stream, double* gbps,
                               double* gbps_plain_loads)
{
    if (!buf || !gbps || reps < 1 || bytes < ((int64_t)64 << 20) || ((uintptr_t)buf % 16))
        return fail(nullptr, GCADA_EINVAL, "hbm_read_calibration: a 16-byte aligned device buffer of at least 64 MiB, reps >= 1 and an output are required");
    double g = 0;
    hipError_t e = gcada::hbm_read_calibration(buf, (size_t)bytes, reps, (hipStream_t)stream, &g, gbps_plain_loads);
    if (e != hipSuccess) return fail_hip(nullptr, e, "hbm_read_calibration");
    *gbps = g;
    return GCADA_OK;
}

int gcada_gather_read_calibration(gcada_ctx* ctx, const int32_t* idx, int64_t idx_stride, int32_t reps,
                                  void* stream, double* gbps)
{
    if (!ctx) return GCADA_EINVAL;
    if (!idx || reps < 1 || !gbps || idx_stride < 0)
        return fail(ctx, GCADA_EINVAL, "gather_read_calibration: row ids, reps >= 1 and an output are required");
    const int64_t d = ctx->hy.p;
    if (ctx->dims.model == GCADA_MLP || ctx->dims.dtype != GCADA_F32 || d % 4096 || d < 8192 || d / 4096 > 16 ||
        ctx->hy.mu % 4)
        return fail(ctx, GCADA_EINVAL, "gather_read_calibration: a linear fp32 model whose width is 2 to 16 times 4096 and a minibatch that is a multiple of 4 are required");
    for (int g = 0; g < ctx->hy.G; ++g) {
        if (!ctx->shard_set[g]) return fail(ctx, GCADA_ESTATE, "gather_read_calibration: a group has no shard");
        if (((uintptr_t)ctx->shards[g].X % 16) || ctx->shards[g].ld % 4)
            return fail(ctx, GCADA_EINVAL, "gather_read_calibration: shard rows must be 16-byte aligned");
    }
    double g = 0;
    hipError_t e = gcada::gather_read_calibration(ctx, idx, idx_stride, reps, (hipStream_t)stream, &g);
    if (e == hipErrorInvalidValue)
        return fail(ctx, GCADA_EINVAL, "gather_read_calibration: the tiles of the minibatches do not divide evenly among the teams of this device");
    if (e != hipSuccess) return fail_hip(ctx, e, "gather_read_calibration");
    *gbps = g;
    return GCADA_OK;
}

int gcada_cost_model(int32_t G, int32_t M_G, int32_t mu, const uint8_t* mask, const double* T,
                     double* time, int64_t* comm, int64_t* comp)
{
    if (G < 1 || M_G < 1 || mu < 1 || !mask) return GCADA_EINVAL;
    if (time && !T) return GCADA_EINVAL;
    int64_t nsel = 0;
    double tmax = 0.0;
    for (int g = 0; g < G; ++g) {
        if (!mask[g]) continue;
        ++nsel;
        if (time) {
            double tmin = T[(size_t)g * M_G];
            for (int m = 1; m < M_G; ++m) tmin = std::min(tmin, T[(size_t)g * M_G + m]);
            tmax = std::max(tmax, tmin);
        }
    }
    if (time) *time = tmax;
    if (comm) *comm = nsel * (int64_t)(M_G + 1);
    if (comp) *comp = nsel * (int64_t)M_G * (int64_t)mu;
    return GCADA_OK;
}

}  // extern "C"
