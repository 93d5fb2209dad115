/*
 * G-CADA reference oracle -- TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow, fp64 CPU statement of one G-CADA iteration (grouping-based
 * communication-adaptive distributed Adam): every worker group evaluates its
 * minibatch gradient at the current iterate and at the iterate of its last
 * upload, the server selects groups, sums the selected groups' innovations
 * into the lazily aggregated gradient and applies the AMSGrad-style update.
 * Only tests, the smoke check and the benchmark's cpu-baseline leg may use
 * this file; it shares no code with the GPU library.
 *
 * What follows the paper directly:
 *   - minibatch gradient = gradient of the SUM of the per-sample losses
 *     over the minibatch (Sec. II-A);
 *   - aggregate = fresh gradients of the selected groups plus the last
 *     uploaded gradients of the others (Sec. IV, the aggregated-gradient
 *     expression; Eq. (3));
 *   - server update h, v, v-hat, theta (Eq. (8a)-(8c)): v is built from the
 *     previous v-hat, epsilon sits inside the square root, no bias correction;
 *   - right-hand side of the selection rule: the sum over the last D squared
 *     iterate differences (Eq. (9)); age-of-information counters with a forced
 *     upload once the age reaches D and "age + 1" for unselected groups
 *     (Algorithm 1).
 * What is a reading (the paper's left-hand side of Eq. (9) needs smoothness
 * constants; this method evaluates the quantity that side estimates, Sec. III):
 *   stat_g = || grad(theta^k; xi_g) - grad(theta_stale_g; xi_g) ||^2 on the
 *   same minibatch, compared against (c/D) * sum of the last D squared
 *   iterate differences; a group is also selected when that threshold is 0.
 *
 * Pins (tests/test_oracle_*.py): closed forms of the moment recursions under
 * a constant gradient, central finite differences of the loss, the logistic
 * loss and gradient at theta = 0, library autograd on tiny networks, the
 * c = 0 collapse to plain distributed AMSGrad, the periodic mask for huge c,
 * the aggregate identity, group-permutation invariance; the ReLU-kink
 * diagnostic against hand-built power-of-two networks.  The figures the
 * paper prints for its experiment (Sec. VI) need its dataset and unstated
 * settings: parity unpinned for those.
 *
 * Parameter vector layout (an interface; the GPU library uses the same):
 *   logistic / quadratic: theta[d]
 *   MLP: for each layer l = 1..L:  W_l (n_l x n_{l-1}, row-major), then b_l (n_l)
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_LOGISTIC = 0, ORC_MLP = 1, ORC_QUADRATIC = 2 };

typedef struct orc_config {
    int32_t model;       /* ORC_* */
    int32_t n_widths;    /* logistic/quadratic: 1 ({d}); MLP: number of layer widths incl. input */
    int32_t widths[8];
    int32_t batch;       /* mu: minibatch size per group */
    int32_t G;           /* number of groups */
    int32_t D;           /* history depth / maximum age */
    int32_t round_bf16;  /* 1: gradients are evaluated at theta rounded fp64->fp32->bf16 (RNE);
                            2: also every hidden activation is rounded to bf16 (every layer's
                               product then has bf16 inputs), see mlp_sample */
    double l2;           /* lambda: each sample's loss gets + (lambda/2)||theta||^2 */
    double c, alpha, beta1, beta2, eps;
} orc_config;

typedef struct orc_ctx {
    orc_config cfg;
    int64_t p;
    int64_t k;
    double *theta, *h, *vhat, *agg;      /* p each                              */
    double *theta_stale, *last;          /* G x p: iterate / gradient at last upload */
    double *grad, *grad_stale;           /* G x p: this step's two gradients    */
    double *stat;                        /* G                                   */
    double *ring;                        /* D squared iterate differences       */
    double *loss_g;                      /* G: minibatch loss sums at theta^k   */
    double *kink;                        /* G: smallest relative distance of a hidden pre-activation
                                            to the ReLU kink in this step (diagnostic; 1 if none) */
    double *kink_unit;                   /* G x H, H = sum of the hidden widths: the same per hidden
                                            unit (layer 1's units first), minimum over the group's
                                            samples and both iterates; 1 if never evaluated */
    int64_t H;
    double rhs, loss;
    int32_t *tau;                        /* G                                   */
    uint8_t *mask;                       /* G                                   */
    int32_t rule;                        /* 0: same-minibatch gradient difference; 1: the server-side
                                            condition of Sec. IV with smoothness constants L_g */
    double *L;                           /* G (rule 1)                          */
} orc_ctx;

/* ---------- helpers ---------------------------------------------------- */

static double bf16_round(double x)
{
    /* fp64 -> fp32 (round to nearest even, the C conversion), then keep the top
       16 bits of the fp32 pattern with round to nearest even. */
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) return (double)f;   /* inf / nan pass through */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

int64_t orc_param_count(const orc_config *cfg)
{
    if (cfg->model != ORC_MLP) return cfg->widths[0];
    int64_t p = 0;
    for (int l = 1; l < cfg->n_widths; ++l)
        p += (int64_t)cfg->widths[l] * cfg->widths[l - 1] + cfg->widths[l];
    return p;
}

/* log(1 + exp(t)) without overflow */
static double softplus(double t)
{
    return t > 0 ? t + log1p(exp(-t)) : log1p(exp(t));
}

static double sigmoid(double t)
{
    if (t >= 0) return 1.0 / (1.0 + exp(-t));
    double e = exp(t);
    return e / (1.0 + e);
}

/* ---------- per-sample losses and gradients ---------------------------- */

/* logistic: y in {-1,+1}; loss = log(1 + exp(-y x.theta));
   gradient = -y * sigmoid(-y x.theta) * x.   No intercept. */
static double logistic_sample(const double *theta, const float *x, double y, int64_t d, double *grad)
{
    double z = 0;
    for (int64_t j = 0; j < d; ++j) z += (double)x[j] * theta[j];
    if (grad) {
        double r = -y * sigmoid(-y * z);
        for (int64_t j = 0; j < d; ++j) grad[j] += r * (double)x[j];
    }
    return softplus(-y * z);
}

/* linear regression with the quadratic error loss, the model of the paper's experiment
 * (Sec. VI), scalar output: loss = 0.5 (x.theta - y)^2 */
static double quadratic_sample(const double *theta, const float *x, double y, int64_t d, double *grad)
{
    double z = 0;
    for (int64_t j = 0; j < d; ++j) z += (double)x[j] * theta[j];
    double r = z - y;
    if (grad)
        for (int64_t j = 0; j < d; ++j) grad[j] += r * (double)x[j];
    return 0.5 * r * r;
}

/* MLP: a_0 = x; z_l = W_l a_{l-1} + b_l; a_l = max(z_l, 0) for l < L; logits = z_L;
   loss = log sum exp(logits) - logits[y].  ReLU'(0) = 0.
   round_bf16 == 2 (the bf16 configuration: "bf16 inputs and weights, fp32 accumulation" read as
   every layer's matrix product taking bf16 inputs): a_l <- bf16(a_l) for the hidden layers, so
   the next layer's pre-activation -- whose SIGN is a discrete decision (which ReLU branch) -- is
   formed from the values a bf16 implementation multiplies; the rounding is treated as the
   identity in the backward pass (the signal passes where a_l > 0) and the weight gradient
   multiplies the rounded activation.  Sums stay fp64 and nothing else is rounded.
   work: 2 * sum(widths) doubles (activations, then deltas). */
static double mlp_sample(const orc_config *cfg, const double *theta, const float *x, int32_t y,
                         double *grad, double *work, double *kink, double *kink_unit)
{
    const int L = cfg->n_widths - 1;
    const int32_t *n = cfg->widths;
    double *act[8], *del[8];
    double *w = work;
    for (int l = 0; l <= L; ++l) { act[l] = w; w += n[l]; }
    for (int l = 0; l <= L; ++l) { del[l] = w; w += n[l]; }

    for (int j = 0; j < n[0]; ++j) act[0][j] = (double)x[j];
    const double *W = theta;
    int64_t unit0 = 0;                   /* index of this layer's first unit among the hidden units */
    for (int l = 1; l <= L; ++l) {
        const double *b = W + (int64_t)n[l] * n[l - 1];
        for (int o = 0; o < n[l]; ++o) {
            double z = b[o], az = fabs(b[o]);
            const double *row = W + (int64_t)o * n[l - 1];
            for (int i = 0; i < n[l - 1]; ++i) {
                z += row[i] * act[l - 1][i];
                az += fabs(row[i] * act[l - 1][i]);
            }
            /* diagnostic only: how close this hidden pre-activation is to the ReLU kink, relative
               to the sum of the magnitudes of its terms (a comparison in lower precision may
               land on the other side of the kink when this is tiny) */
            if (kink && l < L && az > 0 && fabs(z) / az < *kink) *kink = fabs(z) / az;
            if (kink_unit && l < L && az > 0 && fabs(z) / az < kink_unit[unit0 + o]) kink_unit[unit0 + o] = fabs(z) / az;
            act[l][o] = (l < L && z < 0) ? 0.0 : z;      /* z == 0 stays 0 either way */
            if (l < L && cfg->round_bf16 == 2) act[l][o] = bf16_round(act[l][o]);
        }
        W = b + n[l];
        unit0 += n[l];
    }
    /* softmax cross-entropy on the logits act[L] */
    double zmax = act[L][0];
    for (int o = 1; o < n[L]; ++o) if (act[L][o] > zmax) zmax = act[L][o];
    double se = 0;
    for (int o = 0; o < n[L]; ++o) se += exp(act[L][o] - zmax);
    double loss = zmax + log(se) - act[L][y];
    if (!grad) return loss;

    for (int o = 0; o < n[L]; ++o) del[L][o] = exp(act[L][o] - zmax) / se - (o == y ? 1.0 : 0.0);
    /* walk the layers backwards; W points one past the last layer's block */
    const double *Wend = theta + orc_param_count(cfg);
    double *gend = grad + orc_param_count(cfg);
    for (int l = L; l >= 1; --l) {
        int64_t blk = (int64_t)n[l] * n[l - 1] + n[l];
        const double *Wl = Wend - blk;
        double *gW = gend - blk;
        double *gb = gW + (int64_t)n[l] * n[l - 1];
        for (int o = 0; o < n[l]; ++o) {
            double dl = del[l][o];
            gb[o] += dl;
            double *grow = gW + (int64_t)o * n[l - 1];
            for (int i = 0; i < n[l - 1]; ++i) grow[i] += dl * act[l - 1][i];
        }
        if (l > 1) {
            for (int i = 0; i < n[l - 1]; ++i) {
                double s = 0;
                for (int o = 0; o < n[l]; ++o) s += Wl[(int64_t)o * n[l - 1] + i] * del[l][o];
                del[l - 1][i] = act[l - 1][i] > 0 ? s : 0.0;   /* ReLU'(0) = 0 */
            }
        }
        Wend = Wl;
        gend = gW;
    }
    return loss;
}

/* Sum over n samples of [ loss(theta; z) + (l2/2)||theta||^2 ]; if grad != NULL it is
   OVERWRITTEN with the gradient of that sum.  X is n x widths[0] row-major fp32 (promoted
   exactly); y is float[n] (logistic: +-1, quadratic: target) or int32[n] (MLP class id). */
static double loss_grad_sum_k(const orc_config *cfg, const double *theta, const float *X,
                              const void *y, int64_t n, double *grad, double *kink, double *kink_unit)
{
    const int64_t p = orc_param_count(cfg);
    const int64_t d = cfg->widths[0];
    double *work = NULL;
    if (cfg->model == ORC_MLP) {
        int64_t s = 0;
        for (int l = 0; l < cfg->n_widths; ++l) s += cfg->widths[l];
        work = (double *)malloc(sizeof(double) * 2 * s);
    }
    if (grad) memset(grad, 0, sizeof(double) * p);
    double loss = 0;
    for (int64_t i = 0; i < n; ++i) {
        const float *x = X + i * d;
        if (cfg->model == ORC_LOGISTIC)
            loss += logistic_sample(theta, x, (double)((const float *)y)[i], d, grad);
        else if (cfg->model == ORC_QUADRATIC)
            loss += quadratic_sample(theta, x, (double)((const float *)y)[i], d, grad);
        else
            loss += mlp_sample(cfg, theta, x, ((const int32_t *)y)[i], grad, work, kink, kink_unit);
    }
    free(work);
    if (cfg->l2 != 0) {
        double sq = 0;
        for (int64_t j = 0; j < p; ++j) sq += theta[j] * theta[j];
        loss += (double)n * 0.5 * cfg->l2 * sq;
        if (grad)
            for (int64_t j = 0; j < p; ++j) grad[j] += (double)n * cfg->l2 * theta[j];
    }
    return loss;
}

double orc_loss_grad_sum(const orc_config *cfg, const double *theta, const float *X, const void *y,
                         int64_t n, double *grad)
{
    return loss_grad_sum_k(cfg, theta, X, y, n, grad, NULL, NULL);
}

/* Server update, Eq. (8a)-(8c):
     h     <- beta1 h + (1 - beta1) agg
     v     <- beta2 vhat + (1 - beta2) agg^2          (from the previous v-hat)
     vhat  <- max(vhat, v)
     theta <- theta - alpha h / sqrt(eps + vhat)      (eps inside the root)
   Returns || theta_new - theta_old ||^2. */
double orc_amsgrad(double *theta, double *h, double *vhat, const double *agg, int64_t p,
                   double alpha, double beta1, double beta2, double eps)
{
    double sq = 0;
    for (int64_t j = 0; j < p; ++j) {
        h[j] = beta1 * h[j] + (1.0 - beta1) * agg[j];
        double v = beta2 * vhat[j] + (1.0 - beta2) * agg[j] * agg[j];
        if (v > vhat[j]) vhat[j] = v;
        double tn = theta[j] - alpha * h[j] / sqrt(eps + vhat[j]);
        double dt = tn - theta[j];
        sq += dt * dt;
        theta[j] = tn;
    }
    return sq;
}

/* ---------- the iteration ---------------------------------------------- */

void orc_destroy(orc_ctx *c)
{
    if (!c) return;
    free(c->theta); free(c->h); free(c->vhat); free(c->agg);
    free(c->theta_stale); free(c->last); free(c->grad); free(c->grad_stale);
    free(c->stat); free(c->ring); free(c->loss_g); free(c->kink); free(c->kink_unit); free(c->tau); free(c->mask);
    free(c->L);
    free(c);
}

orc_ctx *orc_create(const orc_config *cfg)
{
    if (cfg->G < 1 || cfg->D < 1 || cfg->batch < 1 || cfg->n_widths < 1 || cfg->n_widths > 8)
        return NULL;
    if (cfg->model == ORC_MLP && cfg->n_widths < 2) return NULL;
    orc_ctx *c = (orc_ctx *)calloc(1, sizeof(orc_ctx));
    c->cfg = *cfg;
    c->p = orc_param_count(cfg);
    const int64_t p = c->p, G = cfg->G;
    c->theta = calloc(p, 8); c->h = calloc(p, 8); c->vhat = calloc(p, 8); c->agg = calloc(p, 8);
    c->theta_stale = calloc(G * p, 8); c->last = calloc(G * p, 8);
    c->grad = calloc(G * p, 8); c->grad_stale = calloc(G * p, 8);
    c->stat = calloc(G, 8); c->ring = calloc(cfg->D, 8); c->loss_g = calloc(G, 8); c->kink = calloc(G, 8);
    c->tau = calloc(G, 4); c->mask = calloc(G, 1); c->L = calloc(G, 8);
    c->H = 0;
    if (cfg->model == ORC_MLP)
        for (int l = 1; l < cfg->n_widths - 1; ++l) c->H += cfg->widths[l];
    c->kink_unit = calloc(G * (c->H > 0 ? c->H : 1), 8);
    for (int g = 0; g < G; ++g) c->tau[g] = cfg->D;
    return c;
}

/* Start of a run: theta <- theta0, moments, aggregate and stored gradients 0, every stale
   iterate = theta0, every age = D (so the first step selects everyone), empty history. */
void orc_reset(orc_ctx *c, const double *theta0)
{
    const int64_t p = c->p, G = c->cfg.G;
    memcpy(c->theta, theta0, 8 * p);
    memset(c->h, 0, 8 * p); memset(c->vhat, 0, 8 * p); memset(c->agg, 0, 8 * p);
    memset(c->last, 0, 8 * G * p);
    for (int64_t g = 0; g < G; ++g) {
        memcpy(c->theta_stale + g * p, theta0, 8 * p);
        c->tau[g] = c->cfg.D;
    }
    memset(c->ring, 0, 8 * c->cfg.D);
    c->k = 0;
}

/* Which selection rule the steps use.  rule 0 (default): a group is selected when the squared
   norm of the difference of its two same-minibatch gradients exceeds the threshold.  rule 1:
   the condition the paper states for the server (Sec. IV, the inequality with L_g): a group
   is selected when L_g^2 ||theta^k - theta^{k - tau_g}||^2 exceeds the same threshold; then
   only the selected groups evaluate a gradient, once, at theta^k (Algorithm 1).  L: G
   smoothness constants (an input of Algorithm 1). */
void orc_set_rule(orc_ctx *c, int32_t rule, const double *L)
{
    c->rule = rule;
    if (L) memcpy(c->L, L, 8 * (size_t)c->cfg.G);
}

/* One iteration under rule 1.  The statistic field holds the left side of the condition;
   the loss is the mean over the samples that were evaluated (0 when no group is selected). */
static void orc_step_server_rule(orc_ctx *c, const float *X, const void *y, uint8_t *mask_out,
                                 double *loss_out)
{
    const orc_config *cfg = &c->cfg;
    const int64_t p = c->p, G = cfg->G, mu = cfg->batch, d = cfg->widths[0];

    /* threshold, left sides, selection -- no gradient is needed for this */
    double hist = 0;
    for (int j = 0; j < cfg->D; ++j) hist += c->ring[j];
    c->rhs = cfg->c / (double)cfg->D * hist;
    for (int64_t g = 0; g < G; ++g) {
        double dist = 0;
        for (int64_t j = 0; j < p; ++j) {
            double df = c->theta[j] - c->theta_stale[g * p + j];
            dist += df * df;
        }
        c->stat[g] = c->L[g] * c->L[g] * dist;
        c->mask[g] = (c->stat[g] > c->rhs) || (c->tau[g] >= cfg->D) || (c->rhs == 0.0);
    }

    /* the selected groups evaluate their minibatch gradient at theta^k */
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t g = 0; g < G; ++g) {
        c->kink[g] = 1.0;
        for (int64_t u = 0; u < c->H; ++u) c->kink_unit[g * c->H + u] = 1.0;
        c->loss_g[g] = 0;
        if (!c->mask[g]) continue;
        const float *Xg = X + g * mu * d;
        const void *yg = (const char *)y + g * mu * 4;
        double *pt = c->theta, *ev = NULL;
        if (cfg->round_bf16) {
            ev = malloc(8 * p);
            for (int64_t j = 0; j < p; ++j) ev[j] = bf16_round(pt[j]);
            pt = ev;
        }
        c->loss_g[g] = loss_grad_sum_k(cfg, pt, Xg, yg, mu, c->grad + g * p, c->kink + g, c->kink_unit + g * c->H);
        free(ev);
    }
    double loss = 0;
    int64_t nsel = 0;
    for (int64_t g = 0; g < G; ++g)
        if (c->mask[g]) { loss += c->loss_g[g]; ++nsel; }
    c->loss = nsel ? loss / (double)(nsel * mu) : 0.0;

    for (int64_t g = 0; g < G; ++g) {
        if (c->mask[g]) {
            for (int64_t j = 0; j < p; ++j) {
                c->agg[j] += c->grad[g * p + j] - c->last[g * p + j];
                c->last[g * p + j] = c->grad[g * p + j];
                c->theta_stale[g * p + j] = c->theta[j];
            }
            c->tau[g] = 1;
        } else {
            c->tau[g] += 1;
        }
    }
    double sq = orc_amsgrad(c->theta, c->h, c->vhat, c->agg, p, cfg->alpha, cfg->beta1,
                            cfg->beta2, cfg->eps);
    c->ring[c->k % cfg->D] = sq;
    c->k += 1;
    if (mask_out) memcpy(mask_out, c->mask, G);
    if (loss_out) *loss_out = c->loss;
}

/* One iteration.  X: G x mu x widths[0] fp32 (group g's minibatch rows), y: G x mu
   (float or int32 as for orc_loss_grad_sum).  mask_out: G bytes.  loss_out: mean minibatch
   loss at theta^k over all G*mu samples (+ (l2/2)||theta||^2). */
void orc_step(orc_ctx *c, const float *X, const void *y, uint8_t *mask_out, double *loss_out)
{
    const orc_config *cfg = &c->cfg;
    const int64_t p = c->p, G = cfg->G, mu = cfg->batch, d = cfg->widths[0];
    const int64_t ysz = 4;   /* float and int32 are both 4 bytes */
    if (c->rule == 1) { orc_step_server_rule(c, X, y, mask_out, loss_out); return; }

    /* 1. two gradients per group on the same samples; statistic; loss */
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t g = 0; g < G; ++g) {
        const float *Xg = X + g * mu * d;
        const void *yg = (const char *)y + g * mu * ysz;
        double *pt = c->theta, *ps = c->theta_stale + g * p;
        double *ev = NULL, *evs = NULL;
        if (cfg->round_bf16) {
            ev = malloc(8 * p); evs = malloc(8 * p);
            for (int64_t j = 0; j < p; ++j) { ev[j] = bf16_round(pt[j]); evs[j] = bf16_round(ps[j]); }
            pt = ev; ps = evs;
        }
        c->kink[g] = 1.0;
        for (int64_t u = 0; u < c->H; ++u) c->kink_unit[g * c->H + u] = 1.0;
        c->loss_g[g] = loss_grad_sum_k(cfg, pt, Xg, yg, mu, c->grad + g * p, c->kink + g, c->kink_unit + g * c->H);
        loss_grad_sum_k(cfg, ps, Xg, yg, mu, c->grad_stale + g * p, c->kink + g, c->kink_unit + g * c->H);
        double s = 0;
        for (int64_t j = 0; j < p; ++j) {
            double df = c->grad[g * p + j] - c->grad_stale[g * p + j];
            s += df * df;
        }
        c->stat[g] = s;
        free(ev); free(evs);
    }
    double loss = 0;
    for (int64_t g = 0; g < G; ++g) loss += c->loss_g[g];
    c->loss = loss / (double)(G * mu);

    /* 2. threshold and selection */
    double hist = 0;
    for (int j = 0; j < cfg->D; ++j) hist += c->ring[j];
    c->rhs = cfg->c / (double)cfg->D * hist;
    for (int64_t g = 0; g < G; ++g)
        c->mask[g] = (c->stat[g] > c->rhs) || (c->tau[g] >= cfg->D) || (c->rhs == 0.0);

    /* 3. lazily aggregated gradient: selected groups replace their stored gradient */
    for (int64_t g = 0; g < G; ++g) {
        if (c->mask[g]) {
            for (int64_t j = 0; j < p; ++j) {
                c->agg[j] += c->grad[g * p + j] - c->last[g * p + j];
                c->last[g * p + j] = c->grad[g * p + j];
                c->theta_stale[g * p + j] = c->theta[j];
            }
            c->tau[g] = 1;
        } else {
            c->tau[g] += 1;
        }
    }

    /* 4. server update and history */
    double sq = orc_amsgrad(c->theta, c->h, c->vhat, c->agg, p, cfg->alpha, cfg->beta1,
                            cfg->beta2, cfg->eps);
    c->ring[c->k % cfg->D] = sq;
    c->k += 1;

    if (mask_out) memcpy(mask_out, c->mask, G);
    if (loss_out) *loss_out = c->loss;
}

/* ---------- state access for the tests --------------------------------- */

enum { ORC_F_THETA = 0, ORC_F_H, ORC_F_VHAT, ORC_F_AGG, ORC_F_THETA_STALE, ORC_F_LAST,
       ORC_F_GRAD, ORC_F_GRAD_STALE, ORC_F_STAT, ORC_F_RING, ORC_F_LOSS_G, ORC_F_KINK, ORC_F_KINK_UNIT };

double *orc_field(orc_ctx *c, int32_t id, int64_t *count)
{
    const int64_t p = c->p, G = c->cfg.G;
    switch (id) {
    case ORC_F_THETA: *count = p; return c->theta;
    case ORC_F_H: *count = p; return c->h;
    case ORC_F_VHAT: *count = p; return c->vhat;
    case ORC_F_AGG: *count = p; return c->agg;
    case ORC_F_THETA_STALE: *count = G * p; return c->theta_stale;
    case ORC_F_LAST: *count = G * p; return c->last;
    case ORC_F_GRAD: *count = G * p; return c->grad;
    case ORC_F_GRAD_STALE: *count = G * p; return c->grad_stale;
    case ORC_F_STAT: *count = G; return c->stat;
    case ORC_F_RING: *count = c->cfg.D; return c->ring;
    case ORC_F_LOSS_G: *count = G; return c->loss_g;
    case ORC_F_KINK: *count = G; return c->kink;
    case ORC_F_KINK_UNIT: *count = G * c->H; return c->kink_unit;
    default: *count = 0; return NULL;
    }
}

int32_t *orc_tau(orc_ctx *c) { return c->tau; }
uint8_t *orc_mask(orc_ctx *c) { return c->mask; }
double orc_rhs(const orc_ctx *c) { return c->rhs; }
double orc_loss(const orc_ctx *c) { return c->loss; }
int64_t orc_k(const orc_ctx *c) { return c->k; }
void orc_set_k(orc_ctx *c, int64_t k) { c->k = k; }
int64_t orc_p(const orc_ctx *c) { return c->p; }
double orc_bf16_round(double x) { return bf16_round(x); }
