/*
 * AsyncMesh per-stage update -- plain CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what the
 * update computes.  It is called by the tests, by the smoke check and by the benchmark's CPU
 * baseline leg; the product (the HIP library) never links, loads or calls it, and the two share
 * no code.
 *
 * What is computed, for ONE pipeline stage of n parameters replicated R (= m in the paper) times,
 * at step t = 1, 2, ...:
 *
 *   1. local step      w^_i^t = OPT(w_i^{t-1}, g_i^{t-1})            (sparse-averaging equation, line 1)
 *   2. send            if t mod K == 0: keep a copy of w^_i^t for every replica
 *                                                                    (buffered simulation of the delay)
 *   3. receive         if t mod K == 0 and s = t - tau*K >= 1, for every mu in S^s:
 *                        abar    = (1/R) sum_i w^_i^s[mu]            (old average; async sparse averaging eq.)
 *                        d_i[mu] = (1-lambda) d_i[mu] + lambda (w^_i^t[mu] - w^_i^s[mu])     (EMA equation)
 *                        w_i^t[mu] = abar + d_i[mu]                  (estimated average; corrected update)
 *                      (correction NONE: w_i^t[mu] = abar;  correction EAGER, the eager-DiLoCo special case
 *                       named after the estimated-average equations: d_i[mu] = (1/R)(w^_i^t[mu] - w^_i^s[mu]),
 *                       no memory);  mu not in S^s: w_i^t[mu] = w^_i^t[mu]
 *   4. look-ahead      fwd_i^t = w_i^t + gamma (w^_i^t - w_i^{t-1})  (NAG-style extrapolation of the
 *                                                                    optimizer's last displacement)
 *
 * S^s = { mu : philox4x32_10(counter = (lo32(mu>>2), hi32(mu>>2), lo32(s), hi32(s)),
 *                            key = (lo32(seed), hi32(seed)))[mu & 3]  <  floor(p * 2^32) }
 * i.e. every coordinate is in the subset independently with probability p (the sampling model of
 * the sparse-averaging lemma), the subset is shared by all replicas and redrawn every step.
 *
 * Precision: the paper's implementation is FP32.  All state (w, m, v, d, fwd, the kept copies) is
 * stored in fp32; every expression is evaluated in fp64 from the stored fp32 values and rounded
 * ONCE when stored.  A later expression uses the stored (rounded) value, never the unrounded one.
 *
 * The kept copies are FULL copies of w^_i (tau*K+1 of them): only their subset entries are ever
 * read, so this equals any packed representation, and it is the simplest thing that is right.
 *
 * A slice [mu0, mu0+n) of a longer stage can be evaluated on its own (every operation is
 * coordinate-wise given (seed, step, global mu)); mu0 is the global index of local element 0.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------------------------ */
/* Philox4x32-10, Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",   */
/* SC'11.  Ten rounds; round constants and key schedule as published.                          */
/* ------------------------------------------------------------------------------------------ */
void amo_philox4x32_10(const uint32_t counter[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;   /* multipliers */
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;   /* Weyl key increments */
    uint32_t c0 = counter[0], c1 = counter[1], c2 = counter[2], c3 = counter[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = M0 * (uint64_t)c0;
        uint64_t p1 = M1 * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* threshold T = floor(p * 2^32) as a 64-bit integer; p = 1 gives 2^32 (every coordinate) */
uint64_t amo_threshold(double p)
{
    if (!(p > 0.0)) return 0;
    if (p >= 1.0) return (uint64_t)1 << 32;
    return (uint64_t)floor(p * 4294967296.0);
}

/* is global coordinate mu in the subset drawn for step s ?
 * granule 1: every coordinate is drawn on its own (the paper's sampling model).
 * granule g > 1 (a variant, not the paper's): aligned blocks of g consecutive coordinates are drawn
 * as a whole, block b = mu / g taking the place of the coordinate in the counter; every coordinate
 * is still in the subset with probability p (all the sparse-averaging lemma uses), but coordinates
 * of one block are no longer independent. */
int amo_member(uint64_t seed, uint64_t s, uint64_t mu, uint64_t threshold, uint32_t granule)
{
    if (granule > 1) mu /= granule;
    uint64_t group = mu >> 2;
    uint32_t counter[4] = { (uint32_t)group, (uint32_t)(group >> 32), (uint32_t)s, (uint32_t)(s >> 32) };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t x[4];
    amo_philox4x32_10(counter, key, x);
    return (uint64_t)x[mu & 3] < threshold;
}

/* Stratified VARIANT of the sampling (not the paper's independent draws; the exact-size alternative
 * that keeps the marginal inclusion probability, which is all the sparse-averaging lemma uses):
 * the coordinates are cut into aligned blocks of B = round(1/p) and exactly one coordinate of every
 * block is in S^s, at offset floor(X B / 2^32) inside the block, X the generator word that
 * coordinate number b = mu / B would get.  So |S^s| = ceil-or-floor(n / B) exactly and every
 * coordinate is in S^s with probability 1/B (up to B / 2^32). */
uint64_t amo_block_size(double p)
{
    if (!(p > 0.0)) return 0;
    const long long B = llround(1.0 / p);
    return B < 1 ? 1 : (uint64_t)B;
}

int amo_member_stratified(uint64_t seed, uint64_t s, uint64_t mu, uint64_t B)
{
    const uint64_t b = mu / B, group = b >> 2;
    uint32_t counter[4] = { (uint32_t)group, (uint32_t)(group >> 32), (uint32_t)s, (uint32_t)(s >> 32) };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t x[4];
    amo_philox4x32_10(counter, key, x);
    return mu - b * B == (((uint64_t)x[b & 3] * B) >> 32);
}

/* the sampling rule in force: independent draws (per coordinate or per aligned block of
 * `granule`), or the stratified variant */
static int in_subset(uint64_t seed, uint64_t s, uint64_t mu, double p, uint32_t granule, uint32_t stratified)
{
    if (stratified) return amo_member_stratified(seed, s, mu, amo_block_size(p));
    return amo_member(seed, s, mu, amo_threshold(p), granule);
}

/* ascending list of the members of S^s inside [mu0, mu0+n); returns how many there are
 * (all of them are counted even when out_capacity is too small to hold them) */
uint64_t amo_subset(uint64_t seed, uint64_t s, uint64_t mu0, uint64_t n, double p, uint32_t granule,
                    uint32_t stratified, uint64_t *out, uint64_t out_capacity)
{
    uint64_t count = 0;
    for (uint64_t k = 0; k < n; ++k)
        if (in_subset(seed, s, mu0 + k, p, granule, stratified)) {
            if (out && count < out_capacity) out[count] = mu0 + k;
            ++count;
        }
    return count;
}

/* ------------------------------------------------------------------------------------------ */
/* bfloat16 helpers (1 sign, 8 exponent, 7 fraction bits = the top half of an IEEE binary32)   */
/* ------------------------------------------------------------------------------------------ */
float amo_bf16_to_float(uint16_t h)
{
    uint32_t bits = (uint32_t)h << 16;
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

/* round-to-nearest-even of a double to bfloat16, in one rounding */
uint16_t amo_double_to_bf16(double x)
{
    if (x != x) return 0x7FC0;
    double ax = fabs(x);
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    if (ax == 0.0) return sign;
    int e;
    (void)frexp(ax, &e);                      /* ax = frac * 2^e with frac in [0.5, 1) */
    int exp_unbiased = e - 1;                 /* so ax = (2 frac) * 2^(e-1), 2 frac in [1, 2) */
    if (exp_unbiased < -126) exp_unbiased = -126;       /* subnormal range: fixed quantum */
    double quantum = ldexp(1.0, exp_unbiased - 7);      /* spacing of bf16 numbers near ax */
    double q = nearbyint(ax / quantum);                 /* default rounding mode: ties to even */
    double r = q * quantum;
    if (r >= ldexp(1.0, 128)) return sign | 0x7F80;     /* overflow to infinity */
    float rf = (float)r;                                /* exact: r has <= 8 significant bits */
    uint32_t bits;
    memcpy(&bits, &rf, 4);
    return sign | (uint16_t)(bits >> 16);
}

/* round-to-nearest-even of a double to the 8-bit float E4M3 (OCP "FN" flavour: 1 sign, 4 exponent
 * bits with bias 7, 3 fraction bits, no infinity, largest finite value 448), saturating; returned
 * as the value it represents */
double amo_quantize_e4m3(double x)
{
    if (x != x) return x;
    double ax = fabs(x);
    if (ax == 0.0) return x;
    int e;
    (void)frexp(ax, &e);
    int exp_unbiased = e - 1;
    if (exp_unbiased < -6) exp_unbiased = -6;           /* subnormals: fixed quantum 2^-9 */
    double quantum = ldexp(1.0, exp_unbiased - 3);
    double r = nearbyint(ax / quantum) * quantum;
    if (r > 448.0) r = 448.0;
    return signbit(x) ? -r : r;
}

/* what a replica's value becomes on the wire: 0 = fp32 (unchanged), 1 = bfloat16, 2 = E4M3 */
enum { AMO_MSG_F32 = 0, AMO_MSG_BF16 = 1, AMO_MSG_E4M3 = 2 };
double amo_quantize_message(float x, uint32_t msg_dtype)
{
    if (msg_dtype == AMO_MSG_BF16) return (double)amo_bf16_to_float(amo_double_to_bf16((double)x));
    if (msg_dtype == AMO_MSG_E4M3) return amo_quantize_e4m3((double)x);
    return (double)x;
}

/* ------------------------------------------------------------------------------------------ */
/* state                                                                                       */
/* ------------------------------------------------------------------------------------------ */
enum { AMO_OPT_SGD = 0, AMO_OPT_ADAMW = 1, AMO_OPT_NADAMW = 2 };
enum { AMO_CORR_NONE = 0, AMO_CORR_EMA = 1, AMO_CORR_EAGER = 2 };

typedef struct {
    uint64_t n;            /* coordinates held by this oracle instance                      */
    uint64_t mu0;          /* global index of local coordinate 0                            */
    uint32_t replicas;     /* R (m in the paper)                                            */
    uint32_t delay;        /* tau, in averaging rounds                                      */
    uint32_t avg_interval; /* K                                                             */
    uint32_t optimizer;    /* AMO_OPT_*                                                     */
    double   fraction;     /* p                                                             */
    uint64_t seed;
    double   beta1, beta2, eps, weight_decay;
    double   gamma;        /* look-ahead coefficient; used only when lookahead != 0         */
    uint32_t lookahead;
    uint32_t correction;   /* AMO_CORR_*                                                    */
    uint32_t fwd_bf16;     /* fwd stored as bfloat16 instead of fp32                        */
    uint32_t grad_bf16;    /* gradients arrive as bfloat16                                  */
    double   momentum_decay; /* NAdam's psi (0.004 in Dozat's schedule); NADAMW only        */
    uint32_t granule;        /* subset drawn per coordinate (1) or per aligned block of g   */
    uint32_t msg_dtype;      /* AMO_MSG_*: precision of the exchanged values (the compression
                                experiment: the average is formed from quantised values; a
                                replica's own staleness term uses its own exact old value)  */
    uint32_t stratified;     /* 1: the stratified sampling variant (one coordinate per block) */
    uint32_t reserved;
} amo_config;

typedef struct {
    amo_config c;
    float **w, **m, **v, **d;    /* [R][n] */
    float **fwd;                 /* [R][n] fp32 value of fwd (already rounded to bf16 when fwd_bf16) */
    float **what;                /* [R][n] scratch: w^ of the current step */
    float **w_before;            /* [R][n] scratch: w^{t-1} */
    float ***kept;               /* [tau*K+1][R][n] copies of w^ (one per step) */
    uint32_t nkept;
    uint64_t last_t;
    uint32_t delay_now;          /* the delay in force (<= c.delay, which sizes the buffer) */
    /* per replica, because replicas of unequal speed make unequal numbers of local steps
     * (heterogeneous set-up of the experiments): */
    uint64_t *opt_steps;         /* [R] optimizer steps made so far = the t of the bias corrections */
    double *mu_product;          /* [R] NAdam's running product of momentum coefficients */
} amo_state;

static float **alloc_2d(uint32_t R, uint64_t n)
{
    float **a = (float **)calloc(R, sizeof(float *));
    for (uint32_t i = 0; i < R; ++i) a[i] = (float *)calloc(n ? n : 1, sizeof(float));
    return a;
}
static void free_2d(float **a, uint32_t R)
{
    if (!a) return;
    for (uint32_t i = 0; i < R; ++i) free(a[i]);
    free(a);
}

amo_state *amo_create(const amo_config *c)
{
    amo_state *s = (amo_state *)calloc(1, sizeof(amo_state));
    s->c = *c;
    uint32_t R = c->replicas;
    s->w = alloc_2d(R, c->n);  s->m = alloc_2d(R, c->n);  s->v = alloc_2d(R, c->n);
    s->d = alloc_2d(R, c->n);  s->fwd = alloc_2d(R, c->n);
    s->what = alloc_2d(R, c->n);  s->w_before = alloc_2d(R, c->n);
    s->nkept = c->delay * c->avg_interval + 1;
    s->kept = (float ***)calloc(s->nkept, sizeof(float **));
    for (uint32_t k = 0; k < s->nkept; ++k) s->kept[k] = alloc_2d(R, c->n);
    s->last_t = 0;
    s->delay_now = c->delay;
    s->opt_steps = (uint64_t *)calloc(R ? R : 1, sizeof(uint64_t));
    s->mu_product = (double *)calloc(R ? R : 1, sizeof(double));
    for (uint32_t i = 0; i < R; ++i) s->mu_product[i] = 1.0;
    return s;
}

void amo_destroy(amo_state *s)
{
    if (!s) return;
    uint32_t R = s->c.replicas;
    free_2d(s->w, R); free_2d(s->m, R); free_2d(s->v, R); free_2d(s->d, R); free_2d(s->fwd, R);
    free_2d(s->what, R); free_2d(s->w_before, R);
    for (uint32_t k = 0; k < s->nkept; ++k) free_2d(s->kept[k], R);
    free(s->kept);
    free(s->opt_steps);
    free(s->mu_product);
    free(s);
}

float *amo_w(amo_state *s, uint32_t i)   { return s->w[i]; }
float *amo_m(amo_state *s, uint32_t i)   { return s->m[i]; }
float *amo_v(amo_state *s, uint32_t i)   { return s->v[i]; }
float *amo_d(amo_state *s, uint32_t i)   { return s->d[i]; }
float *amo_fwd(amo_state *s, uint32_t i) { return s->fwd[i]; }
uint64_t amo_last_t(const amo_state *s)  { return s->last_t; }

/* ------------------------------------------------------------------------------------------ */
/* 1. local optimizer step for every replica: w -> what (w itself is left untouched here)       */
/* ------------------------------------------------------------------------------------------ */
static double grad_value(const amo_state *s, const void *g, uint64_t k, double grad_scale)
{
    double raw = s->c.grad_bf16 ? (double)amo_bf16_to_float(((const uint16_t *)g)[k])
                                : (double)((const float *)g)[k];
    return grad_scale * raw;
}

/* replica_scale: NULL, or one more factor per replica on top of grad_scale (each replica clips by
 * its own gradient norm).
 * active: NULL = every replica steps and its optimizer step count becomes t (the homogeneous
 * set-up); else bit i says whether replica i makes a local step in this tick.  A replica that does
 * not step keeps w, m, v (w^ = w) and its step count; one that does counts one more step.  This
 * is the heterogeneous set-up of the experiments (Sec. "Heterogeneous setup": faster devices make
 * more iterations between two averaging steps), simulated in lock-step ticks. */
static void local_step(amo_state *s, uint64_t t, const void *const *grads, double lr, double grad_scale,
                       const float *replica_scale, const uint32_t *active)
{
    const amo_config *c = &s->c;
    const double b1 = c->beta1, b2 = c->beta2, eps = c->eps, wd = c->weight_decay;

    for (uint32_t i = 0; i < c->replicas; ++i) {
        float *w = s->w[i], *m = s->m[i], *v = s->v[i], *what = s->what[i], *wb = s->w_before[i];
        const void *g_i = grads[i];
        if (active && !((*active >> i) & 1u)) {          /* no local step in this tick */
            memcpy(what, w, c->n * sizeof(float));
            memcpy(wb, w, c->n * sizeof(float));
            continue;
        }
        const uint64_t steps = active ? s->opt_steps[i] + 1 : t;
        s->opt_steps[i] = steps;
        /* per-step scalars, evaluated once */
        const double bc1 = 1.0 - pow(b1, (double)steps);       /* Adam bias corrections */
        const double bc2 = 1.0 - pow(b2, (double)steps);
        /* NAdam (Dozat) momentum schedule: mu_t = beta1 (1 - 0.5 * 0.96^(t psi)) */
        const double mu_t  = b1 * (1.0 - 0.5 * pow(0.96, (double)steps * c->momentum_decay));
        const double mu_t1 = b1 * (1.0 - 0.5 * pow(0.96, (double)(steps + 1) * c->momentum_decay));
        const double mu_prod = s->mu_product[i] * mu_t;        /* prod_{k<=t} mu_k */
        if (c->optimizer == AMO_OPT_NADAMW) s->mu_product[i] = mu_prod;
        #pragma omp parallel for schedule(static)
        for (uint64_t k = 0; k < c->n; ++k) {
            const double g = grad_value(s, g_i, k, replica_scale ? grad_scale * (double)replica_scale[i] : grad_scale);
            const double w_old = (double)w[k];
            wb[k] = w[k];
            double w_hat;
            if (c->optimizer == AMO_OPT_SGD) {
                /* SGD with heavy-ball momentum beta1 (0 = plain SGD), decoupled weight decay:
                 *   m <- beta1 m + g ;  w^ = w (1 - lr wd) - lr m                              */
                if (b1 != 0.0) {
                    m[k] = (float)(b1 * (double)m[k] + g);
                    w_hat = w_old * (1.0 - lr * wd) - lr * (double)m[k];
                } else {
                    w_hat = w_old * (1.0 - lr * wd) - lr * g;
                }
            } else {
                /* Adam moments */
                m[k] = (float)(b1 * (double)m[k] + (1.0 - b1) * g);
                v[k] = (float)(b2 * (double)v[k] + (1.0 - b2) * g * g);
                const double mk = (double)m[k], vk = (double)v[k];
                const double denom = sqrt(vk) / sqrt(bc2) + eps;
                if (c->optimizer == AMO_OPT_ADAMW) {
                    /* AdamW (Loshchilov & Hutter): decoupled decay, bias-corrected step */
                    w_hat = w_old * (1.0 - lr * wd) - (lr / bc1) * mk / denom;
                } else {
                    /* NAdamW: Nesterov look-ahead inside Adam (Dozat), decoupled decay:
                     *   w^ = w(1-lr wd) - lr (1-mu_t)/(1-prod_t) g/denom
                     *                   - lr mu_{t+1}/(1-prod_t mu_{t+1}) m/denom               */
                    w_hat = w_old * (1.0 - lr * wd)
                          - lr * (1.0 - mu_t) / (1.0 - mu_prod) * g / denom
                          - lr * mu_t1 / (1.0 - mu_prod * mu_t1) * mk / denom;
                }
            }
            what[k] = (float)w_hat;
        }
    }
}

/* ------------------------------------------------------------------------------------------ */
/* 2.+3. asynchronous sparse averaging acting on what (-> w, d)                                 */
/* ------------------------------------------------------------------------------------------ */
static void sparse_average(amo_state *s, uint64_t t, double lambda)
{
    const amo_config *c = &s->c;
    const uint32_t R = c->replicas, K = c->avg_interval;
    const uint64_t n = c->n;

    /* coordinates outside the received subset keep the local result */
    for (uint32_t i = 0; i < R; ++i) memcpy(s->w[i], s->what[i], n * sizeof(float));

    if (t % K != 0) return;                           /* not an averaging step */

    /* send: this step's w^ is what every replica puts on the wire now */
    float **now = s->kept[t % s->nkept];
    for (uint32_t i = 0; i < R; ++i) memcpy(now[i], s->what[i], n * sizeof(float));

    /* receive: the average that was sent tau rounds (tau*K steps) ago arrives now */
    const uint64_t lag = (uint64_t)s->delay_now * K;
    if (t < lag + 1) return;                          /* nothing was sent that long ago */
    const uint64_t sstep = t - lag;
    float **old = s->kept[sstep % s->nkept];

    #pragma omp parallel for schedule(static)
    for (uint64_t k = 0; k < n; ++k) {
        if (!in_subset(c->seed, sstep, c->mu0 + k, c->fraction, c->granule, c->stratified)) continue;
        double sum = 0.0;
        for (uint32_t i = 0; i < R; ++i) sum += amo_quantize_message(old[i][k], c->msg_dtype);
        const float abar = (float)(sum / (double)R);              /* old average, an fp32 message */
        for (uint32_t i = 0; i < R; ++i) {
            if (c->correction == AMO_CORR_EMA || c->correction == AMO_CORR_EAGER) {
                const double staleness = (double)s->what[i][k] - (double)old[i][k];
                if (c->correction == AMO_CORR_EMA)
                    s->d[i][k] = (float)((1.0 - lambda) * (double)s->d[i][k] + lambda * staleness);
                else
                    s->d[i][k] = (float)(staleness / (double)R);
                s->w[i][k] = (float)((double)abar + (double)s->d[i][k]);
            } else {
                s->w[i][k] = abar;
            }
        }
    }
}

/* ------------------------------------------------------------------------------------------ */
/* 4. look-ahead: the weights the next forward pass uses                                        */
/* ------------------------------------------------------------------------------------------ */
static void look_ahead(amo_state *s)
{
    const amo_config *c = &s->c;
    for (uint32_t i = 0; i < c->replicas; ++i) {
        #pragma omp parallel for schedule(static)
        for (uint64_t k = 0; k < c->n; ++k) {
            double f = (double)s->w[i][k];
            if (c->lookahead)
                f += c->gamma * ((double)s->what[i][k] - (double)s->w_before[i][k]);
            s->fwd[i][k] = c->fwd_bf16 ? amo_bf16_to_float(amo_double_to_bf16(f)) : (float)f;
        }
    }
}

/* one full step (1.-4.) ; grads = R pointers to n fp32 (or bf16) values ; returns 0, or -1 when
 * t is not last_t + 1 */
int amo_step_scaled(amo_state *s, uint64_t t, const void *const *grads, double lr, double lambda,
                    double grad_scale, const float *replica_scale)
{
    if (t != s->last_t + 1) return -1;
    local_step(s, t, grads, lr, grad_scale, replica_scale, NULL);
    sparse_average(s, t, lambda);
    look_ahead(s);
    s->last_t = t;
    return 0;
}

/* one tick of the heterogeneous set-up: only the replicas whose bit is set make a local step
 * (grads[i] of the others is not read and may be NULL); everything else as in amo_step_scaled */
int amo_step_masked(amo_state *s, uint64_t t, const void *const *grads, double lr, double lambda,
                    double grad_scale, const float *replica_scale, uint32_t active)
{
    if (t != s->last_t + 1) return -1;
    local_step(s, t, grads, lr, grad_scale, replica_scale, &active);
    sparse_average(s, t, lambda);
    look_ahead(s);
    s->last_t = t;
    return 0;
}

int amo_step(amo_state *s, uint64_t t, const void *const *grads, double lr, double lambda, double grad_scale)
{
    if (t != s->last_t + 1) return -1;
    local_step(s, t, grads, lr, grad_scale, NULL, NULL);
    sparse_average(s, t, lambda);
    look_ahead(s);
    s->last_t = t;
    return 0;
}

/* sparse averaging alone (2.-3.) on the current w, which plays the role of w^ ; fwd untouched */
int amo_sparse_average(amo_state *s, uint64_t t, double lambda)
{
    if (t != s->last_t + 1) return -1;
    for (uint32_t i = 0; i < s->c.replicas; ++i) {
        memcpy(s->what[i], s->w[i], s->c.n * sizeof(float));
        memcpy(s->w_before[i], s->w[i], s->c.n * sizeof(float));
    }
    sparse_average(s, t, lambda);
    s->last_t = t;
    return 0;
}

/* stateless look-ahead in its literal two-point form: out = w + gamma (w - w_prev) */
void amo_lookahead(float *out, uint16_t *out_bf16, const float *w, const float *w_prev, uint64_t n, double gamma)
{
    for (uint64_t k = 0; k < n; ++k) {
        double f = (double)w[k] + gamma * ((double)w[k] - (double)w_prev[k]);
        if (out) out[k] = (float)f;
        if (out_bf16) out_bf16[k] = amo_double_to_bf16(f);
    }
}

/* the delay in force from the next step on: 0 <= tau <= the delay the state was created with
 * (late or early arrival of an average; the buffer keeps enough copies for the largest delay) */
int amo_set_delay(amo_state *s, uint32_t tau)
{
    if (tau > s->c.delay) return -1;
    s->delay_now = tau;
    return 0;
}

/* variance over the replicas of the EMA estimates, (1/R) sum_i (d_i[mu] - mean_i d_i[mu])^2, as its
 * mean and its maximum over the coordinates (the two curves of the paper's consensus figure) */
void amo_ema_variance(const amo_state *s, double *mean_out, double *max_out)
{
    const uint32_t R = s->c.replicas;
    double total = 0.0, worst = 0.0;
    for (uint64_t k = 0; k < s->c.n; ++k) {
        double mean = 0.0, var = 0.0;
        for (uint32_t i = 0; i < R; ++i) mean += (double)s->d[i][k];
        mean /= (double)R;
        for (uint32_t i = 0; i < R; ++i) {
            double e = (double)s->d[i][k] - mean;
            var += e * e;
        }
        var /= (double)R;
        total += var;
        if (var > worst) worst = var;
    }
    *mean_out = s->c.n ? total / (double)s->c.n : 0.0;
    *max_out = worst;
}

/* consensus error  sum_i || w_i - mean_i w_i ||^2  (diagnostic used by the invariants) */
double amo_consensus_error(const amo_state *s)
{
    const uint32_t R = s->c.replicas;
    double total = 0.0;
    for (uint64_t k = 0; k < s->c.n; ++k) {
        double mean = 0.0;
        for (uint32_t i = 0; i < R; ++i) mean += (double)s->w[i][k];
        mean /= (double)R;
        for (uint32_t i = 0; i < R; ++i) {
            double e = (double)s->w[i][k] - mean;
            total += e * e;
        }
    }
    return total;
}

/* sum of squares of one gradient array (the stage's share of a replica's squared gradient norm,
 * what global-norm clipping needs from every stage) */
double amo_grad_sqnorm(const void *g, uint64_t n, uint32_t is_bf16)
{
    double total = 0.0;
    for (uint64_t k = 0; k < n; ++k) {
        double x = is_bf16 ? (double)amo_bf16_to_float(((const uint16_t *)g)[k]) : (double)((const float *)g)[k];
        total += x * x;
    }
    return total;
}

/* number of threads the coordinate loops above run on */
int amo_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
