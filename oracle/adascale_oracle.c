/*
 * CPU oracle for one AdaScale SGD iteration.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 statement of what the method computes, used to check the GPU
 * library.  It shares no code with that library, and nothing in the product path may
 * call it: only the tests, the smoke check and the benchmark's CPU-baseline leg do.
 *
 * What is computed (one iteration t, S gradient vectors g_1..g_S of length d):
 *   - the mean gradient that scaled SGD applies (Sec. 2, Algorithm 1);
 *   - the variance and squared-mean estimates of App. B.3,
 *         sigma2_hat = (sum_i ||g_i||^2 - S ||gbar||^2) / (S - 1),
 *         mu2_hat    = ||gbar||^2 - sigma2_hat / S,
 *     their clamping (sigma2_hat >= eps, mu2_hat >= 0) and moving averages with
 *     parameter theta, using the plain mean of the samples seen so far while fewer
 *     than 1/(1-theta) samples exist (App. B.3);
 *   - the gain ratio of eq. (3) with the averages plugged in,
 *         r_t = (sbar + mbar) / (sbar / S + mbar);
 *   - the learning rate eta_t = r_t * lr(floor(tau_t)) and the scale-invariant clock
 *     tau_{t+1} = tau_t + r_t (Sec. 3.2);
 *   - the momentum-SGD update (Sec. 3.4 keeps rho fixed across scales).
 *
 * Readings taken where the paper leaves a choice open:
 *   - tau_0 = 0; eta_t uses tau_t (before this iteration's r_t is added).
 *   - r_t uses the averages *including* the current sample (the paper's recommendation
 *     at the end of App. B.3); flag ORACLE_LAGGED_R selects the other variant described
 *     there: averages of prior iterations only, r_0 = 1.
 *   - moving average: xbar <- xbar + alpha_k (x - xbar), alpha_k = max(1 - theta, 1/k),
 *     k = number of samples including the current one.
 *   - mu2_hat is formed from the unclamped sigma2_hat; both are clamped afterwards.
 *   - S = 1: sigma2_hat := 0 (no eps clamp), mu2_hat := ||gbar||^2, so r_t = 1.
 *   - momentum: v <- rho v + (gbar + lambda w);  w <- w - eta_t v.  Weight decay is a
 *     coupled L2 term added after the statistics are taken.
 *   - floor(tau_t) beyond the table: the last entry is used.
 *   - flag ORACLE_EST_M1M2 selects the estimator of Sec. 3.4 instead: moving averages
 *     m1 of (1/S) sum_i ||g_i||^2 and m2 of ||gbar||^2, r_t = (m1 + eps) / (m2 + eps).
 *
 * Arithmetic: every quantity is a double; the two global sums run in long double.
 * Gradients arrive as the same bit patterns the GPU reads (fp32 or bf16) and are
 * widened exactly.
 *
 * parity unpinned by the paper: the moving-average switch-over, the momentum form, the
 * weight-decay placement and the value of eps in App. B.3 have no printed numbers; they
 * are pinned only by the readings above, a library optimizer (S = 1) and a hand-derived
 * two-step example.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum { ORACLE_LAGGED_R = 1u, ORACLE_EST_M1M2 = 2u };

typedef struct {
    int64_t step;      /* iterations completed = samples in the averages */
    double tau;        /* tau_{t+1} */
    double r;          /* r_t of the last iteration */
    double lr_eff;     /* eta_t of the last iteration */
    double sum_sq;     /* A = sum_i ||g_i||^2 */
    double sq_mean;    /* B = ||gbar||^2 */
    double sigma2_hat; /* raw, before clamping */
    double mu2_hat;    /* raw, before clamping */
    double sigma2_bar; /* moving averages after this iteration (m1, m2 for EST_M1M2) */
    double mu2_bar;
    int32_t done;      /* tau >= L */
} oracle_state;

typedef struct oracle_ctx {
    int S, grad_dtype;
    double rho, lambda, theta, eps;
    float *lr;
    int64_t L;
    uint32_t flags;
    long double A, B; /* running sums of the current iteration */
    oracle_state st;
} oracle_ctx;

static double widen(const void *buf, int dtype, int64_t j)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)buf)[j];
    uint32_t bits = (uint32_t)((const uint16_t *)buf)[j] << 16; /* bf16 = top half of an fp32 */
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

oracle_ctx *oracle_create(int S, int grad_dtype, double rho, double lambda, double theta, double eps,
                          const float *lr_table, int64_t L, uint32_t flags)
{
    if (S < 1 || L < 1 || !lr_table || rho < 0 || rho >= 1 || lambda < 0 || theta >= 1) return NULL;
    oracle_ctx *c = calloc(1, sizeof *c);
    if (!c) return NULL;
    c->S = S;
    c->grad_dtype = grad_dtype;
    c->rho = rho;
    c->lambda = lambda;
    c->theta = theta < 0 ? fmax(1.0 - S / 1000.0, 0.0) : theta; /* Sec. 3.4 default */
    c->eps = eps <= 0 ? 1e-6 : eps;
    c->L = L;
    c->flags = flags;
    c->lr = malloc(sizeof(float) * (size_t)L);
    if (!c->lr) { free(c); return NULL; }
    memcpy(c->lr, lr_table, sizeof(float) * (size_t)L);
    return c;
}

void oracle_destroy(oracle_ctx *c)
{
    if (c) { free(c->lr); free(c); }
}

void oracle_get_state(const oracle_ctx *c, oracle_state *out) { *out = c->st; }

/* Resume from (k, tau, averages); the rest of the record is diagnostic. */
void oracle_set_state(oracle_ctx *c, int64_t step, double tau, double sigma2_bar, double mu2_bar, double r)
{
    c->st.step = step;
    c->st.tau = tau;
    c->st.sigma2_bar = sigma2_bar;
    c->st.mu2_bar = mu2_bar;
    c->st.r = r;
}

/* Elastic scaling (Sec. 4, "Elastic AdaScaling"): the scale changes, the state carries on. */
void oracle_set_scale(oracle_ctx *c, int S, double theta)
{
    c->S = S;
    c->theta = theta < 0 ? fmax(1.0 - S / 1000.0, 0.0) : theta;
}

void oracle_begin_step(oracle_ctx *c) { c->A = 0; c->B = 0; }

/* Mean gradient (Sec. 2) over n coordinates and their contribution to
 * A = sum_i ||g_i||^2 and B = ||gbar||^2 (App. B.3).  g[i] points at replica i's slice. */
void oracle_accumulate(oracle_ctx *c, int64_t n, const void *const *g, double *gbar)
{
    const int S = c->S, dt = c->grad_dtype;
    long double A = 0, B = 0;
#ifdef _OPENMP
#pragma omp parallel for reduction(+ : A, B) schedule(static)
#endif
    for (int64_t j = 0; j < n; ++j) {
        double sum = 0, sq = 0;
        for (int i = 0; i < S; ++i) {
            double x = widen(g[i], dt, j);
            sum += x;
            sq += x * x;
        }
        double m = sum / S;
        gbar[j] = m;
        A += sq;
        B += m * m;
    }
    c->A += A;
    c->B += B;
}

static double ema(double avg, double sample, double alpha) { return avg + alpha * (sample - avg); }

static double gain_from(const oracle_ctx *c, double sbar, double mbar)
{
    if (c->flags & ORACLE_EST_M1M2) return (sbar + c->eps) / (mbar + c->eps);
    double den = sbar / c->S + mbar;
    return den > 0 ? (sbar + mbar) / den : 1.0;
}

/* Estimates, clamps, moving averages, gain ratio and learning rate (App. B.3, eq. 3, Sec. 3.2). */
void oracle_gain(oracle_ctx *c)
{
    oracle_state *s = &c->st;
    const int S = c->S;
    const double A = (double)c->A, B = (double)c->B;
    double sig, mu;
    if (S >= 2) {
        sig = (A - S * B) / (S - 1);
        mu = B - sig / S;
    } else {
        sig = 0;
        mu = B;
    }
    s->sum_sq = A;
    s->sq_mean = B;
    s->sigma2_hat = sig;
    s->mu2_hat = mu;

    double x1, x2; /* the two samples that enter the averages */
    if (c->flags & ORACLE_EST_M1M2) {
        x1 = A / S;
        x2 = B;
    } else {
        x1 = S >= 2 ? fmax(sig, c->eps) : 0.0;
        x2 = fmax(mu, 0.0);
    }
    const int64_t k = s->step + 1;
    const double alpha = fmax(1.0 - c->theta, 1.0 / (double)k);

    double r = 1.0;
    if (c->flags & ORACLE_LAGGED_R) /* averages of prior iterations only; r_0 = 1 */
        r = s->step == 0 ? 1.0 : gain_from(c, s->sigma2_bar, s->mu2_bar);
    s->sigma2_bar = ema(s->sigma2_bar, x1, alpha);
    s->mu2_bar = ema(s->mu2_bar, x2, alpha);
    if (!(c->flags & ORACLE_LAGGED_R)) r = gain_from(c, s->sigma2_bar, s->mu2_bar);

    int64_t idx = (int64_t)floor(s->tau);
    if (idx > c->L - 1) idx = c->L - 1;
    s->r = r;
    s->lr_eff = r * (double)c->lr[idx];
}

/* Momentum-SGD update of n coordinates with eta_t (eq. 2 with the mean gradient and momentum). */
void oracle_apply(const oracle_ctx *c, int64_t n, double *w, double *v, const double *gbar)
{
    const double rho = c->rho, lambda = c->lambda, eta = c->st.lr_eff;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t j = 0; j < n; ++j) {
        double u = gbar[j] + lambda * w[j];
        v[j] = rho * v[j] + u;
        w[j] = w[j] - eta * v[j];
    }
}

/* tau_{t+1} = tau_t + r_t (Sec. 3.2); training is over once tau >= T_SI = L. */
void oracle_advance(oracle_ctx *c)
{
    c->st.tau += c->st.r;
    c->st.step += 1;
    c->st.done = c->st.tau >= (double)c->L;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
