/*
 * OD-SGD update oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, one-element-at-a-time CPU statement of what one iteration of
 * the OD-SGD parameter-update pipeline computes.  Only the test-suite, the
 * smoke check and the benchmark's cpu_baseline leg may call it; the GPU
 * library shares no source, header, table or helper with this file.
 *
 * What is computed (paper: Section 3.1, Algorithm 1 "parameter server" and
 * Algorithm 2 "worker m"; Section 3.3 "Local Updater"):
 *
 *   server  (Alg. 1, the step taken once all M gradients have arrived):
 *           aggregate the M worker gradients, then update the global weights
 *           w_t with a momentum-SGD step (momentum is a property of the global
 *           updater only: Section 4.2 sets 0.9 for "the global updater").
 *   worker  (Alg. 2, training stage): the copy w_bak of the *pulled* weights
 *           w_t is updated with the worker's own fresh gradient g_m; the result
 *           is what the worker trains on in the next iteration.  The copy is
 *           of the weights *before* this iteration's server update (caption of
 *           the three-stage overview figure: copied at i-1, updated at i, used
 *           at i+1), which is what makes the delay exactly one step.
 *   warm-up (Alg. 2, while num < wp): plain synchronous SGD -- the worker
 *           trains on the freshly pulled w_{t+1}; no local update.
 *
 * The paper does not print the momentum formula, sum-vs-mean, or where weight
 * decay enters.  Readings taken here (readings, not statements of the paper):
 *   - velocity form  v <- mu*v - lr*(gbar + wd*w);  w <- w + v
 *   - gbar = (g_0 + g_1 + ... + g_{M-1}) * grad_scale, summed strictly left to
 *     right in ascending worker index; grad_scale <= 0 selects 1/M (the mean)
 *   - coupled L2 weight decay wd*w, the same term in the global and the local
 *     update, computed once from the pre-update weight
 *   - the local SGD updater has no momentum state: u_m = w_t - local_lr*(g_m + wd*w_t)
 *
 * Arithmetic: every line below is exactly one IEEE-754 operation in type
 * `real`, round-to-nearest-even, no fused multiply-add (build with
 * -ffp-contract=off, no -ffast-math), subnormals kept.  The file is compiled
 * twice: real=float (the precision the method is run in here) and real=double
 * (same order of operations; used to report how far fp32 is from exact).
 *
 * Layout: one call handles ONE parameter tensor, given as flat arrays of n
 * elements; g and u are arrays of M pointers (one per worker).
 *
 * Delay-compensated local updaters (Section 3.3, equations "DC-ASGD-c" and
 * "DC-ASGD-a" with the MeanSquare recurrence).  The equations are printed for
 * asynchronous SGD; inside OD-SGD their symbols are read as
 *     w_{t+tau}   = the freshly copied global weights w_t the update starts from
 *     w_t         = the weights the gradient g_m was evaluated at, i.e. worker
 *                   m's previous local weights (the old content of u[m])
 *     g(w_t)      = g_m,   eta = local_lr
 * and weight decay enters as in the SGD updater (r = wd * w added to the
 * gradient term only; the compensation term uses the raw gradient, so wd = 0
 * gives the printed equation).  Products are taken left to right as
 * ((g*g) * (w - u_old)) * lambda.
 */
#include <math.h>
#include <stdint.h>

#if !defined(ODSGD_REAL) || !defined(ODSGD_SUFFIX) || !defined(ODSGD_SQRT)
#error "compile with -DODSGD_REAL=float|double -DODSGD_SUFFIX=f32|f64 -DODSGD_SQRT=sqrtf|sqrt"
#endif
#define ODSGD_CAT2(a, b) a##_##b
#define ODSGD_CAT(a, b) ODSGD_CAT2(a, b)
#define ODSGD_NAME(base) ODSGD_CAT(base, ODSGD_SUFFIX)

typedef ODSGD_REAL real;

static real resolve_grad_scale(real grad_scale, int M)
{
    if (grad_scale <= (real)0)
        return (real)1 / (real)M;
    return grad_scale;
}

/*
 * Worker-side local update (Alg. 2, "Update w_bak with g_m"), SGD flavour.
 * Reads the current global weights w (the pulled, one-step-old w_t) and writes
 * u[m] for one worker (worker = m) or for all of them (worker = -1).
 * w is not modified.
 */
void ODSGD_NAME(odsgd_oracle_local)(int64_t n, int M, const real *w,
                                    const real *const *g, real *const *u,
                                    int worker, real local_lr, real weight_decay)
{
    for (int64_t i = 0; i < n; ++i) {
        real w0 = w[i];
        real r = weight_decay * w0;
        for (int m = 0; m < M; ++m) {
            if (worker >= 0 && m != worker)
                continue;
            real dm = g[m][i] + r;
            real pm = local_lr * dm;
            u[m][i] = w0 - pm;
        }
    }
}

/*
 * Local update with the constant delay compensation of equation "DC-ASGD-c":
 *   u_m <- w - local_lr * ( (g_m + r) + lambda * g_m*g_m*(w - u_m_old) ).
 * u[m] is read (old local weights) and then overwritten.
 */
void ODSGD_NAME(odsgd_oracle_local_dcasgd_c)(int64_t n, int M, const real *w,
                                             const real *const *g, real *const *u,
                                             int worker, real local_lr,
                                             real weight_decay, real lambda)
{
    for (int64_t i = 0; i < n; ++i) {
        real w0 = w[i];
        real r = weight_decay * w0;
        for (int m = 0; m < M; ++m) {
            if (worker >= 0 && m != worker)
                continue;
            real gm = g[m][i];
            real dlt = w0 - u[m][i];
            real gg = gm * gm;
            real c1 = gg * dlt;
            real c2 = c1 * lambda;
            real dm = gm + r;
            real em = dm + c2;
            real pm = local_lr * em;
            u[m][i] = w0 - pm;
        }
    }
}

/*
 * Local update with the adaptive compensation of equation "DC-ASGD-a":
 *   MeanSquare <- ms_decay * MeanSquare + (1 - ms_decay) * g_m*g_m   (per worker state)
 *   lambda_eff  = lambda / sqrt(MeanSquare + epsilon)
 *   u_m <- w - local_lr * ( (g_m + r) + lambda_eff * g_m*g_m*(w - u_m_old) ).
 */
void ODSGD_NAME(odsgd_oracle_local_dcasgd_a)(int64_t n, int M, const real *w,
                                             const real *const *g, real *const *u,
                                             real *const *ms, int worker,
                                             real local_lr, real weight_decay,
                                             real lambda, real ms_decay,
                                             real epsilon)
{
    real one_minus_decay = (real)1 - ms_decay;
    for (int64_t i = 0; i < n; ++i) {
        real w0 = w[i];
        real r = weight_decay * w0;
        for (int m = 0; m < M; ++m) {
            if (worker >= 0 && m != worker)
                continue;
            real gm = g[m][i];
            real dlt = w0 - u[m][i];
            real gg = gm * gm;
            real s1 = ms_decay * ms[m][i];
            real s2 = one_minus_decay * gg;
            real msq = s1 + s2;
            ms[m][i] = msq;
            real rad = msq + epsilon;
            real den = ODSGD_SQRT(rad);
            real lam = lambda / den;
            real c1 = gg * dlt;
            real c2 = c1 * lam;
            real dm = gm + r;
            real em = dm + c2;
            real pm = local_lr * em;
            u[m][i] = w0 - pm;
        }
    }
}

/*
 * Local momentum-SGD updater.  Section 4.2 runs the local SGD updater with "the
 * learning rate and momentum of SSGD", which is read here as a per-worker local
 * velocity lv_m that accumulates the worker's own gradients:
 *   lv_m <- local_momentum * lv_m - local_lr * (g_m + r) ;   u_m <- w + lv_m.
 * With local_momentum = 0 this is exactly the plain SGD local updater.
 */
void ODSGD_NAME(odsgd_oracle_local_momentum)(int64_t n, int M, const real *w,
                                             const real *const *g, real *const *u,
                                             real *const *lv, int worker,
                                             real local_lr, real weight_decay,
                                             real local_momentum)
{
    for (int64_t i = 0; i < n; ++i) {
        real w0 = w[i];
        real r = weight_decay * w0;
        for (int m = 0; m < M; ++m) {
            if (worker >= 0 && m != worker)
                continue;
            real dm = g[m][i] + r;
            real am = local_momentum * lv[m][i];
            real pm = local_lr * dm;
            real lv1 = am - pm;
            lv[m][i] = lv1;
            u[m][i] = w0 + lv1;
        }
    }
}

/*
 * Server-side global update (Alg. 1, "Update w_t with aggregated gradient"):
 * M-way sum in ascending worker order, scale, coupled weight decay,
 * momentum-SGD step in velocity form.  w and v are updated in place.
 */
void ODSGD_NAME(odsgd_oracle_global)(int64_t n, int M, real *w, real *v,
                                     const real *const *g, real lr,
                                     real momentum, real weight_decay,
                                     real grad_scale)
{
    real scale = resolve_grad_scale(grad_scale, M);
    for (int64_t i = 0; i < n; ++i) {
        real w0 = w[i];
        real v0 = v[i];
        real s = g[0][i];
        for (int m = 1; m < M; ++m)
            s = s + g[m][i];
        real gb = s * scale;
        real r = weight_decay * w0;
        real d = gb + r;
        real a = momentum * v0;
        real b = lr * d;
        real v1 = a - b;
        real w1 = w0 + v1;
        v[i] = v1;
        w[i] = w1;
    }
}

/*
 * One OD-SGD iteration in the training stage (Alg. 2 repeat-loop together with
 * Alg. 1): every worker's local update is taken from the pre-update weights
 * w_t, then the server moves w_t -> w_{t+1}.  By definition this is the local
 * update of all workers followed by the global update.
 */
void ODSGD_NAME(odsgd_oracle_od_step)(int64_t n, int M, real *w, real *v,
                                      const real *const *g, real *const *u,
                                      real lr, real local_lr, real momentum,
                                      real weight_decay, real grad_scale)
{
    ODSGD_NAME(odsgd_oracle_local)(n, M, w, g, u, -1, local_lr, weight_decay);
    ODSGD_NAME(odsgd_oracle_global)(n, M, w, v, g, lr, momentum, weight_decay,
                                    grad_scale);
}

/*
 * One warm-up iteration (Alg. 2 while-loop before the switch, i.e. plain
 * synchronous SGD): the server updates, and every worker receives the fresh
 * w_{t+1} unchanged as the weights it trains on next.
 */
void ODSGD_NAME(odsgd_oracle_ssgd_step)(int64_t n, int M, real *w, real *v,
                                        const real *const *g, real *const *u,
                                        real lr, real momentum,
                                        real weight_decay, real grad_scale)
{
    ODSGD_NAME(odsgd_oracle_global)(n, M, w, v, g, lr, momentum, weight_decay,
                                    grad_scale);
    for (int m = 0; m < M; ++m)
        for (int64_t i = 0; i < n; ++i)
            u[m][i] = w[i];
}
