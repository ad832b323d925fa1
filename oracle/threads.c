/*
 * Static multi-thread driver for the oracle -- TEST/BENCH INFRASTRUCTURE, NOT
 * THE PRODUCT, and not part of the oracle's definition either.
 *
 * It holds no arithmetic.  The flat element range [0, N) of a tensor list is
 * cut into `threads` equal, contiguous parts; each POSIX thread walks the
 * tensors that intersect its part and hands every piece to the oracle's own
 * per-tensor routine (passed in as a function pointer, so this file does not
 * link against or include the oracle).  The update is element-wise, so the
 * result is the single-thread result bit for bit.  Only the benchmark's
 * "all host cores" baseline uses it.
 */
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>

typedef void (*od_step_f32_fn)(int64_t n, int M, float *w, float *v, const float *const *g, float *const *u,
                               float lr, float local_lr, float momentum, float weight_decay, float grad_scale);

typedef struct {
    od_step_f32_fn fn;
    int K, M;
    const int64_t *numel;
    float *const *w;
    float *const *v;
    const float *const *g; /* [M*K], worker-major */
    float *const *u;       /* [M*K], worker-major */
    float lr, local_lr, momentum, weight_decay, grad_scale;
    int64_t begin, end;    /* flat element range of this thread */
    int failed;
} job_t;

static void *run_job(void *arg)
{
    job_t *j = (job_t *)arg;
    const float **gk = (const float **)malloc(sizeof(*gk) * (size_t)j->M);
    float **uk = (float **)malloc(sizeof(*uk) * (size_t)j->M);
    if (!gk || !uk) {
        j->failed = 1;
        free(gk);
        free(uk);
        return NULL;
    }
    int64_t first = 0; /* flat index of the tensor's first element */
    for (int k = 0; k < j->K; ++k) {
        const int64_t n = j->numel[k];
        const int64_t lo = j->begin > first ? j->begin - first : 0;
        const int64_t hi = j->end < first + n ? j->end - first : n;
        if (lo < hi) {
            for (int m = 0; m < j->M; ++m) {
                gk[m] = j->g[(size_t)m * j->K + k] + lo;
                uk[m] = j->u[(size_t)m * j->K + k] + lo;
            }
            j->fn(hi - lo, j->M, j->w[k] + lo, j->v[k] + lo, gk, uk, j->lr, j->local_lr, j->momentum,
                  j->weight_decay, j->grad_scale);
        }
        first += n;
    }
    free(gk);
    free(uk);
    return NULL;
}

/* Returns 0 on success, -1 on bad arguments or when a thread could not be started. */
int odsgd_oracle_threads_od_step_f32(od_step_f32_fn fn, int threads, int K, const int64_t *numel, float *const *w,
                                     float *const *v, const float *const *g, float *const *u, int M, float lr,
                                     float local_lr, float momentum, float weight_decay, float grad_scale)
{
    if (!fn || threads < 1 || threads > 1024 || K < 1 || M < 1)
        return -1;
    int64_t N = 0;
    for (int k = 0; k < K; ++k)
        N += numel[k];
    job_t *jobs = (job_t *)calloc((size_t)threads, sizeof(*jobs));
    pthread_t *tids = (pthread_t *)calloc((size_t)threads, sizeof(*tids));
    if (!jobs || !tids) {
        free(jobs);
        free(tids);
        return -1;
    }
    int started = 0, rc = 0;
    for (int t = 0; t < threads; ++t) {
        job_t *j = &jobs[t];
        j->fn = fn; j->K = K; j->M = M; j->numel = numel; j->w = w; j->v = v; j->g = g; j->u = u;
        j->lr = lr; j->local_lr = local_lr; j->momentum = momentum; j->weight_decay = weight_decay;
        j->grad_scale = grad_scale;
        j->begin = N / threads * t + (N % threads) * t / threads;
        j->end = N / threads * (t + 1) + (N % threads) * (t + 1) / threads;
        if (pthread_create(&tids[t], NULL, run_job, j) != 0) {
            rc = -1;
            break;
        }
        ++started;
    }
    for (int t = 0; t < started; ++t)
        pthread_join(tids[t], NULL);
    for (int t = 0; t < started; ++t)
        if (jobs[t].failed)
            rc = -1;
    if (started != threads)
        rc = -1; /* part of the range was not processed */
    free(jobs);
    free(tids);
    return rc;
}
