/*
 * odsgd.h -- C ABI of the OD-SGD (One-step Delay SGD) parameter-update engine
 *            for one AMD MI355X (gfx950).
 *
 * The engine runs the per-iteration update pipeline that OD-SGD adds to
 * data-parallel training (paper: Section 3.1, Algorithms 1 and 2; Section 3.3):
 *
 *   global update  (Alg. 1, parameter server, taken once all M gradients are in)
 *       s    = g_0 + g_1 + ... + g_{W-1}          strictly in ascending worker order
 *       gbar = s * grad_scale
 *       r    = weight_decay * w_t
 *       v'   = momentum * v_t - lr * (gbar + r)
 *       w'   = w_t + v'
 *   local update   (Alg. 2, worker m, "update w_bak with g_m"; Section 3.3 "Local Updater")
 *       u_m  = w_t - local_lr * (g_m + r)         w_t = weights BEFORE this
 *                                                 iteration's global update
 *   warm-up iteration (Alg. 2, while-loop before the switch: plain synchronous SGD)
 *       global update, then u_m = w' for every worker
 *
 * All tensors are fp32.  Each arithmetic line above is one IEEE-754 binary32
 * operation, round-to-nearest-even, with no fused multiply-add, so results do
 * not depend on launch shape.  NaN/Inf inputs propagate; subnormals are kept.
 *
 * Memory model.  The caller owns all device memory (weights, momentum,
 * gradients, local weights and the workspace); the library borrows the
 * pointers given to odsgd_init until odsgd_destroy and never allocates or
 * frees device memory.  Every pointer named "device" must be a device address
 * valid on the GPU that is current when odsgd_init is called.  Arrays named
 * "host" are read during the call only.
 *
 * Tuning.  Launch shape is chosen per call from the worker count and entry
 * point; a few environment variables, read by odsgd_init, override it for
 * experiments and never change results: ODSGD_WAVES_PER_CU
 * (resident wavefronts per compute unit; 0 = automatic, negative = uncapped),
 * ODSGD_BLOCKS_PER_CU (> 0: persistent grid), ODSGD_PAIR_BIT (address bit that
 * separates the two halves of a tile, default 15; 0 = contiguous tiles only),
 * ODSGD_LLC_BYTES (size of the last-level cache, default 256 MiB: weights plus
 * momentum beyond it are loaded non-temporally by odsgd_global_update).
 *
 * Layout advice.  The update runs fastest when, for each tensor, all arrays
 * (w, mom, every grads[m] and local_w[m], state) start at the same offset from
 * a 64 KiB boundary -- e.g. each role packed the same way into a bucket whose
 * base is 64 KiB aligned, or every array 64 KiB aligned by itself.
 *
 * Execution model.  odsgd_local_update / odsgd_global_update / odsgd_step /
 * odsgd_ssgd_step enqueue one kernel on the given HIP stream and return
 * without synchronising.  A handle is not thread-safe; distinct handles are
 * independent.  On any error no kernel is launched.
 */
#ifndef ODSGD_H
#define ODSGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Error codes (all entry points returning int: 0 on success, negative on error). */
#define ODSGD_OK 0
#define ODSGD_EINVAL (-1) /* null pointer, K < 1, W < 1 or > ODSGD_MAX_WORKERS, negative numel, bad worker index */
#define ODSGD_EALIGN (-2) /* a device pointer is not 4-byte aligned */
#define ODSGD_EALIAS (-3) /* an output range (w, mom, local_w) overlaps any other registered range */
#define ODSGD_ENOSPC (-4) /* workspace smaller than odsgd_workspace_bytes() */
#define ODSGD_EHIP (-5)   /* a HIP runtime call failed */
#define ODSGD_ERANGE (-6) /* sizes exceed what the tables can index (a tensor >= 2^40 elements, > 2^31-2 chunks) */
#define ODSGD_ESTALE (-7) /* handle of odsgd_init_static whose table memory a later odsgd_init_static took over */

#define ODSGD_MAX_WORKERS 64

typedef struct odsgd_handle odsgd_handle; /* opaque; host memory owned by the library */

/*
 * Hyper-parameters of one call.  The paper names a global and a local learning
 * rate (Section 4.4: "OD(1.6+0.4)"), momentum for the global updater (Section
 * 4.2) and weight decay (Section 4.4).  Passed by pointer, read during the call.
 */
typedef struct {
    float lr;           /* global (server) learning rate */
    float local_lr;     /* local (worker) learning rate */
    float momentum;     /* global updater only */
    float weight_decay; /* coupled L2 term, same value in global and local update */
    float grad_scale;   /* multiplies the W-way gradient sum; <= 0 selects 1.0f/(float)W */
} odsgd_hyper;

/*
 * Bytes of device workspace odsgd_init needs for this tensor list (chunk
 * table + pointer table).  numel: host array of num_tensors element counts.
 * Returns 0 if the arguments are invalid.
 */
size_t odsgd_workspace_bytes(int num_tensors, const int64_t *numel, int num_workers);

/*
 * Register a parameter set and build the launch plan (Section 2.2 keeps one
 * <key, value> pair per parameter tensor; here the K tensors become one chunk
 * table so that a single launch covers all of them).
 *
 *   out            receives the handle
 *   num_tensors    K >= 1
 *   numel          host, [K]; element count of tensor k (0 is legal and skipped)
 *   w, mom         host arrays [K] of device pointers: global weights and
 *                  momentum of tensor k, numel[k] floats each, read and written
 *   grads          host array [W] of host arrays [K] of device pointers:
 *                  worker m's gradient of tensor k, read only.  The buffers are
 *                  registered once; the caller refills them in place each iteration
 *   local_w        host array [W] of host arrays [K] of device pointers:
 *                  worker m's local weights of tensor k; written only with the SGD
 *                  local updater, read and written with the delay-compensated ones
 *   num_workers    1 <= W <= ODSGD_MAX_WORKERS
 *   workspace      device, >= odsgd_workspace_bytes(...) bytes, 256-byte aligned,
 *                  must stay valid and untouched until odsgd_destroy
 *   stream         hipStream_t (as void*) on which the tables are uploaded;
 *                  the call returns after the upload has completed
 *
 * Pointers 16-byte aligned take the 128-bit path; a tensor with any pointer
 * only 4-byte aligned is processed with 32-bit accesses.  Ranges of w, mom and
 * local_w must not overlap each other or any gradient (ODSGD_EALIAS);
 * gradients may alias one another.
 */
int odsgd_init(odsgd_handle **out, int num_tensors, const int64_t *numel,
               float *const *w, float *const *mom,
               const float *const *const *grads, float *const *const *local_w,
               int num_workers, void *workspace, size_t workspace_bytes,
               void *stream);

/*
 * odsgd_init for callers that cannot allocate device memory (code that runs
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): the same registration, but the chunk and pointer tables go into
 * a fixed array of ODSGD_STATIC_PLAN_BYTES that is part of the library's code
 * object (one copy per GPU, held until the process ends) instead of a caller
 * workspace.  The call allocates no device memory and neither does anything
 * done with the handle; host heap is used for the handle only.  Every other
 * argument, every check and every later call (odsgd_step, odsgd_local_update,
 * odsgd_global_update, odsgd_ssgd_step, odsgd_set_local_rule, ...) is as for
 * odsgd_init, and results are bitwise the same.
 *
 * Limit: odsgd_workspace_bytes(num_tensors, numel, num_workers) must not exceed
 * ODSGD_STATIC_PLAN_BYTES (16 MiB: 16 bytes per 256 elements plus
 * 8*(2 + 3*num_workers) bytes per tensor, i.e. about 2.6e8 parameters);
 * ODSGD_ENOSPC otherwise, before any device is touched.
 *
 * All static registrations on one GPU share that GPU's array.  A new call
 * overwrites it, so (a) handles of earlier odsgd_init_static calls on the same
 * GPU become stale: their launches return ODSGD_ESTALE and enqueue nothing;
 * (b) the caller must make sure no kernel of such an earlier handle is still
 * running or enqueued when the new call is made -- the upload would race with
 * it.  The array keeps the previous registration's bytes; each call uploads its
 * complete table image (padding and unset columns included), so no launch reads
 * anything left over.  Handles of odsgd_init are unaffected.
 */
#define ODSGD_STATIC_PLAN_BYTES (16u << 20)
int odsgd_init_static(odsgd_handle **out, int num_tensors, const int64_t *numel,
                      float *const *w, float *const *mom,
                      const float *const *const *grads, float *const *const *local_w,
                      int num_workers, void *stream);

/*
 * Inspection aid: build, in host memory and without touching any device, the
 * exact table image odsgd_init would upload for these arguments.
 *
 * Pointer table: *num_rows rows of 4 + 3*num_workers 64-bit addresses
 * [w, mom, grads[0..], local_w[0..], per-worker state[0..], w_alt, mom_alt]
 * (the last W + 2 are zero until odsgd_set_local_rule / odsgd_set_double_buffer
 * register them).  Rows follow the tensors in order; a tensor of more than 2^29
 * elements takes one row per 2^29 elements (the addresses of row j are those of
 * the tensor advanced by j * 2^29 elements), every other tensor one row.
 *
 * Chunk table, at *chunk_table_offset: *num_chunks descriptors of four 32-bit
 * words {row index | bit 31 set if the chunk takes 128-bit accesses, element
 * count, element offset inside the row, second-half word}.  With a second-half
 * word of 0 the chunk is `count` consecutive elements.  Otherwise it is a
 * two-half tile of 256 elements: 128 consecutive elements at the offset, and 128
 * more starting 4*(32 + second-half word) elements after the offset (32 KiB
 * later by default).  Such tiles are only used where all arrays of the tensor sit
 * at the same offset from a 64 KiB boundary, and only inside aligned 64 KiB blocks.
 *
 * The pointers are only inspected, never dereferenced.  image must hold
 * odsgd_workspace_bytes(...) bytes.  Same validation and error codes as odsgd_init.
 */
int odsgd_plan_host(int num_tensors, const int64_t *numel, float *const *w, float *const *mom,
                    const float *const *const *grads, float *const *const *local_w,
                    int num_workers, void *image, size_t image_bytes, int64_t *num_rows,
                    int64_t *num_chunks, size_t *chunk_table_offset);

/*
 * Inspection aid: the residency decision of a launch, for a CU described by the
 * arguments instead of the one the process runs on.  Each entry point limits how
 * many of its one-wavefront workgroups a CU holds at a time, because with many
 * concurrent streams the memory system delivers more when fewer requests are in
 * flight.  The limit is imposed by requesting dynamic LDS that the kernel never
 * touches.  Side effect to know about: while such a kernel runs, that LDS is
 * not available to kernels of other streams on the same CUs.
 *   entry           ODSGD_ENTRY_*
 *   rule            ODSGD_LOCAL_* in force (matters for STEP and LOCAL_UPDATE)
 *   num_workers     workers the launch touches
 *   waves_override  as ODSGD_WAVES_PER_CU: 0 = automatic, > 0 = that many, < 0 = no limit
 *   lds_per_cu, lds_granule, max_request   LDS per CU, allocation granularity and
 *                   largest request of one workgroup, in bytes
 *   *waves_wanted   wavefronts per CU the launch aims at (0 = no limit)
 *   *lds_bytes      the request that achieves it (0 = launched without a request:
 *                   no limit wanted, or no request lands on the wanted count or,
 *                   failing that, one below it)
 *   *waves_achieved workgroups per CU under that request
 * At run time the same search is driven by hipOccupancyMaxActiveBlocksPerMultiprocessor.
 */
#define ODSGD_ENTRY_STEP 0
#define ODSGD_ENTRY_SSGD_STEP 1
#define ODSGD_ENTRY_GLOBAL_UPDATE 2
#define ODSGD_ENTRY_LOCAL_UPDATE 3
int odsgd_plan_residency(int entry, int rule, int num_workers, int waves_override,
                         size_t lds_per_cu, size_t lds_granule, size_t max_request,
                         int *waves_wanted, size_t *lds_bytes, int *waves_achieved);

/*
 * Local update (Alg. 2, training stage) with the local updater in force (default
 * SGD: local_w[m] = w - local_lr*(grads[m] + wd*w); see odsgd_set_local_rule),
 * for worker m = `worker`, or for all workers if worker == -1.  Reads w as it is
 * when the kernel runs: for iteration t it must be enqueued BEFORE that
 * iteration's odsgd_global_update.  Uses hyper->local_lr and hyper->weight_decay.
 */
int odsgd_local_update(odsgd_handle *h, int worker, const odsgd_hyper *hyper, void *stream);

/*
 * Global update (Alg. 1): W-way gradient reduce and momentum-SGD step on w and
 * mom, in place (out of place once odsgd_set_double_buffer has been called).
 * Uses lr, momentum, weight_decay, grad_scale.  Advances the handle's iteration
 * counter by one.
 */
int odsgd_global_update(odsgd_handle *h, const odsgd_hyper *hyper, void *stream);

/*
 * Running the two halves of an iteration at the same time.  Section 3.1 notes
 * that Push (which feeds the global update) and local_update only read the new
 * gradient and can therefore run in parallel.  With an in-place global update
 * that is not possible on one GPU, because the local update reads the very
 * weights the global update overwrites.  This call registers a second pair of
 * buffers (w_alt, mom_alt: host arrays [K] of device pointers, numel[k] floats
 * each, caller-owned, contents irrelevant).  From then on odsgd_global_update
 * reads the current pair and writes the other one, after which the roles swap;
 * odsgd_local_update only reads the current pair.  Within one iteration the two
 * calls may then be enqueued on two different streams with no ordering between
 * them, and the results are bitwise those of odsgd_step.  Between iterations the
 * caller orders the streams: iteration t+1 of either call must not start before
 * iteration t of both has finished.  odsgd_step and odsgd_ssgd_step keep
 * updating the current pair in place.  odsgd_current_buffers tells where the
 * current weights and momentum are: 0 = the buffers given to odsgd_init, 1 = the
 * second pair.  Must be called while the current pair is 0, and (the tables
 * are rebuilt and uploaded on `stream`) while no kernel of this handle is
 * running or enqueued on another stream.
 */
int odsgd_set_double_buffer(odsgd_handle *h, float *const *w_alt, float *const *mom_alt, void *stream);
int odsgd_current_buffers(const odsgd_handle *h);

/*
 * One iteration of the whole schedule of Alg. 2 in a single launch.  With i the
 * handle's iteration counter and wp the warm-up length (odsgd_set_warmup,
 * default 0):
 *   i >= wp : one-step-delay iteration -- bitwise identical to
 *             odsgd_local_update(h, -1, ...) followed by odsgd_global_update(h, ...)
 *   i <  wp : warm-up iteration        -- identical to odsgd_ssgd_step
 * Reads w, mom and the W gradients once and writes w, mom and the W local
 * weights once.  Advances the iteration counter by one.  The call is a single
 * kernel launch and may be captured into a HIP graph; the counter is host
 * state, so which kind of iteration a captured launch performs is fixed at
 * capture time.
 */
int odsgd_step(odsgd_handle *h, const odsgd_hyper *hyper, void *stream);

/*
 * Warm-up iteration regardless of the counter: global update, then every
 * local_w[m] receives the new global weights.  Advances the iteration counter.
 */
int odsgd_ssgd_step(odsgd_handle *h, const odsgd_hyper *hyper, void *stream);

/*
 * Local updater used by odsgd_local_update and by the one-step-delay iterations
 * of odsgd_step (Section 3.3 "Local Updater": SGD, DC-ASGD-c, DC-ASGD-a).
 * With u_old = the weights worker m evaluated its gradient at (what local_w[m]
 * holds on entry) and g = grads[m]:
 *   ODSGD_LOCAL_SGD       local_w[m] = w - local_lr*((g + r))
 *   ODSGD_LOCAL_DCASGD_C  local_w[m] = w - local_lr*((g + r) + ((g*g)*(w - u_old))*lambda)
 *   ODSGD_LOCAL_DCASGD_A  ms[m]      = ms_decay*ms[m] + (1 - ms_decay)*(g*g)
 *                         local_w[m] = w - local_lr*((g + r) + ((g*g)*(w - u_old))*(lambda/sqrt(ms[m] + epsilon)))
 *   ODSGD_LOCAL_SGD_MOMENTUM  lv[m]  = local_momentum*lv[m] - local_lr*(g + r)
 *                         local_w[m] = w + lv[m]
 *     (Section 4.2 runs the local SGD updater with the server's learning rate
 *     and momentum; read as a per-worker local velocity.  local_momentum = 0
 *     gives exactly ODSGD_LOCAL_SGD.)
 * r = weight_decay*w; sqrt and divide are correctly rounded.  For the two
 * delay-compensated rules local_w[m] is read before it is overwritten, so it
 * must be initialised (to the weights the first gradients were taken at).
 * state: host array [W] of host arrays [K] of device pointers to the per-worker
 * state (MeanSquare for DCASGD_A, local velocity lv for SGD_MOMENTUM; numel[k]
 * floats each, 4-byte aligned (16 for the 128-bit path), read and written,
 * caller-owned, zero for a fresh run); required for those two rules, ignored otherwise.  A new
 * registration replaces the previous one.  The tables are rebuilt and uploaded
 * on `stream` (how a tensor is tiled depends on the alignment of all its
 * arrays, the state included); the call returns after the upload.  No kernel of
 * this handle may be running or enqueued on another stream during the call.  The paper gives lambda = 0.04
 * (c), lambda = 2 with ms_decay 0.95 or 0 (a) and never states epsilon.
 */
#define ODSGD_LOCAL_SGD 0
#define ODSGD_LOCAL_DCASGD_C 1
#define ODSGD_LOCAL_DCASGD_A 2
#define ODSGD_LOCAL_SGD_MOMENTUM 3
typedef struct {
    int rule;
    float lambda;         /* DCASGD_C, DCASGD_A */
    float ms_decay;       /* DCASGD_A */
    float epsilon;        /* DCASGD_A */
    float local_momentum; /* SGD_MOMENTUM */
} odsgd_local_rule;
int odsgd_set_local_rule(odsgd_handle *h, const odsgd_local_rule *rule,
                         float *const *const *state, void *stream);

/*
 * Warm-up length wp >= 0 (Alg. 2 input): iterations 0..wp-1 are synchronous SGD,
 * the first local update happens in iteration wp.
 */
int odsgd_set_warmup(odsgd_handle *h, int64_t warmup_steps);

/* Iteration counter (number of global updates taken); set it to resume a run. */
int64_t odsgd_get_iteration(const odsgd_handle *h);
int odsgd_set_iteration(odsgd_handle *h, int64_t iteration);

/*
 * Measurement aid, not part of the method: copy numel floats from src to dst
 * (both device, 16-byte aligned, numel a multiple of 4, ranges disjoint) with
 * the same 128-bit streaming accesses the update kernels use.  Its traffic is
 * known exactly (4*numel bytes read, 4*numel written), which makes it the
 * yardstick for hardware byte counters and for the copy bandwidth of the box.
 */
int odsgd_probe_copy(float *dst, const float *src, size_t numel, void *stream);

/*
 * Measurement aid, not part of the method: one launch with exactly the memory
 * accesses of the fused odsgd_step with the SGD local updater on this handle
 * (same tables, tiles, cache policies and residency) and none of its
 * arithmetic: w and mom are read and written back unchanged, local_w[m]
 * receives a copy of grads[m].  Its rate is the ceiling of this access shape on
 * the machine at hand.  The iteration counter does not move.
 */
int odsgd_probe_streams(odsgd_handle *h, void *stream);

/* Release the handle.  Does not touch device memory and does not synchronise:
 * the caller must not free the workspace while enqueued kernels may still run. */
int odsgd_destroy(odsgd_handle *h);

/* Static description of an error code; for ODSGD_EHIP, of the last HIP error seen by this thread. */
const char *odsgd_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* ODSGD_H */
