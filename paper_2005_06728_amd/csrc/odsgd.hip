// OD-SGD parameter-update engine for MI355X (gfx950): kernels and C ABI.
//
// One launch covers every parameter tensor ("multi-tensor apply"): odsgd_init
// cuts the K tensors into fixed-size chunks and writes, into caller-provided
// device memory, a chunk table (which tensor, where, how many elements) and a
// pointer table (2 + 3W device pointers per tensor).  A workgroup is a single
// wavefront; it takes one chunk, fetches its descriptor and pointers with scalar
// loads, and streams the chunk with 128-bit loads and stores (by default a chunk
// is 256 elements: one 16-byte access per lane, 1 KiB per wavefront, per array).
// The work is purely element-wise (about half a flop per byte), so the only
// roofline that matters is HBM bandwidth; there is no data reuse, hence no LDS
// staging and no matrix-core use.
//
// Launch shape.  With 2W + 4 concurrent streams (W = 8: 20, W = 16: 36) the
// memory system delivers the most when few requests are in flight and the
// whole chip walks one narrow window of each array: measured on MI355X, one-wavefront workgroups taking consecutive
// 1 KiB tiles in dispatch order, with only about 3-4 wavefronts resident per
// CU, sustain 6.0-6.3 TB/s, against 5.2-5.4 TB/s for the same kernel at full
// occupancy or as a persistent grid.  Residency is capped by requesting (and
// never touching) dynamic LDS, the one launch parameter that limits how many
// workgroups a CU accepts.
//
// Arithmetic (paper: Section 3.1, Algorithms 1 and 2; Section 3.3 Local Updater):
// see include/odsgd.h.  Every statement in the update_* functions below is one
// binary32 operation; FP contraction is disabled for the whole file so that no
// multiply-add pair is fused and results are independent of launch shape.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "odsgd.h"

#pragma clang fp contract(off)

// Table storage of odsgd_init_static: one array per GPU, part of the loaded code
// object, alive until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress; the device address it yields (one per device)
// is what kernels and copies are given.
static __device__ __align__(256) unsigned char odsgd_static_plan[ODSGD_STATIC_PLAN_BYTES];

namespace {

// ---------------------------------------------------------------------------
// compile-time tuning knobs (overridable with -D for sweeps)
// ---------------------------------------------------------------------------
#ifndef ODSGD_NT_GRAD
#define ODSGD_NT_GRAD 1  // gradients are read once: non-temporal loads
#endif
#ifndef ODSGD_NT_LOCAL
#define ODSGD_NT_LOCAL 1  // local weights are written once: non-temporal stores
#endif
#ifndef ODSGD_NT_STATE_LD
// w and momentum are the only arrays the next step reads again.  Loading these
// two with ordinary (cacheable) loads while everything else streams
// non-temporally is 4 % faster even with a cold cache, and lets them stay in the
// 256 MB last-level cache from one step to the next when they fit (ResNet-50:
// 204 MB).  Caching even one gradient stream as well, by contrast, costs 10 %.
#define ODSGD_NT_STATE_LD 0
#endif
#ifndef ODSGD_NT_STATE_ST
#define ODSGD_NT_STATE_ST 1  // w, momentum stores
#endif
#ifndef ODSGD_NT_INPLACE_LD
// per-worker arrays that a delay-compensated or momentum rule updates in place
// (previous local weights, MeanSquare, local velocity): although they share the
// read-then-write pattern of w and momentum, loading them through the cache was
// measured 10 % slower, so they stream like the gradients
#define ODSGD_NT_INPLACE_LD 1
#endif
#define ODSGD_BLOCK 64  // one wavefront per workgroup
#ifndef ODSGD_INFLIGHT_MEMOPS_PER_CU
// target of (resident wavefronts per CU) x (128-bit loads + stores per lane per
// tile); measured optimum 100-120 for every entry point and worker count tried
#define ODSGD_INFLIGHT_MEMOPS_PER_CU 110
#endif

constexpr int kBlock = ODSGD_BLOCK;

typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));

// Data pointers come out of the pointer table as integers.  Giving them the
// global address space (instead of the generic one an integer-to-pointer cast
// would have) lets the compiler emit global_load/global_store with a uniform
// SGPR base and one shared 32-bit VGPR offset, rather than flat accesses with a
// 64-bit VGPR address per array.
#define ODSGD_GLOBAL_AS __attribute__((address_space(1)))
template <typename T>
using gptr = ODSGD_GLOBAL_AS T *;
template <typename T>
using gcptr = const ODSGD_GLOBAL_AS T *;

// Tables live in global memory but never change while a kernel runs; reading
// them through the constant address space makes the compiler use scalar loads
// (one fetch per wavefront, results in SGPRs, usable as the uniform base of
// "SGPR base + VGPR offset" global loads).
#define ODSGD_CONST_AS __attribute__((address_space(4)))
typedef const ODSGD_CONST_AS u4 *chunk_table_t;
typedef const ODSGD_CONST_AS uint64_t *ptr_table_t;

enum Mode : int {
    MODE_OD = 0,      // local update of all workers from w_t, then global update
    MODE_SSGD = 1,    // global update, then every worker receives w_{t+1}
    MODE_GLOBAL = 2,  // global update only
    MODE_LOCAL = 3,   // local update only, workers [wfirst, wfirst + wcount)
};

// local updater applied by MODE_OD / MODE_LOCAL (Section 3.3, "Local Updater")
enum Rule : int {
    RULE_SGD = 0,  // u_m = w - local_lr*(g_m + r)
    RULE_DCC = 1,  // + lambda * g_m*g_m*(w - u_m_old)                         (eq. DC-ASGD-c)
    RULE_DCA = 2,  // + lambda/sqrt(MeanSquare_m + eps) * g_m*g_m*(w - u_m_old) (eq. DC-ASGD-a)
    RULE_MOM = 3,  // lv_m = mu_l*lv_m - local_lr*(g_m + r); u_m = w + lv_m    (local momentum SGD)
};

static_assert(RULE_SGD == ODSGD_LOCAL_SGD && RULE_DCC == ODSGD_LOCAL_DCASGD_C &&
                  RULE_DCA == ODSGD_LOCAL_DCASGD_A && RULE_MOM == ODSGD_LOCAL_SGD_MOMENTUM,
              "kernel rule ids are the public ones");

struct KernelArgs {
    const void *chunks;  // device: nchunks * 16 bytes
    const void *ptrs;    // device: K rows of (2 + 3*wtot) pointers
    int nchunks;
    int wtot;    // workers registered (row = [w, v, g_0.., u_0.., ms_0..], stride 2 + 3*wtot)
    int wfirst;  // first worker this launch touches
    int wcount;  // number of workers this launch touches (== W_T when W_T > 0)
    float lr, local_lr, momentum, weight_decay, grad_scale;
    float lambda, ms_decay, one_minus_ms_decay, epsilon, local_momentum;
};

// chunk descriptor, 16 bytes: {tensor | vec<<31, count, offset_lo, offset_hi}
constexpr uint32_t kVecFlag = 0x80000000u;

// ---------------------------------------------------------------------------
// memory access helpers
// ---------------------------------------------------------------------------
// `base` is a uniform 64-bit address (held in SGPRs), `idx` the lane's element
// index in units of T.  The byte offset is formed in 32 bits (chunks are at
// most 2^24 elements), which is what allows the SGPR-base + VGPR-offset form.
template <bool NT, typename T>
__device__ __forceinline__ T load(uint64_t base, unsigned idx)
{
    const gcptr<T> p = (gcptr<T>)((gcptr<char>)base + idx * (unsigned)sizeof(T));
    if constexpr (NT)
        return __builtin_nontemporal_load(p);
    else
        return *p;
}

template <bool NT, typename T>
__device__ __forceinline__ void store(uint64_t base, unsigned idx, T x)
{
    const gptr<T> p = (gptr<T>)((gptr<char>)base + idx * (unsigned)sizeof(T));
    if constexpr (NT)
        __builtin_nontemporal_store(x, p);
    else
        *p = x;
}

// ---------------------------------------------------------------------------
// the update rules; T is float or f4 (element-wise).  One statement = one
// binary32 operation (sqrt and divide are the correctly rounded ones).
// ---------------------------------------------------------------------------
struct Hyp {
    float lr, local_lr, momentum, weight_decay, grad_scale;
    float lambda, ms_decay, one_minus_ms_decay, epsilon, local_momentum;
};

__device__ __forceinline__ float sqrt_rn(float x) { return __builtin_sqrtf(x); }
__device__ __forceinline__ f4 sqrt_rn(f4 x)
{
    return f4{__builtin_sqrtf(x.x), __builtin_sqrtf(x.y), __builtin_sqrtf(x.z), __builtin_sqrtf(x.w)};
}

// SGD local updater: u_m = w_t - local_lr * (g_m + r)
template <typename T>
__device__ __forceinline__ T update_local(T w0, T g, T r, float local_lr)
{
    T dm = g + r;
    T pm = local_lr * dm;
    return w0 - pm;
}

// local momentum SGD: lv' = mu_l * lv - local_lr * (g + r);  u = w + lv'
template <typename T>
__device__ __forceinline__ T update_local_momentum(T w0, T g, T r, T lv0, const Hyp &h, T &lv1)
{
    T dm = g + r;
    T am = h.local_momentum * lv0;
    T pm = h.local_lr * dm;
    lv1 = am - pm;
    return w0 + lv1;
}

// delay-compensated local updaters; u_old = the weights g was evaluated at.
// lam is the scalar lambda (RULE_DCC) or the per-element lambda/sqrt(ms+eps) (RULE_DCA).
template <typename T, typename L>
__device__ __forceinline__ T update_local_dc(T w0, T g, T gg, T u_old, T r, L lam, float local_lr)
{
    T dlt = w0 - u_old;
    T c1 = gg * dlt;
    T c2 = c1 * lam;
    T dm = g + r;
    T em = dm + c2;
    T pm = local_lr * em;
    return w0 - pm;
}

// MeanSquare_m <- ms_decay * MeanSquare_m + (1 - ms_decay) * g*g; returns lambda / sqrt(ms + eps)
template <typename T>
__device__ __forceinline__ T mean_square_step(T gg, T ms_old, const Hyp &h, T &ms_new)
{
    T s1 = h.ms_decay * ms_old;
    T s2 = h.one_minus_ms_decay * gg;
    ms_new = s1 + s2;
    T rad = ms_new + h.epsilon;
    T den = sqrt_rn(rad);
    return h.lambda / den;
}

// v' = momentum * v_t - lr * (s * grad_scale + r);  w' = w_t + v'
template <typename T>
__device__ __forceinline__ void update_global(T w0, T v0, T s, T r, const Hyp &h, T &w1, T &v1)
{
    T gb = s * h.grad_scale;
    T d = gb + r;
    T a = h.momentum * v0;
    T b = h.lr * d;
    v1 = a - b;
    w1 = w0 + v1;
}

// ---------------------------------------------------------------------------
// one tile, fixed worker count W_T: every load is issued before the first
// store (the compiler cannot prove the outputs do not alias the inputs, so the
// order is written out by hand).
// ---------------------------------------------------------------------------
template <int W_T>
struct Ptrs {
    uint64_t w;
    uint64_t v;
    uint64_t g[W_T];
    uint64_t u[W_T];
    uint64_t ms[W_T];
};

template <int W_T, int MODE, int RULE, typename T>
__device__ __forceinline__ void apply_fixed(const Ptrs<W_T> &p, unsigned i, const Hyp &h)
{
    constexpr bool need_v = (MODE != MODE_LOCAL);
    constexpr bool need_u = (MODE != MODE_GLOBAL);
    constexpr bool local_rule = (MODE == MODE_OD || MODE == MODE_LOCAL);
    constexpr bool need_u_old = local_rule && (RULE == RULE_DCC || RULE == RULE_DCA);
    constexpr bool need_ms = local_rule && (RULE == RULE_DCA || RULE == RULE_MOM);  // per-worker state

    T w0, v0, g[W_T], u_old[W_T], ms_old[W_T];
    w0 = load<ODSGD_NT_STATE_LD, T>(p.w, i);
    if constexpr (need_v)
        v0 = load<ODSGD_NT_STATE_LD, T>(p.v, i);
#pragma unroll
    for (int m = 0; m < W_T; ++m)
        g[m] = load<ODSGD_NT_GRAD, T>(p.g[m], i);
    if constexpr (need_u_old) {
#pragma unroll
        for (int m = 0; m < W_T; ++m)
            u_old[m] = load<ODSGD_NT_INPLACE_LD, T>(p.u[m], i);
    }
    if constexpr (need_ms) {
#pragma unroll
        for (int m = 0; m < W_T; ++m)
            ms_old[m] = load<ODSGD_NT_INPLACE_LD, T>(p.ms[m], i);
    }

    T r = h.weight_decay * w0;
    T w1 = w0, v1;
    if constexpr (MODE != MODE_LOCAL) {
        T s = g[0];
#pragma unroll
        for (int m = 1; m < W_T; ++m)
            s = s + g[m];
        update_global(w0, v0, s, r, h, w1, v1);
    }
    if constexpr (need_u) {
#pragma unroll
        for (int m = 0; m < W_T; ++m) {
            T um;
            if constexpr (MODE == MODE_SSGD) {
                um = w1;
            } else if constexpr (RULE == RULE_SGD) {
                um = update_local(w0, g[m], r, h.local_lr);
            } else if constexpr (RULE == RULE_DCC) {
                T gg = g[m] * g[m];
                um = update_local_dc(w0, g[m], gg, u_old[m], r, h.lambda, h.local_lr);
            } else if constexpr (RULE == RULE_DCA) {
                T gg = g[m] * g[m];
                T ms_new;
                T lam = mean_square_step(gg, ms_old[m], h, ms_new);
                store<ODSGD_NT_LOCAL, T>(p.ms[m], i, ms_new);
                um = update_local_dc(w0, g[m], gg, u_old[m], r, lam, h.local_lr);
            } else {
                T lv1;
                um = update_local_momentum(w0, g[m], r, ms_old[m], h, lv1);
                store<ODSGD_NT_LOCAL, T>(p.ms[m], i, lv1);
            }
            store<ODSGD_NT_LOCAL, T>(p.u[m], i, um);
        }
    }
    if constexpr (MODE != MODE_LOCAL) {
        store<ODSGD_NT_STATE_ST, T>(p.v, i, v1);
        store<ODSGD_NT_STATE_ST, T>(p.w, i, w1);
    }
}

// any worker count: pointers are fetched from the table inside the worker loop
template <int MODE, int RULE, typename T>
__device__ __forceinline__ void apply_generic(ptr_table_t row, uint64_t byte_off, int wtot, int wfirst,
                                              int wcount, unsigned i, const Hyp &h)
{
    const uint64_t pw = row[0] + byte_off;
    const uint64_t pv = row[1] + byte_off;
    T w0 = load<ODSGD_NT_STATE_LD, T>(pw, i);
    T r = h.weight_decay * w0;
    T s;
    for (int m = 0; m < wcount; ++m) {
        T gm = load<ODSGD_NT_GRAD, T>(row[2 + wfirst + m] + byte_off, i);
        s = (m == 0) ? gm : s + gm;
        if constexpr (MODE == MODE_OD || MODE == MODE_LOCAL) {
            const uint64_t pu = row[2 + wtot + wfirst + m] + byte_off;
            T um;
            if constexpr (RULE == RULE_SGD) {
                um = update_local(w0, gm, r, h.local_lr);
            } else if constexpr (RULE == RULE_DCC) {
                T u_old = load<ODSGD_NT_INPLACE_LD, T>(pu, i);
                T gg = gm * gm;
                um = update_local_dc(w0, gm, gg, u_old, r, h.lambda, h.local_lr);
            } else if constexpr (RULE == RULE_DCA) {
                const uint64_t pms = row[2 + 2 * wtot + wfirst + m] + byte_off;
                T u_old = load<ODSGD_NT_INPLACE_LD, T>(pu, i);
                T ms_old = load<ODSGD_NT_INPLACE_LD, T>(pms, i);
                T gg = gm * gm;
                T ms_new;
                T lam = mean_square_step(gg, ms_old, h, ms_new);
                store<ODSGD_NT_LOCAL, T>(pms, i, ms_new);
                um = update_local_dc(w0, gm, gg, u_old, r, lam, h.local_lr);
            } else {
                const uint64_t plv = row[2 + 2 * wtot + wfirst + m] + byte_off;
                T lv0 = load<ODSGD_NT_INPLACE_LD, T>(plv, i);
                T lv1;
                um = update_local_momentum(w0, gm, r, lv0, h, lv1);
                store<ODSGD_NT_LOCAL, T>(plv, i, lv1);
            }
            store<ODSGD_NT_LOCAL, T>(pu, i, um);
        }
    }
    if constexpr (MODE != MODE_LOCAL) {
        T v0 = load<ODSGD_NT_STATE_LD, T>(pv, i);
        T w1, v1;
        update_global(w0, v0, s, r, h, w1, v1);
        if constexpr (MODE == MODE_SSGD) {
            for (int m = 0; m < wcount; ++m) {
                store<ODSGD_NT_LOCAL, T>(row[2 + wtot + wfirst + m] + byte_off, i, w1);
            }
        }
        store<ODSGD_NT_STATE_ST, T>(pv, i, v1);
        store<ODSGD_NT_STATE_ST, T>(pw, i, w1);
    }
}

// ---------------------------------------------------------------------------
// the kernel: grid-stride over the chunk table
// ---------------------------------------------------------------------------
template <int W_T, int MODE, int RULE>
__global__ void __launch_bounds__(kBlock) odsgd_kernel(KernelArgs a)
{
    const chunk_table_t chunks = (chunk_table_t)a.chunks;
    const ptr_table_t ptrs = (ptr_table_t)a.ptrs;
    const Hyp h{a.lr, a.local_lr, a.momentum, a.weight_decay, a.grad_scale,
                a.lambda, a.ms_decay, a.one_minus_ms_decay, a.epsilon, a.local_momentum};
    const unsigned tid = threadIdx.x;
    const int stride = 2 + 3 * a.wtot;

    // Workgroup b takes chunk b (the host never launches more workgroups than
    // chunks, so the first trip needs no bounds check and the descriptor fetch can
    // be issued together with the kernel arguments).  The dispatcher hands
    // consecutive workgroups to the 8 XCDs in turn, so at any moment the chip works
    // on one narrow, sliding window of each array; giving every XCD a contiguous
    // range of its own instead was measured 15 % slower.
    unsigned c = blockIdx.x;
    do {
        const u4 d = chunks[c];
        const uint32_t tensor = d.x & ~kVecFlag;
        const bool vec = (d.x & kVecFlag) != 0;
        const unsigned count = d.y;
        const uint64_t byte_off = (((uint64_t)d.w << 32) | d.z) * sizeof(float);
        const ptr_table_t row = ptrs + (uint64_t)tensor * stride;
        const unsigned nvec = vec ? (count >> 2) : 0u;

        if constexpr (W_T > 0) {
            // Fetch the whole pointer row before touching any of it: the scalar loads
            // are then in flight together instead of one memory latency after another
            // (with 3-4 wavefronts per CU that latency is not hidden by anyone else).
            constexpr bool with_state = (RULE == RULE_DCA || RULE == RULE_MOM);
            uint64_t raw_wv[2], raw_g[W_T], raw_u[W_T], raw_s[W_T];
            raw_wv[0] = row[0];
            raw_wv[1] = row[1];
#pragma unroll
            for (int m = 0; m < W_T; ++m)
                raw_g[m] = row[2 + a.wfirst + m];
#pragma unroll
            for (int m = 0; m < W_T; ++m)
                raw_u[m] = row[2 + a.wtot + a.wfirst + m];
            if constexpr (with_state) {
#pragma unroll
                for (int m = 0; m < W_T; ++m)
                    raw_s[m] = row[2 + 2 * a.wtot + a.wfirst + m];
            }
            Ptrs<W_T> p;
            p.w = raw_wv[0] + byte_off;
            p.v = raw_wv[1] + byte_off;
#pragma unroll
            for (int m = 0; m < W_T; ++m) {
                p.g[m] = raw_g[m] + byte_off;
                p.u[m] = raw_u[m] + byte_off;
                if constexpr (with_state)
                    p.ms[m] = raw_s[m] + byte_off;
            }
            for (unsigned i = tid; i < nvec; i += kBlock)
                apply_fixed<W_T, MODE, RULE, f4>(p, i, h);
            for (unsigned t = nvec * 4 + tid; t < count; t += kBlock)
                apply_fixed<W_T, MODE, RULE, float>(p, t, h);
        } else {
            for (unsigned i = tid; i < nvec; i += kBlock)
                apply_generic<MODE, RULE, f4>(row, byte_off, a.wtot, a.wfirst, a.wcount, i, h);
            for (unsigned t = nvec * 4 + tid; t < count; t += kBlock)
                apply_generic<MODE, RULE, float>(row, byte_off, a.wtot, a.wfirst, a.wcount, t, h);
        }
        c += gridDim.x;
    } while (c < (unsigned)a.nchunks);
}

// Plain copy, one 1 KiB tile per wavefront: a kernel of exactly known traffic
// (n*4 bytes read, n*4 bytes written) for calibrating HBM byte counters.
__global__ void __launch_bounds__(kBlock) odsgd_probe_copy_kernel(uint64_t dst, uint64_t src, uint64_t nvec)
{
    const uint64_t tile = blockIdx.x;
    const uint64_t i = tile * kBlock + threadIdx.x;
    if (i < nvec) {
        const f4 x = load<true, f4>(src + tile * (kBlock * sizeof(f4)), threadIdx.x);
        store<true, f4>(dst + tile * (kBlock * sizeof(f4)), threadIdx.x, x);
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
thread_local hipError_t g_last_hip_error = hipSuccess;

struct Tuning {
    int64_t chunk_elems;  // elements per chunk (multiple of 4 * kBlock)
    int blocks_per_cu;    // grid cap = blocks_per_cu * CUs; 0 = one workgroup per chunk
    int waves_per_cu;     // resident wavefronts per CU: 0 = choose per launch, < 0 = no cap
};

int64_t env_int(const char *name, int64_t dflt)
{
    const char *s = std::getenv(name);
    if (!s || !*s)
        return dflt;
    char *end = nullptr;
    long long v = std::strtoll(s, &end, 10);
    return (end && *end == '\0') ? (int64_t)v : dflt;
}

Tuning current_tuning()
{
    Tuning t;
    t.chunk_elems = env_int("ODSGD_CHUNK_ELEMS", 4 * kBlock);
    const int64_t q = 4 * kBlock;
    if (t.chunk_elems < q)
        t.chunk_elems = q;
    if (t.chunk_elems > (int64_t)1 << 24)
        t.chunk_elems = (int64_t)1 << 24;
    t.chunk_elems = (t.chunk_elems / q) * q;
    t.blocks_per_cu = (int)env_int("ODSGD_BLOCKS_PER_CU", 0);
    if (t.blocks_per_cu < 0)
        t.blocks_per_cu = 0;
    t.waves_per_cu = (int)env_int("ODSGD_WAVES_PER_CU", 0);
    return t;
}

constexpr int64_t kMaxNumel = (int64_t)1 << 40;
// Tiles whose addresses start on a 512-byte boundary stream measurably faster
// (5-6 % on MI355X) than tiles that straddle one; 1 KiB = one full tile.
constexpr uintptr_t kTileAlignBytes = 1024;
constexpr int64_t kMaxChunks = 0x7ffffffe;

// Upper bound on the number of chunks for this tensor list (what the workspace is
// sized for), or -1 on invalid input / overflow.  Each tensor may get one extra
// short head chunk that brings the following chunk starts onto a tile boundary.
int64_t count_chunks(int num_tensors, const int64_t *numel, int64_t chunk_elems, int *err)
{
    int64_t n = 0;
    for (int k = 0; k < num_tensors; ++k) {
        if (numel[k] < 0) {
            *err = ODSGD_EINVAL;
            return -1;
        }
        if (numel[k] >= kMaxNumel) {
            *err = ODSGD_ERANGE;
            return -1;
        }
        n += (numel[k] + chunk_elems - 1) / chunk_elems + (numel[k] > 0 ? 1 : 0);
        if (n > kMaxChunks) {
            *err = ODSGD_ERANGE;
            return -1;
        }
    }
    return n;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

size_t ptr_table_bytes(int num_tensors, int num_workers)
{
    return align_up((size_t)num_tensors * (2 + 3 * (size_t)num_workers) * sizeof(uint64_t), 256);
}

struct Range {
    uintptr_t lo, hi;
    bool is_output;
};

// true if any output range overlaps any other range
bool ranges_alias(std::vector<Range> &r)
{
    std::sort(r.begin(), r.end(), [](const Range &a, const Range &b) { return a.lo < b.lo; });
    uintptr_t max_hi_any = 0, max_hi_out = 0;
    for (const Range &x : r) {
        if (x.lo < max_hi_out)
            return true;
        if (x.is_output && x.lo < max_hi_any)
            return true;
        max_hi_any = std::max(max_hi_any, x.hi);
        if (x.is_output)
            max_hi_out = std::max(max_hi_out, x.hi);
    }
    return false;
}

// The launch plan: host image of the two tables odsgd_init uploads, plus the
// registered address ranges.  Building it touches no device.
struct Plan {
    Tuning tuning;
    std::vector<unsigned char> image;  // [pointer table | chunk table], sized for the upper bound of chunks
    size_t ptr_bytes;                  // offset of the chunk table inside image
    int64_t nchunks;                   // chunks actually emitted
    std::vector<Range> ranges;
};

int make_plan(Plan &plan, int num_tensors, const int64_t *numel, float *const *w, float *const *mom,
              const float *const *const *grads, float *const *const *local_w, int num_workers)
{
    if (num_tensors < 1 || !numel || !w || !mom || !grads || !local_w || num_workers < 1 ||
        num_workers > ODSGD_MAX_WORKERS)
        return ODSGD_EINVAL;
    for (int m = 0; m < num_workers; ++m)
        if (!grads[m] || !local_w[m])
            return ODSGD_EINVAL;

    plan.tuning = current_tuning();
    int err = 0;
    const int64_t max_chunks = count_chunks(num_tensors, numel, plan.tuning.chunk_elems, &err);
    if (max_chunks < 0)
        return err;

    const int W = num_workers;
    const int stride = 2 + 3 * W;
    const int registered = 2 + 2 * W;  // the per-worker state columns stay null until a rule registers them

    // pointer checks: non-null and 4-byte aligned where the tensor is not empty
    plan.ranges.clear();
    plan.ranges.reserve((size_t)num_tensors * stride + 1);
    std::vector<unsigned char> vec_ok(num_tensors, 1);
    // elements before the first tile boundary, when every array of the tensor sits
    // at the same offset from one (packed buckets); 0 = chunks start at element 0
    std::vector<int64_t> head(num_tensors, 0);
    for (int k = 0; k < num_tensors; ++k) {
        if (numel[k] == 0)
            continue;
        const size_t bytes = (size_t)numel[k] * sizeof(float);
        const uintptr_t phase = (uintptr_t)w[k] % kTileAlignBytes;
        bool same_phase = true;
        for (int j = 0; j < registered; ++j) {
            const void *p = j == 0   ? (const void *)w[k]
                            : j == 1 ? (const void *)mom[k]
                            : j < 2 + W ? (const void *)grads[j - 2][k]
                                        : (const void *)local_w[j - 2 - W][k];
            if (!p)
                return ODSGD_EINVAL;
            const uintptr_t a = (uintptr_t)p;
            if (a % 4 != 0)
                return ODSGD_EALIGN;
            if (a % 16 != 0)
                vec_ok[k] = 0;
            if (a % kTileAlignBytes != phase)
                same_phase = false;
            const bool is_output = (j < 2) || (j >= 2 + W);
            plan.ranges.push_back(Range{a, a + bytes, is_output});
        }
        if (same_phase && vec_ok[k] && phase != 0) {
            const int64_t h0 = (int64_t)((kTileAlignBytes - phase) / sizeof(float));
            if (h0 < numel[k])
                head[k] = h0;
        }
    }

    plan.ptr_bytes = ptr_table_bytes(num_tensors, W);
    const size_t chunk_bytes = align_up((size_t)std::max<int64_t>(max_chunks, 1) * 16, 256);
    plan.image.assign(plan.ptr_bytes + chunk_bytes, 0);
    uint64_t *pt = reinterpret_cast<uint64_t *>(plan.image.data());
    for (int k = 0; k < num_tensors; ++k) {
        uint64_t *row = pt + (size_t)k * stride;
        row[0] = (uint64_t)(uintptr_t)w[k];
        row[1] = (uint64_t)(uintptr_t)mom[k];
        for (int m = 0; m < W; ++m) {
            row[2 + m] = (uint64_t)(uintptr_t)grads[m][k];
            row[2 + W + m] = (uint64_t)(uintptr_t)local_w[m][k];
        }
    }
    // chunk table: full chunks of all tensors first, ragged ones (heads and
    // tails) after them, so the short pieces fill the end of the launch
    uint32_t *ct = reinterpret_cast<uint32_t *>(plan.image.data() + plan.ptr_bytes);
    int64_t c = 0;
    const int64_t C = plan.tuning.chunk_elems;
    auto emit = [&](int k, int64_t off, int64_t cnt) {
        uint32_t *dsc = ct + c * 4;
        dsc[0] = (uint32_t)k | (vec_ok[k] ? kVecFlag : 0u);
        dsc[1] = (uint32_t)cnt;
        dsc[2] = (uint32_t)((uint64_t)off & 0xffffffffu);
        dsc[3] = (uint32_t)((uint64_t)off >> 32);
        ++c;
    };
    for (int pass = 0; pass < 2; ++pass) {
        for (int k = 0; k < num_tensors; ++k) {
            const int64_t n = numel[k];
            const int64_t body = n - head[k];
            const int64_t nfull = body / C;
            if (pass == 0) {
                for (int64_t j = 0; j < nfull; ++j)
                    emit(k, head[k] + j * C, C);
            } else {
                if (head[k] > 0)
                    emit(k, 0, head[k]);
                if (body > nfull * C)
                    emit(k, head[k] + nfull * C, body - nfull * C);
            }
        }
    }
    plan.nchunks = c;
    return ODSGD_OK;
}

using KernelFn = void (*)(KernelArgs);

template <int MODE, int RULE>
KernelFn pick_by_workers(int wcount)
{
    switch (wcount) {
    case 1: return odsgd_kernel<1, MODE, RULE>;
    case 2: return odsgd_kernel<2, MODE, RULE>;
    case 4: return odsgd_kernel<4, MODE, RULE>;
    case 8: return odsgd_kernel<8, MODE, RULE>;
    case 12: return odsgd_kernel<12, MODE, RULE>;
    case 16: return odsgd_kernel<16, MODE, RULE>;
    default: return odsgd_kernel<0, MODE, RULE>;
    }
}

template <int MODE>
KernelFn pick_by_rule(int rule, int wcount)
{
    switch (rule) {
    case RULE_DCC: return pick_by_workers<MODE, RULE_DCC>(wcount);
    case RULE_DCA: return pick_by_workers<MODE, RULE_DCA>(wcount);
    case RULE_MOM: return pick_by_workers<MODE, RULE_MOM>(wcount);
    default: return pick_by_workers<MODE, RULE_SGD>(wcount);
    }
}

KernelFn pick_kernel(int mode, int rule, int wcount)
{
    switch (mode) {
    case MODE_OD: return pick_by_rule<MODE_OD>(rule, wcount);
    case MODE_LOCAL: return pick_by_rule<MODE_LOCAL>(rule, wcount);
    case MODE_SSGD: return pick_by_workers<MODE_SSGD, RULE_SGD>(wcount);
    default: return pick_by_workers<MODE_GLOBAL, RULE_SGD>(wcount);
    }
}

}  // namespace

struct odsgd_handle {
    int num_tensors;
    int num_workers;
    int64_t nchunks;
    const void *d_chunks;
    const void *d_ptrs;
    int device;
    int num_cus;
    int lds_per_cu;
    Tuning tuning;
    int64_t iteration;
    int64_t warmup_steps;
    odsgd_local_rule rule;               // local updater of MODE_OD / MODE_LOCAL
    std::vector<int64_t> numel;
    std::vector<Range> ranges;           // every registered buffer, for alias checks of later registrations
    size_t base_ranges;                  // how many of them odsgd_init registered
    bool static_plan;                    // tables live in the per-device static array
    uint64_t static_generation;          // which registration of that array this handle is
};

namespace {

// Dynamic LDS to request so that a CU holds about `waves` one-wavefront
// workgroups.  The kernels never touch LDS; the request only limits residency.
// LDS is handed out in 1280-byte granules; a workgroup may ask for at most 64 KiB
// (so two resident wavefronts per CU is the lowest cap).
size_t occupancy_cap_lds_bytes(const odsgd_handle *h, int mode, int wcount)
{
    int waves = h->tuning.waves_per_cu;
    if (waves < 0)
        return 0;
    if (waves == 0) {
        // memory instructions (loads + stores) one lane issues per tile
        int loads = (mode == MODE_LOCAL) ? wcount + 1 : wcount + 2;
        int stores = (mode == MODE_GLOBAL) ? 2 : (mode == MODE_LOCAL) ? wcount : wcount + 2;
        if (mode == MODE_OD || mode == MODE_LOCAL) {
            const int rl = h->rule.rule;
            if (rl == ODSGD_LOCAL_DCASGD_C || rl == ODSGD_LOCAL_DCASGD_A)
                loads += wcount;  // previous local weights
            if (rl == ODSGD_LOCAL_DCASGD_A || rl == ODSGD_LOCAL_SGD_MOMENTUM) {
                loads += wcount;  // per-worker state in ...
                stores += wcount; // ... and out
            }
        }
        const int ops = loads + stores;
        waves = (ODSGD_INFLIGHT_MEMOPS_PER_CU + ops / 2) / ops;  // nearest integer
        // the adaptive rule spends a correctly rounded sqrt and divide per element and
        // worker: more wavefronts are needed to hide that arithmetic
        if ((mode == MODE_OD || mode == MODE_LOCAL) && h->rule.rule == ODSGD_LOCAL_DCASGD_A)
            waves = std::max(5, (170 + ops / 2) / ops);
        if (waves > 16)
            return 0;  // few streams: full occupancy is best
    }
    if (waves < 2)
        waves = 2;
    const size_t granule = 1280;
    size_t bytes = (size_t)h->lds_per_cu / (size_t)waves / granule * granule;
    if (bytes > 65536)
        bytes = 65536;
    if (bytes < granule)
        return 0;  // more wavefronts than the cap can express: no cap
    return bytes;
}

// Per-device address of odsgd_static_plan and the number of registrations it has
// seen; only the latest registration's handle may still launch.
constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
void *g_static_ptr[kMaxDevices] = {};
uint64_t g_static_generation[kMaxDevices] = {};

// Device address of the static array on `device`, which must be the current device.
int static_plan_address(int device, void **out)
{
    if (device < 0 || device >= kMaxDevices)
        return ODSGD_EINVAL;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[device]) {
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(odsgd_static_plan));
        if (e != hipSuccess || !p) {
            g_last_hip_error = (e != hipSuccess) ? e : hipErrorInvalidSymbol;
            return ODSGD_EHIP;
        }
        g_static_ptr[device] = p;
    }
    *out = g_static_ptr[device];
    return ODSGD_OK;
}

bool handle_is_stale(const odsgd_handle *h)
{
    if (!h->static_plan)
        return false;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    return g_static_generation[h->device] != h->static_generation;
}

int launch(odsgd_handle *h, int mode, int wfirst, int wcount, const odsgd_hyper *hy, void *stream)
{
    if (handle_is_stale(h))
        return ODSGD_ESTALE;
    if (h->nchunks == 0)
        return ODSGD_OK;
    KernelArgs a;
    a.chunks = h->d_chunks;
    a.ptrs = h->d_ptrs;
    a.nchunks = (int)h->nchunks;
    a.wtot = h->num_workers;
    a.wfirst = wfirst;
    a.wcount = wcount;
    a.lr = hy->lr;
    a.local_lr = hy->local_lr;
    a.momentum = hy->momentum;
    a.weight_decay = hy->weight_decay;
    a.grad_scale = (hy->grad_scale <= 0.0f) ? 1.0f / (float)h->num_workers : hy->grad_scale;
    a.lambda = h->rule.lambda;
    a.ms_decay = h->rule.ms_decay;
    a.one_minus_ms_decay = 1.0f - h->rule.ms_decay;
    a.epsilon = h->rule.epsilon;
    a.local_momentum = h->rule.local_momentum;

    // one workgroup per chunk; beyond 2^25 workgroups (2^31 threads, the launch
    // limit is 2^32) the kernel's grid-stride loop takes over
    int64_t grid = std::min<int64_t>(h->nchunks, (int64_t)1 << 25);
    if (h->tuning.blocks_per_cu > 0)
        grid = std::min<int64_t>(grid, (int64_t)h->tuning.blocks_per_cu * h->num_cus);
    KernelFn fn = pick_kernel(mode, h->rule.rule, wcount);
    const size_t lds = occupancy_cap_lds_bytes(h, mode, wcount);
    hipLaunchKernelGGL(fn, dim3((unsigned)grid), dim3(kBlock), lds, (hipStream_t)stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        g_last_hip_error = e;
        return ODSGD_EHIP;
    }
    return ODSGD_OK;
}

// Shared by odsgd_init (tables in the caller's workspace) and odsgd_init_static
// (tables in the per-device static array; `workspace` is then looked up here,
// after every check that needs no device has passed).
int init_common(odsgd_handle **out, int num_tensors, const int64_t *numel, float *const *w, float *const *mom,
                const float *const *const *grads, float *const *const *local_w, int num_workers,
                void *workspace, size_t workspace_bytes, bool static_plan, void *stream)
{
    Plan plan;
    int rc = make_plan(plan, num_tensors, numel, w, mom, grads, local_w, num_workers);
    if (rc != ODSGD_OK)
        return rc;
    if (!static_plan && (uintptr_t)workspace % 256 != 0)
        return ODSGD_EALIGN;
    if (workspace_bytes < plan.image.size())
        return ODSGD_ENOSPC;

    int device = 0;
    if (static_plan) {
        // the caller's buffers cannot overlap the library's own array, but they may
        // not overlap each other either
        std::vector<Range> sorted = plan.ranges;
        if (ranges_alias(sorted))
            return ODSGD_EALIAS;
        hipError_t e = hipGetDevice(&device);
        if (e != hipSuccess) {
            g_last_hip_error = e;
            return ODSGD_EHIP;
        }
        rc = static_plan_address(device, &workspace);
        if (rc != ODSGD_OK)
            return rc;
    }
    plan.ranges.push_back(Range{(uintptr_t)workspace, (uintptr_t)workspace + plan.image.size(), true});
    {
        std::vector<Range> sorted = plan.ranges;
        if (ranges_alias(sorted))
            return ODSGD_EALIAS;
    }

    odsgd_handle *h = new (std::nothrow) odsgd_handle();
    if (!h)
        return ODSGD_EINVAL;
    h->num_tensors = num_tensors;
    h->num_workers = num_workers;
    h->nchunks = plan.nchunks;
    h->tuning = plan.tuning;
    h->iteration = 0;
    h->warmup_steps = 0;
    h->rule = odsgd_local_rule{ODSGD_LOCAL_SGD, 0.0f, 0.0f, 0.0f, 0.0f};
    h->numel.assign(numel, numel + num_tensors);
    h->ranges = std::move(plan.ranges);
    h->base_ranges = h->ranges.size();
    h->d_ptrs = workspace;
    h->d_chunks = (const unsigned char *)workspace + plan.ptr_bytes;
    h->static_plan = static_plan;
    h->static_generation = 0;

    hipError_t e = hipGetDevice(&h->device);
    if (e == hipSuccess) {
        int cus = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, h->device);
        h->num_cus = cus > 0 ? cus : 256;
    }
    if (e == hipSuccess) {
        int lds = 0;
        e = hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, h->device);
        h->lds_per_cu = lds > 0 ? lds : 160 * 1024;
    }
    if (e == hipSuccess && static_plan) {
        // from here on the array holds this registration: handles of earlier ones are stale
        std::lock_guard<std::mutex> lock(g_static_mutex);
        h->static_generation = ++g_static_generation[h->device];
    }
    // The whole image is uploaded, zero padding and the (still null) per-worker
    // state columns included, so nothing a kernel reads is left over from an
    // earlier registration of the same memory.
    if (e == hipSuccess)
        e = hipMemcpyAsync(workspace, plan.image.data(), plan.image.size(), hipMemcpyHostToDevice,
                           (hipStream_t)stream);
    if (e == hipSuccess)
        e = hipStreamSynchronize((hipStream_t)stream);  // plan.image must outlive the copy
    if (e != hipSuccess) {
        g_last_hip_error = e;
        delete h;
        return ODSGD_EHIP;
    }
    *out = h;
    return ODSGD_OK;
}

}  // namespace

extern "C" {

size_t odsgd_workspace_bytes(int num_tensors, const int64_t *numel, int num_workers)
{
    if (num_tensors < 1 || !numel || num_workers < 1 || num_workers > ODSGD_MAX_WORKERS)
        return 0;
    int err = 0;
    const Tuning t = current_tuning();
    const int64_t nchunks = count_chunks(num_tensors, numel, t.chunk_elems, &err);
    if (nchunks < 0)
        return 0;
    return ptr_table_bytes(num_tensors, num_workers) + align_up((size_t)std::max<int64_t>(nchunks, 1) * 16, 256);
}

int odsgd_init(odsgd_handle **out, int num_tensors, const int64_t *numel, float *const *w,
               float *const *mom, const float *const *const *grads, float *const *const *local_w,
               int num_workers, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!out)
        return ODSGD_EINVAL;
    *out = nullptr;
    if (!workspace)
        return ODSGD_EINVAL;
    return init_common(out, num_tensors, numel, w, mom, grads, local_w, num_workers, workspace, workspace_bytes,
                       false, stream);
}

int odsgd_init_static(odsgd_handle **out, int num_tensors, const int64_t *numel, float *const *w,
                      float *const *mom, const float *const *const *grads, float *const *const *local_w,
                      int num_workers, void *stream)
{
    if (!out)
        return ODSGD_EINVAL;
    *out = nullptr;
    return init_common(out, num_tensors, numel, w, mom, grads, local_w, num_workers, nullptr,
                       ODSGD_STATIC_PLAN_BYTES, true, stream);
}

int odsgd_plan_host(int num_tensors, const int64_t *numel, float *const *w, float *const *mom,
                    const float *const *const *grads, float *const *const *local_w, int num_workers,
                    void *image, size_t image_bytes, int64_t *num_chunks, size_t *chunk_table_offset)
{
    if (!image || !num_chunks || !chunk_table_offset)
        return ODSGD_EINVAL;
    Plan plan;
    int rc = make_plan(plan, num_tensors, numel, w, mom, grads, local_w, num_workers);
    if (rc != ODSGD_OK)
        return rc;
    {
        std::vector<Range> sorted = plan.ranges;
        if (ranges_alias(sorted))
            return ODSGD_EALIAS;
    }
    if (image_bytes < plan.image.size())
        return ODSGD_ENOSPC;
    std::memcpy(image, plan.image.data(), plan.image.size());
    *num_chunks = plan.nchunks;
    *chunk_table_offset = plan.ptr_bytes;
    return ODSGD_OK;
}

int odsgd_local_update(odsgd_handle *h, int worker, const odsgd_hyper *hyper, void *stream)
{
    if (!h || !hyper || worker < -1 || worker >= h->num_workers)
        return ODSGD_EINVAL;
    if (worker < 0)
        return launch(h, MODE_LOCAL, 0, h->num_workers, hyper, stream);
    return launch(h, MODE_LOCAL, worker, 1, hyper, stream);
}

int odsgd_global_update(odsgd_handle *h, const odsgd_hyper *hyper, void *stream)
{
    if (!h || !hyper)
        return ODSGD_EINVAL;
    int rc = launch(h, MODE_GLOBAL, 0, h->num_workers, hyper, stream);
    if (rc == ODSGD_OK)
        ++h->iteration;
    return rc;
}

int odsgd_ssgd_step(odsgd_handle *h, const odsgd_hyper *hyper, void *stream)
{
    if (!h || !hyper)
        return ODSGD_EINVAL;
    int rc = launch(h, MODE_SSGD, 0, h->num_workers, hyper, stream);
    if (rc == ODSGD_OK)
        ++h->iteration;
    return rc;
}

int odsgd_step(odsgd_handle *h, const odsgd_hyper *hyper, void *stream)
{
    if (!h || !hyper)
        return ODSGD_EINVAL;
    const int mode = (h->iteration < h->warmup_steps) ? MODE_SSGD : MODE_OD;
    int rc = launch(h, mode, 0, h->num_workers, hyper, stream);
    if (rc == ODSGD_OK)
        ++h->iteration;
    return rc;
}

int odsgd_set_local_rule(odsgd_handle *h, const odsgd_local_rule *rule, float *const *const *state,
                         void *stream)
{
    if (!h || !rule)
        return ODSGD_EINVAL;
    if (handle_is_stale(h))
        return ODSGD_ESTALE;
    if (rule->rule != ODSGD_LOCAL_SGD && rule->rule != ODSGD_LOCAL_DCASGD_C &&
        rule->rule != ODSGD_LOCAL_DCASGD_A && rule->rule != ODSGD_LOCAL_SGD_MOMENTUM)
        return ODSGD_EINVAL;
    if (rule->rule == ODSGD_LOCAL_DCASGD_A || rule->rule == ODSGD_LOCAL_SGD_MOMENTUM) {
        float *const *const *mean_square = state;
        if (!mean_square)
            return ODSGD_EINVAL;
        const int W = h->num_workers, K = h->num_tensors;
        const int stride = 2 + 3 * W;
        // a state registration replaces the previous one (its ranges were appended last)
        std::vector<Range> all(h->ranges.begin(), h->ranges.begin() + (std::ptrdiff_t)h->base_ranges);
        std::vector<uint64_t> cols((size_t)K * W, 0);
        for (int m = 0; m < W; ++m) {
            if (!mean_square[m])
                return ODSGD_EINVAL;
            for (int k = 0; k < K; ++k) {
                if (h->numel[k] == 0)
                    continue;
                const uintptr_t a = (uintptr_t)mean_square[m][k];
                if (!a)
                    return ODSGD_EINVAL;
                // a tensor's 128-bit path was chosen at init from its other pointers, so
                // the state must be able to follow it
                if (a % 16 != 0)
                    return ODSGD_EALIGN;
                all.push_back(Range{a, a + (size_t)h->numel[k] * sizeof(float), true});
                cols[(size_t)k * W + m] = (uint64_t)a;
            }
        }
        std::vector<Range> sorted = all;
        if (ranges_alias(sorted))
            return ODSGD_EALIAS;
        // upload the MeanSquare columns of every pointer-table row
        hipError_t e = hipMemcpy2DAsync((unsigned char *)const_cast<void *>(h->d_ptrs) + (size_t)(2 + 2 * W) * sizeof(uint64_t),
                                        (size_t)stride * sizeof(uint64_t), cols.data(), (size_t)W * sizeof(uint64_t),
                                        (size_t)W * sizeof(uint64_t), (size_t)K, hipMemcpyHostToDevice,
                                        (hipStream_t)stream);
        if (e == hipSuccess)
            e = hipStreamSynchronize((hipStream_t)stream);
        if (e != hipSuccess) {
            g_last_hip_error = e;
            return ODSGD_EHIP;
        }
        h->ranges = std::move(all);
    }
    h->rule = *rule;
    return ODSGD_OK;
}

int odsgd_set_warmup(odsgd_handle *h, int64_t warmup_steps)
{
    if (!h || warmup_steps < 0)
        return ODSGD_EINVAL;
    h->warmup_steps = warmup_steps;
    return ODSGD_OK;
}

int64_t odsgd_get_iteration(const odsgd_handle *h) { return h ? h->iteration : (int64_t)ODSGD_EINVAL; }

int odsgd_set_iteration(odsgd_handle *h, int64_t iteration)
{
    if (!h || iteration < 0)
        return ODSGD_EINVAL;
    h->iteration = iteration;
    return ODSGD_OK;
}

int odsgd_probe_copy(float *dst, const float *src, size_t numel, void *stream)
{
    if (!dst || !src || numel % 4 != 0 || (uintptr_t)dst % 16 != 0 || (uintptr_t)src % 16 != 0)
        return ODSGD_EINVAL;
    const uint64_t nvec = numel / 4;
    const uint64_t tiles = (nvec + kBlock - 1) / kBlock;
    if (tiles > (uint64_t)kMaxChunks)
        return ODSGD_ERANGE;
    if (tiles == 0)
        return ODSGD_OK;
    hipLaunchKernelGGL(odsgd_probe_copy_kernel, dim3((unsigned)tiles), dim3(kBlock), 0, (hipStream_t)stream,
                       (uint64_t)(uintptr_t)dst, (uint64_t)(uintptr_t)src, nvec);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        g_last_hip_error = e;
        return ODSGD_EHIP;
    }
    return ODSGD_OK;
}

int odsgd_destroy(odsgd_handle *h)
{
    if (!h)
        return ODSGD_EINVAL;
    delete h;
    return ODSGD_OK;
}

const char *odsgd_strerror(int code)
{
    switch (code) {
    case ODSGD_OK: return "success";
    case ODSGD_EINVAL: return "invalid argument";
    case ODSGD_EALIGN: return "device pointer not sufficiently aligned";
    case ODSGD_EALIAS: return "an output buffer overlaps another registered buffer";
    case ODSGD_ENOSPC: return "workspace too small";
    case ODSGD_EHIP: return hipGetErrorString(g_last_hip_error);
    case ODSGD_ERANGE: return "tensor list too large for the chunk table";
    case ODSGD_ESTALE: return "a later odsgd_init_static on this GPU took over the static table memory";
    default: return "unknown error code";
    }
}

}  // extern "C"
