// OD-SGD parameter-update engine for MI355X (gfx950): kernels and C ABI.
//
// One launch covers every parameter tensor ("multi-tensor apply"): registration
// cuts the K tensors into chunks of one 256-element tile and writes, into caller-provided
// device memory, a chunk table (which pointer row, where, how many elements)
// and a pointer table (4 + 3W device pointers per row; a row is a tensor, or a
// 2 GiB segment of a larger one, so that offsets inside a row fit 32 bits).  A
// workgroup is a single wavefront; it takes one tile, fetches its descriptor and
// pointers with scalar loads, and moves one 16-byte access per lane per array
// (1 KiB per wavefront per array).  The work is purely element-wise (about half
// a flop per byte), so the only roofline that matters is HBM bandwidth; there is
// no data reuse, hence no LDS staging and no matrix-core use.
//
// Launch shape.  With 2W + 4 concurrent streams (W = 8: 20, W = 16: 36) the
// memory system delivers the most when few requests are in flight and the whole
// chip walks one narrow window of each array, consecutive workgroups taking
// consecutive tiles in dispatch order with only a few wavefronts resident per
// CU.  Residency is capped by requesting (and never touching) dynamic LDS, the
// one launch parameter that limits how many workgroups a CU accepts.
//
// Tile shape.  Where all arrays of a tensor sit at the same offset from a 64 KiB
// boundary, a tile is not 1 KiB contiguous but two 512-byte halves 32 KiB apart
// inside one aligned 64 KiB block (lanes 0-31 take the first half, lanes 32-63
// the second; 64 consecutive workgroups cover the block).  Measured on MI355X
// with 36 streams this sustains 6.5-6.6 TB/s against 6.0 TB/s for contiguous
// 1 KiB tiles; no other address bit shows the effect, and a pair that straddles
// a 64 KiB boundary is slower than a contiguous tile.
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
// target of (resident wavefronts per CU) x (arrays a launch streams through)
#define ODSGD_INFLIGHT_MEMOPS_PER_CU 110
#endif

constexpr int kBlock = ODSGD_BLOCK;
constexpr int kTileElems = 4 * kBlock;  // one 128-bit access per lane

typedef float raw4 __attribute__((ext_vector_type(4)));  // what one 128-bit access moves
typedef unsigned int u4 __attribute__((ext_vector_type(4)));

// Four elements of one lane.  The arithmetic is written per component on a
// plain struct rather than on the compiler's vector type: a scalar operand
// (learning rate, momentum, ...) is then used straight from its one scalar
// register, where the vector type makes the compiler keep a four-register
// broadcast copy of every such scalar.
struct f4 {
    float x, y, z, w;
};
__device__ __forceinline__ f4 operator+(f4 a, f4 b) { return f4{a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w}; }
__device__ __forceinline__ f4 operator-(f4 a, f4 b) { return f4{a.x - b.x, a.y - b.y, a.z - b.z, a.w - b.w}; }
__device__ __forceinline__ f4 operator*(f4 a, f4 b) { return f4{a.x * b.x, a.y * b.y, a.z * b.z, a.w * b.w}; }
__device__ __forceinline__ f4 operator*(float s, f4 b) { return f4{s * b.x, s * b.y, s * b.z, s * b.w}; }
__device__ __forceinline__ f4 operator*(f4 a, float s) { return f4{a.x * s, a.y * s, a.z * s, a.w * s}; }
__device__ __forceinline__ f4 operator+(f4 a, float s) { return f4{a.x + s, a.y + s, a.z + s, a.w + s}; }
__device__ __forceinline__ f4 operator/(float s, f4 b) { return f4{s / b.x, s / b.y, s / b.z, s / b.w}; }

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
    MODE_COPY = 4,    // measurement aid: the memory accesses of MODE_OD without its arithmetic
    MODE_GLOBAL_STREAM = 5,  // MODE_GLOBAL with w and momentum loaded non-temporally (state larger than the cache)
};

__host__ __device__ constexpr bool is_global_only(int mode) { return mode == MODE_GLOBAL || mode == MODE_GLOBAL_STREAM; }

// Cache policy of the w / momentum loads.  Cacheable by default (see ODSGD_NT_STATE_LD).  The
// global-only update is the exception when the two arrays cannot stay in the last-level cache
// anyway: streaming them like the gradients is then 4-5 % faster (vgg16, alexnet at W = 16), while
// for the fused and local-only kernels the cacheable loads stay ahead at every size.
template <int MODE>
constexpr bool nt_state_load() { return ODSGD_NT_STATE_LD || MODE == MODE_GLOBAL_STREAM; }

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

// Pointer-table row: [w, mom, g_0.., u_0.., state_0.., w_alt, mom_alt]; the
// last two are the second buffer pair of the out-of-place global update.
__host__ __device__ constexpr int row_stride(int W) { return 4 + 3 * W; }
__host__ __device__ constexpr int col_grad(int W, int m) { return 2 + m; }
__host__ __device__ constexpr int col_local(int W, int m) { return 2 + W + m; }
__host__ __device__ constexpr int col_state(int W, int m) { return 2 + 2 * W + m; }
__host__ __device__ constexpr int col_alt(int W, int which) { return 2 + 3 * W + which; }

struct KernelArgs {
    const void *chunks;  // device: nchunks * 16 bytes
    const void *ptrs;    // device: rows of row_stride(wtot) pointers
    int nchunks;
    int wtot;    // workers registered
    int wfirst;  // first worker this launch touches
    int wcount;  // number of workers this launch touches (== W_T when W_T > 0)
    int col_w, col_v;          // columns the global weights / momentum are read from
    int col_w_out, col_v_out;  // ... and written to (the same two unless the update is out of place)
    float lr, local_lr, momentum, weight_decay, grad_scale;
    float lambda, ms_decay, one_minus_ms_decay, epsilon, local_momentum;
};

// chunk descriptor, 16 bytes:
//   x = pointer-table row | kVecFlag (128-bit accesses allowed)
//   y = element count
//   z = element offset inside the row (< 2^29 + 2^14, so the byte offset fits 32 bits)
//   w = for a two-half tile, what lanes 32..63 add to their 16-byte index to
//       reach the second half; 0 for a contiguous chunk
constexpr uint32_t kVecFlag = 0x80000000u;
constexpr int64_t kRowElems = (int64_t)1 << 29;  // elements per pointer-table row (2 GiB)

// ---------------------------------------------------------------------------
// memory access helpers
// ---------------------------------------------------------------------------
// `base` is a uniform 64-bit address (held in SGPRs), `boff` the lane's byte
// offset from it, 32 bits wide: together the "SGPR base + VGPR offset" form.
template <typename T>
struct access {
    typedef T type;
    static __device__ __forceinline__ T unpack(T x) { return x; }
    static __device__ __forceinline__ T pack(T x) { return x; }
};
template <>
struct access<f4> {
    typedef raw4 type;
    static __device__ __forceinline__ f4 unpack(raw4 x) { return f4{x.x, x.y, x.z, x.w}; }
    static __device__ __forceinline__ raw4 pack(f4 x) { return raw4{x.x, x.y, x.z, x.w}; }
};

template <bool NT, typename T>
__device__ __forceinline__ T load(uint64_t base, unsigned boff)
{
    typedef typename access<T>::type M;
    const gcptr<M> p = (gcptr<M>)((gcptr<char>)base + boff);
    if constexpr (NT)
        return access<T>::unpack(__builtin_nontemporal_load(p));
    else
        return access<T>::unpack(*p);
}

template <bool NT, typename T>
__device__ __forceinline__ void store(uint64_t base, unsigned boff, T x)
{
    typedef typename access<T>::type M;
    const gptr<M> p = (gptr<M>)((gptr<char>)base + boff);
    if constexpr (NT)
        __builtin_nontemporal_store(access<T>::pack(x), p);
    else
        *p = access<T>::pack(x);
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

// One worker's local update in MODE_OD / MODE_LOCAL, stores included.
template <int RULE, typename T>
__device__ __forceinline__ void local_one(T w0, T gm, T r, T u_old, T st_old, uint64_t pu, uint64_t pst,
                                          unsigned boff, const Hyp &h)
{
    T um;
    if constexpr (RULE == RULE_SGD) {
        um = update_local(w0, gm, r, h.local_lr);
    } else if constexpr (RULE == RULE_DCC) {
        T gg = gm * gm;
        um = update_local_dc(w0, gm, gg, u_old, r, h.lambda, h.local_lr);
    } else if constexpr (RULE == RULE_DCA) {
        T gg = gm * gm;
        T ms_new;
        T lam = mean_square_step(gg, st_old, h, ms_new);
        store<ODSGD_NT_LOCAL, T>(pst, boff, ms_new);
        um = update_local_dc(w0, gm, gg, u_old, r, lam, h.local_lr);
    } else {
        T lv1;
        um = update_local_momentum(w0, gm, r, st_old, h, lv1);
        store<ODSGD_NT_LOCAL, T>(pst, boff, lv1);
    }
    store<ODSGD_NT_LOCAL, T>(pu, boff, um);
}

// ---------------------------------------------------------------------------
// one full tile, fixed worker count W_T.
//
// Workers are taken in groups of G.  The loads of group j+1 are issued before
// the arithmetic and the stores of group j (the compiler cannot prove that
// outputs do not alias inputs, so it keeps this order), which bounds what is
// live at any time to two groups of operands and two groups of pointers instead
// of all W of them: without it the W = 16 variants need more scalar registers
// for pointers than exist, and the adaptive rule more than 230 vector registers.
// (Fencing the groups off from one another with scheduling barriers removes the
// few scalar spills the stateful rules keep at W >= 12, but was measured 1 %
// slower, so the scheduler is left free.)
// The gradient sum is accumulated as the groups go by, in ascending worker
// order: the same left-to-right sum a single loop over the workers gives.
// ---------------------------------------------------------------------------
template <int W_T, int MODE, int RULE>
constexpr int group_size()
{
    constexpr bool local_rule = (MODE == MODE_OD || MODE == MODE_LOCAL);
    if (local_rule && RULE != RULE_SGD)
        return W_T >= 8 ? 4 : W_T;  // 2 or 3 loads and 1 or 2 stores per worker
    return W_T > 12 ? 8 : W_T;      // 1 load and at most 1 store per worker
}

template <int W_T, int MODE, int RULE, typename T>
__device__ __forceinline__ void apply_fixed(ptr_table_t row, const KernelArgs &a, unsigned boff, const Hyp &h)
{
    constexpr bool need_v = (MODE != MODE_LOCAL);
    constexpr bool local_rule = (MODE == MODE_OD || MODE == MODE_LOCAL);
    constexpr bool need_u_old = local_rule && (RULE == RULE_DCC || RULE == RULE_DCA);
    constexpr bool need_state = local_rule && (RULE == RULE_DCA || RULE == RULE_MOM);  // per-worker state
    constexpr int G = group_size<W_T, MODE, RULE>();
    constexpr int NG = (W_T + G - 1) / G;  // the last group may be short

    const ptr_table_t pg = row + col_grad(a.wtot, a.wfirst);
    const ptr_table_t pu = row + col_local(a.wtot, a.wfirst);
    const ptr_table_t ps = row + col_state(a.wtot, a.wfirst);

    T w0, v0, g[2][G], u_old[2][G], st_old[2][G];
    w0 = load<nt_state_load<MODE>(), T>(row[a.col_w], boff);
    if constexpr (need_v)
        v0 = load<nt_state_load<MODE>(), T>(row[a.col_v], boff);

    auto issue_loads = [&](int grp, int buf) {
#pragma unroll
        for (int j = 0; j < G; ++j)
            if (grp * G + j < W_T)
                g[buf][j] = load<ODSGD_NT_GRAD, T>(pg[grp * G + j], boff);
        if constexpr (need_u_old) {
#pragma unroll
            for (int j = 0; j < G; ++j)
                if (grp * G + j < W_T)
                    u_old[buf][j] = load<ODSGD_NT_INPLACE_LD, T>(pu[grp * G + j], boff);
        }
        if constexpr (need_state) {
#pragma unroll
            for (int j = 0; j < G; ++j)
                if (grp * G + j < W_T)
                    st_old[buf][j] = load<ODSGD_NT_INPLACE_LD, T>(ps[grp * G + j], boff);
        }
    };

    issue_loads(0, 0);
    const T r = h.weight_decay * w0;
    T s = w0;  // overwritten by the first gradient below
#pragma unroll
    for (int grp = 0; grp < NG; ++grp) {
        const int buf = grp & 1;
        if (grp + 1 < NG)
            issue_loads(grp + 1, buf ^ 1);
#pragma unroll
        for (int j = 0; j < G; ++j) {
            if (grp * G + j >= W_T)
                break;
            const T gm = g[buf][j];
            if constexpr (MODE != MODE_LOCAL)
                s = (grp == 0 && j == 0) ? gm : s + gm;
            if constexpr (local_rule) {
                T uo = gm, so = gm;
                uint64_t pst = 0;
                if constexpr (need_u_old)
                    uo = u_old[buf][j];
                if constexpr (need_state) {
                    so = st_old[buf][j];
                    pst = ps[grp * G + j];
                }
                local_one<RULE, T>(w0, gm, r, uo, so, pu[grp * G + j], pst, boff, h);
            } else if constexpr (MODE == MODE_COPY) {
                store<ODSGD_NT_LOCAL, T>(pu[grp * G + j], boff, gm);
            }
        }
    }
    if constexpr (MODE == MODE_COPY) {
        store<ODSGD_NT_STATE_ST, T>(row[a.col_v_out], boff, v0);
        store<ODSGD_NT_STATE_ST, T>(row[a.col_w_out], boff, w0);
    } else if constexpr (MODE != MODE_LOCAL) {
        T w1, v1;
        update_global(w0, v0, s, r, h, w1, v1);
        if constexpr (MODE == MODE_SSGD) {
#pragma unroll
            for (int m = 0; m < W_T; ++m)
                store<ODSGD_NT_LOCAL, T>(pu[m], boff, w1);
        }
        store<ODSGD_NT_STATE_ST, T>(row[a.col_v_out], boff, v1);
        store<ODSGD_NT_STATE_ST, T>(row[a.col_w_out], boff, w1);
    }
}

// any worker count, any chunk length: pointers are fetched from the table inside the worker loop
template <int MODE, int RULE, typename T>
__device__ __forceinline__ void apply_generic(ptr_table_t row, const KernelArgs &a, unsigned boff, const Hyp &h)
{
    constexpr bool local_rule = (MODE == MODE_OD || MODE == MODE_LOCAL);
    constexpr bool need_u_old = local_rule && (RULE == RULE_DCC || RULE == RULE_DCA);
    constexpr bool need_state = local_rule && (RULE == RULE_DCA || RULE == RULE_MOM);
    const ptr_table_t pg = row + col_grad(a.wtot, a.wfirst);
    const ptr_table_t pu = row + col_local(a.wtot, a.wfirst);
    const ptr_table_t ps = row + col_state(a.wtot, a.wfirst);
    T w0 = load<nt_state_load<MODE>(), T>(row[a.col_w], boff);
    T r = h.weight_decay * w0;
    T s = w0;
    for (int m = 0; m < a.wcount; ++m) {
        T gm = load<ODSGD_NT_GRAD, T>(pg[m], boff);
        s = (m == 0) ? gm : s + gm;
        if constexpr (local_rule) {
            T uo = gm, so = gm;
            uint64_t pst = 0;
            if constexpr (need_u_old)
                uo = load<ODSGD_NT_INPLACE_LD, T>(pu[m], boff);
            if constexpr (need_state) {
                pst = ps[m];
                so = load<ODSGD_NT_INPLACE_LD, T>(pst, boff);
            }
            local_one<RULE, T>(w0, gm, r, uo, so, pu[m], pst, boff, h);
        } else if constexpr (MODE == MODE_COPY) {
            store<ODSGD_NT_LOCAL, T>(pu[m], boff, gm);
        }
    }
    if constexpr (MODE != MODE_LOCAL) {
        T v0 = load<nt_state_load<MODE>(), T>(row[a.col_v], boff);
        T w1 = w0, v1 = v0;
        if constexpr (MODE != MODE_COPY)
            update_global(w0, v0, s, r, h, w1, v1);
        if constexpr (MODE == MODE_SSGD) {
            for (int m = 0; m < a.wcount; ++m)
                store<ODSGD_NT_LOCAL, T>(pu[m], boff, w1);
        }
        store<ODSGD_NT_STATE_ST, T>(row[a.col_v_out], boff, v1);
        store<ODSGD_NT_STATE_ST, T>(row[a.col_w_out], boff, w1);
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
    const int stride = row_stride(a.wtot);

    // Workgroup b takes chunk b (the host never launches more workgroups than
    // chunks, so the first trip needs no bounds check and the descriptor fetch can
    // be issued together with the kernel arguments).  The dispatcher hands
    // consecutive workgroups to the 8 XCDs in turn, so at any moment the chip works
    // on one narrow, sliding window of each array; giving every XCD a contiguous
    // range of its own instead was measured 15 % slower.
    unsigned c = blockIdx.x;
    do {
        const u4 d = chunks[c];
        const uint32_t rowi = d.x & ~kVecFlag;
        const bool vec = (d.x & kVecFlag) != 0;
        const unsigned count = d.y;
        const unsigned base_off = d.z * (unsigned)sizeof(float);
        const unsigned second_half = d.w;
        const ptr_table_t row = ptrs + (uint64_t)rowi * stride;

        const unsigned nvec = vec ? (count >> 2) : 0u;
        if constexpr (W_T > 0) {
            // straight-line: one 128-bit access per lane per array (a chunk never
            // exceeds one tile; lanes beyond a short chunk sit this out), then the
            // up to three elements that do not fill a 128-bit access -- or, where an
            // array is only 4-byte aligned, the whole chunk -- one element per lane
            if (tid < nvec) {
                const unsigned idx = tid + (tid >> 5) * second_half;
                apply_fixed<W_T, MODE, RULE, f4>(row, a, base_off + idx * 16u, h);
            }
            for (unsigned t = nvec * 4 + tid; t < count; t += kBlock)
                apply_generic<MODE, RULE, float>(row, a, base_off + t * 4u, h);
        } else {
            if (tid < nvec)
                apply_generic<MODE, RULE, f4>(row, a, base_off + (tid + (tid >> 5) * second_half) * 16u, h);
            for (unsigned t = nvec * 4 + tid; t < count; t += kBlock)
                apply_generic<MODE, RULE, float>(row, a, base_off + t * 4u, h);
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
        const f4 x = load<true, f4>(src + tile * (kBlock * 16u), threadIdx.x * 16u);
        store<true, f4>(dst + tile * (kBlock * 16u), threadIdx.x * 16u, x);
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
thread_local hipError_t g_last_hip_error = hipSuccess;

struct Tuning {
    int blocks_per_cu;    // grid cap = blocks_per_cu * CUs; 0 = one workgroup per chunk
    int waves_per_cu;     // resident wavefronts per CU: 0 = choose per launch, < 0 = no cap
    int pair_bit;         // address bit that separates the two halves of a tile; 0 = contiguous tiles only
    int64_t llc_bytes;    // last-level cache: w + momentum beyond this size are streamed by the global-only update
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
    t.blocks_per_cu = (int)env_int("ODSGD_BLOCKS_PER_CU", 0);
    if (t.blocks_per_cu < 0)
        t.blocks_per_cu = 0;
    t.waves_per_cu = (int)env_int("ODSGD_WAVES_PER_CU", 0);
    t.pair_bit = (int)env_int("ODSGD_PAIR_BIT", 15);
    if (t.pair_bit != 0 && (t.pair_bit < 10 || t.pair_bit > 20))
        t.pair_bit = 0;
    t.llc_bytes = env_int("ODSGD_LLC_BYTES", (int64_t)256 << 20);  // MI355X: 256 MB Infinity Cache
    return t;
}

constexpr int64_t kMaxNumel = (int64_t)1 << 40;
// Tiles whose addresses start on a 512-byte boundary stream measurably faster
// (5-6 % on MI355X) than tiles that straddle one; 1 KiB = one full tile.
constexpr uintptr_t kTileAlignBytes = 1024;
constexpr int64_t kMaxChunks = 0x7ffffffe;

int64_t rows_of(int64_t numel) { return numel <= kRowElems ? 1 : (numel + kRowElems - 1) / kRowElems; }

// Upper bounds on pointer-table rows and chunks for this tensor list (what the
// workspace is sized for; they depend on the element counts only, not on any
// address), or false on invalid input / overflow.  A row gets at most two
// ragged chunks besides its full ones: a short head that brings the following
// chunk starts onto a tile boundary, and a tail.
bool count_tables(int num_tensors, const int64_t *numel, int64_t *rows, int64_t *chunks, int *err)
{
    int64_t r = 0, n = 0;
    for (int k = 0; k < num_tensors; ++k) {
        if (numel[k] < 0) {
            *err = ODSGD_EINVAL;
            return false;
        }
        if (numel[k] >= kMaxNumel) {
            *err = ODSGD_ERANGE;
            return false;
        }
        const int64_t rk = rows_of(numel[k]);
        r += rk;
        n += (numel[k] + kTileElems - 1) / kTileElems + (numel[k] > 0 ? 2 * rk : 0);
        if (n > kMaxChunks) {
            *err = ODSGD_ERANGE;
            return false;
        }
    }
    *rows = r;
    *chunks = n;
    return true;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

size_t ptr_table_bytes(int64_t rows, int num_workers)
{
    return align_up((size_t)rows * (size_t)row_stride(num_workers) * sizeof(uint64_t), 256);
}

struct Range {
    uintptr_t lo, hi;
    bool is_output;
};

// true if any output range overlaps any other range
bool ranges_alias(std::vector<Range> r)
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

// What a handle has registered: per tensor the addresses of every array, in
// pointer-table column order (0 = not registered).
struct Registration {
    int num_tensors = 0;
    int num_workers = 0;
    std::vector<int64_t> numel;
    std::vector<uint64_t> cols;  // [K][row_stride(W)]
    uint64_t &at(int k, int col) { return cols[(size_t)k * row_stride(num_workers) + col]; }
    uint64_t at(int k, int col) const { return cols[(size_t)k * row_stride(num_workers) + col]; }
};

// The launch plan: host image of the two tables, built without touching a device.
struct Plan {
    std::vector<unsigned char> image;  // [pointer table | chunk table], sized for the upper bounds
    size_t ptr_bytes = 0;              // offset of the chunk table inside image
    int64_t nrows = 0;
    int64_t nchunks = 0;  // chunks actually emitted
};

// Validate the arguments of a registration and collect them.  Pointer checks:
// non-null and 4-byte aligned where the tensor is not empty.
int collect_registration(Registration &reg, std::vector<Range> &ranges, int num_tensors, const int64_t *numel,
                         float *const *w, float *const *mom, const float *const *const *grads,
                         float *const *const *local_w, int num_workers)
{
    if (num_tensors < 1 || !numel || !w || !mom || !grads || !local_w || num_workers < 1 ||
        num_workers > ODSGD_MAX_WORKERS)
        return ODSGD_EINVAL;
    for (int m = 0; m < num_workers; ++m)
        if (!grads[m] || !local_w[m])
            return ODSGD_EINVAL;
    const int W = num_workers;
    int err = 0;
    int64_t rows = 0, chunks = 0;
    if (!count_tables(num_tensors, numel, &rows, &chunks, &err))
        return err;
    reg.num_tensors = num_tensors;
    reg.num_workers = W;
    reg.numel.assign(numel, numel + num_tensors);
    reg.cols.assign((size_t)num_tensors * row_stride(W), 0);
    ranges.clear();
    ranges.reserve((size_t)num_tensors * (2 + 2 * W) + 1);
    for (int k = 0; k < num_tensors; ++k) {
        if (numel[k] == 0)
            continue;
        const size_t bytes = (size_t)numel[k] * sizeof(float);
        for (int j = 0; j < 2 + 2 * W; ++j) {
            const void *p = j == 0   ? (const void *)w[k]
                            : j == 1 ? (const void *)mom[k]
                            : j < 2 + W ? (const void *)grads[j - 2][k]
                                        : (const void *)local_w[j - 2 - W][k];
            if (!p)
                return ODSGD_EINVAL;
            const uintptr_t a = (uintptr_t)p;
            if (a % 4 != 0)
                return ODSGD_EALIGN;
            const bool is_output = (j < 2) || (j >= 2 + W);
            ranges.push_back(Range{a, a + bytes, is_output});
            reg.at(k, j) = (uint64_t)a;
        }
    }
    return ODSGD_OK;
}

// Build the table image for a registration.
//
// Per tensor: `vec` = every registered array is 16-byte aligned (128-bit
// accesses); the arrays' common offset from a 1 KiB boundary, if they have one,
// decides where contiguous chunks start; their common offset from a
// 2^(pair_bit+1) boundary, if they have one, allows two-half tiles inside the
// aligned blocks of that size.
int make_plan(Plan &plan, const Registration &reg, const Tuning &tuning)
{
    const int K = reg.num_tensors, W = reg.num_workers, stride = row_stride(W);
    int err = 0;
    int64_t max_rows = 0, max_chunks = 0;
    if (!count_tables(K, reg.numel.data(), &max_rows, &max_chunks, &err))
        return err;
    plan.ptr_bytes = ptr_table_bytes(max_rows, W);
    const size_t chunk_bytes = align_up((size_t)std::max<int64_t>(max_chunks, 1) * 16, 256);
    plan.image.assign(plan.ptr_bytes + chunk_bytes, 0);
    uint64_t *pt = reinterpret_cast<uint64_t *>(plan.image.data());
    uint32_t *ct = reinterpret_cast<uint32_t *>(plan.image.data() + plan.ptr_bytes);

    const int64_t C = kTileElems;
    const bool pairing = tuning.pair_bit > 0;
    const uintptr_t half_bytes = pairing ? ((uintptr_t)1 << tuning.pair_bit) : 0;  // distance between the halves
    const uintptr_t block_bytes = pairing ? 2 * half_bytes : 1;
    const int64_t block_elems = (int64_t)(block_bytes / sizeof(float));
    const int64_t half_tile = kTileElems / 2;
    const uint32_t second_half = pairing ? (uint32_t)(half_bytes / 16 - kBlock / 2) : 0;

    int64_t c = 0, r = 0;
    auto emit = [&](int64_t row, bool vec, int64_t off, int64_t cnt, uint32_t second) {
        if (c >= max_chunks) {  // never taken (see count_tables); keeps a counting mistake from becoming an overrun
            ++c;
            return;
        }
        uint32_t *dsc = ct + c * 4;
        dsc[0] = (uint32_t)row | (vec ? kVecFlag : 0u);
        dsc[1] = (uint32_t)cnt;
        dsc[2] = (uint32_t)off;
        dsc[3] = second;
        ++c;
    };
    // chunk table: full chunks of all rows first, ragged ones (heads and tails)
    // after them, so the short pieces fill the end of the launch
    for (int pass = 0; pass < 2; ++pass) {
        r = 0;
        for (int k = 0; k < K; ++k) {
            const int64_t n = reg.numel[k];
            bool vec = true, same_tile_phase = true, same_block_phase = pairing;
            uintptr_t first = 0;
            for (int j = 0; j < stride; ++j) {
                const uintptr_t a = (uintptr_t)reg.at(k, j);
                if (!a)
                    continue;
                if (!first)
                    first = a;
                if (a % 16 != 0)
                    vec = false;
                if (a % kTileAlignBytes != first % kTileAlignBytes)
                    same_tile_phase = false;
                if (pairing && a % block_bytes != first % block_bytes)
                    same_block_phase = false;
            }
            const int64_t nrows = rows_of(n);
            for (int64_t seg = 0; seg < nrows; ++seg, ++r) {
                const int64_t seg_off = seg * kRowElems;
                const int64_t len = std::min(kRowElems, n - seg_off);
                if (pass == 0) {
                    for (int j = 0; j < stride; ++j)
                        if (reg.at(k, j))
                            pt[(size_t)r * stride + j] = reg.at(k, j) + (uint64_t)seg_off * sizeof(float);
                }
                if (len <= 0)
                    continue;
                const uintptr_t start = first + (uintptr_t)seg_off * sizeof(float);
                // [0, pre) contiguous, [pre, post) two-half tiles, [post, len) contiguous
                int64_t pre = len, blocks = 0;
                if (vec && same_block_phase) {
                    const int64_t to_block =
                        (int64_t)((block_bytes - start % block_bytes) % block_bytes / sizeof(float));
                    if (to_block < len && (len - to_block) / block_elems > 0) {
                        pre = to_block;
                        blocks = (len - to_block) / block_elems;
                    }
                }
                const int64_t post = pre + blocks * block_elems;
                // contiguous region [lo, hi): a head up to the first tile boundary when
                // all arrays share their offset from one, full chunks, a tail
                auto contiguous = [&](int64_t lo, int64_t hi) {
                    if (lo >= hi)
                        return;
                    int64_t head = 0;
                    if (vec && same_tile_phase) {
                        const uintptr_t at = start + (uintptr_t)lo * sizeof(float);
                        const int64_t h0 =
                            (int64_t)((kTileAlignBytes - at % kTileAlignBytes) % kTileAlignBytes / sizeof(float));
                        if (h0 < hi - lo)
                            head = h0;
                    }
                    const int64_t body = hi - lo - head;
                    const int64_t nfull = body / C;
                    if (pass == 0) {
                        for (int64_t j = 0; j < nfull; ++j)
                            emit(r, vec, lo + head + j * C, C, 0);
                    } else {
                        if (head > 0)
                            emit(r, vec, lo, head, 0);
                        if (body > nfull * C)
                            emit(r, vec, lo + head + nfull * C, body - nfull * C, 0);
                    }
                };
                contiguous(0, pre);
                if (pass == 0) {
                    for (int64_t b = 0; b < blocks; ++b)
                        for (int64_t s = 0; s < block_elems / kTileElems; ++s)
                            emit(r, true, pre + b * block_elems + s * half_tile, kTileElems, second_half);
                }
                if (blocks > 0)
                    contiguous(post, len);
            }
        }
    }
    plan.nrows = r;
    plan.nchunks = c;
    if (c > max_chunks || r > max_rows)
        return ODSGD_ERANGE;  // cannot happen: the bounds above cover every case
    return ODSGD_OK;
}

using KernelFn = void (*)(KernelArgs);

template <int MODE, int RULE>
KernelFn pick_by_workers(int wcount)
{
    switch (wcount) {
    case 1: return odsgd_kernel<1, MODE, RULE>;
    case 2: return odsgd_kernel<2, MODE, RULE>;
    case 3: return odsgd_kernel<3, MODE, RULE>;
    case 4: return odsgd_kernel<4, MODE, RULE>;
    case 5: return odsgd_kernel<5, MODE, RULE>;
    case 6: return odsgd_kernel<6, MODE, RULE>;
    case 7: return odsgd_kernel<7, MODE, RULE>;
    case 8: return odsgd_kernel<8, MODE, RULE>;
    case 9: return odsgd_kernel<9, MODE, RULE>;
    case 10: return odsgd_kernel<10, MODE, RULE>;
    case 11: return odsgd_kernel<11, MODE, RULE>;
    case 12: return odsgd_kernel<12, MODE, RULE>;
    case 13: return odsgd_kernel<13, MODE, RULE>;
    case 14: return odsgd_kernel<14, MODE, RULE>;
    case 15: return odsgd_kernel<15, MODE, RULE>;
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
    case MODE_COPY: return pick_by_workers<MODE_COPY, RULE_SGD>(wcount);
    case MODE_GLOBAL_STREAM: return pick_by_workers<MODE_GLOBAL_STREAM, RULE_SGD>(wcount);
    default: return pick_by_workers<MODE_GLOBAL, RULE_SGD>(wcount);
    }
}

// ---------------------------------------------------------------------------
// residency: how many one-wavefront workgroups a CU should hold, and the dynamic
// LDS request that makes it so
// ---------------------------------------------------------------------------
constexpr int kMaxUnrolledWorkers = 16;  // odsgd_kernel<W_T, ...> exists for W_T = 1..16; more workers take W_T = 0

// distinct arrays a launch streams through (an array updated in place counts once)
int arrays_per_tile(int mode, int rule, int wcount)
{
    int arrays = 1 + wcount;  // w and the gradients
    if (mode != MODE_LOCAL)
        ++arrays;  // momentum
    if (!is_global_only(mode))
        arrays += wcount;  // local weights
    if ((mode == MODE_OD || mode == MODE_LOCAL) && (rule == RULE_DCA || rule == RULE_MOM))
        arrays += wcount;  // per-worker state
    return arrays;
}

// Resident wavefronts per CU wanted for a launch; 0 = no cap (full occupancy).
// Measured on MI355X for every entry point and rule at W = 8 and W = 16: the
// best residency is the one that keeps (wavefronts per CU) x (arrays) near
// ODSGD_INFLIGHT_MEMOPS_PER_CU, i.e. the chip-wide window of open 1 KiB tiles
// about constant -- 3 wavefronts for the 34 arrays of the fused step at W = 16,
// 6 for the 18 arrays at W = 8.
int wanted_waves(int mode, int rule, int wcount, int override_waves)
{
    if (override_waves < 0)
        return 0;
    int waves = override_waves;
    if (waves == 0) {
        // beyond the unrolled worker counts the kernel walks the workers one after the other,
        // one memory latency each: that loop needs every wavefront it can get (W = 32 on the
        // ResNet-50-shaped set: 0.82 of peak unlimited, 0.23 at two wavefronts per CU)
        if (wcount > kMaxUnrolledWorkers)
            return 0;
        const int arrays = arrays_per_tile(mode, rule, wcount);
        waves = (ODSGD_INFLIGHT_MEMOPS_PER_CU + arrays / 2) / arrays;  // nearest integer
        // the adaptive rule spends a correctly rounded sqrt and divide per element and
        // worker: at least one wavefront per SIMD and one more to hide that arithmetic
        if ((mode == MODE_OD || mode == MODE_LOCAL) && rule == RULE_DCA)
            waves = std::max(5, waves);
        if (waves > 16)
            return 0;  // few streams: full occupancy is best
    }
    return std::max(waves, 2);
}

// Smallest dynamic-LDS request (multiple of 256 bytes, at most max_request) for
// which `occupancy(bytes)` -- workgroups a CU accepts with that request, a
// non-increasing function -- is at most `waves`.  Returns the request and what
// it achieves; 0 and 0 if no request within the limit gets there.
template <typename Occupancy>
void lds_request_for(int waves, size_t max_request, Occupancy occupancy, size_t *bytes, int *achieved)
{
    *bytes = 0;
    *achieved = 0;
    const size_t step = 256;
    size_t lo = 0, hi = max_request / step;  // invariant: occupancy(lo*step) > waves (or lo == 0)
    if (hi == 0 || occupancy(hi * step) > waves)
        return;
    while (hi - lo > 1) {
        const size_t mid = (lo + hi) / 2;
        if (occupancy(mid * step) > waves)
            lo = mid;
        else
            hi = mid;
    }
    *bytes = hi * step;
    *achieved = occupancy(hi * step);
}

// A request is used if it lands on the wanted count or, where the allocation
// granularity steps over it, one below (never below two); otherwise the launch
// goes without a request rather than with a residency nobody asked for.
bool residency_acceptable(int wanted, int achieved)
{
    return achieved <= wanted && achieved >= std::max(2, wanted - 1);
}

}  // namespace

struct odsgd_handle {
    Registration reg;
    int64_t nchunks;
    void *workspace;
    size_t workspace_bytes;
    const void *d_chunks;
    const void *d_ptrs;
    int device;
    int num_cus;
    int lds_per_cu;
    int max_lds_request;
    Tuning tuning;
    int64_t iteration;
    int64_t warmup_steps;
    odsgd_local_rule rule;               // local updater of MODE_OD / MODE_LOCAL
    bool has_alt;                        // a second (w, mom) buffer pair is registered
    int current;                         // which pair holds the current weights: 0 = w/mom, 1 = the second pair
    std::vector<Range> base_ranges;      // what odsgd_init registered (incl. the table memory)
    std::vector<Range> state_ranges;     // per-worker state of the rule in force
    std::vector<Range> alt_ranges;       // the second buffer pair
    bool static_plan;                    // tables live in the per-device static array
    uint64_t static_generation;          // which registration of that array this handle is
    struct CapEntry {
        KernelFn fn;
        int waves;
        size_t lds;
        int achieved;
    };
    std::vector<CapEntry> caps;          // residency requests already worked out
};

namespace {

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

// Rebuild the tables from the handle's registration and upload them.  The whole
// image is uploaded, zero padding and unregistered (null) columns included, so
// nothing a kernel reads is left over from an earlier use of the same memory.
int upload_plan(odsgd_handle *h, void *stream)
{
    Plan plan;
    int rc = make_plan(plan, h->reg, h->tuning);
    if (rc != ODSGD_OK)
        return rc;
    if (plan.image.size() > h->workspace_bytes)
        return ODSGD_ENOSPC;
    hipError_t e = hipMemcpyAsync(h->workspace, plan.image.data(), plan.image.size(), hipMemcpyHostToDevice,
                                  (hipStream_t)stream);
    if (e == hipSuccess)
        e = hipStreamSynchronize((hipStream_t)stream);  // plan.image must outlive the copy
    if (e != hipSuccess) {
        g_last_hip_error = e;
        return ODSGD_EHIP;
    }
    h->nchunks = plan.nchunks;
    h->d_ptrs = h->workspace;
    h->d_chunks = (const unsigned char *)h->workspace + plan.ptr_bytes;
    return ODSGD_OK;
}

// Dynamic LDS to request so that a CU holds the wanted number of one-wavefront
// workgroups of kernel `fn`.  The kernels never touch LDS; the request only
// limits residency.  The size is found by asking the runtime how many
// workgroups a CU accepts for a given request; if the wanted count cannot be
// reached (see residency_acceptable) the launch goes uncapped.
size_t residency_lds_bytes(odsgd_handle *h, KernelFn fn, int mode, int wcount)
{
    const int waves = wanted_waves(mode, h->rule.rule, wcount, h->tuning.waves_per_cu);
    if (waves == 0)
        return 0;
    for (const auto &e : h->caps)
        if (e.fn == fn && e.waves == waves)
            return residency_acceptable(waves, e.achieved) ? e.lds : 0;
    auto occupancy = [&](size_t bytes) {
        int blocks = 0;
        hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, (const void *)fn, kBlock, bytes);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return 1 << 30;  // unknown: treated as "not capped"
        }
        return blocks;
    };
    odsgd_handle::CapEntry entry{fn, waves, 0, 0};
    lds_request_for(waves, (size_t)h->max_lds_request, occupancy, &entry.lds, &entry.achieved);
    h->caps.push_back(entry);
    return residency_acceptable(waves, entry.achieved) ? entry.lds : 0;
}

// Which global-only kernel a handle uses: w and momentum that cannot stay in the
// last-level cache from one step to the next anyway are streamed.
int global_only_mode(const odsgd_handle *h)
{
    int64_t n = 0;
    for (int64_t x : h->reg.numel)
        n += x;
    return 2 * n * (int64_t)sizeof(float) > h->tuning.llc_bytes ? MODE_GLOBAL_STREAM : MODE_GLOBAL;
}

// Work out the residency requests of every entry point for the rule in force,
// so that no launch has to query the runtime (a launch may be under stream capture).
void warm_residency(odsgd_handle *h)
{
    const int W = h->reg.num_workers;
    const int rule = h->rule.rule;
    (void)residency_lds_bytes(h, pick_kernel(MODE_OD, rule, W), MODE_OD, W);
    (void)residency_lds_bytes(h, pick_kernel(MODE_LOCAL, rule, W), MODE_LOCAL, W);
    (void)residency_lds_bytes(h, pick_kernel(MODE_LOCAL, rule, 1), MODE_LOCAL, 1);
    (void)residency_lds_bytes(h, pick_kernel(MODE_SSGD, rule, W), MODE_SSGD, W);
    const int gmode = global_only_mode(h);
    (void)residency_lds_bytes(h, pick_kernel(gmode, rule, W), gmode, W);
}

int launch(odsgd_handle *h, int mode, int wfirst, int wcount, bool out_of_place, const odsgd_hyper *hy, void *stream)
{
    if (handle_is_stale(h))
        return ODSGD_ESTALE;
    if (h->nchunks == 0)
        return ODSGD_OK;
    const int W = h->reg.num_workers;
    KernelArgs a;
    a.chunks = h->d_chunks;
    a.ptrs = h->d_ptrs;
    a.nchunks = (int)h->nchunks;
    a.wtot = W;
    a.wfirst = wfirst;
    a.wcount = wcount;
    a.col_w = h->current ? col_alt(W, 0) : 0;
    a.col_v = h->current ? col_alt(W, 1) : 1;
    a.col_w_out = a.col_w;
    a.col_v_out = a.col_v;
    if (out_of_place) {
        a.col_w_out = h->current ? 0 : col_alt(W, 0);
        a.col_v_out = h->current ? 1 : col_alt(W, 1);
    }
    a.lr = hy->lr;
    a.local_lr = hy->local_lr;
    a.momentum = hy->momentum;
    a.weight_decay = hy->weight_decay;
    a.grad_scale = (hy->grad_scale <= 0.0f) ? 1.0f / (float)W : hy->grad_scale;
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
    const size_t lds = residency_lds_bytes(h, fn, mode, wcount);
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
    Registration reg;
    std::vector<Range> ranges;
    int rc = collect_registration(reg, ranges, num_tensors, numel, w, mom, grads, local_w, num_workers);
    if (rc != ODSGD_OK)
        return rc;
    const Tuning tuning = current_tuning();
    int64_t rows = 0, chunks = 0;
    if (!count_tables(num_tensors, numel, &rows, &chunks, &rc))
        return rc;
    const size_t need = ptr_table_bytes(rows, num_workers) + align_up((size_t)std::max<int64_t>(chunks, 1) * 16, 256);
    if (!static_plan && (uintptr_t)workspace % 256 != 0)
        return ODSGD_EALIGN;
    if (workspace_bytes < need)
        return ODSGD_ENOSPC;

    if (static_plan) {
        // the caller's buffers cannot overlap the library's own array, but they may
        // not overlap each other either
        if (ranges_alias(ranges))
            return ODSGD_EALIAS;
        int device = 0;
        hipError_t e = hipGetDevice(&device);
        if (e != hipSuccess) {
            g_last_hip_error = e;
            return ODSGD_EHIP;
        }
        rc = static_plan_address(device, &workspace);
        if (rc != ODSGD_OK)
            return rc;
    }
    ranges.push_back(Range{(uintptr_t)workspace, (uintptr_t)workspace + need, true});
    if (ranges_alias(ranges))
        return ODSGD_EALIAS;

    odsgd_handle *h = new (std::nothrow) odsgd_handle();
    if (!h)
        return ODSGD_EINVAL;
    h->reg = std::move(reg);
    h->nchunks = 0;
    h->workspace = workspace;
    h->workspace_bytes = workspace_bytes;
    h->d_chunks = nullptr;
    h->d_ptrs = nullptr;
    h->tuning = tuning;
    h->iteration = 0;
    h->warmup_steps = 0;
    h->rule = odsgd_local_rule{ODSGD_LOCAL_SGD, 0.0f, 0.0f, 0.0f, 0.0f};
    h->has_alt = false;
    h->current = 0;
    h->base_ranges = std::move(ranges);
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
    if (e == hipSuccess) {
        int lds = 0;
        e = hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, h->device);
        h->max_lds_request = lds > 0 ? lds : 64 * 1024;
    }
    if (e != hipSuccess) {
        g_last_hip_error = e;
        delete h;
        return ODSGD_EHIP;
    }
    if (static_plan) {
        // from here on the array holds this registration: handles of earlier ones are stale
        std::lock_guard<std::mutex> lock(g_static_mutex);
        h->static_generation = ++g_static_generation[h->device];
    }
    rc = upload_plan(h, stream);
    if (rc != ODSGD_OK) {
        delete h;
        return rc;
    }
    warm_residency(h);
    *out = h;
    return ODSGD_OK;
}

// Register, replace or drop extra arrays (per-worker state, the second buffer
// pair) in columns [col0, col0 + ncols) of every tensor's row, then rebuild and
// upload the tables: how a tensor is tiled depends on the alignment of all its arrays.
int register_columns(odsgd_handle *h, int col0, int ncols, const uintptr_t *addr /* [ncols][K] */,
                     std::vector<Range> &own_ranges, const std::vector<Range> &other_ranges, void *stream)
{
    const int K = h->reg.num_tensors;
    std::vector<Range> fresh;
    Registration reg = h->reg;
    for (int j = 0; j < ncols; ++j) {
        for (int k = 0; k < K; ++k) {
            reg.at(k, col0 + j) = 0;
            if (reg.numel[k] == 0)
                continue;
            const uintptr_t a = addr[(size_t)j * K + k];
            if (!a)
                return ODSGD_EINVAL;
            if (a % 4 != 0)
                return ODSGD_EALIGN;
            fresh.push_back(Range{a, a + (size_t)reg.numel[k] * sizeof(float), true});
            reg.at(k, col0 + j) = (uint64_t)a;
        }
    }
    std::vector<Range> all = h->base_ranges;
    all.insert(all.end(), other_ranges.begin(), other_ranges.end());
    all.insert(all.end(), fresh.begin(), fresh.end());
    if (ranges_alias(all))
        return ODSGD_EALIAS;
    Registration old = std::move(h->reg);
    h->reg = std::move(reg);
    int rc = upload_plan(h, stream);
    if (rc != ODSGD_OK) {
        h->reg = std::move(old);
        return rc;
    }
    own_ranges = std::move(fresh);
    return ODSGD_OK;
}

}  // namespace

extern "C" {

size_t odsgd_workspace_bytes(int num_tensors, const int64_t *numel, int num_workers)
{
    if (num_tensors < 1 || !numel || num_workers < 1 || num_workers > ODSGD_MAX_WORKERS)
        return 0;
    int err = 0;
    int64_t rows = 0, chunks = 0;
    if (!count_tables(num_tensors, numel, &rows, &chunks, &err))
        return 0;
    return ptr_table_bytes(rows, num_workers) + align_up((size_t)std::max<int64_t>(chunks, 1) * 16, 256);
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
                    void *image, size_t image_bytes, int64_t *num_rows, int64_t *num_chunks,
                    size_t *chunk_table_offset)
{
    if (!image || !num_rows || !num_chunks || !chunk_table_offset)
        return ODSGD_EINVAL;
    Registration reg;
    std::vector<Range> ranges;
    int rc = collect_registration(reg, ranges, num_tensors, numel, w, mom, grads, local_w, num_workers);
    if (rc != ODSGD_OK)
        return rc;
    if (ranges_alias(ranges))
        return ODSGD_EALIAS;
    Plan plan;
    rc = make_plan(plan, reg, current_tuning());
    if (rc != ODSGD_OK)
        return rc;
    if (image_bytes < plan.image.size())
        return ODSGD_ENOSPC;
    std::memcpy(image, plan.image.data(), plan.image.size());
    *num_rows = plan.nrows;
    *num_chunks = plan.nchunks;
    *chunk_table_offset = plan.ptr_bytes;
    return ODSGD_OK;
}

int odsgd_plan_residency(int entry, int rule, int num_workers, int waves_override, size_t lds_per_cu,
                         size_t lds_granule, size_t max_request, int *waves_wanted, size_t *lds_bytes,
                         int *waves_achieved)
{
    if (!waves_wanted || !lds_bytes || !waves_achieved || num_workers < 1 || num_workers > ODSGD_MAX_WORKERS ||
        lds_granule == 0 || lds_per_cu == 0)
        return ODSGD_EINVAL;
    int mode;
    switch (entry) {
    case ODSGD_ENTRY_STEP: mode = MODE_OD; break;
    case ODSGD_ENTRY_SSGD_STEP: mode = MODE_SSGD; break;
    case ODSGD_ENTRY_GLOBAL_UPDATE: mode = MODE_GLOBAL; break;
    case ODSGD_ENTRY_LOCAL_UPDATE: mode = MODE_LOCAL; break;
    default: return ODSGD_EINVAL;
    }
    if (rule < ODSGD_LOCAL_SGD || rule > ODSGD_LOCAL_SGD_MOMENTUM)
        return ODSGD_EINVAL;
    *waves_wanted = wanted_waves(mode, rule, num_workers, waves_override);
    *lds_bytes = 0;
    *waves_achieved = 0;
    if (*waves_wanted == 0)
        return ODSGD_OK;
    // the model of a CU that the run-time query stands in for on a real device
    auto occupancy = [&](size_t bytes) {
        const size_t alloc = align_up(bytes, lds_granule);
        return alloc == 0 ? 1 << 30 : (int)(lds_per_cu / alloc);
    };
    lds_request_for(*waves_wanted, max_request, occupancy, lds_bytes, waves_achieved);
    if (!residency_acceptable(*waves_wanted, *waves_achieved))
        *lds_bytes = 0;  // the launch would go uncapped
    return ODSGD_OK;
}

int odsgd_local_update(odsgd_handle *h, int worker, const odsgd_hyper *hyper, void *stream)
{
    if (!h || !hyper || worker < -1 || worker >= h->reg.num_workers)
        return ODSGD_EINVAL;
    if (worker < 0)
        return launch(h, MODE_LOCAL, 0, h->reg.num_workers, false, hyper, stream);
    return launch(h, MODE_LOCAL, worker, 1, false, hyper, stream);
}

int odsgd_global_update(odsgd_handle *h, const odsgd_hyper *hyper, void *stream)
{
    if (!h || !hyper)
        return ODSGD_EINVAL;
    int rc = launch(h, global_only_mode(h), 0, h->reg.num_workers, h->has_alt, hyper, stream);
    if (rc == ODSGD_OK) {
        ++h->iteration;
        if (h->has_alt)
            h->current ^= 1;
    }
    return rc;
}

int odsgd_ssgd_step(odsgd_handle *h, const odsgd_hyper *hyper, void *stream)
{
    if (!h || !hyper)
        return ODSGD_EINVAL;
    int rc = launch(h, MODE_SSGD, 0, h->reg.num_workers, false, hyper, stream);
    if (rc == ODSGD_OK)
        ++h->iteration;
    return rc;
}

int odsgd_step(odsgd_handle *h, const odsgd_hyper *hyper, void *stream)
{
    if (!h || !hyper)
        return ODSGD_EINVAL;
    const int mode = (h->iteration < h->warmup_steps) ? MODE_SSGD : MODE_OD;
    int rc = launch(h, mode, 0, h->reg.num_workers, false, hyper, stream);
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
        if (!state)
            return ODSGD_EINVAL;
        const int W = h->reg.num_workers, K = h->reg.num_tensors;
        std::vector<uintptr_t> addr((size_t)W * K, 0);
        for (int m = 0; m < W; ++m) {
            if (!state[m])
                return ODSGD_EINVAL;
            for (int k = 0; k < K; ++k)
                addr[(size_t)m * K + k] = (uintptr_t)state[m][k];
        }
        // a state registration replaces the previous one
        int rc = register_columns(h, col_state(W, 0), W, addr.data(), h->state_ranges, h->alt_ranges, stream);
        if (rc != ODSGD_OK)
            return rc;
    }
    h->rule = *rule;
    warm_residency(h);
    return ODSGD_OK;
}

int odsgd_set_double_buffer(odsgd_handle *h, float *const *w_alt, float *const *mom_alt, void *stream)
{
    if (!h || !w_alt || !mom_alt)
        return ODSGD_EINVAL;
    if (handle_is_stale(h))
        return ODSGD_ESTALE;
    if (h->current != 0)
        return ODSGD_EINVAL;  // the current weights must be in the buffers given to odsgd_init
    const int W = h->reg.num_workers, K = h->reg.num_tensors;
    std::vector<uintptr_t> addr((size_t)2 * K, 0);
    for (int k = 0; k < K; ++k) {
        addr[k] = (uintptr_t)w_alt[k];
        addr[(size_t)K + k] = (uintptr_t)mom_alt[k];
    }
    int rc = register_columns(h, col_alt(W, 0), 2, addr.data(), h->alt_ranges, h->state_ranges, stream);
    if (rc != ODSGD_OK)
        return rc;
    h->has_alt = true;
    return ODSGD_OK;
}

int odsgd_current_buffers(const odsgd_handle *h) { return h ? h->current : ODSGD_EINVAL; }

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

int odsgd_probe_streams(odsgd_handle *h, void *stream)
{
    if (!h)
        return ODSGD_EINVAL;
    const odsgd_hyper none = {0.0f, 0.0f, 0.0f, 0.0f, 1.0f};
    // launched with the residency of the fused SGD step it stands in for
    const odsgd_local_rule saved = h->rule;
    h->rule.rule = ODSGD_LOCAL_SGD;
    int rc = launch(h, MODE_COPY, 0, h->reg.num_workers, false, &none, stream);
    h->rule = saved;
    return rc;
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
