// AdaScale SGD step for MI355X (gfx950): the device code (kernels, their argument records and
// the tables that pick a kernel instance), shared by the translation units of the library.  The
// fused kernel's many instances are compiled in several units (one per register-slot level) so
// that the build runs in parallel; everything here is in an unnamed namespace or a template.
#pragma once

#include <hip/hip_runtime.h>
#include <type_traits>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "adascale_diag.h"

namespace {

// Gradient buffers are read exactly once per step: mark those loads non-temporal.
#ifndef ADASCALE_NT_LOADS
#define ADASCALE_NT_LOADS 1
#endif
#ifndef ADASCALE_THREADS
#define ADASCALE_THREADS 256
#endif

constexpr int kThreads = ADASCALE_THREADS;
constexpr int kWave = 64;
constexpr int kWaves = kThreads / kWave;
constexpr int kTables = 8;  // pointer tables kept on the device, each with a pinned host mirror

struct DevState {
    long long step;
    double tau, r, lr_eff, A, B, sig_hat, mu_hat, sig_bar, mu_bar;
    float eta_f32;
    int done;
};

// Everything about a context's progress that changes from one launch to the next lives on the
// device, in this record, and the kernels advance it themselves.  The host passes the same kernel
// arguments at every step, so a step captured into a HIP graph can be replayed.
struct DevBook {
    // Steps completed.  State record st[epoch & 1] is the current one; a step reads it, writes
    // the other record and then raises epoch (the kernel that evaluates the scalars does).
    alignas(128) unsigned long long epoch;
    // Fused launches with a grid barrier so far: the arrival counter stands at barrier_gen * grid
    // between launches, and a launch waits for (barrier_gen + 1) * grid.
    unsigned long long barrier_gen;
    alignas(128) unsigned long long barrier;  // arrivals, monotonically increasing
    alignas(128) int fault;                   // raised when a bounded wait at the barrier gave up
    alignas(128) unsigned claim;              // streaming reduce: tile pairs handed out (zero between launches)
    alignas(128) DevState st[2];
};

__device__ __forceinline__ unsigned long long book_epoch(const DevBook *bk)
{
    return __hip_atomic_load(&bk->epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
// Same vectors with element alignment only: tensors inside flat buffers start anywhere.
typedef f4 f4e __attribute__((aligned(4)));
typedef u4 u4e __attribute__((aligned(2)));
// Tensor pointers arrive as integers in a table; tell the compiler they are global memory so
// that it emits global_* rather than flat_* accesses.
#define AS_GLOBAL __attribute__((address_space(1)))
typedef const AS_GLOBAL f4e *gp_cf4;
typedef AS_GLOBAL f4e *gp_f4;
typedef const AS_GLOBAL u4e *gp_cu4;

struct Bf16 {
    unsigned short bits;
};

template <typename GT>
struct Traits;
template <>
struct Traits<float> {
    static constexpr int VEC = 4;
};
template <>
struct Traits<Bf16> {
    static constexpr int VEC = 8;
};

__device__ __forceinline__ float widen(float x) { return x; }
__device__ __forceinline__ float widen(Bf16 x) { return __uint_as_float((unsigned)x.bits << 16); }

template <int VEC>
__device__ __forceinline__ void load_f32(const float *p, float (&x)[VEC])
{
#pragma unroll
    for (int q = 0; q < VEC / 4; ++q) {
        f4 t = *(gp_cf4)(p + 4 * q);
        x[4 * q] = t.x; x[4 * q + 1] = t.y; x[4 * q + 2] = t.z; x[4 * q + 3] = t.w;
    }
}
// STREAM: streaming store, for the mean gradient on its way to the HBM scratch (measured: the
// gradient sweep that writes it runs 4-11 % faster than with plain stores, which linger in L2
// and leave it in no particular order).
template <int VEC, bool STREAM = false>
__device__ __forceinline__ void store_f32(float *p, const float (&x)[VEC])
{
#pragma unroll
    for (int q = 0; q < VEC / 4; ++q) {
        f4 t = {x[4 * q], x[4 * q + 1], x[4 * q + 2], x[4 * q + 3]};
        if constexpr (STREAM) __builtin_nontemporal_store(t, (gp_f4)(p + 4 * q));
        else *(gp_f4)(p + 4 * q) = t;
    }
}

__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) x += __shfl_xor(x, off, kWave);
    return x;
}

// Pointer table row of tensor k: [w, v, gbar, g_0 .. g_{S-1}].
constexpr int kRowW = 0, kRowV = 1, kRowGbar = 2, kRowG = 3;

// ---------------------------------------------------------------------------------------------
// reduce: mean gradient + partial sums of A and B.  The S replicas of a tile are consumed in
// half-groups of HG replicas that alternate between two register buffers, so that the loads of
// the next half-group are in flight while the current one is accumulated.
//
// fp32 gradients are accumulated in fp64 (their squares are not exact in fp32).  bf16 gradients
// are accumulated in fp32 and flushed to fp64 after every half-group: a product of two bf16
// values is exact in fp32, and so is a sum of up to 64 bf16 values whose magnitudes lie within
// 2^10 of each other; what rounding remains is random, below 2^-24 per operation, and averages
// out over the ~1e5..1e9 flushed partials.
__device__ __forceinline__ u4 load_raw(const void *p)
{
#if ADASCALE_NT_LOADS
    return __builtin_nontemporal_load((gp_cu4)p);
#else
    return *(gp_cu4)p;
#endif
}

struct AccF32 {  // for fp32 gradients
    double s[4], a;
    __device__ __forceinline__ void init() { s[0] = s[1] = s[2] = s[3] = 0.0; a = 0.0; }
    __device__ __forceinline__ void add(u4 raw, bool live)
    {
        const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const double xd = live ? (double)__uint_as_float(w[e]) : 0.0;
            s[e] += xd;
            a = fma(xd, xd, a);
        }
    }
    __device__ __forceinline__ void flush() {}
    __device__ __forceinline__ double sum(int e) const { return s[e]; }
    __device__ __forceinline__ double squares() const { return a; }
};

struct AccBf16 {  // for bf16 gradients
    float s[8], af;
    double a;
    __device__ __forceinline__ void init()
    {
#pragma unroll
        for (int e = 0; e < 8; ++e) s[e] = 0.f;
        af = 0.f;
        a = 0.0;
    }
    __device__ __forceinline__ void add(u4 raw, bool live)
    {
        const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float lo = live ? __uint_as_float(w[j] << 16) : 0.f;
            const float hi = live ? __uint_as_float(w[j] & 0xffff0000u) : 0.f;
            s[2 * j] += lo;
            s[2 * j + 1] += hi;
            af = fmaf(lo, lo, af);
            af = fmaf(hi, hi, af);
        }
    }
    __device__ __forceinline__ void flush()
    {
        a += (double)af;
        af = 0.f;
    }
    __device__ __forceinline__ double sum(int e) const { return (double)s[e]; }
    __device__ __forceinline__ double squares() const { return a; }
};

template <typename GT> struct AccOf;
template <> struct AccOf<float> { typedef AccF32 type; };
template <> struct AccOf<Bf16> { typedef AccBf16 type; };

// Mean of the S replicas at one lane's VEC elements (all inside the tensor), and the lane's
// contribution to A and B.
template <typename GT, int HG>
__device__ __forceinline__ void reduce_lane_full(const unsigned long long *__restrict__ row, long long base, int S,
                                                 double inv_S, float (&out)[Traits<GT>::VEC], double &acc_a,
                                                 double &acc_b)
{
    constexpr int VEC = Traits<GT>::VEC;
    typename AccOf<GT>::type acc;
    acc.init();
    u4 xa[HG], xb[HG];
    auto issue = [&](u4(&x)[HG], int first) {
#pragma unroll
        for (int g = 0; g < HG; ++g) {
            const int i = min(first + g, S - 1);  // past-the-end slots re-read the last replica
            x[g] = load_raw(reinterpret_cast<const GT *>(row[kRowG + i]) + base);
        }
    };
    auto consume = [&](const u4(&x)[HG], int first) {
#pragma unroll
        for (int g = 0; g < HG; ++g) acc.add(x[g], first + g < S);
        acc.flush();
    };
    issue(xa, 0);
    for (int i0 = 0; i0 < S; i0 += 2 * HG) {
        const bool second = i0 + HG < S;
        if (second) issue(xb, i0 + HG);
        consume(xa, i0);
        if (i0 + 2 * HG < S) issue(xa, i0 + 2 * HG);
        if (second) consume(xb, i0 + HG);
    }
    double b = 0.0;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        const double m = acc.sum(e) * inv_S;
        out[e] = (float)m;
        b = fma(m, m, b);
    }
    acc_a += acc.squares();
    acc_b += b;
}

// The same for one element at the ragged end of a tensor (fp64 throughout).
template <typename GT>
__device__ __forceinline__ float reduce_element(const unsigned long long *__restrict__ row, long long idx, int S,
                                                double inv_S, double &acc_a, double &acc_b)
{
    double se = 0.0, a = 0.0;
    for (int i = 0; i < S; ++i) {
        const double xd = (double)widen(reinterpret_cast<const GT *>(row[kRowG + i])[idx]);
        se += xd;
        a = fma(xd, xd, a);
    }
    const double m = se * inv_S;
    acc_a += a;
    acc_b = fma(m, m, acc_b);
    return (float)m;
}

// Workgroup sum of the lanes' (a, b) into the span's fixed partial slot.
__device__ __forceinline__ void reduce_store_partial(double acc_a, double acc_b, double (&sh)[kWaves][2],
                                                     double *__restrict__ partials, int span)
{
    const int tid = threadIdx.x;
    acc_a = wave_sum(acc_a);
    acc_b = wave_sum(acc_b);
    if ((tid & (kWave - 1)) == 0) {
        sh[tid >> 6][0] = acc_a;
        sh[tid >> 6][1] = acc_b;
    }
    __syncthreads();
    if (tid < 2) {  // fixed order over the waves
        double tsum = sh[0][tid];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) tsum += sh[w][tid];
        partials[(size_t)span * 2 + tid] = tsum;
    }
    __syncthreads();
}

template <typename GT, int HG>
__global__ __launch_bounds__(kThreads) void k_reduce(const int *__restrict__ span_first,
                                                     const int *__restrict__ tile_prefix,
                                                     const long long *__restrict__ numel,
                                                     const unsigned long long *__restrict__ ptrs,
                                                     double *__restrict__ partials, int n_tiles, int span_tiles,
                                                     int n_spans, int S, int row_len, double inv_S)
{
    constexpr int VEC = Traits<GT>::VEC;
    constexpr int TILE = kThreads * VEC;
    const int tid = threadIdx.x;
    __shared__ double sh[kWaves][2];

    for (int span = blockIdx.x; span < n_spans; span += gridDim.x) {
        const int t0 = span * span_tiles;
        const int t1 = min(t0 + span_tiles, n_tiles);
        int k = span_first[span];
        double acc_a = 0.0, acc_b = 0.0;
        for (int t = t0; t < t1; ++t) {
            while (t >= tile_prefix[k + 1]) ++k;
            const long long base = (long long)(t - tile_prefix[k]) * TILE + (long long)tid * VEC;
            const long long rem = numel[k] - base;
            if (rem <= 0) continue;
            const unsigned long long *row = ptrs + (size_t)k * row_len;
            float *gbar = reinterpret_cast<float *>(row[kRowGbar]) + base;
            if (rem >= VEC) {
                float out[VEC];
                reduce_lane_full<GT, HG>(row, base, S, inv_S, out, acc_a, acc_b);
                store_f32<VEC, true>(gbar, out);
            } else {
                for (int e = 0; e < (int)rem; ++e) gbar[e] = reduce_element<GT>(row, base + e, S, inv_S, acc_a, acc_b);
            }
        }
        reduce_store_partial(acc_a, acc_b, sh, partials, span);
    }
}

// ---------------------------------------------------------------------------------------------
// scalars: fixed-order fp64 sum of the partials, then the estimator and the clock.
struct ScalarArgs {
    int S;
    unsigned flags;
    double theta, eps;
    long long L;
};

__device__ __forceinline__ double gain_from(const ScalarArgs &c, double sbar, double mbar)
{
    if (c.flags & ADASCALE_EST_NORM_RATIO) return (sbar + c.eps) / (mbar + c.eps);
    const double den = sbar / c.S + mbar;
    return den > 0.0 ? (sbar + mbar) / den : 1.0;
}

// What the scalar evaluation needs of the state before the step, and the learning rate of the
// step: lr(floor(tau_t)), with tau_t of BEFORE the step (Sec. 3.2) -- none of it depends on this
// step's gradients, so it can be fetched while they are still being summed.
struct ScalarIn {
    long long step;
    double tau, sig_bar, mu_bar;
    float lr_now;
};

// Which record is current is itself read from memory (the epoch): both records are fetched
// beside it and the choice is made in registers, one memory latency instead of two in a row.
__device__ __forceinline__ ScalarIn load_scalar_in(const DevBook *__restrict__ book, const float *__restrict__ lr,
                                                   const ScalarArgs &c, unsigned long long &epoch)
{
    epoch = book_epoch(book);
    const DevState &r0 = book->st[0], &r1 = book->st[1];
    const long long step0 = r0.step, step1 = r1.step;
    const double tau0 = r0.tau, tau1 = r1.tau, sb0 = r0.sig_bar, sb1 = r1.sig_bar, mb0 = r0.mu_bar, mb1 = r1.mu_bar;
    const bool odd = (epoch & 1) != 0;
    ScalarIn s;
    s.step = odd ? step1 : step0;
    s.tau = odd ? tau1 : tau0;
    s.sig_bar = odd ? sb1 : sb0;
    s.mu_bar = odd ? mb1 : mb0;
    long long idx = (long long)floor(s.tau);
    if (idx > c.L - 1) idx = c.L - 1;
    if (idx < 0) idx = 0;
    s.lr_now = lr[idx];
    return s;
}

// The estimator and the clock, evaluated by one lane from the sums A, B and the state of before
// the step; writes the state of after the step to `out` (another record than the one `in` was
// read from: other workgroups may still be reading that).  Returns eta_t.
__device__ __forceinline__ float eval_scalars(double A, double B, const ScalarIn &in, DevState *__restrict__ out,
                                              const ScalarArgs &c, bool write)
{
    const int S = c.S;
    double sig, mu;
    if (S >= 2) {
        sig = (A - S * B) / (S - 1);
        mu = B - sig / S;
    } else {
        sig = 0.0;
        mu = B;
    }
    double x1, x2;
    if (c.flags & ADASCALE_EST_NORM_RATIO) {
        x1 = A / S;
        x2 = B;
    } else {
        x1 = S >= 2 ? fmax(sig, c.eps) : 0.0;
        x2 = fmax(mu, 0.0);
    }
    const long long step = in.step;
    const long long k = step + 1;
    const double alpha = fmax(1.0 - c.theta, 1.0 / (double)k);
    double sbar = in.sig_bar, mbar = in.mu_bar;
    double r = 1.0;
    if (c.flags & ADASCALE_LAGGED_R) r = step == 0 ? 1.0 : gain_from(c, sbar, mbar);
    sbar += alpha * (x1 - sbar);
    mbar += alpha * (x2 - mbar);
    if (!(c.flags & ADASCALE_LAGGED_R)) r = gain_from(c, sbar, mbar);

    const double tau = in.tau;
    const double eta = r * (double)in.lr_now;
    if (write) {
        out->A = A;
        out->B = B;
        out->sig_hat = sig;
        out->mu_hat = mu;
        out->sig_bar = sbar;
        out->mu_bar = mbar;
        out->r = r;
        out->lr_eff = eta;
        out->eta_f32 = (float)eta;
        out->tau = tau + r;
        out->step = k;
        out->done = (tau + r) >= (double)c.L;
    }
    return (float)eta;
}

constexpr int kScalarThreads = 1024;

__global__ __launch_bounds__(kScalarThreads) void k_scalars(const double *__restrict__ partials, int n_partials,
                                                            DevBook *__restrict__ book,
                                                            const float *__restrict__ lr, ScalarArgs c)
{
    __shared__ double sh_a[kScalarThreads], sh_b[kScalarThreads];
    const int tid = threadIdx.x;
    ScalarIn sin{};
    unsigned long long epoch = 0;
    if (tid == 0) sin = load_scalar_in(book, lr, c, epoch);  // in flight while the partials are summed
    typedef double d2 __attribute__((ext_vector_type(2)));
    const d2 *p2 = reinterpret_cast<const d2 *>(partials);
    double a = 0.0, b = 0.0;
    constexpr int U = 8;  // independent loads in flight per thread; the add order stays fixed
    for (int j0 = tid; j0 < n_partials; j0 += kScalarThreads * U) {
        d2 x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + u * kScalarThreads;
            x[u] = j < n_partials ? p2[j] : d2{0.0, 0.0};
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a += x[u].x;
            b += x[u].y;
        }
    }
    sh_a[tid] = a;
    sh_b[tid] = b;
    __syncthreads();
    for (int w = kScalarThreads / 2; w > 0; w >>= 1) {
        if (tid < w) {
            sh_a[tid] += sh_a[tid + w];
            sh_b[tid] += sh_b[tid + w];
        }
        __syncthreads();
    }
    if (tid == 0) {
        eval_scalars(sh_a[0], sh_b[0], sin, &book->st[(epoch + 1) & 1], c, true);
        // the streaming reduce kernel of this step, if any, has finished with its counter
        __hip_atomic_store(&book->claim, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&book->epoch, epoch + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// eta_t of the prior-iteration variant (App. B.3): r_t from the averages as they stand before
// the step (r_0 = 1), so it is known before any gradient is read.
__device__ __forceinline__ float lagged_eta(const DevBook *__restrict__ book, const float *__restrict__ lr,
                                            const ScalarArgs &c)
{
    unsigned long long epoch;
    const ScalarIn in = load_scalar_in(book, lr, c, epoch);
    const double r = in.step == 0 ? 1.0 : gain_from(c, in.sig_bar, in.mu_bar);
    return (float)(r * (double)in.lr_now);
}

// ---------------------------------------------------------------------------------------------
// single pass (prior-iteration gain): reduce and update in one sweep, S*d*b + 16*d bytes.  The
// mean gradient never goes to memory; k_scalars afterwards folds A and B into the averages.
template <typename GT, int HG>
__global__ __launch_bounds__(kThreads) void k_reduce_update(const int *__restrict__ span_first,
                                                            const int *__restrict__ tile_prefix,
                                                            const long long *__restrict__ numel,
                                                            const unsigned long long *__restrict__ ptrs,
                                                            double *__restrict__ partials,
                                                            const DevBook *__restrict__ book,
                                                            const float *__restrict__ lr, ScalarArgs sc, int n_tiles,
                                                            int span_tiles, int n_spans, int S, int row_len,
                                                            double inv_S, float rho, float lambda)
{
    constexpr int VEC = Traits<GT>::VEC;
    constexpr int TILE = kThreads * VEC;
    const int tid = threadIdx.x;
    __shared__ double sh[kWaves][2];
    const float eta = lagged_eta(book, lr, sc);  // k_scalars, behind this kernel, raises the epoch

    for (int span = blockIdx.x; span < n_spans; span += gridDim.x) {
        const int t0 = span * span_tiles;
        const int t1 = min(t0 + span_tiles, n_tiles);
        int k = span_first[span];
        double acc_a = 0.0, acc_b = 0.0;
        for (int t = t0; t < t1; ++t) {
            while (t >= tile_prefix[k + 1]) ++k;
            const long long base = (long long)(t - tile_prefix[k]) * TILE + (long long)tid * VEC;
            const long long rem = numel[k] - base;
            if (rem <= 0) continue;
            const unsigned long long *row = ptrs + (size_t)k * row_len;
            float *w = reinterpret_cast<float *>(row[kRowW]) + base;
            float *v = reinterpret_cast<float *>(row[kRowV]) + base;
            if (rem >= VEC) {
                float wv[VEC], vv[VEC], gv[VEC];
                load_f32<VEC>(w, wv);
                load_f32<VEC>(v, vv);
                reduce_lane_full<GT, HG>(row, base, S, inv_S, gv, acc_a, acc_b);
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float u = fmaf(lambda, wv[e], gv[e]);
                    vv[e] = fmaf(rho, vv[e], u);
                    wv[e] = fmaf(-eta, vv[e], wv[e]);
                }
                store_f32<VEC>(v, vv);
                store_f32<VEC>(w, wv);
            } else {
                for (int e = 0; e < (int)rem; ++e) {
                    const float g = reduce_element<GT>(row, base + e, S, inv_S, acc_a, acc_b);
                    const float u = fmaf(lambda, w[e], g);
                    const float vn = fmaf(rho, v[e], u);
                    v[e] = vn;
                    w[e] = fmaf(-eta, vn, w[e]);
                }
            }
        }
        reduce_store_partial(acc_a, acc_b, sh, partials, span);
    }
}

// ---------------------------------------------------------------------------------------------
// update: momentum-SGD with eta_t taken from device memory.
// (Streaming loads and stores were measured here too: 4 % slower at d = 351 M, and smaller
// lists profit from finding w and v in the memory-side cache at the next step.)
template <int VEC>
__global__ __launch_bounds__(kThreads) void k_update(const int *__restrict__ span_first,
                                                     const int *__restrict__ tile_prefix,
                                                     const long long *__restrict__ numel,
                                                     const unsigned long long *__restrict__ ptrs,
                                                     const DevBook *__restrict__ book, int n_tiles, int span_tiles,
                                                     int n_spans, int row_len, float rho, float lambda)
{
    constexpr int TILE = kThreads * VEC;
    const int tid = threadIdx.x;
    const float eta = book->st[book_epoch(book) & 1].eta_f32;  // the record k_scalars has just written

    for (int span = blockIdx.x; span < n_spans; span += gridDim.x) {
        const int t0 = span * span_tiles;
        const int t1 = min(t0 + span_tiles, n_tiles);
        int k = span_first[span];
        for (int t = t0; t < t1; ++t) {
            while (t >= tile_prefix[k + 1]) ++k;
            const long long base = (long long)(t - tile_prefix[k]) * TILE + (long long)tid * VEC;
            const long long rem = numel[k] - base;
            if (rem <= 0) continue;
            const unsigned long long *row = ptrs + (size_t)k * row_len;
            float *w = reinterpret_cast<float *>(row[kRowW]) + base;
            float *v = reinterpret_cast<float *>(row[kRowV]) + base;
            const float *g = reinterpret_cast<const float *>(row[kRowGbar]) + base;
            if (rem >= VEC) {
                float gv[VEC], wv[VEC], vv[VEC];
                load_f32<VEC>(g, gv);
                load_f32<VEC>(w, wv);
                load_f32<VEC>(v, vv);
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float u = fmaf(lambda, wv[e], gv[e]);
                    vv[e] = fmaf(rho, vv[e], u);
                    wv[e] = fmaf(-eta, vv[e], wv[e]);
                }
                store_f32<VEC>(v, vv);
                store_f32<VEC>(w, wv);
            } else {
                for (int e = 0; e < (int)rem; ++e) {
                    const float u = fmaf(lambda, w[e], g[e]);
                    const float vn = fmaf(rho, v[e], u);
                    v[e] = vn;
                    w[e] = fmaf(-eta, vn, w[e]);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// fused step: one persistent launch, one workgroup per compute unit.
//
// Writing the mean gradient to HBM between the two passes is what the three-kernel step pays
// most for: a small write stream mixed into the gradient reads lowers the read rate of the whole
// pass, and the vector is read again by the update.  The chip can hold it instead: 256 CUs x
// (160 KB LDS + 512 KB VGPR).  Phase 1 streams the S gradient buffers (reads only) and leaves
// each lane's share of gbar in registers and LDS; a grid barrier makes A and B global; every
// workgroup then sums the per-workgroup partials in the same fixed order, derives eta_t itself,
// and phase 2 applies the momentum update from the retained values.
//
// Tiles here are 512 lanes x 4 elements.  Tiles that lie wholly inside a tensor ("full") take
// the hot path: straight-line code without per-lane predicates.  Slot q of workgroup b is full
// tile q * gridDim.x + b; slots [0, R) live in VGPRs (R up to 44), the next lds_tiles slots in
// LDS; for any further slots the sweep leaves the new momentum in v (it does not depend on
// eta_t) and phase 2 only applies it.  The ragged last tile of each tensor ("cold", at most one
// per tensor) takes a simple predicated path through a small HBM scratch.
constexpr int kFThreads = 512;                 // 8 waves: 2 per SIMD, up to 256 VGPRs each
constexpr int kFWaves = kFThreads / kWave;
constexpr int kFRegTiles = 44;                 // most f4 per lane kept in VGPRs (176 of the 256 registers)
constexpr int kFTile = kFThreads * 4;          // elements per tile (fp32 gradients)
constexpr int kFMaxGrid = 256;                 // workgroups (one per CU) = partial slots
constexpr long long kFSpinLimit = 1LL << 22;   // polls of the bounded wait at the grid barrier (several seconds)

struct FTile {
    int k;      // tensor
    int local;  // tile index inside the tensor
};

typedef const AS_GLOBAL char *gp_cchar;
typedef AS_GLOBAL char *gp_char;
// The tile, numel and pointer tables are never written while a kernel runs: reading them through
// the constant address space lets the compiler use scalar loads even though the kernel stores to
// other global memory (with plain global pointers it falls back to vector loads plus a full wait).
#define AS_CONST __attribute__((address_space(4)))
typedef const AS_CONST unsigned long long *cp_u64;

// Where a full tile lives, in wave-uniform terms only (so it costs scalar registers): the
// tensor's pointer row and the tile's byte offset inside the tensor (the same for w, v, the
// scratch and every fp32 gradient buffer).  A lane adds its own constant byte offset 16 * tid.
struct FLoc {
    cp_u64 row;
    unsigned long long tile_off;
};

// How the fused kernel fetches and accumulates a lane's 4 gradient elements of one replica.
// fp32: one 16-byte load, fp64 accumulation (squares of fp32 values are not exact in fp32).
// bf16: one 8-byte load, fp32 accumulation flushed to fp64 after every half-group (products of
// bf16 values are exact in fp32; see the reduce kernel for the argument).
typedef unsigned int u2 __attribute__((ext_vector_type(2)));
typedef u2 u2e __attribute__((aligned(2)));

template <typename GT>
struct FGrad;

template <>
struct FGrad<float> {
    typedef f4 raw;
    static constexpr int kShift = 0;  // gradient byte offset = fp32 byte offset >> kShift
    static __device__ __forceinline__ raw load(gp_cchar p) { return __builtin_nontemporal_load((gp_cf4)p); }
    static __device__ __forceinline__ raw load_partial(gp_cchar p, int c4)
    {
        const AS_GLOBAL float *e = (const AS_GLOBAL float *)p;
        raw x = {e[0], 0.f, 0.f, 0.f};
        if (c4 > 1) x.y = e[1];
        if (c4 > 2) x.z = e[2];
        return x;
    }
    struct Acc {
        double s[4], a;
        __device__ __forceinline__ void init() { s[0] = s[1] = s[2] = s[3] = 0.0; a = 0.0; }
        __device__ __forceinline__ void add(raw x, bool live)
        {
            const float xv[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const double xd = live ? (double)xv[e] : 0.0;
                s[e] += xd;
                a = fma(xd, xd, a);
            }
        }
        __device__ __forceinline__ void flush() {}
        __device__ __forceinline__ double sum(int e) const { return s[e]; }
    };
};

template <>
struct FGrad<Bf16> {
    typedef u2 raw;
    static constexpr int kShift = 1;
    static __device__ __forceinline__ raw load(gp_cchar p) { return __builtin_nontemporal_load((const AS_GLOBAL u2e *)p); }
    static __device__ __forceinline__ raw load_partial(gp_cchar p, int c4)
    {
        const AS_GLOBAL unsigned short *e = (const AS_GLOBAL unsigned short *)p;
        raw x = {(unsigned)e[0], 0u};
        if (c4 > 1) x.x |= (unsigned)e[1] << 16;
        if (c4 > 2) x.y = (unsigned)e[2];
        return x;
    }
    struct Acc {
        float s[4], af;
        double a;
        __device__ __forceinline__ void init() { s[0] = s[1] = s[2] = s[3] = 0.f; af = 0.f; a = 0.0; }
        __device__ __forceinline__ void add(raw x, bool live)
        {
            const unsigned w[2] = {x.x, x.y};
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const float lo = live ? __uint_as_float(w[j] << 16) : 0.f;
                const float hi = live ? __uint_as_float(w[j] & 0xffff0000u) : 0.f;
                s[2 * j] += lo;
                s[2 * j + 1] += hi;
                af = fmaf(lo, lo, af);
                af = fmaf(hi, hi, af);
            }
        }
        __device__ __forceinline__ void flush() { a += (double)af; af = 0.f; }
        __device__ __forceinline__ double sum(int e) const { return (double)s[e]; }
    };
};

// A tile's S = HG * NH replicas are consumed in NH (even) half-groups of HG replicas, alternating
// between two register buffers: while one half-group is accumulated, the loads of the next one
// (of the same tile, or of the next tile after the last half-group) are in flight.
// MASK: S may be smaller than HG * NH; the host pads every pointer row to HG * NH replica slots
// by repeating the last replica, so slots at or past S re-read it (no branch, no index clamp:
// the pointers of a half-group are adjacent in the row and come with one scalar load) and count
// as zero when accumulated.
template <typename GT, int HG, bool MASK>
__device__ __forceinline__ void fused_issue(const FLoc &L, unsigned lane_off, int first, int /*S*/,
                                            typename FGrad<GT>::raw (&x)[HG])
{
#pragma unroll
    for (int g = 0; g < HG; ++g)
        x[g] = FGrad<GT>::load((gp_cchar)(L.row[kRowG + first + g] + (L.tile_off >> FGrad<GT>::kShift)) +
                               (lane_off >> FGrad<GT>::kShift));
}

template <typename GT, int HG, bool MASK>
__device__ __forceinline__ void fused_accumulate(const typename FGrad<GT>::raw (&x)[HG], int first, int S,
                                                 typename FGrad<GT>::Acc &acc)
{
#pragma unroll
    for (int g = 0; g < HG; ++g) {
        acc.add(x[g], !MASK || first + g < S);
        // keep the replicas in order: hoisting all the conversions costs registers
        __builtin_amdgcn_sched_barrier(0);
    }
    acc.flush();
}

// Workgroup barrier that publishes this wave's LDS writes; global loads stay in flight.
__device__ __forceinline__ void lds_release_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

struct NoHook {
    __device__ __forceinline__ void operator()() const {}
};

// Mean gradient of one full tile plus its contribution to A and B.  On entry `xa` holds (in
// flight) half-group 0 of this tile; on return half-group 0 of the NEXT tile is in flight there
// (the last tile of a workgroup names itself as next: a few redundant loads, no branch).
// `hook` runs once, right after the second half-group has been issued: work with long latencies
// of its own (cross-lane sums) hides there behind loads that have to be waited for anyway; LDS
// writes it makes are published by the barrier at the end.
// NH = 0: the (even) number of half-groups is the run-time value nh_rt (scales beyond 8 half-groups).
template <typename GT, int HG, int NH, bool MASK, typename HOOK = NoHook>
__device__ __forceinline__ f4 fused_tile_mean(const FLoc &cur, const FLoc &next, unsigned lane_off, int S, double inv_S,
                                              typename FGrad<GT>::raw (&xa)[HG], double &acc_a, double &acc_b,
                                              const HOOK &hook = HOOK(), int nh_rt = 0)
{
    static_assert(NH % 2 == 0, "half-groups alternate between two buffers");
    typename FGrad<GT>::Acc acc;
    acc.init();
    typename FGrad<GT>::raw xb[HG];
    // Eight or more half-groups stay a loop (unrolled they cost more registers than there are).
    // Its body must be one basic block: what the second issue of a pair fetches -- the next
    // half-group of this tile or, after the last pair, the first one of the next tile -- is
    // chosen with scalar selects, not a branch (with a branch the compiler sinks the accumulation
    // below it, the loads then overwrite registers still in use, and it drains the memory
    // pipeline every iteration to stay correct).
    constexpr int kUnroll = NH > 4 || NH == 0 ? 1 : NH;
    const int nh = NH > 0 ? NH : nh_rt;
    auto pair = [&](int h, auto &&between) {
        fused_issue<GT, HG, MASK>(cur, lane_off, (h + 1) * HG, S, xb);
        __builtin_amdgcn_sched_barrier(0);
        between();
        fused_accumulate<GT, HG, MASK>(xa, h * HG, S, acc);
        __builtin_amdgcn_sched_barrier(0);
        const bool last = h + 2 >= nh;
        const FLoc from{last ? next.row : cur.row, last ? next.tile_off : cur.tile_off};
        fused_issue<GT, HG, MASK>(from, lane_off, last ? 0 : (h + 2) * HG, S, xa);
        __builtin_amdgcn_sched_barrier(0);
        fused_accumulate<GT, HG, MASK>(xb, (h + 1) * HG, S, acc);
        __builtin_amdgcn_sched_barrier(0);
    };
    int h = 0;
    if constexpr (!std::is_same<HOOK, NoHook>::value) {  // first pair apart, with the hook
        pair(0, [&] {
            hook();
            __builtin_amdgcn_sched_barrier(0);
        });
        h = 2;
    }
#pragma unroll kUnroll
    for (; h < nh; h += 2) pair(h, [] {});
    float o[4];
    double b = 0.0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const double m = acc.sum(e) * inv_S;
        o[e] = (float)m;
        b = fma(m, m, b);
    }
    acc_a += acc.a;
    acc_b += b;
    // The sums are brought up to date and the means rounded to fp32 here: left free, the compiler
    // postpones the squares of the means of every retained tile, or their rounding, to the end of
    // phase 1 and keeps their fp64 values alive until then (8 more registers per retained tile).
    asm volatile("" : "+v"(acc_a), "+v"(acc_b), "+v"(o[0]), "+v"(o[1]), "+v"(o[2]), "+v"(o[3]));
    // Keep the 8 waves of the workgroup on the same tile: left alone, the older waves win the
    // arbitration for the memory pipeline and the workgroup then waits for its youngest wave.
    if constexpr (std::is_same<HOOK, NoHook>::value) __builtin_amdgcn_s_barrier();
    else lds_release_barrier();
    return f4{o[0], o[1], o[2], o[3]};
}

// Phase 2 reads and writes w and v with streaming loads and stores (both; either alone changes
// nothing).  With plain accesses the 8 bytes per parameter written here linger in the memory-side
// cache and are written back during the next step's gradient sweep, where a write stream costs
// far more than its volume; streamed, they are out of the way when the phase ends.  Measured with
// parameters that are cold at the start of a step: cfg3 319.6 -> 307.4 us, cfg2 98.4 -> 96.0 us,
// cfg4 (with fused_tile_apply) 780.5 -> 759.5 us.  (A loop that steps on the same 204 MB of w, v
// again and again, and so finds them cached, is 1 % slower for it at cfg3.)
__device__ __forceinline__ void fused_tile_finish(const FLoc &L, unsigned lane_off, f4 wv, f4 vv, f4 g, float eta, float rho,
                                                  float lambda)
{
    gp_char w = (gp_char)(L.row[kRowW] + L.tile_off) + lane_off;
    gp_char v = (gp_char)(L.row[kRowV] + L.tile_off) + lane_off;
    const float gv[4] = {g.x, g.y, g.z, g.w};
    float wn[4] = {wv.x, wv.y, wv.z, wv.w}, vn[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float u = fmaf(lambda, wn[e], gv[e]);
        vn[e] = fmaf(rho, vn[e], u);
        wn[e] = fmaf(-eta, vn[e], wn[e]);
    }
    __builtin_nontemporal_store(f4{vn[0], vn[1], vn[2], vn[3]}, (gp_f4)v);
    __builtin_nontemporal_store(f4{wn[0], wn[1], wn[2], wn[3]}, (gp_f4)w);
}

__device__ __forceinline__ void fused_tile_update(const FLoc &L, unsigned lane_off, f4 g, float eta, float rho,
                                                  float lambda)
{
    const f4 wv = __builtin_nontemporal_load((gp_cf4)((gp_cchar)(L.row[kRowW] + L.tile_off) + lane_off));
    const f4 vv = __builtin_nontemporal_load((gp_cf4)((gp_cchar)(L.row[kRowV] + L.tile_off) + lane_off));
    fused_tile_finish(L, lane_off, wv, vv, g, eta, rho, lambda);
}

// w <- w - eta v for one full tile whose new momentum is already in v.
__device__ __forceinline__ void fused_tile_apply(const FLoc &L, unsigned lane_off, float eta)
{
    gp_char w = (gp_char)(L.row[kRowW] + L.tile_off) + lane_off;
    const f4 wv = __builtin_nontemporal_load((gp_cf4)w),
             vv = __builtin_nontemporal_load((gp_cf4)((gp_cchar)(L.row[kRowV] + L.tile_off) + lane_off));
    __builtin_nontemporal_store(f4{fmaf(-eta, vv.x, wv.x), fmaf(-eta, vv.y, wv.y), fmaf(-eta, vv.z, wv.z), fmaf(-eta, vv.w, wv.w)},
                                (gp_f4)w);
}

// Write bursts.  A sweep that writes as it reads runs well below the rate of one that only reads
// on this memory system, whatever the cache policy of the stores, and the loss does not shrink
// with the volume written.  What does help is to make the whole chip write at the same moments:
// each wave keeps its part of the tiles it has finished in LDS and writes them out when a clock
// that all compute units share enters a new window (or when its ring is full), so between the
// windows the memory system sees reads only.  Measured at d = 351 M, S = 64 bf16: the sweep takes
// 7.23 ms against 7.68 ms with every tile written at once; windows of 130-180 us are equally
// good when the ring takes 200 us to fill, longer ones let it fill up first and lose the effect.
// The ring is private to a wave: a lane keeps and later writes its own 16 bytes of a tile and
// lane 0 of the wave the tile's address, so no barrier is involved and nothing needs to be agreed.
constexpr int kBurstMax = 19;  // tiles of kFThreads x 16 bytes
struct BurstRing {
    f4 *slots;                    // LDS [n][kFThreads]
    unsigned long long *dst;      // LDS [kBurstMax] of this wave: where each kept tile goes
    unsigned long long inv;       // 2^64 / window length in clock ticks
    unsigned long long window;
    int n, kept, hslot, tslot;
    __device__ __forceinline__ void init(f4 *lds, unsigned long long *dst_of_wave, int tiles, unsigned long long win_inv)
    {
        slots = lds;
        dst = dst_of_wave;
        inv = win_inv;
        n = tiles;
        kept = hslot = tslot = 0;
        window = __umul64hi(wall_clock64(), inv);
    }
    __device__ __forceinline__ void write_kept(int tid, unsigned lane_off)
    {
        for (; kept > 0; --kept) {
            const unsigned long long d = dst[tslot];
            __builtin_nontemporal_store(slots[tslot * kFThreads + tid], (gp_f4)((gp_char)d + lane_off));
            tslot = tslot + 1 == n ? 0 : tslot + 1;
        }
    }
    // d: address of the tile; n = 0 writes at once
    __device__ __forceinline__ void put(unsigned long long d, f4 o, int tid, unsigned lane_off)
    {
        if (n == 0) {
            __builtin_nontemporal_store(o, (gp_f4)((gp_char)d + lane_off));
            return;
        }
        if (kept == n) write_kept(tid, lane_off);
        slots[hslot * kFThreads + tid] = o;
        if ((tid & (kWave - 1)) == 0) dst[hslot] = d;
        hslot = hslot + 1 == n ? 0 : hslot + 1;
        ++kept;
        const unsigned long long now = __umul64hi(wall_clock64(), inv);
        if (now != window) {
            window = now;
            write_kept(tid, lane_off);
        }
    }
};

struct FusedArgs {
    const FTile *tiles;            // full tiles   } read through the constant address space
    const FTile *cold;             // ragged tiles }
    const long long *numel;
    const unsigned long long *ptrs;
    double *partials;              // [gridDim.x][2]
    DevBook *book;                 // state records, epoch, barrier counter and generation, fault flag
    const float *lr;
    long long spin_limit;          // polls after which the wait at the barrier gives up
    int barrier_extra;             // test hook: arrivals to wait for beyond the grid's (they never come)
    int n_tiles, n_cold, tiles_per_block, lds_tiles, S, row_len;
    int nh;                        // half-groups per tile (used by the instances with NH = 0)
    double inv_S;
    float rho, lambda;
    unsigned long long win_inv;    // write bursts of the tiles beyond the chip's capacity: 2^64 / window in clock ticks, 0 = none
    ScalarArgs sc;
};

// Ragged last tile of a tensor, phase 1: per-lane predicates, mean gradient to the HBM scratch.
// Lanes wholly inside the tensor use one 16-byte load per replica, the lane on the boundary
// single elements; the replicas are loaded HG at a time so that their latencies overlap.
template <typename GT, int HG, typename ARGS>
__device__ __forceinline__ void fused_cold_mean(const ARGS &p, int c, int tid, double &acc_a, double &acc_b)
{
    const AS_CONST int *tp = (const AS_CONST int *)p.cold + 2 * (size_t)c;
    const int k = tp[0], local = tp[1];
    cp_u64 row = (cp_u64)p.ptrs + (size_t)k * p.row_len;
    const long long first = (long long)local * kFTile + (long long)tid * 4;
    const long long rem = ((const AS_CONST long long *)p.numel)[k] - first;
    if (rem <= 0) return;
    const int c4 = rem < 4 ? (int)rem : 4;
    typename FGrad<GT>::Acc acc;
    acc.init();
    // nothing overlaps these loads (no double buffering here), so two half-groups go out together
    // (the pointer rows are padded to an even number of half-groups): a ragged tile costs
    // ceil(S / (2 HG)) memory latencies
    auto fetch = [&](typename FGrad<GT>::raw (&x)[HG], int i0) {
#pragma unroll
        for (int g = 0; g < HG; ++g) {
            gp_cchar gp = (gp_cchar)row[kRowG + i0 + g] + ((first * 4) >> FGrad<GT>::kShift);
            x[g] = c4 == 4 ? FGrad<GT>::load(gp) : FGrad<GT>::load_partial(gp, c4);
        }
    };
    for (int i0 = 0; i0 < p.S; i0 += 2 * HG) {
        typename FGrad<GT>::raw x0[HG], x1[HG];
        fetch(x0, i0);
        fetch(x1, i0 + HG);
        fused_accumulate<GT, HG, true>(x0, i0, p.S, acc);
        fused_accumulate<GT, HG, true>(x1, i0 + HG, p.S, acc);
    }
    AS_GLOBAL float *gb = (AS_GLOBAL float *)row[kRowGbar] + first;
    float o[4];
    double b = 0.0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const double m = acc.sum(e) * p.inv_S;   // elements past the end were loaded as zeros: m = 0
        o[e] = (float)m;
        b = fma(m, m, b);
    }
    if (c4 == 4) {
        *(gp_f4)gb = f4{o[0], o[1], o[2], o[3]};
    } else {
        gb[0] = o[0];
        if (c4 > 1) gb[1] = o[1];
        if (c4 > 2) gb[2] = o[2];
    }
    acc_a += acc.a;
    acc_b += b;
}

__device__ __forceinline__ void fused_cold_update(const FusedArgs &p, int c, int tid, float eta)
{
    const AS_CONST int *tp = (const AS_CONST int *)p.cold + 2 * (size_t)c;
    const int k = tp[0], local = tp[1];
    cp_u64 row = (cp_u64)p.ptrs + (size_t)k * p.row_len;
    const long long first = (long long)local * kFTile + (long long)tid * 4;
    const long long rem = ((const AS_CONST long long *)p.numel)[k] - first;
    if (rem <= 0) return;
    AS_GLOBAL float *w = (AS_GLOBAL float *)row[kRowW] + first;
    AS_GLOBAL float *v = (AS_GLOBAL float *)row[kRowV] + first;
    const AS_GLOBAL float *gb = (const AS_GLOBAL float *)row[kRowGbar] + first;
    if (rem >= 4) {
        const f4 gv = *(gp_cf4)gb, wv = *(gp_cf4)w, vv = *(gp_cf4)v;
        const float g4[4] = {gv.x, gv.y, gv.z, gv.w};
        float wn[4] = {wv.x, wv.y, wv.z, wv.w}, vn[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float u = fmaf(p.lambda, wn[e], g4[e]);
            vn[e] = fmaf(p.rho, vn[e], u);
            wn[e] = fmaf(-eta, vn[e], wn[e]);
        }
        *(gp_f4)v = f4{vn[0], vn[1], vn[2], vn[3]};
        *(gp_f4)w = f4{wn[0], wn[1], wn[2], wn[3]};
    } else {
#pragma unroll
        for (int e = 0; e < 3; ++e) {
            if (e < (int)rem) {
                const float u = fmaf(p.lambda, w[e], gb[e]);
                const float vn = fmaf(p.rho, v[e], u);
                v[e] = vn;
                w[e] = fmaf(-eta, vn, w[e]);
            }
        }
    }
}

// The full-tile slots of one workgroup (wave-uniform).  Slot q holds full tile q * G + b; the
// workgroup's slots [0, n_valid) exist.  Slots [0, R) are kept in VGPRs (the host picks R so that
// every workgroup has at least R tiles: that part is straight-line code without branches),
// [R, q_hbm) in LDS; for [q_hbm, n_valid) nothing is kept (the momentum is updated in the sweep).
template <int R>
struct FCtx {
    const FusedArgs &p;
    int b, G, row_len, q_hbm, n_valid;

    __device__ __forceinline__ FLoc locate(int q) const
    {
        const AS_CONST int *tp = (const AS_CONST int *)p.tiles + 2 * ((size_t)q * G + b);
        return FLoc{(cp_u64)p.ptrs + (size_t)tp[0] * row_len, (unsigned long long)tp[1] * (kFTile * 4ULL)};
    }
    // Phase 1 visits the HBM-spilled slots first (the only ones that write), then the LDS slots,
    // then the register slots; after(q) is the slot visited after q, or q itself at the end.
    __device__ __forceinline__ int after(int q) const
    {
        const int lds_end = min(q_hbm, n_valid);
        if (q >= q_hbm) return q + 1 < n_valid ? q + 1 : (R < lds_end ? R : 0);
        if (q >= R) return q + 1 < lds_end ? q + 1 : (R > 0 ? 0 : q);
        return q + 1 < R ? q + 1 : q;
    }
};

// Register slots, addressed at compile time (template recursion instead of a loop so that the
// retained values are plain registers whatever the unroller decides).
template <typename GT, int HG, int NH, bool MASK, int R, int Q>
__device__ __forceinline__ void fused_regs_phase1(const FCtx<R> &cx, unsigned lane_off, f4 (&keep)[R > 0 ? R : 1],
                                                  FLoc &cur, typename FGrad<GT>::raw (&xa)[HG], double &acc_a,
                                                  double &acc_b)
{
    if constexpr (Q < R) {
        const FLoc next = cx.locate(cx.after(Q));
        keep[Q] = fused_tile_mean<GT, HG, NH, MASK>(cur, next, lane_off, cx.p.S, cx.p.inv_S, xa, acc_a, acc_b, NoHook(),
                                                    cx.p.nh);
        cur = next;
        fused_regs_phase1<GT, HG, NH, MASK, R, Q + 1>(cx, lane_off, keep, cur, xa, acc_a, acc_b);
    }
}

template <int R, int Q>
__device__ __forceinline__ void fused_regs_phase2(const FCtx<R> &cx, unsigned lane_off, const f4 (&keep)[R > 0 ? R : 1],
                                                  float eta)
{
    if constexpr (Q < R) {
        fused_tile_update(cx.locate(Q), lane_off, keep[Q], eta, cx.p.rho, cx.p.lambda);
        fused_regs_phase2<R, Q + 1>(cx, lane_off, keep, eta);
    }
}

// S == HG * NH (MASK: S <= HG * NH); R = register slots per lane (every workgroup has at least R full tiles).
// LAG: prior-iteration gain (App. B.3) -- eta_t is known at the start, so there is no grid
// barrier and no scalar evaluation here; k_scalars runs afterwards on the partials.
template <typename GT, int HG, int NH, bool MASK, int R, bool LAG>
__global__ __launch_bounds__(kFThreads) void k_fused(FusedArgs p)
{
    extern __shared__ f4 lds_gbar[];  // [lds_tiles][kFThreads]
    __shared__ double red[kFMaxGrid][2];
    __shared__ float sh_eta;
    __shared__ int sh_fault;
    __shared__ unsigned long long s_dst[kFWaves][kBurstMax];
    const int tid = threadIdx.x, b = blockIdx.x, G = gridDim.x;
    // this workgroup's slots: full tiles b, b + G, b + 2G, ...
    const int n_valid = b < p.n_tiles ? (p.n_tiles - 1 - b) / G + 1 : 0;
    const int q_hbm = min(R + p.lds_tiles, p.tiles_per_block);
    const int q_lds_end = min(q_hbm, n_valid);
    const FCtx<R> cx{p, b, G, p.row_len, q_hbm, n_valid};
    const unsigned lane_off = (unsigned)tid * 16u;

    f4 keep[R > 0 ? R : 1];
    double acc_a = 0.0, acc_b = 0.0;

    // phase 1
    // ragged tiles go to the workgroups from the top: those are the ones with one full tile less
    for (int c = G - 1 - b; c < p.n_cold; c += G) fused_cold_mean<GT, HG, FusedArgs>(p, c, tid, acc_a, acc_b);

    if (n_valid > 0) {
        typename FGrad<GT>::raw xa[HG];
        const int q_first = q_hbm < n_valid ? q_hbm : (R < q_lds_end ? R : 0);
        FLoc cur = cx.locate(q_first);
        fused_issue<GT, HG, MASK>(cur, lane_off, 0, p.S, xa);
        // Tiles beyond the chip's capacity: their sweep leaves the new momentum
        // v <- rho v + gbar + lambda w (which does not depend on eta_t) in v, and phase 2 only
        // applies it.  That writes 8 bytes per parameter where a round trip of the mean gradient
        // through a scratch writes 12, and writes are what this memory system charges most for.
        // v (and w when there is weight decay) are requested before the tile's gradients, so
        // they have arrived when the mean is known.
        // The LDS slots are still empty while these tiles are swept: they serve as the ring the
        // new momentum is written from in bursts.
        const bool decay = p.lambda != 0.f;
        BurstRing ring;
        ring.init(lds_gbar, s_dst[tid >> 6], p.win_inv != 0 ? min(p.lds_tiles, kBurstMax) : 0, p.win_inv);
        for (int q = q_hbm; q < n_valid; ++q) {
            const FLoc next = cx.locate(cx.after(q));
            gp_char vp = (gp_char)(cur.row[kRowV] + cur.tile_off) + lane_off;
            const f4 vv = __builtin_nontemporal_load((gp_cf4)vp);
            f4 wv = {0.f, 0.f, 0.f, 0.f};
            if (decay) wv = __builtin_nontemporal_load((gp_cf4)((gp_cchar)(cur.row[kRowW] + cur.tile_off) + lane_off));
            const f4 m = fused_tile_mean<GT, HG, NH, MASK>(cur, next, lane_off, p.S, p.inv_S, xa, acc_a, acc_b, NoHook(), p.nh);
            const float g4[4] = {m.x, m.y, m.z, m.w}, v4[4] = {vv.x, vv.y, vv.z, vv.w}, w4[4] = {wv.x, wv.y, wv.z, wv.w};
            float o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = fmaf(p.rho, v4[e], decay ? fmaf(p.lambda, w4[e], g4[e]) : g4[e]);
            ring.put(cur.row[kRowV] + cur.tile_off, f4{o[0], o[1], o[2], o[3]}, tid, lane_off);
            cur = next;
        }
        ring.write_kept(tid, lane_off);
        for (int q = R; q < q_lds_end; ++q) {
            const FLoc next = cx.locate(cx.after(q));
            lds_gbar[(q - R) * kFThreads + tid] =
                fused_tile_mean<GT, HG, NH, MASK>(cur, next, lane_off, p.S, p.inv_S, xa, acc_a, acc_b, NoHook(), p.nh);
            cur = next;
        }
        fused_regs_phase1<GT, HG, NH, MASK, R, 0>(cx, lane_off, keep, cur, xa, acc_a, acc_b);
    }

    // w and v of the first kPre slots (register slots first, then LDS slots: the order of phase 2)
    // are requested right after the workgroup has arrived at the grid barrier: the loads travel
    // while it waits for the others, and phase 2 finds them in registers.  How many depends on the
    // registers the instance has to spare (the load buffers of phase 1 are free again by then).
    constexpr int kPre = LAG ? 0 : R == 0 ? 16 : R <= 10 ? 20 : R <= 30 ? 10 : 4;  // the most that leaves no spills
    f4 pre_w[kPre > 0 ? kPre : 1], pre_v[kPre > 0 ? kPre : 1];

    // workgroup partial -> fixed slot
    acc_a = wave_sum(acc_a);
    acc_b = wave_sum(acc_b);
    if ((tid & (kWave - 1)) == 0) {
        red[tid >> 6][0] = acc_a;
        red[tid >> 6][1] = acc_b;
    }
    __syncthreads();
    float eta;
    if constexpr (LAG) {
        if (tid < 2) {
            double t = red[0][tid];
#pragma unroll
            for (int w = 1; w < kFWaves; ++w) t += red[w][tid];
            p.partials[(size_t)b * 2 + tid] = t;
        }
        eta = lagged_eta(p.book, p.lr, p.sc);  // k_scalars, behind this kernel, raises the epoch
    } else {
        // The partials cross workgroups (and XCDs, whose L2s are not coherent with each other): they
        // are written and read with agent-scope atomic accesses, which are performed at the memory
        // side, and the arrival count is bumped only after this workgroup's stores have completed.
        // That avoids a whole-L2 write-back and invalidate at the barrier; nothing else written in
        // phase 1 (scratch tiles) is read by another workgroup.
        // (the state of before the step and lr(floor(tau_t)) do not depend on the sums: lane 0
        // fetches them here, behind the wait for the partial store and for the other workgroups)
        // So are the epoch (which state record is current) and the barrier's generation: workgroup 0
        // raises both after the barrier, that is after this workgroup has arrived.
        ScalarIn sin{};
        unsigned long long epoch = 0, barrier_target = 0;
        if (tid == 0) {
            const unsigned long long gen = __hip_atomic_load(&p.book->barrier_gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sin = load_scalar_in(p.book, p.lr, p.sc, epoch);
            barrier_target = (gen + 1) * (unsigned long long)G + (unsigned long long)p.barrier_extra;
        }
        if (tid < 2) {
            double t = red[0][tid];
    #pragma unroll
            for (int w = 1; w < kFWaves; ++w) t += red[w][tid];
            __hip_atomic_store(&p.partials[(size_t)b * 2 + tid], t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_s_waitcnt(0);  // vmcnt(0) expcnt(0) lgkmcnt(0): the store has been acknowledged
        }

        // Grid barrier with a bounded wait.  A workgroup whose wait runs out raises the fault flag;
        // every poll reads the flag beside the counter (two loads in flight, one latency), so the
        // others stop waiting too.  A workgroup that has seen the flag leaves without evaluating the
        // scalars and without phase 2: its retained tiles leave w and v as they were and the state
        // record is not advanced by it.  (Workgroups that saw all arrivals before the flag went up
        // carry on; tiles beyond the chip's capacity already hold the new momentum in v.  The host
        // reports the step as failed either way.)
        __syncthreads();
        if (tid == 0) __hip_atomic_fetch_add(&p.book->barrier, 1ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if constexpr (kPre > 0) {
#pragma unroll
            for (int q = 0; q < kPre; ++q) {
                if (q < R || q < q_lds_end) {  // register slots always exist
                    const FLoc L = cx.locate(q);
                    pre_w[q] = __builtin_nontemporal_load((gp_cf4)((gp_cchar)(L.row[kRowW] + L.tile_off) + lane_off));
                    pre_v[q] = __builtin_nontemporal_load((gp_cf4)((gp_cchar)(L.row[kRowV] + L.tile_off) + lane_off));
                }
            }
        }
        if (tid == 0) {
            long long spins = 0;
            int failed = 0;
            for (;;) {
                const unsigned long long seen = __hip_atomic_load(&p.book->barrier, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                failed = __hip_atomic_load(&p.book->fault, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (failed || seen >= barrier_target) break;
                if (++spins > p.spin_limit) {
                    __hip_atomic_store(&p.book->fault, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    failed = 1;
                    break;
                }
                __builtin_amdgcn_s_sleep(16);  // poll not too often: 256 pollers share one address
            }
            sh_fault = failed;
            // The counter receives this grid's arrivals whatever happens (a workgroup that gives up
            // has arrived; one that was not resident arrives when it runs), so the generation moves
            // on with it even when the step is void.
            if (b == 0) {
                const unsigned long long gen = (barrier_target - (unsigned long long)p.barrier_extra) / (unsigned long long)G;
                __hip_atomic_store(&p.book->barrier_gen, gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        __syncthreads();
        if (sh_fault) return;

        // every workgroup: the same fixed-order sum of all partials, then the scalars
        for (int j = tid; j < kFMaxGrid; j += kFThreads) {
            red[j][0] = j < G ? __hip_atomic_load(&p.partials[(size_t)j * 2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.0;
            red[j][1] =
                j < G ? __hip_atomic_load(&p.partials[(size_t)j * 2 + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.0;
        }
        __syncthreads();
        for (int w = kFMaxGrid / 2; w > 0; w >>= 1) {
            for (int j = tid; j < w; j += kFThreads) {
                red[j][0] += red[j + w][0];
                red[j][1] += red[j + w][1];
            }
            __syncthreads();
        }
        if (tid == 0) {
            sh_eta = eval_scalars(red[0][0], red[0][1], sin, &p.book->st[(epoch + 1) & 1], p.sc, b == 0);
            if (b == 0) __hip_atomic_store(&p.book->epoch, epoch + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        eta = sh_eta;
    }
    // phase 2: momentum update from the retained mean gradient
    if constexpr (kPre > 0) {
#pragma unroll
        for (int q = 0; q < kPre; ++q) {
            if (q < R) {
                if (n_valid > 0) fused_tile_finish(cx.locate(q), lane_off, pre_w[q], pre_v[q], keep[q < R ? q : 0], eta, p.rho, p.lambda);
            } else if (q < q_lds_end) {
                fused_tile_finish(cx.locate(q), lane_off, pre_w[q], pre_v[q], lds_gbar[(q - R) * kFThreads + tid], eta, p.rho, p.lambda);
            }
        }
    }
    constexpr int kRegFrom = kPre < R ? kPre : R;
    if (n_valid > 0) fused_regs_phase2<R, kRegFrom>(cx, lane_off, keep, eta);
    for (int q = kPre > R ? kPre : R; q < q_lds_end; ++q)
        fused_tile_update(cx.locate(q), lane_off, lds_gbar[(q - R) * kFThreads + tid], eta, p.rho, p.lambda);
    for (int q = q_hbm; q < n_valid; ++q) fused_tile_apply(cx.locate(q), lane_off, eta);
    for (int c = G - 1 - b; c < p.n_cold; c += G) fused_cold_update(p, c, tid, eta);  // same owner as in phase 1
}

// ---------------------------------------------------------------------------------------------
// streaming reduce: the first kernel of the three-kernel step for parameter lists far larger
// than the chip (the fused step then keeps little of the mean gradient on chip).
//
// Measured on this memory system: a gradient sweep that also writes the mean gradient reads at
// ~5.1 TB/s instead of ~6.9 TB/s, however small the write stream is -- unless the accesses of
// the whole chip stay close together in memory and the writes bypass the cache: one persistent
// workgroup per CU, tiles handed out in memory order from one global counter (the front is then
// 256 tiles wide), streaming stores.  That reads at ~6.1 TB/s.
//
// Unit of work: a pair of consecutive full tiles (512 lanes x 4 elements each).  A workgroup
// claims pairs two ahead (the counter's latency is hidden behind a pair of tiles), the first
// half-group of a tile is in flight before the previous tile ends, and each pair leaves its
// contribution to A and B in the pair's own slot, so the sums do not depend on which workgroup
// took which pair: k_scalars adds the slots in index order.  The ragged last tiles of the
// tensors are shared out statically; their contribution goes to the workgroup's slot.
struct StreamArgs {
    const FTile *tiles;            // full tiles   } read through the constant address space
    const FTile *cold;             // ragged tiles }
    const long long *numel;
    const unsigned long long *ptrs;
    double *partials;              // [gridDim.x + pairs][2]
    unsigned *claim;               // pairs handed out so far in this launch (zero on entry; k_scalars zeroes it again)
    int n_tiles, n_cold, S, row_len;
    int nh;                        // half-groups per tile (used by the instances with NH = 0)
    double inv_S;
    // momentum: 0 = write the mean gradient to the scratch (k_update follows); 1 = write
    // v <- rho v + gbar + lambda w, which does not depend on eta_t, in place of it (k_apply
    // follows).  Same arithmetic, same results; the step then writes 8 instead of 12 bytes per
    // parameter, reads v here instead of the mean gradient later, and needs no scratch.
    int momentum;
    float rho, lambda;
    // Write bursts (BurstRing): tiles kept in the dynamic LDS (0: every tile written at once)
    // and 2^64 / window length in clock ticks.
    int keep;
    unsigned long long win_inv;
};
constexpr int kStreamKeepMax = 18;

// Ragged tile, momentum variant: turn the mean gradient the same lane has just left in the
// scratch into the new momentum.
template <typename ARGS>
__device__ __forceinline__ void fused_cold_momentum(const ARGS &p, int c, int tid)
{
    const AS_CONST int *tp = (const AS_CONST int *)p.cold + 2 * (size_t)c;
    const int k = tp[0], local = tp[1];
    cp_u64 row = (cp_u64)p.ptrs + (size_t)k * p.row_len;
    const long long first = (long long)local * kFTile + (long long)tid * 4;
    const long long rem = ((const AS_CONST long long *)p.numel)[k] - first;
    if (rem <= 0) return;
    const AS_GLOBAL float *w = (const AS_GLOBAL float *)row[kRowW] + first;
    AS_GLOBAL float *v = (AS_GLOBAL float *)row[kRowV] + first;
    const AS_GLOBAL float *gb = (const AS_GLOBAL float *)row[kRowGbar] + first;
    const int n = rem < 4 ? (int)rem : 4;
    for (int e = 0; e < n; ++e) v[e] = fmaf(p.rho, v[e], fmaf(p.lambda, w[e], gb[e]));
}

// (The prior-iteration-gain variant uses this kernel too, followed by k_scalars and k_update:
// updating w and v inside the sweep would save 8 bytes per parameter, but measured at d = 351 M
// the sweep then runs at the rate of a pass with twice the writes, 9.7 ms against 9.2 ms.)
template <typename GT, int HG, int NH, bool MASK>
__global__ __launch_bounds__(kFThreads) void k_reduce_stream(StreamArgs p)
{
    __shared__ double red[1][kFWaves][2];
    __shared__ int s_claim[2];
    extern __shared__ f4 s_keep[];                              // [keep][kFThreads]
    __shared__ unsigned long long s_dst[kFWaves][kBurstMax];
    const int tid = threadIdx.x, b = blockIdx.x, G = gridDim.x;
    const unsigned lane_off = (unsigned)tid * 16u;
    const int row_len = p.row_len;
    const int n_pairs = (p.n_tiles + 1) >> 1;

    BurstRing ring;
    ring.init(s_keep, s_dst[tid >> 6], p.keep, p.win_inv);

    auto claim = [&]() -> int {
        const unsigned c = __hip_atomic_fetch_add(p.claim, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return c < (unsigned)n_pairs ? (int)c : -1;
    };
    int pend = -1;  // lane 0: the pair after the next one
    if (tid == 0) {
        s_claim[0] = claim();
        s_claim[1] = claim();
        pend = claim();
    }

    // ragged tiles -> this workgroup's slot
    {
        double acc_a = 0.0, acc_b = 0.0;
        for (int c = b; c < p.n_cold; c += G) {
            fused_cold_mean<GT, HG, StreamArgs>(p, c, tid, acc_a, acc_b);
            if (p.momentum) fused_cold_momentum(p, c, tid);
        }
        acc_a = wave_sum(acc_a);
        acc_b = wave_sum(acc_b);
        if ((tid & (kWave - 1)) == 0) {
            red[0][tid >> 6][0] = acc_a;
            red[0][tid >> 6][1] = acc_b;
        }
        __syncthreads();
        if (tid < 2) {
            double t = red[0][0][tid];
#pragma unroll
            for (int w = 1; w < kFWaves; ++w) t += red[0][w][tid];
            p.partials[(size_t)b * 2 + tid] = t;
        }
        __syncthreads();
    }

    auto locate = [&](int t) -> FLoc {
        const AS_CONST int *tp = (const AS_CONST int *)p.tiles + 2 * (size_t)t;
        return FLoc{(cp_u64)p.ptrs + (size_t)tp[0] * row_len, (unsigned long long)tp[1] * (kFTile * 4ULL)};
    };
    // Momentum variant: v (and w when there is weight decay) of a tile are requested before its
    // gradients, so they have arrived when the mean is known.
    const bool momentum = p.momentum != 0, decay = p.lambda != 0.f;
    auto fetch_params = [&](const FLoc &L, f4 &vv, f4 &wv) {
        if (momentum) {
            vv = __builtin_nontemporal_load((gp_cf4)((gp_cchar)(L.row[kRowV] + L.tile_off) + lane_off));
            if (decay) wv = __builtin_nontemporal_load((gp_cf4)((gp_cchar)(L.row[kRowW] + L.tile_off) + lane_off));
        }
    };
    auto store_mean = [&](const FLoc &L, f4 m, f4 vv, f4 wv) {
        if (momentum) {
            const float g4[4] = {m.x, m.y, m.z, m.w}, v4[4] = {vv.x, vv.y, vv.z, vv.w}, w4[4] = {wv.x, wv.y, wv.z, wv.w};
            float o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = fmaf(p.rho, v4[e], decay ? fmaf(p.lambda, w4[e], g4[e]) : g4[e]);
            ring.put(L.row[kRowV] + L.tile_off, f4{o[0], o[1], o[2], o[3]}, tid, lane_off);
        } else {
            ring.put(L.row[kRowGbar] + L.tile_off, m, tid, lane_off);
        }
    };
    auto finish = [&](int pair) {  // after a barrier: the pair's contribution in wave order
        if (tid < 2) {
            double t = red[0][0][tid];
#pragma unroll
            for (int w = 1; w < kFWaves; ++w) t += red[0][w][tid];
            p.partials[((size_t)G + pair) * 2 + tid] = t;
        }
    };

    int cur = __builtin_amdgcn_readfirstlane(s_claim[0]);
    int nxt = __builtin_amdgcn_readfirstlane(s_claim[1]);
    if (cur < 0) return;
    int par = 0, prev = -1;
    double prev_a = 0.0, prev_b = 0.0;  // this lane's contributions of the previous pair
    // The cross-lane sum of a pair's contributions is a chain of long-latency lane exchanges: it
    // runs inside the next pair's first tile, behind that tile's loads.
    auto wave_partials = [&]() {
        if (prev >= 0) {
            const double a = wave_sum(prev_a), bsum = wave_sum(prev_b);
            if ((tid & (kWave - 1)) == 0) {
                red[0][tid >> 6][0] = a;
                red[0][tid >> 6][1] = bsum;
            }
        }
    };
    typename FGrad<GT>::raw xa[HG];
    FLoc L0 = locate(2 * cur);
    fused_issue<GT, HG, MASK>(L0, lane_off, 0, p.S, xa);
    while (cur >= 0) {
        const bool two = 2 * cur + 1 < p.n_tiles;
        const FLoc L1 = locate(two ? 2 * cur + 1 : 2 * cur);
        const FLoc LN = locate(nxt >= 0 ? 2 * nxt : 2 * cur);  // at the end: a few redundant loads, no branch
        double acc_a = 0.0, acc_b = 0.0;
        f4 vv = {0.f, 0.f, 0.f, 0.f}, wv = {0.f, 0.f, 0.f, 0.f};
        fetch_params(L0, vv, wv);
        f4 m = fused_tile_mean<GT, HG, NH, MASK>(L0, two ? L1 : LN, lane_off, p.S, p.inv_S, xa, acc_a, acc_b,
                                                 wave_partials, p.nh);
        store_mean(L0, m, vv, wv);
        if (prev >= 0) finish(prev);
        if (two) {
            fetch_params(L1, vv, wv);
            m = fused_tile_mean<GT, HG, NH, MASK>(L1, LN, lane_off, p.S, p.inv_S, xa, acc_a, acc_b, NoHook(), p.nh);
            store_mean(L1, m, vv, wv);
        }
        prev_a = acc_a;
        prev_b = acc_b;
        if (tid == 0) {
            s_claim[par] = pend;
            pend = pend >= 0 ? claim() : -1;
        }
        lds_release_barrier();  // the claim is published; the reads of `red` above are done
        prev = cur;
        cur = nxt;
        nxt = __builtin_amdgcn_readfirstlane(s_claim[par]);
        par ^= 1;
        L0 = LN;
    }
    ring.write_kept(tid, lane_off);
    wave_partials();
    lds_release_barrier();
    finish(prev);
}

// Also lowers the fault flag a fused step raises when its grid barrier gives up: the caller has
// restored w, v and this state from a checkpoint.
__global__ void k_set_state(DevBook *book, long long step, double tau, double sbar, double mbar, long long L)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        DevState *st = &book->st[book_epoch(book) & 1];
        book->fault = 0;
        st->step = step;
        st->tau = tau;
        st->sig_bar = sbar;
        st->mu_bar = mbar;
        st->done = tau >= (double)L;
    }
}

// ---------------------------------------------------------------------------------------------
// apply: w <- w - eta_t v, the last kernel of the three-kernel step whose gradient sweep has left
// the new momentum in v (12 bytes per parameter instead of the 20 of k_update).  Persistent
// workgroups, one per compute unit, walk the full tiles in memory order, two tiles a stride of
// the grid apart per round with all four loads ahead of the two stores (the chip then works on a
// front 2 x 256 tiles wide).  Measured against one workgroup per span of two 256-lane tiles in
// dispatch order, at d = 351 M: 705 against 757 us; one tile per round 776, three 772, four 796,
// two adjacent tiles 772, two workgroups per compute unit 860; streaming stores change nothing
// and streaming loads cost 4-15 %, so the accesses are plain ones.
struct ApplyArgs {
    const FTile *tiles, *cold;     // full and ragged tiles, read through the constant address space
    const long long *numel;
    const unsigned long long *ptrs;
    const DevBook *book;
    int n_tiles, n_cold, row_len;
};

constexpr int kApplyRound = 2;  // tiles per workgroup and round

__global__ __launch_bounds__(kFThreads) void k_apply(ApplyArgs p)
{
    constexpr int U = kApplyRound;
    const int tid = threadIdx.x, b = blockIdx.x, G = gridDim.x;
    const unsigned lane_off = (unsigned)tid * 16u;
    const float eta = p.book->st[book_epoch(p.book) & 1].eta_f32;  // the record k_scalars has just written
    auto locate = [&](int t) -> FLoc {
        const AS_CONST int *tp = (const AS_CONST int *)p.tiles + 2 * (size_t)t;
        return FLoc{(cp_u64)p.ptrs + (size_t)tp[0] * p.row_len, (unsigned long long)tp[1] * (kFTile * 4ULL)};
    };
    int t = b;
    for (; t + (U - 1) * G < p.n_tiles; t += U * G) {
        gp_char w[U];
        f4 wv[U], vv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const FLoc L = locate(t + u * G);
            w[u] = (gp_char)(L.row[kRowW] + L.tile_off) + lane_off;
            wv[u] = *(gp_cf4)w[u];
            vv[u] = *(gp_cf4)((gp_cchar)(L.row[kRowV] + L.tile_off) + lane_off);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            *(gp_f4)w[u] = f4{fmaf(-eta, vv[u].x, wv[u].x), fmaf(-eta, vv[u].y, wv[u].y), fmaf(-eta, vv[u].z, wv[u].z),
                              fmaf(-eta, vv[u].w, wv[u].w)};
    }
    for (; t < p.n_tiles; t += G) {  // the last, incomplete round
        const FLoc L = locate(t);
        gp_char w = (gp_char)(L.row[kRowW] + L.tile_off) + lane_off;
        const f4 wv = *(gp_cf4)w, vv = *(gp_cf4)((gp_cchar)(L.row[kRowV] + L.tile_off) + lane_off);
        *(gp_f4)w = f4{fmaf(-eta, vv.x, wv.x), fmaf(-eta, vv.y, wv.y), fmaf(-eta, vv.z, wv.z), fmaf(-eta, vv.w, wv.w)};
    }
    for (int c = b; c < p.n_cold; c += G) {  // ragged last tiles of the tensors
        const AS_CONST int *tp = (const AS_CONST int *)p.cold + 2 * (size_t)c;
        const int k = tp[0], local = tp[1];
        cp_u64 row = (cp_u64)p.ptrs + (size_t)k * p.row_len;
        const long long first = (long long)local * kFTile + (long long)tid * 4;
        const long long rem = ((const AS_CONST long long *)p.numel)[k] - first;
        if (rem <= 0) continue;
        AS_GLOBAL float *w = (AS_GLOBAL float *)row[kRowW] + first;
        const AS_GLOBAL float *v = (const AS_GLOBAL float *)row[kRowV] + first;
        const int n = rem < 4 ? (int)rem : 4;
        for (int e = 0; e < n; ++e) w[e] = fmaf(-eta, v[e], w[e]);
    }
}

// ---------------------------------------------------------------------------------------------
// Step on one flat tensor without a context (adascale_step_flat): every byte of device memory the
// kernels need beyond the caller's buffers -- the pointer row, two state records, the partial
// sums -- lies in one fixed block whose address the host passes in.  Three launches plus a set-up
// kernel: the gradient sweep leaves the new momentum in v (it does not depend on eta_t), k_scalars
// evaluates the estimator, the last kernel applies w <- w - eta_t v and hands the state back.
constexpr int kFlatMaxScale = 64;     // gradient pointers travel as a kernel argument
constexpr int kFlatMaxGrid = 2048;    // workgroups of the sweep = partial slots

struct FlatScratch {
    unsigned long long row[kRowG + kFlatMaxScale];  // [w, v, unused, g_0 .. g_{S-1}]
    DevBook book;                                   // st[0] / st[1]: before / after the step
    alignas(16) double partials[kFlatMaxGrid][2];   // k_scalars reads them as pairs
};

struct FlatPointers {
    unsigned long long w, v, g[kFlatMaxScale];
};

// The block keeps whatever the last call left in it: everything a call reads is written here or
// by its own sweep first (pointer row, the epoch -- zero, so that k_scalars reads record 0 and
// writes record 1 --, the state record of before the step, and, by the sweep, exactly the partial
// slots k_scalars is told to add).
__global__ void k_flat_setup(FlatScratch *sc, FlatPointers ptrs, int S, const adascale_state *user)
{
    const int tid = threadIdx.x;
    if (tid == 0) {
        sc->row[kRowW] = ptrs.w;
        sc->row[kRowV] = ptrs.v;
        sc->row[kRowGbar] = 0;
        DevState st{};
        st.step = user->step;
        st.tau = user->tau;
        st.sig_bar = user->sigma2_bar;
        st.mu_bar = user->mu2_bar;
        sc->book.epoch = 0;
        sc->book.st[0] = st;
    }
    if (tid < S) sc->row[kRowG + tid] = ptrs.g[tid];
}

template <typename GT, int HG>
__global__ __launch_bounds__(kThreads) void k_flat_sweep(FlatScratch *sc, long long numel, int n_tiles, int S,
                                                         double inv_S, float rho, float lambda)
{
    constexpr int VEC = Traits<GT>::VEC;
    constexpr int TILE = kThreads * VEC;
    const int tid = threadIdx.x;
    __shared__ double sh[kWaves][2];
    const unsigned long long *row = sc->row;
    double acc_a = 0.0, acc_b = 0.0;
    for (int t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const long long base = (long long)t * TILE + (long long)tid * VEC;
        const long long rem = numel - base;
        if (rem <= 0) continue;
        const float *w = reinterpret_cast<const float *>(row[kRowW]) + base;
        float *v = reinterpret_cast<float *>(row[kRowV]) + base;
        if (rem >= VEC) {
            float wv[VEC], vv[VEC], gv[VEC];
            load_f32<VEC>(v, vv);
            if (lambda != 0.f) load_f32<VEC>(w, wv);
            reduce_lane_full<GT, HG>(row, base, S, inv_S, gv, acc_a, acc_b);
#pragma unroll
            for (int e = 0; e < VEC; ++e) vv[e] = fmaf(rho, vv[e], lambda != 0.f ? fmaf(lambda, wv[e], gv[e]) : gv[e]);
            store_f32<VEC>(v, vv);
        } else {
            for (int e = 0; e < (int)rem; ++e) {
                const float g = reduce_element<GT>(row, base + e, S, inv_S, acc_a, acc_b);
                v[e] = fmaf(rho, v[e], lambda != 0.f ? fmaf(lambda, w[e], g) : g);
            }
        }
    }
    reduce_store_partial(acc_a, acc_b, sh, &sc->partials[0][0], blockIdx.x);
}

template <int VEC>
__global__ __launch_bounds__(kThreads) void k_flat_finish(const FlatScratch *sc, long long numel, int n_tiles,
                                                          adascale_state *user)
{
    constexpr int TILE = kThreads * VEC;
    const int tid = threadIdx.x;
    const DevState &st = sc->book.st[1];
    const float eta = st.eta_f32;
    float *wp = reinterpret_cast<float *>(sc->row[kRowW]);
    const float *vp = reinterpret_cast<const float *>(sc->row[kRowV]);
    for (int t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const long long base = (long long)t * TILE + (long long)tid * VEC;
        const long long rem = numel - base;
        if (rem <= 0) continue;
        if (rem >= VEC) {
            float wv[VEC], vv[VEC];
            load_f32<VEC>(wp + base, wv);
            load_f32<VEC>(vp + base, vv);
#pragma unroll
            for (int e = 0; e < VEC; ++e) wv[e] = fmaf(-eta, vv[e], wv[e]);
            store_f32<VEC>(wp + base, wv);
        } else {
            for (int e = 0; e < (int)rem; ++e) wp[base + e] = fmaf(-eta, vp[base + e], wp[base + e]);
        }
    }
    if (blockIdx.x == 0 && tid == 0) {
        user->step = st.step;
        user->tau = st.tau;
        user->r = st.r;
        user->lr_eff = st.lr_eff;
        user->sum_sq = st.A;
        user->sq_mean = st.B;
        user->sigma2_hat = st.sig_hat;
        user->mu2_hat = st.mu_hat;
        user->sigma2_bar = st.sig_bar;
        user->mu2_bar = st.mu_bar;
        user->done = st.done;
    }
}

// Register-slot counts the fused kernel is instantiated for (the host uses the largest one that
// every workgroup can fill).
constexpr int kFRegLevels = 4;
constexpr int fused_regs_at(int level) { return level == 0 ? 0 : level == 1 ? 10 : level == 2 ? 30 : kFRegTiles; }
constexpr int kFMaxScaleF32 = 32, kFMaxScaleBf16 = 64;  // largest scales with a compile-time shape
constexpr int kStreamMaxScale = 4096;                   // largest scale of the run-time shapes

// Half-group shape (HG, NH) of the 512-lane kernels for a gradient type and scale; false: none.
// The count is the smallest even one that covers S; 2, 4 and 8 are template parameters, any other
// count is taken at run time (one more instance per kernel family and gradient type).
inline bool fused_shape(int dtype, int S, int *hg, int *nh)
{
    if (S < 1 || S > kStreamMaxScale) return false;
    // fp32: half-groups of up to 4 16-byte loads; bf16: 8-byte loads, so twice the replicas per
    // half-group for the same bytes in flight
    const int cap = dtype == ADASCALE_F32 ? 4 : 8;
    int h = 1;
    while (h < cap && 2 * h < S) h *= 2;  // smallest HG with 2 * HG >= S, at most cap
    *hg = h;
    *nh = 2 * ((S + 2 * h - 1) / (2 * h));
    return true;
}

inline int padded_scale(int dtype, int S)
{
    int hg = 0, nh = 0;
    return fused_shape(dtype, S, &hg, &nh) ? hg * nh : S;
}

template <int LEVEL, bool LAG>
const void *fused_kernel_at(int dtype, int S)
{
#define KF(GT, HG, NH, MASK) reinterpret_cast<const void *>(k_fused<GT, HG, NH, MASK, fused_regs_at(LEVEL), LAG>)
    int hg = 0, nh = 0;
    if (!fused_shape(dtype, S, &hg, &nh)) return nullptr;
    if (nh != 2 && nh != 4 && nh != 8) return dtype == ADASCALE_F32 ? KF(float, 4, 0, true) : KF(Bf16, 8, 0, true);
    const bool exact = hg * nh == S;
    if (dtype == ADASCALE_F32) {
        switch (hg * 100 + nh) {
        case 102: return exact ? KF(float, 1, 2, false) : KF(float, 1, 2, true);
        case 202: return exact ? KF(float, 2, 2, false) : KF(float, 2, 2, true);
        case 402: return exact ? KF(float, 4, 2, false) : KF(float, 4, 2, true);
        case 404: return exact ? KF(float, 4, 4, false) : KF(float, 4, 4, true);
        case 408: return KF(float, 4, 8, true);
        default: return nullptr;
        }
    }
    switch (hg * 100 + nh) {
    case 102: return KF(Bf16, 1, 2, true);
    case 202: return KF(Bf16, 2, 2, true);
    case 402: return KF(Bf16, 4, 2, true);
    case 802: return KF(Bf16, 8, 2, true);
    case 804: return KF(Bf16, 8, 4, true);
    case 808: return KF(Bf16, 8, 8, true);
    default: return nullptr;
    }
#undef KF
}

}  // namespace
