// AdaScale SGD step for MI355X (gfx950): HIP kernels and the C ABI declared in adascale.h.
//
// One step is three launches on the caller's stream, none of which needs the host:
//   reduce  : one streaming pass over the S gradient buffers; writes the mean gradient
//             (Sec. 2, Algorithm 1) and per-wave fp64 partial sums of A = sum_i ||g_i||^2
//             and B = ||gbar||^2 (App. B.3);
//   scalars : one workgroup sums the partials in a fixed order and evaluates the estimates,
//             clamps, moving averages, gain ratio r_t, eta_t and tau (App. B.3, eq. 3, Sec. 3.2);
//   update  : v <- rho v + gbar + lambda w, w <- w - eta_t v with eta_t read from device memory.
// The path is bandwidth bound (about half a flop per byte), so there is no matrix-core work:
// the kernels are 16-byte-per-lane coalesced streams, 64-lane shuffle reductions and fp64
// accumulation of exact squares.
//
// Work decomposition: every tensor is cut into tiles of 256 lanes x 16 bytes of gradient; the
// tiles of all tensors form one list, cut into spans of `span_tiles` consecutive tiles.  A
// workgroup handles whole spans and every workgroup writes its span partial to a slot fixed by
// the span, so the reduction result does not depend on scheduling.

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "adascale.h"

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
constexpr int kRing = 4;  // pinned staging slots for pointer-table uploads

struct DevState {
    long long step;
    double tau, r, lr_eff, A, B, sig_hat, mu_hat, sig_bar, mu_bar;
    float eta_f32;
    int done;
};

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

// One 16-byte gradient load, unpacked to VEC floats.
__device__ __forceinline__ void load_grad_vec(const float *p, float (&x)[4])
{
#if ADASCALE_NT_LOADS
    f4 t = __builtin_nontemporal_load((gp_cf4)(p));
#else
    f4 t = *(gp_cf4)(p);
#endif
    x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
}
__device__ __forceinline__ void load_grad_vec(const Bf16 *p, float (&x)[8])
{
#if ADASCALE_NT_LOADS
    u4 t = __builtin_nontemporal_load((gp_cu4)(p));
#else
    u4 t = *(gp_cu4)(p);
#endif
    const unsigned w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        x[2 * j] = __uint_as_float(w[j] << 16);
        x[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
    }
}

template <int VEC>
__device__ __forceinline__ void load_f32(const float *p, float (&x)[VEC])
{
#pragma unroll
    for (int q = 0; q < VEC / 4; ++q) {
        f4 t = *(gp_cf4)(p + 4 * q);
        x[4 * q] = t.x; x[4 * q + 1] = t.y; x[4 * q + 2] = t.z; x[4 * q + 3] = t.w;
    }
}
template <int VEC>
__device__ __forceinline__ void store_f32(float *p, const float (&x)[VEC])
{
#pragma unroll
    for (int q = 0; q < VEC / 4; ++q) {
        f4 t = {x[4 * q], x[4 * q + 1], x[4 * q + 2], x[4 * q + 3]};
        *(gp_f4)(p + 4 * q) = t;
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
// reduce: mean gradient + partial sums of A and B.  G = replicas loaded per batch of loads.
template <typename GT, int G>
__global__ __launch_bounds__(kThreads) void k_reduce(const int *__restrict__ span_first,
                                                     const int *__restrict__ tile_prefix,
                                                     const long long *__restrict__ numel,
                                                     const unsigned long long *__restrict__ ptrs,
                                                     double *__restrict__ partials, int n_tiles,
                                                     int span_tiles, int n_spans, int S, double inv_S)
{
    constexpr int VEC = Traits<GT>::VEC;
    constexpr int TILE = kThreads * VEC;
    const int tid = threadIdx.x;
    const int row_len = S + kRowG;
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

            double s[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) s[e] = 0.0;
            double a = 0.0;

            if (rem >= VEC) {
                for (int i0 = 0; i0 < S; i0 += G) {
                    float x[G][VEC];
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        const int i = min(i0 + g, S - 1);  // past-the-end slots re-read the last replica
                        load_grad_vec(reinterpret_cast<const GT *>(row[kRowG + i]) + base, x[g]);
                    }
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        const bool live = (i0 + g) < S;
#pragma unroll
                        for (int e = 0; e < VEC; ++e) {
                            const double xd = live ? (double)x[g][e] : 0.0;
                            s[e] += xd;
                            a = fma(xd, xd, a);
                        }
                    }
                }
                float out[VEC];
                double b = 0.0;
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const double m = s[e] * inv_S;
                    out[e] = (float)m;
                    b = fma(m, m, b);
                }
                store_f32<VEC>(gbar, out);
                acc_a += a;
                acc_b += b;
            } else {  // ragged end of a tensor: element by element
                const int c = (int)rem;
                double b = 0.0;
                for (int e = 0; e < c; ++e) {
                    double se = 0.0;
                    for (int i = 0; i < S; ++i) {
                        const double xd = (double)widen(reinterpret_cast<const GT *>(row[kRowG + i])[base + e]);
                        se += xd;
                        a = fma(xd, xd, a);
                    }
                    const double m = se * inv_S;
                    gbar[e] = (float)m;
                    b = fma(m, m, b);
                }
                acc_a += a;
                acc_b += b;
            }
        }

        acc_a = wave_sum(acc_a);
        acc_b = wave_sum(acc_b);
        if ((tid & (kWave - 1)) == 0) {
            sh[tid >> 6][0] = acc_a;
            sh[tid >> 6][1] = acc_b;
        }
        __syncthreads();
        if (tid < 2) {  // fixed order over the waves
            double t = sh[0][tid];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) t += sh[w][tid];
            partials[(size_t)span * 2 + tid] = t;
        }
        __syncthreads();
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

constexpr int kScalarThreads = 1024;

__global__ __launch_bounds__(kScalarThreads) void k_scalars(const double *__restrict__ partials, int n_partials,
                                                            DevState *__restrict__ st, const float *__restrict__ lr,
                                                            ScalarArgs c)
{
    __shared__ double sh_a[kScalarThreads], sh_b[kScalarThreads];
    const int tid = threadIdx.x;
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
    if (tid != 0) return;

    const double A = sh_a[0], B = sh_b[0];
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
    const long long k = st->step + 1;
    const double alpha = fmax(1.0 - c.theta, 1.0 / (double)k);
    double sbar = st->sig_bar, mbar = st->mu_bar;
    double r = 1.0;
    if (c.flags & ADASCALE_LAGGED_R) r = st->step == 0 ? 1.0 : gain_from(c, sbar, mbar);
    sbar += alpha * (x1 - sbar);
    mbar += alpha * (x2 - mbar);
    if (!(c.flags & ADASCALE_LAGGED_R)) r = gain_from(c, sbar, mbar);

    const double tau = st->tau;
    long long idx = (long long)floor(tau);
    if (idx > c.L - 1) idx = c.L - 1;
    if (idx < 0) idx = 0;
    const double eta = r * (double)lr[idx];

    st->A = A;
    st->B = B;
    st->sig_hat = sig;
    st->mu_hat = mu;
    st->sig_bar = sbar;
    st->mu_bar = mbar;
    st->r = r;
    st->lr_eff = eta;
    st->eta_f32 = (float)eta;
    st->tau = tau + r;
    st->step = k;
    st->done = (tau + r) >= (double)c.L;
}

// ---------------------------------------------------------------------------------------------
// update: momentum-SGD with eta_t taken from device memory.
template <int VEC>
__global__ __launch_bounds__(kThreads) void k_update(const int *__restrict__ span_first,
                                                     const int *__restrict__ tile_prefix,
                                                     const long long *__restrict__ numel,
                                                     const unsigned long long *__restrict__ ptrs,
                                                     const DevState *__restrict__ st, int n_tiles, int span_tiles,
                                                     int n_spans, int row_len, float rho, float lambda,
                                                     int reverse)
{
    constexpr int TILE = kThreads * VEC;
    const int tid = threadIdx.x;
    const float eta = st->eta_f32;

    for (int sp = blockIdx.x; sp < n_spans; sp += gridDim.x) {
        // reverse: start with the spans whose mean gradient was written last
        const int span = reverse ? n_spans - 1 - sp : sp;
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

__global__ void k_set_state(DevState *st, long long step, double tau, double sbar, double mbar, long long L)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        st->step = step;
        st->tau = tau;
        st->sig_bar = sbar;
        st->mu_bar = mbar;
        st->done = tau >= (double)L;
    }
}

thread_local char g_init_error[256] = "";

}  // namespace

// ---------------------------------------------------------------------------------------------
struct adascale_ctx {
    adascale_config cfg{};
    std::vector<long long> numel;
    std::vector<int> tile_prefix;   // [N+1]
    std::vector<int> span_first;    // [n_spans]
    std::vector<size_t> gbar_off;   // element offset of tensor k in the mean-gradient scratch
    long long d = 0;
    int vec = 4, tile = 1024;
    int n_tiles = 0, span_tiles = 2, n_spans = 0, max_blocks = 1 << 30, group = 0;
    int update_reverse = 0;
    int S_cap = 0;                  // pointer table capacity in replicas

    int *d_span_first = nullptr, *d_tile_prefix = nullptr;
    long long *d_numel = nullptr;
    unsigned long long *d_ptrs = nullptr;
    float *d_gbar = nullptr, *d_lr = nullptr;
    double *d_partials = nullptr;
    DevState *d_state = nullptr;

    DevState *h_state = nullptr;    // pinned
    unsigned long long *h_ring[kRing] = {};
    hipEvent_t ring_ev[kRing] = {};
    bool ring_used[kRing] = {};
    int ring_next = 0;
    std::vector<unsigned long long> last_table;  // what the device table holds
    bool table_valid = false;

    std::vector<hipEvent_t> prof_ev;  // 4 per recorded step
    int prof_cap = 0, prof_n = 0;
    bool prof_on = false;

    char err[256] = "";
};

namespace {

int fail(adascale_ctx *c, int code, const char *fmt, ...)
{
    char *dst = c ? c->err : g_init_error;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 256, fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(ctx, call)                                                                         \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess) return fail(ctx, ADASCALE_EHIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

int env_int(const char *name, int dflt)
{
    const char *s = getenv(name);
    if (!s || !*s) return dflt;
    const long v = strtol(s, nullptr, 10);
    return v > 0 ? (int)v : dflt;
}

size_t table_len(const adascale_ctx *c, int S) { return (size_t)c->numel.size() * (size_t)(S + kRowG); }

int alloc_pointer_tables(adascale_ctx *c, int S)
{
    if (S <= c->S_cap) return ADASCALE_OK;
    const size_t bytes = std::max<size_t>(table_len(c, S), 1) * sizeof(unsigned long long);
    if (c->d_ptrs) {
        HIP_TRY(c, hipDeviceSynchronize());
        HIP_TRY(c, hipFree(c->d_ptrs));
        c->d_ptrs = nullptr;
    }
    for (int i = 0; i < kRing; ++i) {
        if (c->h_ring[i]) HIP_TRY(c, hipHostFree(c->h_ring[i]));
        c->h_ring[i] = nullptr;
        c->ring_used[i] = false;
    }
    HIP_TRY(c, hipMalloc(&c->d_ptrs, bytes));
    for (int i = 0; i < kRing; ++i) HIP_TRY(c, hipHostMalloc(&c->h_ring[i], bytes, hipHostMallocDefault));
    c->S_cap = S;
    c->table_valid = false;
    return ADASCALE_OK;
}

// Is [p, p + bytes) inside one device allocation on this device?  `lo`/`hi` cache the last range.
bool device_range_ok(const void *p, size_t bytes, int device, uintptr_t &lo, uintptr_t &hi)
{
    const uintptr_t a = (uintptr_t)p;
    if (a >= lo && a + bytes <= hi) return true;
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged) return false;
    if (attr.type == hipMemoryTypeDevice && attr.device != device) return false;
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    if (hipMemGetAddressRange(&base, &size, const_cast<void *>(p)) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    lo = (uintptr_t)base;
    hi = lo + size;
    return a >= lo && a + bytes <= hi;
}

template <typename GT>
void launch_reduce(const adascale_ctx *c, int grid, hipStream_t s, int S)
{
    const double inv_S = 1.0 / (double)S;
    int G = c->group;
    if (G <= 0) G = S >= 16 ? 16 : S >= 8 ? 8 : S >= 4 ? 4 : S >= 2 ? 2 : 1;
#define LAUNCH(GG)                                                                                   \
    hipLaunchKernelGGL((k_reduce<GT, GG>), dim3(grid), dim3(kThreads), 0, s, c->d_span_first,        \
                       c->d_tile_prefix, c->d_numel, c->d_ptrs, c->d_partials, c->n_tiles,           \
                       c->span_tiles, c->n_spans, S, inv_S)
    if (G >= 16) LAUNCH(16);
    else if (G >= 8) LAUNCH(8);
    else if (G >= 4) LAUNCH(4);
    else if (G >= 2) LAUNCH(2);
    else LAUNCH(1);
#undef LAUNCH
}

}  // namespace

// ---------------------------------------------------------------------------------------------
extern "C" {

const char *adascale_last_error(const adascale_ctx *ctx) { return ctx ? ctx->err : g_init_error; }

int64_t adascale_step_bytes(const adascale_ctx *c)
{
    if (!c) return 0;
    const int64_t b = c->cfg.grad_dtype == ADASCALE_F32 ? 4 : 2;
    return (int64_t)c->cfg.S * c->d * b + 24 * c->d;
}

int adascale_init(const adascale_config *cfg, adascale_ctx **out)
{
    if (out) *out = nullptr;
    if (!cfg || !out) return fail(nullptr, ADASCALE_EINVAL, "null cfg or out");
    if (cfg->S < 1) return fail(nullptr, ADASCALE_EINVAL, "S must be >= 1");
    if (cfg->n_tensors < 0 || (cfg->n_tensors > 0 && !cfg->numel))
        return fail(nullptr, ADASCALE_EINVAL, "bad tensor list");
    if (cfg->grad_dtype != ADASCALE_F32 && cfg->grad_dtype != ADASCALE_BF16)
        return fail(nullptr, ADASCALE_EINVAL, "unknown gradient dtype");
    if (!(cfg->momentum >= 0.0 && cfg->momentum < 1.0)) return fail(nullptr, ADASCALE_EINVAL, "momentum outside [0,1)");
    if (!(cfg->weight_decay >= 0.0)) return fail(nullptr, ADASCALE_EINVAL, "negative weight decay");
    if (!(cfg->theta < 1.0)) return fail(nullptr, ADASCALE_EINVAL, "theta must be < 1");
    if (!cfg->lr_table || cfg->lr_table_len < 1) return fail(nullptr, ADASCALE_EINVAL, "empty lr table");
    if (cfg->flags & ~(ADASCALE_LAGGED_R | ADASCALE_EST_NORM_RATIO | ADASCALE_NO_POINTER_CHECK))
        return fail(nullptr, ADASCALE_EINVAL, "unknown flag bits");
    for (int k = 0; k < cfg->n_tensors; ++k)
        if (cfg->numel[k] < 0) return fail(nullptr, ADASCALE_EINVAL, "negative numel");

    adascale_ctx *c = new (std::nothrow) adascale_ctx();
    if (!c) return fail(nullptr, ADASCALE_ENOMEM, "host allocation failed");
    c->cfg = *cfg;
    c->cfg.numel = nullptr;
    c->cfg.lr_table = nullptr;
    if (c->cfg.theta < 0.0) c->cfg.theta = std::max(1.0 - cfg->S / 1000.0, 0.0);
    if (c->cfg.eps <= 0.0) c->cfg.eps = 1e-6;
    c->vec = cfg->grad_dtype == ADASCALE_F32 ? 4 : 8;
    c->tile = kThreads * c->vec;
    c->span_tiles = env_int("ADASCALE_SPAN_TILES", 2);
    c->max_blocks = env_int("ADASCALE_MAX_BLOCKS", 1 << 30);
    c->group = env_int("ADASCALE_GROUP", 0);
    c->update_reverse = env_int("ADASCALE_UPDATE_REVERSE", 0);

    const int N = cfg->n_tensors;
    c->numel.assign(cfg->numel, cfg->numel + N);
    c->tile_prefix.assign(N + 1, 0);
    c->gbar_off.assign(N, 0);
    size_t goff = 0;
    long long tiles = 0;
    for (int k = 0; k < N; ++k) {
        c->d += c->numel[k];
        tiles += (c->numel[k] + c->tile - 1) / c->tile;
        if (tiles > 0x7fffff00LL) {
            delete c;
            return fail(nullptr, ADASCALE_EINVAL, "parameter list too large");
        }
        c->tile_prefix[k + 1] = (int)tiles;
        c->gbar_off[k] = goff;
        goff += ((size_t)c->numel[k] + 63) / 64 * 64;  // 256-byte aligned starts
    }
    c->n_tiles = (int)tiles;
    c->n_spans = (c->n_tiles + c->span_tiles - 1) / c->span_tiles;
    c->span_first.assign(std::max(c->n_spans, 1), 0);
    for (int s = 0, k = 0; s < c->n_spans; ++s) {
        const int t = s * c->span_tiles;
        while (t >= c->tile_prefix[k + 1]) ++k;
        c->span_first[s] = k;
    }

    int rc = ADASCALE_OK;
    auto body = [&]() -> int {
        int ndev = 0;
        HIP_TRY(c, hipGetDeviceCount(&ndev));
        if (cfg->device < 0 || cfg->device >= ndev) return fail(c, ADASCALE_EINVAL, "no such device");
        HIP_TRY(c, hipSetDevice(cfg->device));
        HIP_TRY(c, hipMalloc(&c->d_span_first, sizeof(int) * c->span_first.size()));
        HIP_TRY(c, hipMalloc(&c->d_tile_prefix, sizeof(int) * (N + 1)));
        HIP_TRY(c, hipMalloc(&c->d_numel, sizeof(long long) * std::max(N, 1)));
        HIP_TRY(c, hipMalloc(&c->d_gbar, sizeof(float) * std::max<size_t>(goff, 64)));
        HIP_TRY(c, hipMalloc(&c->d_lr, sizeof(float) * cfg->lr_table_len));
        HIP_TRY(c, hipMalloc(&c->d_partials, sizeof(double) * 2 * std::max(c->n_spans, 1)));
        HIP_TRY(c, hipMalloc(&c->d_state, sizeof(DevState)));
        HIP_TRY(c, hipHostMalloc(&c->h_state, sizeof(DevState), hipHostMallocDefault));
        for (int i = 0; i < kRing; ++i) HIP_TRY(c, hipEventCreateWithFlags(&c->ring_ev[i], hipEventDisableTiming));
        HIP_TRY(c, hipMemcpy(c->d_span_first, c->span_first.data(), sizeof(int) * c->span_first.size(),
                             hipMemcpyHostToDevice));
        HIP_TRY(c, hipMemcpy(c->d_tile_prefix, c->tile_prefix.data(), sizeof(int) * (N + 1), hipMemcpyHostToDevice));
        if (N > 0)
            HIP_TRY(c, hipMemcpy(c->d_numel, c->numel.data(), sizeof(long long) * N, hipMemcpyHostToDevice));
        HIP_TRY(c, hipMemcpy(c->d_lr, cfg->lr_table, sizeof(float) * cfg->lr_table_len, hipMemcpyHostToDevice));
        HIP_TRY(c, hipMemset(c->d_state, 0, sizeof(DevState)));
        HIP_TRY(c, hipMemset(c->d_partials, 0, sizeof(double) * 2 * std::max(c->n_spans, 1)));
        return alloc_pointer_tables(c, cfg->S);
    };
    rc = body();
    if (rc != ADASCALE_OK) {
        snprintf(g_init_error, sizeof g_init_error, "%s", c->err);
        adascale_destroy(c);
        return rc;
    }
    *out = c;
    return ADASCALE_OK;
}

void adascale_destroy(adascale_ctx *c)
{
    if (!c) return;
    (void)hipSetDevice(c->cfg.device);
    (void)hipDeviceSynchronize();
    (void)hipFree(c->d_span_first);
    (void)hipFree(c->d_tile_prefix);
    (void)hipFree(c->d_numel);
    (void)hipFree(c->d_ptrs);
    (void)hipFree(c->d_gbar);
    (void)hipFree(c->d_lr);
    (void)hipFree(c->d_partials);
    (void)hipFree(c->d_state);
    if (c->h_state) (void)hipHostFree(c->h_state);
    for (int i = 0; i < kRing; ++i) {
        if (c->h_ring[i]) (void)hipHostFree(c->h_ring[i]);
        if (c->ring_ev[i]) (void)hipEventDestroy(c->ring_ev[i]);
    }
    for (hipEvent_t e : c->prof_ev) (void)hipEventDestroy(e);
    delete c;
}

int adascale_set_scale(adascale_ctx *c, int32_t S_new, double theta)
{
    if (!c) return ADASCALE_EINVAL;
    if (S_new < 1) return fail(c, ADASCALE_EINVAL, "S must be >= 1");
    if (!(theta < 1.0)) return fail(c, ADASCALE_EINVAL, "theta must be < 1");
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    const int rc = alloc_pointer_tables(c, S_new);
    if (rc != ADASCALE_OK) return rc;
    c->cfg.S = S_new;
    c->cfg.theta = theta < 0.0 ? std::max(1.0 - S_new / 1000.0, 0.0) : theta;
    c->table_valid = false;
    return ADASCALE_OK;
}

int adascale_set_state(adascale_ctx *c, int64_t step, double tau, double sigma2_bar, double mu2_bar, void *hip_stream)
{
    if (!c) return ADASCALE_EINVAL;
    if (step < 0 || !(tau >= 0.0) || !(sigma2_bar >= 0.0) || !(mu2_bar >= 0.0))
        return fail(c, ADASCALE_EINVAL, "state values must be non-negative");
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    hipLaunchKernelGGL(k_set_state, dim3(1), dim3(64), 0, (hipStream_t)hip_stream, c->d_state, (long long)step, tau,
                       sigma2_bar, mu2_bar, (long long)c->cfg.lr_table_len);
    HIP_TRY(c, hipGetLastError());
    return ADASCALE_OK;
}

int adascale_get_state(adascale_ctx *c, adascale_state *out, void *hip_stream)
{
    if (!c) return ADASCALE_EINVAL;
    if (!out) return fail(c, ADASCALE_EINVAL, "null out");
    hipStream_t s = (hipStream_t)hip_stream;
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    HIP_TRY(c, hipMemcpyAsync(c->h_state, c->d_state, sizeof(DevState), hipMemcpyDeviceToHost, s));
    HIP_TRY(c, hipStreamSynchronize(s));
    const DevState &h = *c->h_state;
    out->step = h.step;
    out->tau = h.tau;
    out->r = h.r;
    out->lr_eff = h.lr_eff;
    out->sum_sq = h.A;
    out->sq_mean = h.B;
    out->sigma2_hat = h.sig_hat;
    out->mu2_hat = h.mu_hat;
    out->sigma2_bar = h.sig_bar;
    out->mu2_bar = h.mu_bar;
    out->done = h.done;
    return ADASCALE_OK;
}

int adascale_step(adascale_ctx *c, void *const *w, void *const *mom, const void *const *grads, void *hip_stream)
{
    if (!c) return ADASCALE_EINVAL;
    const int N = (int)c->numel.size();
    const int S = c->cfg.S;
    if (N > 0 && (!w || !mom || !grads)) return fail(c, ADASCALE_EINVAL, "null pointer array");
    hipStream_t s = (hipStream_t)hip_stream;
    HIP_TRY(c, hipSetDevice(c->cfg.device));

    // Build the device pointer table [N][3 + S] in a pinned slot; upload only when it changed.
    const int row_len = S + kRowG;
    const size_t len = table_len(c, S);
    if (len > 0) {
        int slot = c->ring_next;
        if (c->ring_used[slot]) HIP_TRY(c, hipEventSynchronize(c->ring_ev[slot]));
        unsigned long long *tab = c->h_ring[slot];
        for (int k = 0; k < N; ++k) {
            unsigned long long *row = tab + (size_t)k * row_len;
            row[kRowW] = (unsigned long long)(uintptr_t)w[k];
            row[kRowV] = (unsigned long long)(uintptr_t)mom[k];
            row[kRowGbar] = (unsigned long long)(uintptr_t)(c->d_gbar + c->gbar_off[k]);
            for (int i = 0; i < S; ++i) row[kRowG + i] = (unsigned long long)(uintptr_t)grads[(size_t)i * N + k];
        }
        const bool same = c->table_valid && c->last_table.size() == len &&
                          memcmp(c->last_table.data(), tab, len * sizeof(unsigned long long)) == 0;
        if (!same) {
            const size_t gb = c->cfg.grad_dtype == ADASCALE_F32 ? 4 : 2;
            uintptr_t lo = 1, hi = 0;
            for (int k = 0; k < N; ++k) {
                if (c->numel[k] == 0) continue;
                const unsigned long long *row = tab + (size_t)k * row_len;
                for (int j = 0; j < row_len; ++j) {
                    if (j == kRowGbar) continue;
                    if (!row[j]) return fail(c, ADASCALE_EINVAL, "null tensor pointer (tensor %d, slot %d)", k, j);
                    const size_t eb = j < kRowG ? 4 : gb;
                    if (row[j] % eb) return fail(c, ADASCALE_EINVAL, "misaligned tensor pointer (tensor %d, slot %d)", k, j);
                    if (!(c->cfg.flags & ADASCALE_NO_POINTER_CHECK) &&
                        !device_range_ok((const void *)(uintptr_t)row[j], (size_t)c->numel[k] * eb, c->cfg.device, lo, hi))
                        return fail(c, ADASCALE_EINVAL, "tensor %d, slot %d: not device memory of %lld elements", k, j,
                                    c->numel[k]);
                }
            }
            HIP_TRY(c, hipMemcpyAsync(c->d_ptrs, tab, len * sizeof(unsigned long long), hipMemcpyHostToDevice, s));
            HIP_TRY(c, hipEventRecord(c->ring_ev[slot], s));
            c->ring_used[slot] = true;
            c->ring_next = (slot + 1) % kRing;
            c->last_table.assign(tab, tab + len);
            c->table_valid = true;
        }
    }

    hipEvent_t *pe = nullptr;
    if (c->prof_on && c->prof_n < c->prof_cap) pe = &c->prof_ev[(size_t)4 * c->prof_n++];
    if (pe) HIP_TRY(c, hipEventRecord(pe[0], s));
    const int grid = std::min(c->n_spans, c->max_blocks);
    if (grid > 0) {
        if (c->cfg.grad_dtype == ADASCALE_F32) launch_reduce<float>(c, grid, s, S);
        else launch_reduce<Bf16>(c, grid, s, S);
        HIP_TRY(c, hipGetLastError());
    }
    if (pe) HIP_TRY(c, hipEventRecord(pe[1], s));
    ScalarArgs sa{S, c->cfg.flags, c->cfg.theta, c->cfg.eps, (long long)c->cfg.lr_table_len};
    hipLaunchKernelGGL(k_scalars, dim3(1), dim3(kScalarThreads), 0, s, c->d_partials, c->n_spans,
                       c->d_state, c->d_lr, sa);
    HIP_TRY(c, hipGetLastError());
    if (pe) HIP_TRY(c, hipEventRecord(pe[2], s));
    if (grid > 0) {
        const float rho = (float)c->cfg.momentum, lambda = (float)c->cfg.weight_decay;
        if (c->vec == 4)
            hipLaunchKernelGGL((k_update<4>), dim3(grid), dim3(kThreads), 0, s, c->d_span_first, c->d_tile_prefix,
                               c->d_numel, c->d_ptrs, c->d_state, c->n_tiles, c->span_tiles, c->n_spans, row_len, rho,
                               lambda, c->update_reverse);
        else
            hipLaunchKernelGGL((k_update<8>), dim3(grid), dim3(kThreads), 0, s, c->d_span_first, c->d_tile_prefix,
                               c->d_numel, c->d_ptrs, c->d_state, c->n_tiles, c->span_tiles, c->n_spans, row_len, rho,
                               lambda, c->update_reverse);
        HIP_TRY(c, hipGetLastError());
    }
    if (pe) HIP_TRY(c, hipEventRecord(pe[3], s));
    return ADASCALE_OK;
}

int adascale_profile_begin(adascale_ctx *c, int32_t max_steps)
{
    if (!c) return ADASCALE_EINVAL;
    if (max_steps < 1 || max_steps > 100000) return fail(c, ADASCALE_EINVAL, "max_steps out of range");
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    while ((int)c->prof_ev.size() < 4 * max_steps) {
        hipEvent_t e;
        HIP_TRY(c, hipEventCreate(&e));
        c->prof_ev.push_back(e);
    }
    c->prof_cap = max_steps;
    c->prof_n = 0;
    c->prof_on = true;
    return ADASCALE_OK;
}

int adascale_profile_end(adascale_ctx *c, double ms[3], int32_t *n_steps)
{
    if (!c) return ADASCALE_EINVAL;
    if (!ms || !n_steps) return fail(c, ADASCALE_EINVAL, "null output");
    if (!c->prof_on) return fail(c, ADASCALE_ESTATE, "profiling is not on");
    c->prof_on = false;
    ms[0] = ms[1] = ms[2] = 0.0;
    *n_steps = c->prof_n;
    if (c->prof_n == 0) return ADASCALE_OK;
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    HIP_TRY(c, hipEventSynchronize(c->prof_ev[(size_t)4 * (c->prof_n - 1) + 3]));
    for (int i = 0; i < c->prof_n; ++i)
        for (int j = 0; j < 3; ++j) {
            float t = 0.f;
            HIP_TRY(c, hipEventElapsedTime(&t, c->prof_ev[(size_t)4 * i + j], c->prof_ev[(size_t)4 * i + j + 1]));
            ms[j] += t;
        }
    for (int j = 0; j < 3; ++j) ms[j] /= c->prof_n;
    return ADASCALE_OK;
}

}  // extern "C"
