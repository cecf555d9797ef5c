/*
 * adascale.h -- C ABI of the MI355X (gfx950) AdaScale SGD step.
 *
 * One call to adascale_step performs a whole iteration of AdaScale SGD (Algorithm 2,
 * Sec. 3.2) on one GPU, given the S per-batch gradients of that iteration:
 *
 *   gbar   = (1/S) sum_i g_i                               mean gradient, Sec. 2 / Algorithm 1
 *   A      = sum_i ||g_i||^2,  B = ||gbar||^2              App. B.3 (norms over ALL tensors)
 *   s2_hat = (A - S B) / (S - 1),  m2_hat = B - s2_hat / S App. B.3
 *   clamp s2_hat >= eps, m2_hat >= 0; theta-moving averages (plain mean of the samples
 *   while fewer than 1/(1-theta) exist)                    App. B.3
 *   r_t    = (s2_bar + m2_bar) / (s2_bar / S + m2_bar)     eq. (3) with the averages plugged in
 *   eta_t  = r_t * lr[min(floor(tau_t), L-1)]              Sec. 3.2
 *   v <- rho v + gbar + lambda w;  w <- w - eta_t v        momentum-SGD, Sec. 3.4
 *   tau_{t+1} = tau_t + r_t                                Sec. 3.2
 *
 * Everything runs in the library's own HIP kernels on the caller's stream; no call except
 * adascale_get_state waits for the device.  All functions return an ADASCALE_* code and
 * never throw, abort or print.  A context belongs to one device (each call makes it current while
 * it runs and leaves the caller's current device as it found it); calls on one context must
 * be issued in order on one stream at a time (the context owns scratch that consecutive
 * steps reuse), different contexts are independent.
 */
#ifndef ADASCALE_H
#define ADASCALE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct adascale_ctx adascale_ctx; /* opaque, owned by the library */

enum {
    ADASCALE_OK = 0,
    ADASCALE_EINVAL = 1, /* bad argument; nothing was launched or changed */
    ADASCALE_ENOMEM = 2, /* host or device allocation failed */
    ADASCALE_EHIP = 3,   /* a HIP runtime call failed; see adascale_last_error */
    ADASCALE_ESTATE = 4  /* call not valid in the context's current state */
};

enum { ADASCALE_F32 = 0, ADASCALE_BF16 = 1 }; /* gradient element type */

/* adascale_config.flags */
enum {
    /* r_t from the averages of PRIOR iterations only, r_0 = 1 (the variant App. B.3 says
     * its experiments used); eta_t is then known before the gradients are read, so the fused
     * step needs no grid barrier and the general step is a single sweep.  Default (flag
     * clear): current-iteration estimate, which App. B.3 recommends. */
    ADASCALE_LAGGED_R = 1u,
    /* Estimator of Sec. 3.4: moving averages m1 of A/S and m2 of B,
     * r_t = (m1 + eps) / (m2 + eps), instead of the (s2, m2) estimator of App. B.3. */
    ADASCALE_EST_NORM_RATIO = 2u,
    /* Skip the host-side check that every tensor pointer lies inside a device allocation
     * large enough for its tensor (done whenever the pointer set changes). */
    ADASCALE_NO_POINTER_CHECK = 4u,
    /* Launch the fused single-kernel step (see adascale_uses_fused_step) with
     * hipLaunchCooperativeKernel.  Its grid barrier needs every workgroup resident at once; the
     * grid is one workgroup per compute unit, so an ordinary launch (the default, about 15 us
     * cheaper per step) satisfies that as soon as the compute units are free, and the library
     * chains its own fused launches on a device so that two of them never hold half the chip
     * each.  Set this flag if the process runs OTHER grid-synchronising kernels concurrently on
     * the same device: the HIP runtime then serialises all of them.  In either mode the wait at
     * the barrier is bounded; if it ever gives up, adascale_get_state returns ADASCALE_ESTATE. */
    ADASCALE_COOPERATIVE_LAUNCH = 8u
};

typedef struct {
    int32_t S;              /* scale: number of gradient buffers per step, >= 1 (Sec. 2) */
    int32_t n_tensors;      /* N >= 0 parameter tensors */
    const int64_t *numel;   /* host [N], elements per tensor, each >= 0; copied */
    int32_t grad_dtype;     /* ADASCALE_F32 or ADASCALE_BF16; w and momentum are always fp32 */
    double momentum;        /* rho in [0, 1), constant across scales (Sec. 3.4) */
    double weight_decay;    /* lambda >= 0, coupled L2 added after the statistics are taken */
    double theta;           /* in [0, 1); negative selects max(1 - S/1000, 0) (Sec. 3.4) */
    double eps;             /* > 0; <= 0 selects 1e-6 (Sec. 3.4, App. B.3) */
    const float *lr_table;  /* host [lr_table_len], lr(0..L-1) of Sec. 2; copied to the device */
    int64_t lr_table_len;   /* L = T_SI >= 1, total scale-invariant iterations (Sec. 3.2) */
    int32_t device;         /* HIP device ordinal */
    uint32_t flags;         /* ADASCALE_* flag bits, 0 = default */
} adascale_config;

typedef struct {
    int64_t step;      /* iterations completed (= samples in the moving averages) */
    double tau;        /* tau_{t+1} after the last step; tau_0 = 0 */
    double r;          /* r_t used by the last step */
    double lr_eff;     /* eta_t = r_t * lr[min(floor(tau_t), L-1)] of the last step */
    double sum_sq;     /* A = sum_i ||g_i||^2 */
    double sq_mean;    /* B = ||gbar||^2 */
    double sigma2_hat; /* raw estimates of the last step, before clamping */
    double mu2_hat;
    double sigma2_bar; /* moving averages after the last step (m1, m2 with EST_NORM_RATIO) */
    double mu2_bar;
    int32_t done;      /* tau >= L: Algorithm 2 would stop; further steps use lr[L-1] */
} adascale_state;

/*
 * Create a context for a fixed parameter list (Algorithm 2's inputs S, lr, T_SI plus rho).
 * cfg and the arrays it points to are host memory, read during the call only.  Allocates the
 * device scratch (tile tables, reduction partials, state, lr table, a tile per tensor for the
 * mean gradient of ragged ends) on cfg->device.  On success *out receives the context; on
 * failure *out is NULL.
 * EINVAL: null cfg/out, S < 1, N < 0, negative numel, unknown dtype or flag, rho outside
 * [0,1), lambda < 0, theta >= 1, L < 1, null numel (N > 0) or lr_table.
 */
int adascale_init(const adascale_config *cfg, adascale_ctx **out);

/*
 * One AdaScale iteration, asynchronous on hip_stream (a hipStream_t; NULL = default stream).
 *   w, mom : host arrays [N] of DEVICE pointers to fp32 tensors (numel[k] contiguous
 *            elements), updated in place: mom is v of the momentum update.
 *   grads  : host array [S*N] of DEVICE pointers, grads[i*N + k] = replica i, tensor k,
 *            numel[k] contiguous elements of grad_dtype; read only.
 * Pointers need only element alignment (16-byte alignment is the fast case).  The host arrays
 * are copied before the call returns; the device tensors must stay valid, and the gradients
 * unmodified, until the stream work completes.  Never blocks on the device except when more
 * than a few distinct pointer sets are in flight at once, and allocates nothing except the
 * first time a context takes the general kernels (see adascale_step_path), which pass the whole
 * mean gradient through a scratch of d floats.  A tensor with numel 0 may have
 * null pointers.  EINVAL on a null required pointer, or (unless NO_POINTER_CHECK) a pointer
 * that is not device memory of sufficient extent; nothing is launched in that case.
 */
int adascale_step(adascale_ctx *ctx, void *const *w, void *const *mom, const void *const *grads,
                  void *hip_stream);

/*
 * Copy the scalar state (Algorithm 2's tau, the gain ratio, the estimates) to host memory.
 * Waits for the work queued on hip_stream; it is the only call that synchronises.
 */
int adascale_get_state(adascale_ctx *ctx, adascale_state *out, void *hip_stream);

/*
 * Overwrite the resumable part of the state: step count k, tau and the two moving averages
 * (the remaining fields of adascale_state are per-step diagnostics).  With (w, mom) this is
 * a full checkpoint.  Asynchronous on hip_stream.
 */
int adascale_set_state(adascale_ctx *ctx, int64_t step, double tau, double sigma2_bar, double mu2_bar,
                       void *hip_stream);

/*
 * Elastic AdaScaling (Sec. 4): change the scale to S_new between steps; tau and the moving
 * averages carry on.  theta < 0 selects max(1 - S_new/1000, 0).  The next adascale_step
 * expects S_new * N gradient pointers.  EINVAL if S_new < 1 or theta >= 1.
 */
int adascale_set_scale(adascale_ctx *ctx, int32_t S_new, double theta);

/* Free the context and its device scratch.  Waits for the device to go idle.  NULL is allowed. */
void adascale_destroy(adascale_ctx *ctx);

/* Message for the last non-OK code returned on this context (or by the last failed
 * adascale_init when ctx is NULL).  The string is owned by the library. */
const char *adascale_last_error(const adascale_ctx *ctx);

/* Algorithmic bytes one step moves for this context: S*d*b gradient bytes read once plus the
 * per-parameter traffic of a two-sweep step that keeps nothing on chip: 24 bytes (the new momentum
 * written and read back, v read, w read twice and written), 20 without weight decay, where the
 * first sweep does not need w.  For benchmarks; host only. */
int64_t adascale_step_bytes(const adascale_ctx *ctx);

/*
 * Which implementation the next adascale_step on this context runs; all compute the same thing
 * (the choice depends on the gradient type, the scale of the moment and the size of the
 * parameter list, and can be steered with the environment for tests and measurements):
 *   ADASCALE_PATH_FUSED      one persistent launch that keeps the mean gradient on chip as far
 *                            as it fits (S <= 4096 and at least a fifth of the mean
 *                            gradient fitting in registers + LDS);
 *   ADASCALE_PATH_STREAMING  three kernels (reduce, scalars, update), the first one a persistent
 *                            sweep in memory order: S <= 4096, parameter lists far larger than
 *                            the chip;
 *   ADASCALE_PATH_GENERAL    three kernels for any scale (or two with ADASCALE_LAGGED_R: one
 *                            sweep that reduces and updates, then the scalars).
 */
enum { ADASCALE_PATH_GENERAL = 0, ADASCALE_PATH_FUSED = 1, ADASCALE_PATH_STREAMING = 2 };
int adascale_step_path(const adascale_ctx *ctx);

/* 1 if adascale_step_path is ADASCALE_PATH_FUSED, else 0. */
int adascale_uses_fused_step(const adascale_ctx *ctx);

/*
 * How the fused and streaming kernels consume the S gradients of a tile (Algorithm 1's sum over
 * the batches): in shape[1] half-groups of shape[0] loads each, alternating between two register
 * buffers; the pointer table rows are padded to shape[2] = shape[0] * shape[1] replica slots.
 * Host only, needs no device.  Returns a bit mask: 1 = the fused step has a kernel instance for
 * this gradient type and scale (at every register level, both gain variants), 2 = the streaming
 * reduce kernel has one; 0 (shape untouched) if the scale is outside their range, in which case
 * the general kernels run.  For tests and diagnostics.
 */
int adascale_kernel_shape(int32_t grad_dtype, int32_t S, int32_t shape[3]);

/*
 * What adascale_init would decide for cfg's parameter list, gradient type, scale and flags on a
 * device with `compute_units` compute units and `lds_bytes` of LDS per workgroup (MI355X: 256 and
 * 163840): how the list splits into whole 512-lane tiles (2048 elements, inside one tensor) and
 * ragged last tiles, the grids, how many tiles of the mean gradient each workgroup of the fused
 * step keeps in registers and in LDS, and the path.  Host only: no device is touched, cfg's
 * lr_table, device and the optimizer constants are not read.  The fields of a path that does not
 * apply are 0.  (adascale_init additionally asks the runtime whether the fused grid can be
 * resident at once; on MI355X it can.)  For tests and diagnostics.
 */
typedef struct {
    int64_t full_tiles, ragged_tiles;
    int32_t path;                 /* ADASCALE_PATH_* */
    int32_t fused_grid;           /* workgroups of the fused step, one per compute unit at most */
    int32_t tiles_per_workgroup;  /* whole tiles per workgroup, rounded up */
    int32_t register_tiles;       /* of those, kept in registers ... */
    int32_t lds_tiles;            /* ... and in LDS; the rest passes through memory */
    int32_t on_chip_percent;
    int32_t stream_grid;          /* workgroups of the streaming reduce kernel */
} adascale_plan_info;
int adascale_plan(const adascale_config *cfg, int32_t compute_units, int64_t lds_bytes, adascale_plan_info *out);

/*
 * Benchmark instrumentation: while profiling is on, every adascale_step also records HIP
 * events on its stream before and after each of its kernels (up to max_steps steps).
 * adascale_profile_end waits for the stream work, writes the average duration in
 * milliseconds of the reduce, scalars and update kernels over the recorded steps to ms[0..2]
 * (a fused step reports its single kernel in ms[0])
 * and the number of recorded steps to *n_steps, and turns profiling off.
 */
int adascale_profile_begin(adascale_ctx *ctx, int32_t max_steps);
int adascale_profile_end(adascale_ctx *ctx, double ms[3], int32_t *n_steps);

#ifdef __cplusplus
}
#endif
#endif /* ADASCALE_H */
