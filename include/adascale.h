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
 * adascale_get_state waits for the device (adascale_set_scale may, see there).  What a call does
 * depends on its arguments alone: the library reads no environment variables.  Diagnostics,
 * benchmark instrumentation and the knobs the tests steer the choice of kernels with are declared
 * in adascale_diag.h.  All functions return an ADASCALE_* code and
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
     * its experiments used); eta_t is then known before the gradients are read, so the general
     * step is a single sweep and the fused step runs without its grid barrier where that is the
     * faster form (small parameter lists).  Default (flag clear): current-iteration estimate,
     * which App. B.3 recommends. */
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
     * the same device, or if OTHER PROCESSES run such kernels (this library's fused step included)
     * on the same device: the chaining is per process, and two grids that each hold part of the
     * chip and wait for the rest can only be told apart by the runtime.  In either mode the wait
     * at the barrier is bounded (a few seconds); what happens when it gives up is described at
     * adascale_get_state. */
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
 * than a few distinct pointer sets are in flight at once (the device keeps the tables of the last
 * eight pointer sets, so a caller that alternates between a few sets of buffers uploads nothing),
 * and allocates nothing except the first time a context takes the general kernels (scales above
 * 4096, see adascale_diag.h), which pass the whole mean gradient through a scratch of d floats.
 * A tensor with numel 0 may have
 * null pointers.  EINVAL on a null required pointer, or (unless NO_POINTER_CHECK) a pointer
 * that is not device memory of sufficient extent; nothing is launched in that case.
 *
 * HIP graphs.  A step may be captured (hip_stream in capture mode) and the graph replayed: all
 * that changes from step to step -- which state record is current, the generation of the fused
 * step's grid barrier, the work counters -- is kept on the device and advanced by the kernels, so
 * every replay is one more iteration on whatever the gradient buffers hold at that moment.
 * Conditions: the same tensor pointers must have been through one adascale_step outside the
 * capture (their table is then on the device; during capture nothing is uploaded, checked or
 * allocated, and ADASCALE_ESTATE says so otherwise); not with ADASCALE_COOPERATIVE_LAUNCH; the
 * graph is void after adascale_set_scale or adascale_destroy; replays, like direct calls, must
 * not overlap other steps of the same context, and keeping a replayed fused step apart from
 * fused steps running on other streams is the caller's business (direct calls are chained by the
 * library).  adascale_set_state may be captured too; adascale_get_state may not (it waits).
 */
int adascale_step(adascale_ctx *ctx, void *const *w, void *const *mom, const void *const *grads,
                  void *hip_stream);

/*
 * Copy the scalar state (Algorithm 2's tau, the gain ratio, the estimates) to host memory.
 * Waits for the work queued on hip_stream; it is the only call that synchronises.
 * ADASCALE_ESTATE: a fused step's grid barrier gave up waiting (its workgroups were never all
 * resident at once).  That step is void: workgroups that saw the failure left w and v of the
 * tiles they keep on chip untouched and did not advance the state, but others may have finished,
 * and tiles beyond the chip's capacity already hold the new momentum in v -- so w, v and the state
 * are to be taken as lost.  From then on adascale_step on this context returns ADASCALE_ESTATE
 * too, until the caller has restored w and v from a checkpoint and called adascale_set_state.
 */
int adascale_get_state(adascale_ctx *ctx, adascale_state *out, void *hip_stream);

/*
 * Overwrite the resumable part of the state: step count k, tau and the two moving averages
 * (the remaining fields of adascale_state are per-step diagnostics).  With (w, mom) this is
 * a full checkpoint.  Asynchronous on hip_stream.  Also ends the failed state described at
 * adascale_get_state.
 */
int adascale_set_state(adascale_ctx *ctx, int64_t step, double tau, double sigma2_bar, double mu2_bar,
                       void *hip_stream);

/*
 * Elastic AdaScaling (Sec. 4): change the scale to S_new between steps; tau and the moving
 * averages carry on.  theta < 0 selects max(1 - S_new/1000, 0).  The next adascale_step
 * expects S_new * N gradient pointers.  EINVAL if S_new < 1 or theta >= 1.  Host only, except
 * when S_new needs a larger pointer table than any scale before it on this context: the table is
 * then reallocated, which waits for the device to go idle (hipDeviceSynchronize) first.
 */
int adascale_set_scale(adascale_ctx *ctx, int32_t S_new, double theta);

/*
 * One AdaScale iteration on a single flat parameter tensor, for callers that cannot allocate
 * device memory or keep a context: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  No context: everything comes in the argument record, and the call
 * allocates nothing on the host or the device (no hipMalloc, hipFree or any call that does).
 * What its kernels need beyond the caller's buffers (pointer row, state records, partial sums)
 * lies in a fixed block of about 34 KB of device memory inside the library's image, one per GPU,
 * held until the process ends.  Consequences:
 *   - at most ADASCALE_FLAT_MAX_SCALE gradient buffers and ADASCALE_FLAT_MAX_NUMEL elements;
 *     anything beyond is ADASCALE_EINVAL with a message (adascale_last_error(NULL));
 *   - all calls on one GPU share that block: calls that may overlap on one GPU (different
 *     streams or threads of one process; another process has its own copy) race; issue them on
 *     one stream, or order the streams with events;
 *   - the first call on each device looks up the block's address (hipGetSymbolAddress); make that
 *     call outside graph capture.
 * It computes what adascale_step computes for a context with this one tensor (same readings,
 * same flags LAGGED_R / EST_NORM_RATIO / NO_POINTER_CHECK), as a gradient sweep that leaves the new
 * momentum in `mom`, the scalar kernel, and w <- w - eta_t mom; results agree with adascale_step
 * to rounding (the sums are taken in another order).  Asynchronous on hip_stream.
 */
#define ADASCALE_FLAT_MAX_SCALE 64
#define ADASCALE_FLAT_MAX_NUMEL (((int64_t)1 << 40) - 1)
typedef struct {
    int32_t S;               /* 1 .. ADASCALE_FLAT_MAX_SCALE */
    int32_t grad_dtype;      /* ADASCALE_F32 or ADASCALE_BF16 */
    int64_t numel;           /* 0 .. ADASCALE_FLAT_MAX_NUMEL */
    double momentum, weight_decay, theta, eps;   /* as in adascale_config */
    uint32_t flags;          /* ADASCALE_LAGGED_R | ADASCALE_EST_NORM_RATIO | ADASCALE_NO_POINTER_CHECK */
    int32_t device;          /* HIP device ordinal of every pointer below */
    void *w, *mom;           /* DEVICE fp32 [numel], updated in place */
    const void *const *grads; /* HOST array [S] of DEVICE pointers to [numel] elements of grad_dtype; read only */
    const float *lr_table;   /* DEVICE [lr_table_len]: lr(0..L-1) */
    int64_t lr_table_len;
    adascale_state *state;   /* DEVICE record, 8-byte aligned, read (step, tau, sigma2_bar, mu2_bar) and
                                rewritten whole; zero-filled = start of a run */
} adascale_flat_step;
int adascale_step_flat(const adascale_flat_step *args, void *hip_stream);

/* Free the context and its device scratch.  Waits for the device to go idle.  NULL is allowed. */
void adascale_destroy(adascale_ctx *ctx);

/* Message for the last non-OK code returned on this context (or by the last failed
 * adascale_init when ctx is NULL).  The string is owned by the library. */
const char *adascale_last_error(const adascale_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* ADASCALE_H */
