/*
 * adascale_diag.h -- diagnostics, benchmark instrumentation and test knobs of the AdaScale step
 * library.  Nothing here is needed to run Algorithm 2 (adascale.h is the whole interface for
 * that); these calls tell which kernels a context runs and why, count the bytes they move, time
 * them, and let tests take a path the library would not choose for an input.  They describe the
 * implementation, not the method, and may change with it.
 */
#ifndef ADASCALE_DIAG_H
#define ADASCALE_DIAG_H

#include "adascale.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Which implementation the next adascale_step on a context runs; all compute the same thing (the
 * choice depends on the gradient type, the scale of the moment and the size of the parameter
 * list, and on adascale_tuning when the context was created with one):
 *   ADASCALE_PATH_FUSED      one persistent launch that keeps the mean gradient of Algorithm 1 on
 *                            chip as far as it fits (S <= 4096 and at least 8 % of the mean
 *                            gradient fitting in registers + LDS: lists up to about 400 M
 *                            parameters on MI355X);
 *   ADASCALE_PATH_STREAMING  three kernels (reduce, scalars, update), the first one a persistent
 *                            sweep in memory order: S <= 4096, parameter lists beyond that;
 *   ADASCALE_PATH_GENERAL    three kernels for any scale (or two with ADASCALE_LAGGED_R: one
 *                            sweep that reduces and updates, then the scalars).
 */
enum { ADASCALE_PATH_GENERAL = 0, ADASCALE_PATH_FUSED = 1, ADASCALE_PATH_STREAMING = 2 };
int adascale_step_path(const adascale_ctx *ctx);

/* 1 if adascale_step_path is ADASCALE_PATH_FUSED, else 0. */
int adascale_uses_fused_step(const adascale_ctx *ctx);

/*
 * Knobs for tests and measurements; a zero-filled record means the library's own choices.
 */
enum { ADASCALE_FORCE_NONE = 0, ADASCALE_FORCE_GENERAL = 1, ADASCALE_FORCE_FUSED = 2, ADASCALE_FORCE_STREAMING = 3 };
typedef struct {
    int32_t force_path;          /* ADASCALE_FORCE_*: FUSED takes the fused step however little of the mean
                                    gradient fits on chip, STREAMING never takes it, GENERAL takes neither
                                    512-lane kernel; a scale without an instance of the forced kernel still
                                    falls through to the next path */
    int32_t fused_max_grid;      /* > 0: at most this many workgroups in the fused step (fewer than compute
                                    units: forces tiles beyond the chip's capacity on small inputs) */
    int32_t fused_min_percent;   /* > 0: least share of the mean gradient on chip for the fused step
                                    (default 8; ignored under ADASCALE_FORCE_FUSED) */
    int32_t stream_via_scratch;  /* 1: the streaming sweep writes the mean gradient to a scratch of d floats
                                    and the full update kernel follows, instead of leaving the new momentum
                                    in v (12 instead of 8 bytes written per parameter) */
    int64_t barrier_spin_limit;  /* > 0: polls after which the fused step's grid barrier gives up
                                    (default 2^22, several seconds) */
    int32_t burst_tiles;         /* sweeps that write as they read (the streaming sweep; the fused step on its
                                    tiles beyond the chip's capacity) keep finished tiles in LDS and write them
                                    in bursts that all workgroups issue in the same clock windows, from 32
                                    (fused step: 16) gradient bytes per parameter (S x element size) upwards: < 0 no bursts
                                    (every tile written at once), > 0 bursts at any scale, with at most this
                                    many tiles kept by the streaming sweep (up to 18, the default) */
    int32_t burst_window_ticks;  /* > 0: bursts at any scale, in windows of this many ticks of the device's
                                    wall clock, 10 ns each on MI355X (default: from the scale, 0.8 x the time
                                    the ring of kept tiles takes to fill) */
} adascale_tuning;

/* adascale_init with knobs; tuning == NULL is adascale_init. */
int adascale_init_tuned(const adascale_config *cfg, const adascale_tuning *tuning, adascale_ctx **out);

/*
 * Test hook for the failure path of the fused step: the next fused step's grid barrier waits for
 * one arrival more than its grid provides, so every workgroup's bounded wait runs out (set
 * barrier_spin_limit small to keep that short), every kernel exits normally, and the context ends
 * up in the failed state adascale_get_state describes.  ESTATE if the context does not take the
 * fused step with a barrier (see adascale_step_path; with ADASCALE_LAGGED_R small parameter lists
 * run instances of the fused step that have none).
 */
int adascale_fail_next_barrier(adascale_ctx *ctx);

/* Algorithmic bytes one step moves for this context: S*d*b gradient bytes read once plus the
 * per-parameter traffic of a two-sweep step that keeps nothing on chip: 24 bytes (the new momentum
 * written and read back, v read, w read twice and written), 20 without weight decay, where the
 * first sweep does not need w.  Host only. */
int64_t adascale_step_bytes(const adascale_ctx *ctx);

/* Bytes the kernels of the next step actually read from and write to device memory, counted from
 * the context's tile tables: S*d*b for the gradients and, per parameter, 16 where the mean gradient
 * stays on chip (w and v read and written once), 20 or 24 where the gradient sweep leaves the new
 * momentum in v (without / with weight decay), 24 where the mean gradient passes through a
 * scratch, a few more for the ragged last tile of each tensor.  Host only.  rocprofv3's
 * FETCH_SIZE / WRITE_SIZE counters read within a fraction of a percent of this figure. */
int64_t adascale_step_moved_bytes(const adascale_ctx *ctx);

/*
 * How the fused and streaming kernels consume the S gradients of a tile (Algorithm 1's sum over
 * the batches): in shape[1] half-groups of shape[0] loads each, alternating between two register
 * buffers; the pointer table rows are padded to shape[2] = shape[0] * shape[1] replica slots.
 * Host only, needs no device.  Returns a bit mask: 1 = the fused step has a kernel instance for
 * this gradient type and scale (at every register level, both gain variants), 2 = the streaming
 * reduce kernel has one; 0 (shape untouched) if the scale is outside their range, in which case
 * the general kernels run.
 */
int adascale_kernel_shape(int32_t grad_dtype, int32_t S, int32_t shape[3]);

/*
 * What adascale_init_tuned would decide for cfg's parameter list, gradient type, scale and flags
 * (and the knobs, NULL = none) on a device with `compute_units` compute units and `lds_bytes` of
 * LDS per workgroup (MI355X: 256 and 163840): how the list splits into whole 512-lane tiles (2048
 * elements, inside one tensor) and ragged last tiles, the grids, how many tiles of the mean
 * gradient each workgroup of the fused step keeps in registers and in LDS, and the path.  A pure
 * function of its arguments: no device is touched, cfg's lr_table, device and the optimizer
 * constants are not read.  The fields of a path that does not apply are 0.  (adascale_init
 * additionally asks the runtime whether the fused grid can be resident at once; on MI355X it can.)
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
int adascale_plan(const adascale_config *cfg, const adascale_tuning *tuning, int32_t compute_units, int64_t lds_bytes,
                  adascale_plan_info *out);

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
#endif /* ADASCALE_DIAG_H */
