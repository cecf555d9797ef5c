"""The oracle's C under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a small
C driver, compiled together with oracle/adascale_oracle.c, steps it through the hand-derived
example and through a ragged multi-tensor bf16 / fp32 run whose buffers are allocated at their
exact sizes, so that any read past a gradient, w or v buffer is reported."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r'''
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct { int64_t step; double tau, r, lr_eff, sum_sq, sq_mean, sigma2_hat, mu2_hat, sigma2_bar, mu2_bar; int32_t done; } oracle_state;
typedef struct oracle_ctx oracle_ctx;
oracle_ctx *oracle_create(int, int, double, double, double, double, const float *, int64_t, uint32_t);
void oracle_destroy(oracle_ctx *);
void oracle_get_state(const oracle_ctx *, oracle_state *);
void oracle_set_state(oracle_ctx *, int64_t, double, double, double, double);
void oracle_set_scale(oracle_ctx *, int, double);
void oracle_begin_step(oracle_ctx *);
void oracle_accumulate(oracle_ctx *, int64_t, const void *const *, double *);
void oracle_gain(oracle_ctx *);
void oracle_apply(const oracle_ctx *, int64_t, double *, double *, const double *);
void oracle_advance(oracle_ctx *);

static uint32_t rng = 12345u;
static float next(void) { rng = rng * 1664525u + 1013904223u; return (float)((rng >> 8) & 0xffff) / 65536.0f - 0.4f; }

static int run(int S, int dtype, uint32_t flags, const int64_t *numel, int n_tensors, int steps)
{
    float lr[3] = {0.1f, 0.05f, 0.025f};
    oracle_ctx *c = oracle_create(S, dtype, 0.9, 1e-3, -1.0, 0.0, lr, 3, flags);
    if (!c) return 1;
    double **w = malloc(sizeof *w * n_tensors), **v = malloc(sizeof *v * n_tensors), **gb = malloc(sizeof *gb * n_tensors);
    void ***g = malloc(sizeof *g * n_tensors);
    for (int k = 0; k < n_tensors; ++k) {
        w[k] = calloc(numel[k] ? numel[k] : 1, sizeof(double));
        v[k] = calloc(numel[k] ? numel[k] : 1, sizeof(double));
        gb[k] = malloc(sizeof(double) * (numel[k] ? numel[k] : 1));
        g[k] = malloc(sizeof(void *) * S);
        for (int i = 0; i < S; ++i) g[k][i] = malloc((dtype ? 2 : 4) * (numel[k] ? numel[k] : 1));   /* exact size */
    }
    oracle_state st;
    for (int t = 0; t < steps; ++t) {
        if (t == 2) oracle_set_scale(c, S, 0.5);
        for (int k = 0; k < n_tensors; ++k)
            for (int i = 0; i < S; ++i)
                for (int64_t j = 0; j < numel[k]; ++j) {
                    float x = next();
                    if (dtype) { uint32_t b; memcpy(&b, &x, 4); ((uint16_t *)g[k][i])[j] = (uint16_t)(b >> 16); }
                    else ((float *)g[k][i])[j] = x;
                }
        oracle_begin_step(c);
        for (int k = 0; k < n_tensors; ++k) oracle_accumulate(c, numel[k], (const void *const *)g[k], gb[k]);
        oracle_gain(c);
        for (int k = 0; k < n_tensors; ++k) oracle_apply(c, numel[k], w[k], v[k], gb[k]);
        oracle_advance(c);
        oracle_get_state(c, &st);
        if (!(st.r >= 1.0 - 1e-12 && st.r <= S * (1 + 1e-12)) || !isfinite(st.tau)) return 2;
    }
    oracle_set_state(c, st.step, st.tau, st.sigma2_bar, st.mu2_bar, st.r);
    for (int k = 0; k < n_tensors; ++k) {
        for (int i = 0; i < S; ++i) free(g[k][i]);
        free(g[k]); free(w[k]); free(v[k]); free(gb[k]);
    }
    free(g); free(w); free(v); free(gb);
    oracle_destroy(c);
    return 0;
}

int main(void)
{
    const int64_t numel[5] = {1001, 1, 0, 64, 7};
    int rc = 0;
    for (int dtype = 0; dtype < 2; ++dtype)
        for (uint32_t flags = 0; flags < 4; ++flags) {
            rc |= run(1, dtype, flags, numel, 5, 4);
            rc |= run(3, dtype, flags, numel, 5, 4);
            rc |= run(8, dtype, flags, numel, 5, 4);
        }
    /* the hand-derived example: r of iteration 1 is 1.4 */
    {
        float lr[2] = {0.125f, 0.0625f}, g1[2] = {1, 2}, g2[2] = {3, 0};
        const void *g[2] = {g1, g2};
        double w[2] = {0, 0}, v[2] = {0, 0}, gb[2];
        oracle_ctx *c = oracle_create(2, 0, 0.9, 0.0, 0.9, 1e-6, lr, 2, 0);
        oracle_state st;
        oracle_begin_step(c); oracle_accumulate(c, 2, g, gb); oracle_gain(c); oracle_apply(c, 2, w, v, gb); oracle_advance(c);
        oracle_get_state(c, &st);
        if (fabs(st.r - 1.4) > 1e-15 || fabs(w[0] + 0.35) > 1e-15) rc |= 4;
        oracle_destroy(c);
    }
    printf("rc %d\n", rc);
    return rc;
}
'''


@pytest.mark.parametrize("openmp", [False, True])
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path, openmp):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "driver.c"
    src.write_text(DRIVER)
    exe = tmp_path / "driver"
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer", "-static-libasan", "-ffp-contract=off", *(["-fopenmp"] if openmp else []),
           str(src), os.path.join(ROOT, "oracle", "adascale_oracle.c"), "-o", str(exe), "-lm"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "asan" in built.stderr.lower():
        pytest.skip("no static sanitizer runtime: " + built.stderr[-200:])
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", OMP_NUM_THREADS="4")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0 and "rc 0" in r.stdout, (r.stdout[-500:], r.stderr[-2000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
