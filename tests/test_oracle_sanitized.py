"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer: a small C driver runs every
oracle routine on seeded inputs with ragged lengths, invalid rows and the edge sizes; any report aborts."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r"""
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
int oracle_topp_select(const float *, int64_t, int, const int32_t *, float, int32_t *, int64_t, int32_t *, float *, uint32_t *, double *);
int oracle_bisection_select(const float *, int64_t, int, const int32_t *, float, int, int32_t *, int64_t, int32_t *, float *, uint32_t *);
int oracle_chunk_masses(const float *, int64_t, int, const int32_t *, int, int, float *);
int oracle_nucleus_bisection(const float *, int, double, int, double *, double *, double *);
int oracle_masked_attention_tail(const void *, const void *, const void *, int, int, int, int, int, int, int, const uint8_t *,
                                 const int32_t *, const void *, const void *, double, const int32_t *, int, double *, double *);
static uint32_t s = 12345u;
static float rnd(void) { s = s * 1664525u + 1013904223u; return (float)(s >> 8) / 16777216.0f; }
int main(void)
{
    enum { ROWS = 7, N = 131, B = 2, HQ = 4, HK = 2, T = 3, D = 8 };
    float *p = malloc(sizeof(float) * ROWS * N);
    for (int i = 0; i < ROWS * N; ++i) p[i] = rnd() * rnd();
    int32_t lens[ROWS] = {N, 0, 1, 16, 17, N - 1, 64};
    p[3 * N + 5] = NAN;                                   /* an invalid row */
    for (int i = 0; i < N; ++i) p[6 * N + i] = 0.0f;      /* a row without mass */
    int32_t *idx = malloc(sizeof(int32_t) * ROWS * N), counts[ROWS];
    float tau[ROWS];
    uint32_t flags[ROWS];
    double diag[4 * ROWS];
    const float ps[] = {1e-6f, 0.5f, 0.9f, 1.0f};
    for (int k = 0; k < 4; ++k) {
        if (oracle_topp_select(p, N, ROWS, lens, ps[k], idx, N, counts, tau, flags, diag)) return 1;
        if (oracle_bisection_select(p, N, ROWS, lens, ps[k], 10, idx, N, counts, tau, flags)) return 2;
    }
    float mass[ROWS * 9];
    if (oracle_chunk_masses(p, N, ROWS, lens, 16, 9, mass)) return 3;
    double lo, hi, mid;
    oracle_nucleus_bisection(p, N, 0.9, 60, &lo, &hi, &mid);
    float *q = malloc(sizeof(float) * B * HQ * T * D), *k = malloc(sizeof(float) * B * HK * N * D);
    float *v = malloc(sizeof(float) * B * HK * N * D), *kn = malloc(sizeof(float) * B * HK * T * D);
    for (int i = 0; i < B * HQ * T * D; ++i) q[i] = rnd() - 0.5f;
    for (int i = 0; i < B * HK * N * D; ++i) { k[i] = rnd() - 0.5f; v[i] = rnd() - 0.5f; }
    for (int i = 0; i < B * HK * T * D; ++i) kn[i] = rnd() - 0.5f;
    uint8_t *mask = malloc(B * HK * N);
    for (int i = 0; i < B * HK * N; ++i) mask[i] = rnd() < 0.3f;
    int32_t alens[B] = {N, 0};
    int32_t which[B * HQ * T * 3];
    int w = 0;
    for (int b = 0; b < B; ++b) for (int h = 0; h < HQ; ++h) for (int t = 0; t < T; ++t) { which[3 * w] = b; which[3 * w + 1] = h; which[3 * w + 2] = t; ++w; }
    double *out = malloc(sizeof(double) * w * D), *lse = malloc(sizeof(double) * w);
    if (oracle_masked_attention_tail(q, k, v, 0, B, HQ, HK, T, D, N, mask, alens, NULL, NULL, 0.35, which, w, out, lse)) return 4;
    if (oracle_masked_attention_tail(q, k, v, 0, B, HQ, HK, T, D, N, mask, alens, kn, kn, 0.35, which, w, out, lse)) return 5;
    /* 16-bit bit patterns: reinterpret the same memory as half the number of elements */
    if (oracle_masked_attention_tail(q, k, v, 1, 1, HQ, HK, T, D / 2, N, mask, alens, NULL, NULL, 0.35, which, HQ * T, out, lse)) return 6;
    if (oracle_masked_attention_tail(q, k, v, 2, 1, HQ, HK, T, D / 2, N, mask, alens, NULL, NULL, 0.35, which, HQ * T, out, lse)) return 7;
    free(p); free(idx); free(q); free(k); free(v); free(kn); free(mask); free(out); free(lse);
    puts("sanitized run ok");
    return 0;
}
"""


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    (tmp_path / "driver.c").write_text(DRIVER)
    exe = tmp_path / "driver"
    cmd = ["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           os.path.join(ROOT, "oracle", "specattn_oracle.c"), str(tmp_path / "driver.c"), "-lm", "-o", str(exe)]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and "sanitize" in build.stderr:
        pytest.skip("sanitizer runtimes are not installed")
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300, env=env)
    assert run.returncode == 0 and "sanitized run ok" in run.stdout, run.stdout + run.stderr
