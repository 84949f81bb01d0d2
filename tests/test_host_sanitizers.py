"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

Two small C drivers are compiled together with (a) the library's host-only
translation units (plan, kernel selection: no HIP call is made by them) and
(b) the fp64 oracle, with ``-fsanitize=address,undefined
-fno-sanitize-recover``, and run over a sweep of geometries that includes the
error paths and the size limits.  Any out-of-bounds access, signed overflow or
leak ends the driver with a non-zero status.
"""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2601_11608_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-g", "-O1"]

PLAN_DRIVER = r"""
#include <stdio.h>
#include <string.h>
#include "foldconv.h"
int main(void) {
    long plans = 0, errors = 0;
    const int dims[] = {1, 2, 3, 7, 8, 16, 33, 224};
    const int chans[] = {1, 3, 8, 12, 20, 64, 132};
    const int folds[] = {1, 2, 4, 8, 16, 32, 224};
    for (unsigned a = 0; a < sizeof dims / sizeof *dims; ++a)
    for (unsigned b = 0; b < sizeof dims / sizeof *dims; ++b)
    for (unsigned c = 0; c < sizeof chans / sizeof *chans; ++c)
    for (unsigned f = 0; f < sizeof folds / sizeof *folds; ++f)
    for (int k = 1; k <= 5; k += 2)
    for (int pad = 0; pad <= 2; ++pad)
    for (int dt = 0; dt <= 2; ++dt) {
        foldconv_plan_t p = 0;
        int st = foldconv_plan(2, dims[a], dims[b], chans[c], chans[(c + 3) % 7], k, (k + 2) % 6 + 1, pad, folds[f],
                               (foldconv_dtype_t)dt, &p);
        if (st == FOLDCONV_OK) {
            foldconv_shapes_t s;
            if (foldconv_plan_query(p, &s) != FOLDCONV_OK || s.W_fold * s.F != s.W || s.filter_compact_bytes <= 0) return 2;
            foldconv_plan_destroy(p);
            ++plans;
        } else {
            if (p) return 3;
            ++errors;
        }
    }
    /* limits, bad arguments, the GEMM and channels-first front ends, the fold-factor model */
    foldconv_plan_t p = 0;
    if (foldconv_plan(1 << 20, 1 << 12, 1 << 12, 64, 64, 3, 3, 1, 1, FOLDCONV_F16, &p) != FOLDCONV_ERR_UNSUPPORTED) return 4;
    if (foldconv_plan(1, 8, 8, 3, 4, 3, 3, 1, 3, FOLDCONV_F16, &p) != FOLDCONV_ERR_INDIVISIBLE) return 5;
    if (foldconv_plan(1, 8, 8, 3, 4, 3, 3, 1, 4, FOLDCONV_F16, 0) != FOLDCONV_ERR_BADARG) return 6;
    if (foldconv_plan_gemm(1 << 21, 12, 64, 4, FOLDCONV_F16, &p) != FOLDCONV_OK) return 7;
    foldconv_plan_destroy(p);
    if (foldconv_plan_gemm(1LL << 28, 8, 8, 1, FOLDCONV_BF16, &p) != FOLDCONV_OK) return 8;
    foldconv_plan_destroy(p);
    if (foldconv_plan_gemm(2147483647LL, 8, 8, 1, FOLDCONV_BF16, &p) != FOLDCONV_ERR_UNSUPPORTED || p) return 14;
    if (foldconv_plan_nchw(2, 3, 32, 48, 16, 3, 5, 2, 8, FOLDCONV_FOLD_H, FOLDCONV_F16, &p) != FOLDCONV_OK) return 9;
    foldconv_plan_destroy(p);
    foldconv_plan_destroy(0);            /* NULL is ignored */
    int F = 0;
    if (foldconv_choose_fold(64, 224, 224, 3, 64, 3, 3, 1, FOLDCONV_F16, &F) != FOLDCONV_OK || F < 1) return 10;
    if (foldconv_plan_query(0, 0) != FOLDCONV_ERR_BADARG) return 11;
    if (!foldconv_strerror(-3) || !foldconv_strerror(12345)) return 12;
    printf("plans %ld errors %ld\n", plans, errors);
    return plans > 1000 && errors > 1000 ? 0 : 13;
}
"""

ORACLE_DRIVER = r"""
#include <stdio.h>
#include <stdlib.h>
void oracle_conv2d_nhwc(const double*, const double*, const double*, double*, int, int, int, int, int, int, int, int, int, int, int, int);
void oracle_conv2d_nchw(const double*, const double*, const double*, double*, int, int, int, int, int, int, int, int, int, int, int, int);
void oracle_fold_input(const double*, double*, int, int, int, int, int);
void oracle_folded_shapes(int, int, int, int, int*);
void oracle_expand_filter(const double*, double*, int, int, int, int, int, int);
void oracle_unfold_output(const double*, double*, int, int, int, int, int, int);
void oracle_fold_input_h_nchw(const double*, double*, int, int, int, int, int);
void oracle_expand_filter_h_oihw(const double*, double*, int, int, int, int, int, int);
void oracle_unfold_output_h_nchw(const double*, double*, int, int, int, int, int, int);
static double *buf(size_t n) { double *p = malloc(n * sizeof(double)); for (size_t i = 0; i < n; ++i) p[i] = (double)(i % 7) - 3; return p; }
int main(void) {
    const int N = 2, C = 3, Co = 5;
    for (int H = 4; H <= 8; H += 4) for (int F = 1; F <= 4; F *= 2) for (int K = 1; K <= 4; ++K) for (int p = 0; p <= 2; ++p) {
        const int W = 8;
        int sh[8];
        oracle_folded_shapes(W, K, p, F, sh);
        const int Wf = sh[0], KWf = sh[3], W_out = sh[4], Wf_out = sh[5], H_out = H + 2 * p - K + 1;
        if (H_out <= 0 || W_out <= 0) continue;
        double *x = buf((size_t)N * H * W * C), *w = buf((size_t)K * K * C * Co), *b = buf(Co);
        double *y = buf((size_t)N * H_out * W_out * Co), *xf = buf((size_t)N * H * Wf * F * C);
        double *we = buf((size_t)K * KWf * F * C * F * Co), *yf = buf((size_t)N * H_out * Wf_out * F * Co), *y2 = buf((size_t)N * H_out * W_out * Co);
        oracle_conv2d_nhwc(x, w, b, y, N, H, W, C, Co, K, K, p, p, H_out, W_out, 1);
        oracle_fold_input(x, xf, N, H, W, C, F);
        oracle_expand_filter(w, we, K, K, C, Co, F, p);
        oracle_conv2d_nhwc(xf, we, 0, yf, N, H, Wf, F * C, F * Co, K, KWf, p, sh[6], H_out, Wf_out, 0);
        oracle_unfold_output(yf, y2, N, H_out, Wf_out, F, Co, W_out);
        /* channels-first, folding H (H % F == 0 here) */
        oracle_folded_shapes(H, K, p, F, sh);
        double *xh = buf((size_t)N * F * C * (H / F) * W), *wh = buf((size_t)F * Co * F * C * sh[3] * K);
        double *yh = buf((size_t)N * F * Co * sh[5] * W_out), *y3 = buf((size_t)N * Co * H_out * W_out);
        oracle_conv2d_nchw(x, w, b, y3, N, C, H, W, Co, K, K, p, p, H_out, W_out, 0);
        oracle_fold_input_h_nchw(x, xh, N, C, H, W, F);
        oracle_expand_filter_h_oihw(w, wh, Co, C, K, K, F, p);
        oracle_conv2d_nchw(xh, wh, 0, yh, N, F * C, H / F, W, F * Co, sh[3], K, sh[6], p, sh[5], W_out, 0);
        oracle_unfold_output_h_nchw(yh, y3, N, Co, sh[5], W_out, F, H_out);
        free(x); free(w); free(b); free(y); free(xf); free(we); free(yf); free(y2); free(xh); free(wh); free(yh); free(y3);
    }
    puts("oracle ok");
    return 0;
}
"""


def build_and_run(tmp, name, compiler, sources, driver_text, extra):
    drv = os.path.join(tmp, name + (".c" if compiler == "gcc" else ".cpp"))
    with open(drv, "w") as f:
        f.write(driver_text)
    exe = os.path.join(tmp, name)
    subprocess.check_call([compiler] + SAN + extra + [drv] + sources + ["-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1")
    env.pop("LD_PRELOAD", None)
    return subprocess.run([exe], env=env, capture_output=True, text=True)


@pytest.fixture(scope="module")
def tmp():
    if not shutil.which("gcc") or not shutil.which("g++"):
        pytest.skip("no host compiler")
    d = tempfile.mkdtemp()
    probe = os.path.join(d, "p.c")
    open(probe, "w").write("int main(void){return 0;}\n")
    if subprocess.call(["gcc", "-fsanitize=address,undefined", probe, "-o", os.path.join(d, "p")],
                       stderr=subprocess.DEVNULL) != 0:
        pytest.skip("sanitizer runtimes not installed")
    yield d
    shutil.rmtree(d, ignore_errors=True)


def test_plan_and_selection_under_sanitizers(tmp):
    srcs = [os.path.join(CSRC, "plan.cpp"), os.path.join(CSRC, "select.cpp")]
    r = build_and_run(tmp, "plan_driver", "g++", srcs, PLAN_DRIVER,
                      ["-std=c++17", "-x", "c++", "-I", os.path.join(ROOT, "include")])
    assert r.returncode == 0, r.stdout + r.stderr
    assert "plans" in r.stdout


def test_oracle_under_sanitizers(tmp):
    r = build_and_run(tmp, "oracle_driver", "gcc", [os.path.join(ROOT, "oracle", "foldconv_oracle.c")], ORACLE_DRIVER,
                      ["-std=c11", "-fopenmp"])
    assert r.returncode == 0, r.stdout + r.stderr
    assert "oracle ok" in r.stdout
