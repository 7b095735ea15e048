"""The oracle's C source under AddressSanitizer and UndefinedBehaviorSanitizer (host only): every function is
driven once from a small C main over ragged shapes (anchors shorter and longer than the segment, one
unselected), so that an out-of-bounds index or a misuse of the per-anchor lengths aborts the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "kvcomm_oracle.c")

MAIN = r'''
#include <stdio.h>
#include <stdlib.h>
#include <math.h>
#include <stddef.h>
void kvo_rope_rotate(const double *, double *, int, double, double);
void kvo_distances(const double *, const double *const *, const int *, int, int, int, int, int, int, double *, int *);
void kvo_weights(const double *, const int *, int, size_t, double, double *, int *);
void kvo_align(const double *, const double *, const double *const *, const double *const *, const int *, const double *,
               int, int, int, int, int, int, double, const double *, double, double *, double *);
void kvo_suffix_attn(const double *, const double *, const double *, int, int, int, int, int, int, double, double *, double *);
void kvo_capture(const double *, const double *, const double *, const double *, int, int, int, int, double, double, double *, double *);
int kvo_predict(const double *, const int *, const int *, int, size_t, int, double, double *, double *);
void kvo_cosine(const double *, const double *const *, const int *, int, int, int, int, int, int, double *, int *);
void kvo_weights_from_sim(const double *, const int *, int, size_t, double, double *, int *);
void kvo_weights_nearest(const double *, const int *, int, size_t, double *, int *);
void kvo_quantize(const double *, size_t, double, unsigned char *);
void kvo_dequantize(const unsigned char *, size_t, double, double *);

static double *rnd(size_t n) { double *p = malloc(sizeof(double) * n); for (size_t i = 0; i < n; ++i) p[i] = (double)rand() / RAND_MAX - 0.5; return p; }

int main(void)
{
    enum { L = 2, H = 3, S = 7, D = 8, A = 4 };
    int anc_len[A] = {7, 9, 5, 12};               /* anchor 2 is shorter than the segment: never read past 5 tokens */
    double *seg_k = rnd(L * H * S * D), *seg_v = rnd(L * H * S * D);
    const double *ak[A], *dk[A], *dv[A];
    for (int a = 0; a < A; ++a) { size_t n = (size_t)L * H * anc_len[a] * D; ak[a] = rnd(n); dk[a] = rnd(n); dv[a] = rnd(n); }
    for (int gran = 0; gran < 3; ++gran) {
        size_t n = gran == 0 ? S : gran == 1 ? (size_t)L * H * S : 1;
        double *dist = malloc(sizeof(double) * A * n), *w = malloc(sizeof(double) * A * n), *ent = malloc(sizeof(double) * n);
        int sel[A], *near = malloc(sizeof(int) * n);
        kvo_distances(seg_k, ak, anc_len, A, L, H, S, D, gran, dist, sel);
        kvo_weights(dist, sel, A, n, 0.7, w, near);
        double ad[A] = {0, 3, 5, 64}, *ok = malloc(sizeof(double) * L * H * S * D), *ov = malloc(sizeof(double) * L * H * S * D);
        kvo_align(seg_k, seg_v, dk, dv, anc_len, w, gran, A, L, H, S, D, 64.0, ad, 1e4, ok, ov);
        kvo_align(seg_k, seg_v, dk, dv, anc_len, w, gran, A, L, H, S, D, 0.0, NULL, 1e4, ok, ov);
        double mean; (void)kvo_predict(w, sel, anc_len, A, n, S, 0.3, ent, &mean);
        kvo_cosine(seg_k, ak, anc_len, A, L, H, S, D, gran, dist, sel);
        kvo_weights_from_sim(dist, sel, A, n, 0.5, w, near);
        kvo_weights_nearest(dist, sel, A, n, w, near);
        free(dist); free(w); free(ent); free(near); free(ok); free(ov);
    }
    {   /* attention: GQA, no context, single query */
        enum { Hq = 6, Tq = 5, NC = 3 };
        double *q = rnd(L * Hq * Tq * D), *k = rnd(L * H * (NC + Tq) * D), *v = rnd(L * H * (NC + Tq) * D);
        double *o = malloc(sizeof(double) * L * Hq * Tq * D), *lse = malloc(sizeof(double) * L * Hq * Tq);
        kvo_suffix_attn(q, k, v, L, Hq, H, D, NC, Tq, 0.35, o, lse);
        kvo_suffix_attn(q, k, v, L, Hq, H, D, 0, 1, 0.35, o, lse);
        free(q); free(k); free(v); free(o); free(lse);
    }
    {
        double *rk = rnd(L * H * S * D), *rv = rnd(L * H * S * D), *ck = malloc(sizeof(double) * L * H * S * D), *cv = malloc(sizeof(double) * L * H * S * D);
        kvo_capture(seg_k, seg_v, rk, rv, L, H, S, D, 300.0, 5e5, ck, cv);
        unsigned char *b = malloc(L * H * S * D);
        kvo_quantize(ck, L * H * S * D, 0.0009765625, b);
        kvo_dequantize(b, L * H * S * D, 0.0009765625, cv);
        double x[8] = {1e9, -1e9, 0.0, -0.0, NAN, 448.0, 1e-30, -1e-30}; unsigned char bx[8];
        kvo_quantize(x, 8, 1.0, bx);
        free(rk); free(rv); free(ck); free(cv); free(b);
    }
    for (int a = 0; a < A; ++a) { free((void *)ak[a]); free((void *)dk[a]); free((void *)dv[a]); }
    free(seg_k); free(seg_v);
    puts("ok");
    return 0;
}
'''


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_oracle_under_asan_ubsan(tmp_path):
    main_c = tmp_path / "main.c"
    main_c.write_text(MAIN)
    exe = tmp_path / "oracle_san"
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-fno-omit-frame-pointer", "-o", str(exe), str(main_c), SRC, "-lm"], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stderr[-2000:]
    assert "ok" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
