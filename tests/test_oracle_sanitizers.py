"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host only): a small driver
calls every exported function on seeded inputs, including ragged shapes, excluded tokens, padding
in the neighbour table and rows that fall back to p; any report fails the run."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r'''
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include "cool_sd_oracle.c"

static unsigned long long s = 88172645463325252ULL;
static double rnd(void) { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return (double)(s >> 11) / 9007199254740992.0; }
static float gauss(void) { double u = rnd() + 1e-12, v = rnd(); return (float)(sqrt(-2.0 * log(u)) * cos(6.283185307179586 * v)); }

int main(void) {
    const int shapes[][3] = {{1, 1, 1}, {2, 3, 7}, {3, 4, 33}, {2, 9, 130}};
    for (int sh = 0; sh < 4; ++sh) {
        int B = shapes[sh][0], L = shapes[sh][1], V = shapes[sh][2];
        for (int variant = 0; variant < 4; ++variant) {
            int bonus = variant & 1, guided = variant >> 1;
            int k = V > 3 ? 3 : 0;
            size_t nt = (size_t)B * (L + bonus) * V, nd = (size_t)B * L * V;
            float *t = malloc(nt * 4), *tu = malloc(nt * 4), *d = malloc(nd * 4), *du = malloc(nd * 4);
            for (size_t i = 0; i < nt; ++i) { t[i] = 3 * gauss(); tu[i] = t[i] + gauss(); if (rnd() < 0.05) t[i] = tu[i] = -INFINITY; }
            for (size_t i = 0; i < nd; ++i) { d[i] = 3 * gauss(); du[i] = d[i] + gauss(); }
            for (size_t r = 0; r < (size_t)B * (L + bonus); ++r) t[r * V] = tu[r * V] = 1.0f;   /* a finite entry per row */
            int *tok = malloc((size_t)B * L * sizeof(int));
            float *ua = malloc((size_t)B * L * 4), *ur = malloc((size_t)B * 4), *om = malloc((size_t)L * 4);
            for (int i = 0; i < B * L; ++i) { tok[i] = (int)(rnd() * V); ua[i] = (float)rnd(); }
            for (int b = 0; b < B; ++b) ur[b] = (float)rnd();
            double *omd = malloc((size_t)L * 8);
            if (csd_oracle_schedule(CSD_SCHED_EXP, L, 1.1, 0.7, omd)) return 2;
            for (int i = 0; i < L; ++i) om[i] = (float)omd[i];
            if (csd_oracle_schedule(CSD_SCHED_LINEAR, L, 2.0, (double)(L + 1), omd)) return 2;
            int *al = malloc((size_t)B * sizeof(int)), *nx = malloc((size_t)B * sizeof(int));
            double *rm = malloc((size_t)B * 8), *pt = malloc((size_t)B * L * 8), *qt = malloc((size_t)B * L * 8), *ff = malloc((size_t)B * L * 8);
            double *pa = malloc((size_t)B * L * 8);
            int *cnt = malloc((size_t)B * L * sizeof(int));
            unsigned char *acc = malloc((size_t)B * L);
            int top_k = V > 4 ? V / 2 : 0;
            for (int mode = 0; mode < 2; ++mode) {
                int rc = csd_oracle_verify(B, L, V, bonus, t, guided ? tu : NULL, (long long)(L + bonus) * V, V,
                                           d, guided ? du : NULL, (long long)L * V, V, 4.0f, 0.9f, top_k, mode,
                                           tok, om, 0, ua, ur, al, nx, rm, pt, qt, ff, acc, 2);
                if (rc) return 3;
                for (int b = 0; b < B; ++b) if (al[b] < 0 || al[b] > L || nx[b] < -1 || nx[b] >= V) return 4;
            }
            int *nbr = malloc((size_t)V * (k ? k : 1) * sizeof(int));
            for (int x = 0; x < V; ++x) for (int j = 0; j < k; ++j) nbr[x * k + j] = rnd() < 0.2 ? -1 : (x + 1 + j) % V;
            for (int mode = 0; mode < 3; ++mode) {
                int rc = csd_oracle_verify_lantern(B, L, V, bonus, t, guided ? tu : NULL, (long long)(L + bonus) * V, V,
                                                   d, guided ? du : NULL, (long long)L * V, V, 4.0f, 1.0f, top_k, mode,
                                                   tok, nbr, k, 0.7f, ua, ur, al, nx, rm, pt, qt, ff, acc, pa, cnt, 1);
                if (rc) return 5;
            }
            double *g = malloc((size_t)B * V * 8), *mass = malloc((size_t)B * 8);
            float *omr = malloc((size_t)B * 4);
            for (int b = 0; b < B; ++b) omr[b] = 0.5f + (float)rnd();
            if (csd_oracle_resample(B, V, t, guided ? tu : NULL, (long long)(L + bonus) * V, d, guided ? du : NULL,
                                    (long long)L * V, 4.0f, 1.0f, top_k, 0, omr, ur, nx, mass, g)) return 6;
            if (csd_oracle_resample(B, V, t, NULL, (long long)(L + bonus) * V, NULL, NULL, 0, 1.0f, 1.0f, 0, 0, NULL, ur,
                                    nx, mass, NULL)) return 7;
            double *row = malloc((size_t)V * 8), *p = malloc((size_t)V * 8), *q = malloc((size_t)V * 8), alpha, beta;
            csd_oracle_transform_row(t, NULL, V, 1.0f, 1.0f, 0, row); csd_oracle_softmax(row, V, p);
            csd_oracle_transform_row(d, NULL, V, 1.0f, 1.0f, 0, row); csd_oracle_softmax(row, V, q);
            csd_oracle_position_diagnostics(p, q, V, 1.7, &alpha, &beta);
            if (!(alpha >= 0 && alpha <= 1.0000001 && beta >= -1e-15)) return 8;
            /* identical rows: no rejection possible, the law falls back to p */
            if (fabs(csd_oracle_residual(p, p, V, 1.0, 0, row) - 1.0) > 1e-12) return 9;
            free(t); free(tu); free(d); free(du); free(tok); free(ua); free(ur); free(om); free(omd); free(al); free(nx);
            free(rm); free(pt); free(qt); free(ff); free(pa); free(cnt); free(acc); free(nbr); free(g); free(mass);
            free(omr); free(row); free(p); free(q);
        }
    }
    printf("sanitizer driver ok, threads %d\n", csd_oracle_max_threads());
    return 0;
}
'''


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    src = tmp_path / "driver.c"
    src.write_text(DRIVER)
    exe = tmp_path / "driver"
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-I", os.path.join(ROOT, "oracle"), "-o", str(exe), str(src), "-lm"]
    subprocess.run(cmd, check=True)
    # other preloaded libraries may precede the sanitizer runtime in the driver process
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               OMP_NUM_THREADS="2")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, "rc=%d\n%s\n%s" % (r.returncode, r.stdout[-2000:], r.stderr[-4000:])
    assert "sanitizer driver ok" in r.stdout
