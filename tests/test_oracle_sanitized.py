"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): every exported
function is driven on small exactly-sized heap buffers, with odd shapes (d_k != d_v, T not a multiple of
the backward's block length), so that an out-of-bounds index or a use of uninitialised output would be
reported.  The driver also re-checks one identity (segmented run with scanned states and correction ==
unsegmented run, App. A.1) so that the sanitized build is known to compute, not only to run."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r"""
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
void oracle_gla_recurrent(int, int, int, int, int, const double *, const double *, const double *, const double *,
                          double, const double *, double *, double *);
void oracle_gla_local(int, int, int, int, int, int, const double *, const double *, const double *, const double *,
                      double, double *, double *, double *, double *);
void oracle_state_scan(int, int, int, int, const double *, const double *, const double *, double *, double *);
void oracle_apply_init_state(int, int, int, int, int, int, const double *, const double *, const double *, double,
                             double *);
void oracle_gla_recurrent_bwd(int, int, int, int, int, const double *, const double *, const double *,
                              const double *, double, const double *, const double *, const double *, double *,
                              double *, double *, double *, double *);
static unsigned long long s = 88172645463325252ull;
static double rnd(void) { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return (double)(s >> 11) / 9007199254740992.0 - 0.5; }
static double *buf(size_t n, int fill) {
    double *p = malloc(n * sizeof(double));
    for (size_t i = 0; i < n; ++i) p[i] = fill ? rnd() : NAN;
    return p;
}
int main(void) {
    const int B = 2, P = 3, H = 3, L = 67, dk = 5, dv = 7, T = P * L;
    const size_t nk = (size_t)B * T * H * dk, nv = (size_t)B * T * H * dv, ns = (size_t)B * H * dk * dv;
    double *q = buf(nk, 1), *k = buf(nk, 1), *v = buf(nv, 1), *g = buf(nk, 1), *S0 = buf(ns, 1);
    for (size_t i = 0; i < nk; ++i) g[i] = -0.2 * fabs(g[i]);
    double *o = buf(nv, 0), *Sf = buf(ns, 0);
    oracle_gla_recurrent(B, T, H, dk, dv, q, k, v, g, 0.7, S0, o, Sf);
    double *ol = buf(nv, 0), *Sl = buf(P * ns, 0), *Gc = buf(nk, 0), *Gt = buf((size_t)P * B * H * dk, 0);
    oracle_gla_local(B, P, H, L, dk, dv, q, k, v, g, 0.7, ol, Sl, Gc, Gt);
    double *Si = buf(P * ns, 0), *Sla = buf(ns, 0);
    oracle_state_scan(P, B * H, dk, dv, Sl, Gt, S0, Si, Sla);
    oracle_apply_init_state(B, P, H, L, dk, dv, q, Gc, Si, 0.7, ol);
    double err = 0, mx = 0;
    for (size_t i = 0; i < nv; ++i) { err = fmax(err, fabs(ol[i] - o[i])); mx = fmax(mx, fabs(o[i])); }
    for (size_t i = 0; i < ns; ++i) err = fmax(err, fabs(Sla[i] - Sf[i]));
    double *dO = buf(nv, 1), *dST = buf(ns, 1);
    double *dq = buf(nk, 0), *dkk = buf(nk, 0), *dvv = buf(nv, 0), *dg = buf(nk, 0), *dS0 = buf(ns, 0);
    oracle_gla_recurrent_bwd(B, T, H, dk, dv, q, k, v, g, 0.7, S0, dO, dST, dq, dkk, dvv, dg, dS0);
    double chk = 0;
    for (size_t i = 0; i < nk; ++i) chk += dq[i] + dkk[i] + dg[i];
    for (size_t i = 0; i < nv; ++i) chk += dvv[i];
    for (size_t i = 0; i < ns; ++i) chk += dS0[i];
    printf("segmented-vs-unsegmented err %.3e (max |o| %.3e), gradient checksum %.6e\n", err, mx, chk);
    free(q); free(k); free(v); free(g); free(S0); free(o); free(Sf); free(ol); free(Sl); free(Gc); free(Gt);
    free(Si); free(Sla); free(dO); free(dST); free(dq); free(dkk); free(dvv); free(dg); free(dS0);
    return !(err < 1e-12 * (1 + mx)) || !(chk == chk);
}
"""


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    drv = tmp_path / "driver.c"
    drv.write_text(DRIVER)
    exe = tmp_path / "oracle_san"
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", str(drv), os.path.join(ROOT, "oracle", "gla_oracle.c"), "-lm", "-o", str(exe)]
    subprocess.check_call(cmd)
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0")
    res = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    sys.stdout.write(res.stdout)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "ERROR: AddressSanitizer" not in res.stderr and "runtime error" not in res.stderr, res.stderr
