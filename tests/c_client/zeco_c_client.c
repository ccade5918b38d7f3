/* A client of libzeco.so written in plain C (no Python, no torch, no C++): device memory from hipMalloc,
 * the three calls of the method on the null stream, and a comparison with the fp64 oracle (Eq. (1) token by
 * token) linked into the same program.  It checks what the Python tests cannot: that the header compiles as
 * C, that the descriptor struct and the enums have the layout the library was built with, and that the
 * library needs nothing from its caller but device pointers and a stream.  Test infrastructure: built by
 * tests/c_client/build_c_client.py, run by tests/test_gpu_c_client.py.  Exit status 0 = all checks passed. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "zeco.h"

void oracle_gla_recurrent(int B, int T, int H, int dk, int dv, const double *q, const double *k,
                          const double *v, const double *g, double scale, const double *S0, double *o,
                          double *S_final);

#define CHECK_HIP(x)                                                                        \
    do {                                                                                    \
        hipError_t e_ = (x);                                                                \
        if (e_ != hipSuccess) {                                                             \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                         \
            return 2;                                                                       \
        }                                                                                   \
    } while (0)
#define CHECK_ZECO(x)                                                                       \
    do {                                                                                    \
        zeco_status s_ = (x);                                                               \
        if (s_ != ZECO_OK) {                                                                \
            fprintf(stderr, "%s: %s\n", #x, zeco_status_string(s_));                        \
            return 3;                                                                       \
        }                                                                                   \
    } while (0)

static uint64_t lcg_state = 0x9E3779B97F4A7C15ull;
static double uniform01(void) {
    lcg_state = lcg_state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(lcg_state >> 11) / 9007199254740992.0;
}
static double gaussian(void) {   /* sum of 12 uniforms: close enough to N(0,1) for test data */
    double s = -6.0;
    for (int i = 0; i < 12; ++i) s += uniform01();
    return s;
}
static uint16_t to_bf16(double x) {   /* round to nearest even */
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
static double from_bf16(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}
static double rel_err(const double *x, const double *ref, size_t n) {
    double num = 0.0, den = 1e-30;
    for (size_t i = 0; i < n; ++i) {
        const double d = fabs(x[i] - ref[i]);
        if (d > num) num = d;
        if (fabs(ref[i]) > den) den = fabs(ref[i]);
    }
    return num / den;
}

int main(void) {
    enum { B = 1, H = 2, P = 3, L = 200, DK = 128, DV = 128, T = P * L };   /* L is no multiple of 64 on purpose */
    const size_t nk = (size_t)B * T * H * DK, nv = (size_t)B * T * H * DV, ns = (size_t)B * H * DK * DV;
    printf("libzeco version %d\n", (int)zeco_version());

    /* inputs: q, v ~ N(0,1), k normalised per token, slow decay so that the scanned state reaches every token */
    double *q = malloc(nk * 8), *k = malloc(nk * 8), *g = malloc(nk * 8), *v = malloc(nv * 8);
    uint16_t *qh = malloc(nk * 2), *kh = malloc(nk * 2), *vh = malloc(nv * 2);
    float *gh = malloc(nk * 4);
    if (!q || !k || !g || !v || !qh || !kh || !vh || !gh) return 2;
    for (size_t r = 0; r < (size_t)B * T * H; ++r) {
        double norm = 0.0;
        for (int i = 0; i < DK; ++i) {
            q[r * DK + i] = gaussian();
            k[r * DK + i] = gaussian();
            norm += k[r * DK + i] * k[r * DK + i];
            gh[r * DK + i] = (float)(-0.004 * (1.0 + uniform01()));
        }
        for (int i = 0; i < DK; ++i) k[r * DK + i] /= sqrt(norm);
        for (int j = 0; j < DV; ++j) v[r * DV + j] = gaussian();
    }
    for (size_t i = 0; i < nk; ++i) {   /* the oracle sees the values the GPU sees */
        qh[i] = to_bf16(q[i]); q[i] = from_bf16(qh[i]);
        kh[i] = to_bf16(k[i]); k[i] = from_bf16(kh[i]);
        g[i] = (double)gh[i];
    }
    for (size_t i = 0; i < nv; ++i) { vh[i] = to_bf16(v[i]); v[i] = from_bf16(vh[i]); }

    zeco_gla_desc d;
    memset(&d, 0, sizeof d);
    d.B = B; d.P = P; d.H = H; d.L = L; d.d_k = DK; d.d_v = DV; d.C = 64;
    d.io_dtype = ZECO_BF16; d.g_dtype = ZECO_F32; d.scale = 0.5f;
    d.stride_b = (int64_t)T * H * DK; d.stride_t = H * DK; d.stride_h = DK;
    d.vstride_b = (int64_t)T * H * DV; d.vstride_t = H * DV; d.vstride_h = DV;
    d.g_per_head = 0; d.wide_gates = 0;

    /* error paths answer before any HIP call */
    zeco_gla_desc bad = d;
    bad.C = 32;
    if (zeco_gla_local_fwd(&bad, qh, qh, qh, qh, qh, NULL, NULL, NULL, NULL, 0, NULL) != ZECO_ERR_UNSUPPORTED) return 4;
    if (zeco_gla_local_fwd(&d, NULL, qh, qh, qh, qh, NULL, NULL, NULL, NULL, 0, NULL) != ZECO_ERR_INVALID_ARG) return 4;

    void *dq, *dk, *dv, *dg, *dout, *ws = NULL;
    float *S_loc, *G_cum, *G_tot, *S_init, *S_last;
    CHECK_HIP(hipSetDevice(0));
    CHECK_HIP(hipMalloc(&dq, nk * 2)); CHECK_HIP(hipMalloc(&dk, nk * 2)); CHECK_HIP(hipMalloc(&dv, nv * 2));
    CHECK_HIP(hipMalloc(&dg, nk * 4)); CHECK_HIP(hipMalloc(&dout, nv * 2));
    CHECK_HIP(hipMalloc((void **)&S_loc, P * ns * 4)); CHECK_HIP(hipMalloc((void **)&S_init, P * ns * 4));
    CHECK_HIP(hipMalloc((void **)&S_last, ns * 4)); CHECK_HIP(hipMalloc((void **)&G_cum, nk * 4));
    CHECK_HIP(hipMalloc((void **)&G_tot, (size_t)P * B * H * DK * 4));
    const size_t ws_bytes = zeco_gla_local_fwd_workspace(&d);
    if (ws_bytes) CHECK_HIP(hipMalloc(&ws, ws_bytes));
    CHECK_HIP(hipMemcpy(dq, qh, nk * 2, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dk, kh, nk * 2, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dv, vh, nv * 2, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dg, gh, nk * 4, hipMemcpyHostToDevice));

    /* the three calls of the method, on the null stream */
    CHECK_ZECO(zeco_gla_local_fwd(&d, dq, dk, dv, dg, dout, S_loc, G_cum, G_tot, ws, ws_bytes, NULL));
    CHECK_ZECO(zeco_state_scan(P, B * H, DK, DV, 16, S_loc, G_tot, NULL, S_init, S_last, 0, 0, NULL));
    CHECK_ZECO(zeco_apply_init_state(&d, dq, G_cum, S_init, dout, ZECO_APPLY_FIRST_SEGMENT_ZERO, NULL));
    CHECK_HIP(hipDeviceSynchronize());

    uint16_t *oh = malloc(nv * 2);
    float *Sh = malloc(ns * 4);
    double *o = malloc(nv * 8), *S = malloc(ns * 8), *o_ref = malloc(nv * 8), *S_ref = malloc(ns * 8);
    if (!oh || !Sh || !o || !S || !o_ref || !S_ref) return 2;
    CHECK_HIP(hipMemcpy(oh, dout, nv * 2, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(Sh, S_last, ns * 4, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < nv; ++i) o[i] = from_bf16(oh[i]);
    for (size_t i = 0; i < ns; ++i) S[i] = (double)Sh[i];
    oracle_gla_recurrent(B, T, H, DK, DV, q, k, v, g, 0.5, NULL, o_ref, S_ref);
    const double eo = rel_err(o, o_ref, nv), es = rel_err(S, S_ref, ns);
    printf("three calls from C against the oracle: rel err o %.3e, final state %.3e (bound 2e-2)\n", eo, es);

    /* the whole forward in one call must agree too */
    const size_t fb = zeco_gla_fused_fwd_workspace(&d);
    void *fws;
    CHECK_HIP(hipMalloc(&fws, fb ? fb : 16));
    CHECK_ZECO(zeco_gla_fused_fwd(&d, dq, dk, dv, dg, NULL, dout, S_last, NULL, ZECO_SCHEDULE_AUTO, fws, fb, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(oh, dout, nv * 2, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < nv; ++i) o[i] = from_bf16(oh[i]);
    const double ef = rel_err(o, o_ref, nv);
    printf("fused forward from C against the oracle: rel err o %.3e\n", ef);

    /* the same tokens cut into three segments of unequal length, given as a device table of int64 offsets */
    const int64_t start[P + 1] = {0, 70, 407, T};
    int64_t *dstart;
    CHECK_HIP(hipMalloc((void **)&dstart, sizeof start));
    CHECK_HIP(hipMemcpy(dstart, start, sizeof start, hipMemcpyHostToDevice));
    zeco_gla_desc dvar = d;
    dvar.L = 400;   /* any bound on the segment lengths (the longest is 337) */
    CHECK_ZECO(zeco_gla_local_fwd_varlen(&dvar, dstart, T, dq, dk, dv, dg, dout, S_loc, G_cum, G_tot, NULL));
    CHECK_ZECO(zeco_state_scan(P, B * H, DK, DV, 16, S_loc, G_tot, NULL, S_init, S_last, 0, 0, NULL));
    CHECK_ZECO(zeco_apply_init_state_varlen(&dvar, dstart, T, dq, G_cum, S_init, dout, ZECO_APPLY_FIRST_SEGMENT_ZERO, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(oh, dout, nv * 2, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(Sh, S_last, ns * 4, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < nv; ++i) o[i] = from_bf16(oh[i]);
    for (size_t i = 0; i < ns; ++i) S[i] = (double)Sh[i];
    const double ev = rel_err(o, o_ref, nv), evs = rel_err(S, S_ref, ns);
    printf("unequal segments from C against the oracle: rel err o %.3e, final state %.3e\n", ev, evs);

    hipFree(dq); hipFree(dk); hipFree(dv); hipFree(dg); hipFree(dout); hipFree(S_loc); hipFree(S_init);
    hipFree(S_last); hipFree(G_cum); hipFree(G_tot); hipFree(fws); hipFree(dstart);
    if (ws) hipFree(ws);
    if (!(eo <= 2e-2 && es <= 2e-2 && ef <= 2e-2 && ev <= 2e-2 && evs <= 2e-2)) { printf("FAILED\n"); return 1; }
    printf("OK\n");
    return 0;
}
