/*
 * CPU oracle for the ZeCO gated-linear-attention (GLA) hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, fp64, written straight from the paper's definitions.  It shares no code with
 * the HIP library and must never be reached from the product path: only tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it.
 *
 * Layouts (all contiguous, row-major, double):
 *   q, k, g, G_cum : [B, T, H, d_k]      v, o : [B, T, H, d_v]       T = P * L
 *   states         : [.., d_k, d_v]      decay scales ROW i (the d_k index) of a state
 *   g is the LOG decay, alpha = exp(g)  (the paper's G holds alpha itself; Alg. 1 input line)
 *
 * Parity pins (tests/test_oracle_pins.py): brute-force quadratic unrolling of Eq. (1), the
 * geometric-series closed form, g == 0 -> causal linear attention, the single-chunk masked
 * matmul of Sec. 2.1, segmentation invariance (Eq. (global-correction), App. A.1), cumsum /
 * product forms of the segment scan, linearity; for the backward pass: reverse-mode
 * differentiation of an independent quadratic-form forward, central finite differences of the
 * forward oracle, the reverse-cumulative-sum identity of App. A.4 for the gate gradient, chaining
 * of segments through dS, and the g == 0 matmul closed form.  No function here is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

/* One (b, h) stream of the recurrence of Sec. 2.1, Eq. (1):
 *     S_t = (alpha_t^T 1) .* S_{t-1} + k_t^T v_t ,   o_t = scale * q_t S_t
 * token by token, no chunking, no segmentation.  S (d_k x d_v) is updated in place. */
static void recur_stream(int T, int dk, int dv, ptrdiff_t sk, ptrdiff_t sv,
                         const double *q, const double *k, const double *v, const double *g,
                         double scale, double *S, double *o)
{
    for (int t = 0; t < T; ++t) {
        const double *qt = q + t * sk, *kt = k + t * sk, *gt = g + t * sk;
        const double *vt = v + t * sv;
        double *ot = o + t * sv;
        for (int i = 0; i < dk; ++i) {
            const double a = exp(gt[i]);
            double *Si = S + (size_t)i * dv;
            for (int j = 0; j < dv; ++j) Si[j] = a * Si[j] + kt[i] * vt[j];
        }
        for (int j = 0; j < dv; ++j) ot[j] = 0.0;
        for (int i = 0; i < dk; ++i) {
            const double *Si = S + (size_t)i * dv;
            const double qi = scale * qt[i];
            for (int j = 0; j < dv; ++j) ot[j] += qi * Si[j];
        }
    }
}

/* Eq. (1) over the whole sequence of T tokens for every (b, h).
 * S0      [B,H,d_k,d_v] or NULL (zero state)
 * S_final [B,H,d_k,d_v] or NULL */
void oracle_gla_recurrent(int B, int T, int H, int dk, int dv,
                          const double *q, const double *k, const double *v, const double *g,
                          double scale, const double *S0, double *o, double *S_final)
{
    const ptrdiff_t sk = (ptrdiff_t)H * dk, sv = (ptrdiff_t)H * dv;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            double *S = (double *)malloc(sizeof(double) * dk * dv);
            const size_t bh = (size_t)b * H + h;
            if (S0) memcpy(S, S0 + bh * dk * dv, sizeof(double) * dk * dv);
            else memset(S, 0, sizeof(double) * dk * dv);
            const size_t ok = ((size_t)b * T * H + h) * dk, ov = ((size_t)b * T * H + h) * dv;
            recur_stream(T, dk, dv, sk, sv, q + ok, k + ok, v + ov, g + ok, scale, S, o + ov);
            if (S_final) memcpy(S_final + bh * dk * dv, S, sizeof(double) * dk * dv);
            free(S);
        }
}

/* Local pass of Sec. 3.1: every segment p (L tokens) runs Eq. (1) from the ZERO state.
 * Emits the local output, the final local state S_[N] of each segment, and the cumulative
 * decay of Eq. (gamma) kept per token and in the log domain:
 *   G_cum[t] = sum of g over the segment's tokens up to and including t
 *   G_tot[p] = G_cum at the segment's last token  (log of gamma~_[N])
 * S_loc [P,B,H,d_k,d_v], G_tot [P,B,H,d_k]. */
void oracle_gla_local(int B, int P, int H, int L, int dk, int dv,
                      const double *q, const double *k, const double *v, const double *g,
                      double scale, double *o_local, double *S_loc, double *G_cum, double *G_tot)
{
    const int T = P * L;
    const ptrdiff_t sk = (ptrdiff_t)H * dk, sv = (ptrdiff_t)H * dv;
#pragma omp parallel for collapse(3) schedule(dynamic)
    for (int b = 0; b < B; ++b)
        for (int p = 0; p < P; ++p)
            for (int h = 0; h < H; ++h) {
                const size_t t0 = (size_t)p * L;
                const size_t ok = (((size_t)b * T + t0) * H + h) * dk;
                const size_t ov = (((size_t)b * T + t0) * H + h) * dv;
                double *S = S_loc + (((size_t)p * B + b) * H + h) * dk * dv;
                memset(S, 0, sizeof(double) * dk * dv);
                recur_stream(L, dk, dv, sk, sv, q + ok, k + ok, v + ov, g + ok, scale, S,
                             o_local + ov);
                for (int i = 0; i < dk; ++i) {
                    double acc = 0.0;
                    for (int t = 0; t < L; ++t) {
                        acc += g[ok + (size_t)t * sk + i];
                        G_cum[ok + (size_t)t * sk + i] = acc;
                    }
                    G_tot[(((size_t)p * B + b) * H + h) * dk + i] = acc;
                }
            }
}

/* All-Scan recurrence of Sec. 3.2 (block equation), read as an exclusive scan over segments:
 *   S_init[0] = S0 (or 0),   S_init[p+1] = (exp(G_tot[p])^T 1) .* S_init[p] + S_loc[p]
 * S_init[p] is what rank p receives (S_recv), S_init[p+1] what it sends (S_send).
 * S_loc, S_init [P,BH,d_k,d_v]; G_tot [P,BH,d_k]; S0, S_last [BH,d_k,d_v] (nullable). */
void oracle_state_scan(int P, int BH, int dk, int dv, const double *S_loc, const double *G_tot,
                       const double *S0, double *S_init, double *S_last)
{
    const size_t ss = (size_t)dk * dv;
#pragma omp parallel for schedule(static)
    for (int bh = 0; bh < BH; ++bh) {
        double *cur = (double *)malloc(sizeof(double) * ss);
        if (S0) memcpy(cur, S0 + bh * ss, sizeof(double) * ss);
        else memset(cur, 0, sizeof(double) * ss);
        for (int p = 0; p < P; ++p) {
            memcpy(S_init + ((size_t)p * BH + bh) * ss, cur, sizeof(double) * ss);
            const double *loc = S_loc + ((size_t)p * BH + bh) * ss;
            const double *gt = G_tot + ((size_t)p * BH + bh) * dk;
            for (int i = 0; i < dk; ++i) {
                const double a = exp(gt[i]);
                for (int j = 0; j < dv; ++j)
                    cur[(size_t)i * dv + j] = a * cur[(size_t)i * dv + j] + loc[(size_t)i * dv + j];
            }
        }
        if (S_last) memcpy(S_last + bh * ss, cur, sizeof(double) * ss);
        free(cur);
    }
}

/* Initial-state correction (Alg. 1 output pass, the term added to S_[n-1]; with
 * Lambda_t .* gamma~_[n-1] = exp(G_cum[t])):
 *   o_t += (scale * q_t .* exp(G_cum[t])) S_init[p]        for every token t of segment p
 * S_init [P,B,H,d_k,d_v]; o is updated in place. */
void oracle_apply_init_state(int B, int P, int H, int L, int dk, int dv, const double *q,
                             const double *G_cum, const double *S_init, double scale, double *o)
{
    const int T = P * L;
#pragma omp parallel for collapse(3) schedule(dynamic)
    for (int b = 0; b < B; ++b)
        for (int p = 0; p < P; ++p)
            for (int h = 0; h < H; ++h) {
                const double *S = S_init + (((size_t)p * B + b) * H + h) * dk * dv;
                for (int t = 0; t < L; ++t) {
                    const size_t tok = (size_t)b * T + (size_t)p * L + t;
                    const double *qt = q + (tok * H + h) * dk;
                    const double *Gt = G_cum + (tok * H + h) * dk;
                    double *ot = o + (tok * H + h) * dv;
                    for (int i = 0; i < dk; ++i) {
                        const double w = scale * qt[i] * exp(Gt[i]);
                        const double *Si = S + (size_t)i * dv;
                        for (int j = 0; j < dv; ++j) ot[j] += w * Si[j];
                    }
                }
            }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Backward of Eq. (1) (App. A.4 computes the same gradients chunk by chunk).  For the scalar
 *     loss = sum_t <o_t, dO_t> + <S_T, dS_T>
 * reverse-mode differentiation of  S_t = (alpha_t^T 1) .* S_{t-1} + k_t^T v_t,  o_t = scale q_t S_t,
 * alpha_t = exp(g_t), gives, walking t = T-1 .. 0 with E = d loss / d S_t from the later tokens
 * (E = dS_T at the last token):
 *     dS_t  = E + scale q_t^T dO_t
 *     dq_t  = scale dO_t S_t^T           dk_t = (dS_t v_t^T)^T          dv_t = k_t dS_t
 *     dg_t[i] = alpha_t[i] * sum_j dS_t[i,j] S_{t-1}[i,j]
 *     E    <- (alpha_t^T 1) .* dS_t      (after t = 0 this is d loss / d S0)
 * The forward states are kept at block boundaries and recomputed inside one block at a time.
 * dO [B,T,H,d_v]; S0, dS_T, dS0 [B,H,d_k,d_v] (S0, dS_T, dS0 nullable). */
void oracle_gla_recurrent_bwd(int B, int T, int H, int dk, int dv,
                              const double *q, const double *k, const double *v, const double *g,
                              double scale, const double *S0, const double *dO, const double *dS_T,
                              double *dq, double *dk_out, double *dv_out, double *dg, double *dS0)
{
    const ptrdiff_t sk = (ptrdiff_t)H * dk, sv = (ptrdiff_t)H * dv;
    const size_t ss = (size_t)dk * dv;
    const int BLK = 128;
    const int nblk = (T + BLK - 1) / BLK;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            const size_t bh = (size_t)b * H + h;
            const size_t ok = ((size_t)b * T * H + h) * dk, ov = ((size_t)b * T * H + h) * dv;
            /* forward sweep: state before the first token of every block */
            double *ckpt = (double *)malloc(sizeof(double) * ss * nblk);
            double *Sblk = (double *)malloc(sizeof(double) * ss * (BLK + 1));   /* S_{t0-1} .. S_{t1-1} */
            double *S = (double *)malloc(sizeof(double) * ss);
            double *E = (double *)malloc(sizeof(double) * ss);
            double *dS = (double *)malloc(sizeof(double) * ss);
            if (S0) memcpy(S, S0 + bh * ss, sizeof(double) * ss);
            else memset(S, 0, sizeof(double) * ss);
            for (int t = 0; t < T; ++t) {
                if (t % BLK == 0) memcpy(ckpt + (size_t)(t / BLK) * ss, S, sizeof(double) * ss);
                for (int i = 0; i < dk; ++i) {
                    const double a = exp(g[ok + t * sk + i]);
                    for (int j = 0; j < dv; ++j)
                        S[i * dv + j] = a * S[i * dv + j] + k[ok + t * sk + i] * v[ov + t * sv + j];
                }
            }
            if (dS_T) memcpy(E, dS_T + bh * ss, sizeof(double) * ss);
            else memset(E, 0, sizeof(double) * ss);
            for (int blk = nblk - 1; blk >= 0; --blk) {
                const int t0 = blk * BLK, t1 = (t0 + BLK < T) ? t0 + BLK : T;
                memcpy(Sblk, ckpt + (size_t)blk * ss, sizeof(double) * ss);
                for (int t = t0; t < t1; ++t) {   /* Sblk[t - t0 + 1] = S_t */
                    const double *prev = Sblk + (size_t)(t - t0) * ss;
                    double *cur = Sblk + (size_t)(t - t0 + 1) * ss;
                    for (int i = 0; i < dk; ++i) {
                        const double a = exp(g[ok + t * sk + i]);
                        for (int j = 0; j < dv; ++j)
                            cur[i * dv + j] = a * prev[i * dv + j] + k[ok + t * sk + i] * v[ov + t * sv + j];
                    }
                }
                for (int t = t1 - 1; t >= t0; --t) {
                    const double *St = Sblk + (size_t)(t - t0 + 1) * ss;
                    const double *Sp = Sblk + (size_t)(t - t0) * ss;
                    const double *qt = q + ok + t * sk, *kt = k + ok + t * sk, *gt = g + ok + t * sk;
                    const double *vt = v + ov + t * sv, *dOt = dO + ov + t * sv;
                    for (int j = 0; j < dv; ++j) dv_out[ov + t * sv + j] = 0.0;
                    for (int i = 0; i < dk; ++i) {
                        const double a = exp(gt[i]);
                        double accq = 0.0, acck = 0.0, accg = 0.0;
                        for (int j = 0; j < dv; ++j) {
                            const double d = E[i * dv + j] + scale * qt[i] * dOt[j];
                            dS[i * dv + j] = d;
                            accq += dOt[j] * St[i * dv + j];
                            acck += d * vt[j];
                            accg += d * Sp[i * dv + j];
                            dv_out[ov + t * sv + j] += kt[i] * d;
                        }
                        dq[ok + t * sk + i] = scale * accq;
                        dk_out[ok + t * sk + i] = acck;
                        dg[ok + t * sk + i] = a * accg;
                        for (int j = 0; j < dv; ++j) E[i * dv + j] = a * dS[i * dv + j];
                    }
                }
            }
            if (dS0) memcpy(dS0 + bh * ss, E, sizeof(double) * ss);
            free(ckpt); free(Sblk); free(S); free(E); free(dS);
        }
}
