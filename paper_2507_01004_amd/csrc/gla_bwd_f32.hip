// Backward of the chunkwise GLA forward for the two gated operands (App. A.4), fp32 inputs and outputs,
// fp32 MFMA (16x16x4): dQ, dK and the gate gradient dG.  The accuracy path beside gla_bwd_qk.hip, which
// is the throughput path; same equations, one workgroup per (batch, segment, head) stream, no pipelining.
//
// With Lambda the in-chunk cumulative decay, gamma the chunk decay, S the forward state entering a chunk,
// dS the state gradient entering it from the later chunks, dA = mask(dO V^T):
//   dQ_t = Lambda_t   .* [ dO_t S^T                    + sum_{s<=t} dA_ts (K_s / Lambda_s) ]      forward over chunks
//   dK_s = 1/Lambda_s .* [ V_s ((gamma^T 1) .* dS)^T   + sum_{t>=s} dA_ts (Q_t .* Lambda_t) ]    backward over chunks
// i.e.  out_r = F_r .* [ X_r W + sum_{r'<=r} (X_r . Y_r') Z~_r' ]  with
//   dQ: X = dO, Y = V, Z~ = K / Lambda, F = Lambda,     W = S^T
//   dK: X = V, Y = dO, Z~ = Q .* Lambda, F = 1/Lambda,  W = dS^T, chunks last to first, token t at tile row C-1-t
// log Lambda is counted from half the chunk's total log decay (no exponent beyond |total| / 2, so the sum of
// |g| over a chunk may reach 160), and W takes sqrt(gamma) twice: before the chunk's products with it and
// after its update W <- W + Y^T Z~.  W (d_v x d_k, the transposed state) stays in MFMA accumulators, wave w
// owns the output channels [16w, 16w+16); an accumulator register is the B operand of the 16x16x4 step
// whose k-slots are its rows, so X W needs no copy of W.
//
// A segment length that is no multiple of C makes the LAST chunk the short one in both passes (its missing
// tokens count as zero rows), so that both cut a segment at the same tokens.
//
// dG (last line of the backward listing of App. A.4): dG_t = sum over later tokens s >= t of
// (Q_s .* dQ_s - K_s .* dK_s); what the later segments contribute is row_sum(dS_end .* S_end) of the
// segment's final state and its gradient.  The dQ pass leaves Q .* dQ in the dG array; the dK pass, which
// walks the tokens from the last to the first anyway, subtracts K .* dK, accumulates and overwrites the
// array with dG.  The terms nearly cancel, so the running sum collects their rounding noise; at every
// chunk boundary its exact value is row_sum(dS .* S), and with a checkpoint array (S_ck) the dQ pass stores
// the state at every 512th token of a segment and the dK pass replaces its running value there.
#include "zeco_device.h"
#include "zeco_internal.h"

namespace zeco {

template <int DK, int DV, int C> struct QKF32Cfg {
    static constexpr int kWaves = DK / 16;          // 16 output channels each
    static constexpr int kThreads = 64 * kWaves;
    static constexpr int kNIT = DV / 16;            // row tiles of W per wave
    static constexpr int kTG = kThreads / DK;       // token groups in the gate pass (4)
    static constexpr int kTPT = C / kTG;            // tokens per thread in the gate pass
    static constexpr int kNT = C / 16;              // 16-token tiles per chunk
    static constexpr int kTiles = kNT * (kNT + 1) / 2;
    static constexpr int kAnchor = 512 / C;         // chunks between two checkpoints of the forward state
    static constexpr int kXS = DV + 4;              // row strides (floats)
    static constexpr int kZS = DK + 16;
    static constexpr int kFS = DK + 4;
    static constexpr int kPS = C + 4;
    static constexpr int kOffX = 0;
    static constexpr int kOffY = kOffX + C * kXS;
    static constexpr int kOffZ = kOffY + C * kXS;
    static constexpr int kOffF = kOffZ + C * kZS;
    static constexpr int kOffP = kOffF + C * kFS;
    static constexpr int kOffTot = kOffP + C * kPS;
    static constexpr int kOffTot2 = kOffTot + kTG * DK;
    static constexpr int kOffGam = kOffTot2 + kTG * DK;
    static constexpr int kOffCarry = kOffGam + DK;
    static constexpr int kOffAnchor = kOffCarry + DK;
    static constexpr int kFloats = kOffAnchor + DK;
    static constexpr size_t kBytes = sizeof(float) * kFloats;
    static_assert(kTPT >= 1 && C % 16 == 0 && 512 % C == 0 && kBytes <= 163840, "chunk length");
};

// REV = false: dQ (x = dO, y = v, z = k, z2 = q, W_init = forward states; the query scale multiplies the
// output).  REV = true: dK and dG (x = v, y = dO, z = q, z2 = k, W_init = state gradients entering each
// segment's final state; the query scale rides on Q .* Lambda, so that the running dS is the true gradient).
template <int DK, int DV, int C, bool REV>
__global__ __launch_bounds__(DK * 4) void gla_bwd_qk_f32_kernel(BwdQKParams p) {
    typedef QKF32Cfg<DK, DV, C> Cfg;
    constexpr float SZ = REV ? 1.f : -1.f;   // exponent sign of the operand Z~; the factor F takes the other
    extern __shared__ __align__(16) float lds[];
    float *Xs = lds + Cfg::kOffX, *Ys = lds + Cfg::kOffY, *Zs = lds + Cfg::kOffZ;
    float *Fs = lds + Cfg::kOffF;      // the factor F [row][i]; then the finished gradient tile
    float *Ps = lds + Cfg::kOffP;      // masked X Y^T [row][row']
    float *tot = lds + Cfg::kOffTot;   // [token group][channel] gate sums
    float *tot2 = lds + Cfg::kOffTot2; // [token group][channel] sums of the dG terms
    float *gam = lds + Cfg::kOffGam;   // sqrt(gamma) [channel]
    float *carry0 = lds + Cfg::kOffCarry;
    float *anchor = lds + Cfg::kOffAnchor;

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int l16 = lane & 15, kg = lane >> 4;

    const size_t sbh = blockIdx.x;                  // (seg * B + b) * H + h
    int sidx = blockIdx.x;
    const int h = sidx % p.H;
    sidx /= p.H;
    const int b = sidx % p.B, seg = sidx / p.B;
    long long tok0 = (long long)seg * p.L, T = (long long)p.P * p.L, len = p.L;
    if (p.seg_start) {
        // segments of unequal length: this one's bounds from the table; a segment that cannot be taken (under
        // 64 tokens, over the bound L, outside the tensor) is left alone
        tok0 = p.seg_start[seg];
        T = p.T;
        len = p.seg_start[seg + 1] - tok0;
        if (tok0 < 0 || len < 64 || len > p.L || tok0 > T - len) return;   // (in this order: no sum can overflow)
    }
    const int N = (int)((len + C - 1) / C);
    const long long kbase = b * p.sb + tok0 * p.st + h * p.sh;
    const long long vbase = b * p.vb + tok0 * p.vt + h * p.vh;
    const float *x = (const float *)p.x + vbase, *y = (const float *)p.y + vbase;
    const float *z = (const float *)p.z + kbase, *z2 = (const float *)p.z2 + kbase;
    const float *g = (const float *)p.g + kbase;
    float *out = (float *)p.out + kbase;
    float *dg = p.dg + (((long long)b * T + tok0) * p.H + h) * DK;   // [B,T,H,d_k] contiguous
    const long long gcs = (long long)p.H * DK;

    // W^T tile init: Wacc[it][r] = W[row 16 it + 4 kg + r][col 16 w + l16] = W_init[col][row]
    f32x4 Wacc[Cfg::kNIT];
    {
        const float *Wi = p.W_init + sbh * DK * DV + (size_t)(w * 16 + l16) * DV + 4 * kg;
#pragma unroll
        for (int it = 0; it < Cfg::kNIT; ++it) Wacc[it] = *reinterpret_cast<const f32x4 *>(Wi + it * 16);
    }

    const int gc = tid % DK, tg = tid / DK;      // gate pass: channel and token group
    auto row_of = [](int t) { return REV ? C - 1 - t : t; };

    // dG carried in from the later segments: c[i] = sum_j dS_end[i][j] S_end[i][j]  (4 threads per row)
    float carry = 0.f;
    if constexpr (REV) {
        const float *A = p.W_init + sbh * DK * DV;
        const float *Bm = (seg + 1 < p.P) ? p.S_init + (sbh + (size_t)p.B * p.H) * DK * DV
                                          : p.S_last + ((size_t)b * p.H + h) * DK * DV;
        const int i = tid >> 2, part = tid & 3;
        float acc = 0.f;
        for (int j = part * 4; j < DV; j += 16) {
            const f32x4 a4 = *reinterpret_cast<const f32x4 *>(A + (size_t)i * DV + j);
            const f32x4 b4 = *reinterpret_cast<const f32x4 *>(Bm + (size_t)i * DV + j);
            acc += a4[0] * b4[0] + a4[1] * b4[1] + a4[2] * b4[2] + a4[3] * b4[3];
        }
        acc += __shfl_xor(acc, 1, 64);
        acc += __shfl_xor(acc, 2, 64);
        if (part == 0) carry0[i] = acc;
        __syncthreads();
        carry = carry0[gc];
    }

    for (int n = 0; n < N; ++n) {
        const int c = REV ? N - 1 - n : n;                       // chunk index in the segment
        const long long tc = (long long)c * C;                   // its first token
        const int rows = (c == N - 1) ? (int)(len - tc) : C;     // its real tokens
        if constexpr (!REV) {
            // checkpoint: the forward state entering this chunk, for the dK pass to re-anchor dG with (the
            // accumulators as they are: the dK pass holds the gradient in the same layout)
            if (p.S_ck && c > 0 && c % Cfg::kAnchor == 0) {
                float *ck = p.S_ck + (sbh * p.n_ck + (c / Cfg::kAnchor - 1)) * DK * DV + (size_t)tid * (Cfg::kNIT * 4);
#pragma unroll
                for (int it = 0; it < Cfg::kNIT; ++it) *reinterpret_cast<f32x4 *>(ck + it * 4) = Wacc[it];
            }
        }

        // ---- gate pass, part 1: inclusive cumulative sum of g over the chunk, per channel; X, Y -> LDS ----
        float cs[Cfg::kTPT];
        {
            float run = 0.f;
#pragma unroll
            for (int u = 0; u < Cfg::kTPT; ++u) {
                const int t = tg * Cfg::kTPT + u;
                run += t < rows ? g[(tc + t) * p.st + gc] : 0.f;
                cs[u] = run;
            }
            tot[tg * DK + gc] = run;
        }
        for (int e = tid; e < C * DV; e += Cfg::kThreads) {
            const int t = e / DV, j = e % DV;
            Xs[row_of(t) * Cfg::kXS + j] = t < rows ? x[(tc + t) * p.vt + j] : 0.f;
            Ys[row_of(t) * Cfg::kXS + j] = t < rows ? y[(tc + t) * p.vt + j] : 0.f;
        }
        __syncthreads();

        // ---- gate pass, part 2: Z~ and the factor tile -> LDS ------------------------------------------
        {
            float pre = 0.f, total = 0.f;
#pragma unroll
            for (int u = 0; u < Cfg::kTG; ++u) {
                const float v = tot[u * DK + gc];
                if (u < tg) pre += v;
                total += v;
            }
            const float mid = 0.5f * total;
#pragma unroll
            for (int u = 0; u < Cfg::kTPT; ++u) {
                const int t = tg * Cfg::kTPT + u;
                const float cc = pre + cs[u] - mid;
                const float zv = t < rows ? z[(tc + t) * p.st + gc] : 0.f;
                Zs[row_of(t) * Cfg::kZS + gc] = zv * fast_exp(SZ * cc) * p.zscale;
                Fs[row_of(t) * Cfg::kFS + gc] = fast_exp(-SZ * cc) * p.oscale;
            }
            if (tg == 0) gam[gc] = fast_exp(mid);
        }
        __syncthreads();

        // ---- W <- sqrt(gamma) .* W (columns); scores; X W ----------------------------------------------
        const float gcol = gam[w * 16 + l16];
#pragma unroll
        for (int it = 0; it < Cfg::kNIT; ++it)
#pragma unroll
            for (int r = 0; r < 4; ++r) Wacc[it][r] *= gcol;
        for (int idx = w; idx < Cfg::kTiles; idx += Cfg::kWaves) {
            int tt = 0, rem = idx;
            while (rem > tt) { rem -= tt + 1; ++tt; }
            const int ts = rem;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            const float *xa = Xs + (16 * tt + l16) * Cfg::kXS + kg;
            const float *yb = Ys + (16 * ts + l16) * Cfg::kXS + kg;
#pragma unroll 8
            for (int ks = 0; ks < DV / 4; ++ks) acc = mma_f32(xa[4 * ks], yb[4 * ks], acc);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int rr = 16 * tt + 4 * kg + r, rc = 16 * ts + l16;
                Ps[rr * Cfg::kPS + rc] = (rc <= rr) ? acc[r] : 0.f;
            }
        }
        f32x4 Oacc[Cfg::kNT];
#pragma unroll
        for (int mt = 0; mt < Cfg::kNT; ++mt) Oacc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int it = 0; it < Cfg::kNIT; ++it) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float bval = Wacc[it][r];
#pragma unroll
                for (int mt = 0; mt < Cfg::kNT; ++mt) {
                    const float a = Xs[(16 * mt + l16) * Cfg::kXS + 16 * it + 4 * kg + r];
                    Oacc[mt] = mma_f32(a, bval, Oacc[mt]);
                }
            }
        }
        __syncthreads();

        // ---- + (masked scores) Z~, times F: the finished tile replaces F ---------------------------------
#pragma unroll
        for (int mt = 0; mt < Cfg::kNT; ++mt) {
            for (int ks = 0; ks < 4 * (mt + 1); ++ks) {
                const float a = Ps[(16 * mt + l16) * Cfg::kPS + 4 * ks + kg];
                const float bv = Zs[(4 * ks + kg) * Cfg::kZS + 16 * w + l16];
                Oacc[mt] = mma_f32(a, bv, Oacc[mt]);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) Fs[(16 * mt + 4 * kg + r) * Cfg::kFS + 16 * w + l16] *= Oacc[mt][r];
        }

        // ---- W <- sqrt(gamma) .* (W + Y^T Z~) ------------------------------------------------------------
#pragma unroll
        for (int it = 0; it < Cfg::kNIT; ++it) {
            f32x4 acc = Wacc[it];
#pragma unroll 4
            for (int ks = 0; ks < C / 4; ++ks) {
                const float a = Ys[(4 * ks + kg) * Cfg::kXS + 16 * it + l16];
                const float bv = Zs[(4 * ks + kg) * Cfg::kZS + 16 * w + l16];
                acc = mma_f32(a, bv, acc);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r] *= gcol;
            Wacc[it] = acc;
        }
        bool at_anchor = false;
        if constexpr (REV) {
            // the pass has arrived at a checkpoint: what the tokens from here on contribute to dG is exactly
            // row_sum(dS .* S) of the state at this boundary and its gradient
            at_anchor = p.S_ck && c > 0 && c % Cfg::kAnchor == 0;
            if (at_anchor) {
                const float *ck = p.S_ck + (sbh * p.n_ck + (c / Cfg::kAnchor - 1)) * DK * DV + (size_t)tid * (Cfg::kNIT * 4);
                float part = 0.f;
#pragma unroll
                for (int it = 0; it < Cfg::kNIT; ++it) {
                    const f32x4 sv = *reinterpret_cast<const f32x4 *>(ck + it * 4);
                    part += Wacc[it][0] * sv[0] + Wacc[it][1] * sv[1] + Wacc[it][2] * sv[2] + Wacc[it][3] * sv[3];
                }
                part += __shfl_xor(part, 16, 64);
                part += __shfl_xor(part, 32, 64);
                if (kg == 0) anchor[w * 16 + l16] = part;
            }
        }
        __syncthreads();

        // ---- the gradient rows and the dG terms, in the gate pass's layout (coalesced rows) ---------------
        if constexpr (!REV) {
#pragma unroll
            for (int u = 0; u < Cfg::kTPT; ++u) {
                const int t = tg * Cfg::kTPT + u;
                if (t >= rows) continue;
                const float val = Fs[row_of(t) * Cfg::kFS + gc];
                out[(tc + t) * p.st + gc] = val;
                dg[(tc + t) * gcs + gc] = z2[(tc + t) * p.st + gc] * val;   // Q .* dQ, for the dK pass
            }
        } else {
            float dterm[Cfg::kTPT];
            float run = 0.f;
#pragma unroll
            for (int u = Cfg::kTPT - 1; u >= 0; --u) {   // sums over this thread's tokens >= u
                const int t = tg * Cfg::kTPT + u;
                if (t < rows) {
                    const float val = Fs[row_of(t) * Cfg::kFS + gc];
                    out[(tc + t) * p.st + gc] = val;
                    run += dg[(tc + t) * gcs + gc] - z2[(tc + t) * p.st + gc] * val;
                }
                dterm[u] = run;
            }
            tot2[tg * DK + gc] = run;
            __syncthreads();
            float later = carry, total = 0.f;
#pragma unroll
            for (int u = 0; u < Cfg::kTG; ++u) {
                const float v = tot2[u * DK + gc];
                if (u > tg) later += v;
                total += v;
            }
#pragma unroll
            for (int u = 0; u < Cfg::kTPT; ++u) {
                const int t = tg * Cfg::kTPT + u;
                if (t < rows) dg[(tc + t) * gcs + gc] = dterm[u] + later;
            }
            carry = at_anchor ? anchor[gc] : carry + total;
        }
        __syncthreads();
    }
}

template <int DK, int DV, int C, bool REV> static hipError_t launch_qk_f32(const BwdQKParams &p, hipStream_t s) {
    typedef QKF32Cfg<DK, DV, C> Cfg;
    auto kern = gla_bwd_qk_f32_kernel<DK, DV, C, REV>;
    static LdsLimit limit;   // one per instantiation
    hipError_t e = limit.raise((const void *)kern, (int)Cfg::kBytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(p.B * p.P * p.H), dim3(Cfg::kThreads), Cfg::kBytes, s, p);
    return hipGetLastError();
}

template <int DK, int DV> static hipError_t dispatch_qk_f32(const BwdQKParams &p, int C, bool reverse, hipStream_t s) {
    if (C == 16) return reverse ? launch_qk_f32<DK, DV, 16, true>(p, s) : launch_qk_f32<DK, DV, 16, false>(p, s);
    if (C == 32) return reverse ? launch_qk_f32<DK, DV, 32, true>(p, s) : launch_qk_f32<DK, DV, 32, false>(p, s);
    if (C == 64) return reverse ? launch_qk_f32<DK, DV, 64, true>(p, s) : launch_qk_f32<DK, DV, 64, false>(p, s);
    return hipErrorInvalidValue;
}

hipError_t launch_bwd_qk_f32(const BwdQKParams &p, int d_k, int d_v, int C, bool reverse, hipStream_t s) {
    if (d_k == 64 && d_v == 64) return dispatch_qk_f32<64, 64>(p, C, reverse, s);
    if (d_k == 64 && d_v == 128) return dispatch_qk_f32<64, 128>(p, C, reverse, s);
    if (d_k == 128 && d_v == 64) return dispatch_qk_f32<128, 64>(p, C, reverse, s);
    if (d_k == 128 && d_v == 128) return dispatch_qk_f32<128, 128>(p, C, reverse, s);
    return hipErrorInvalidValue;
}

}  // namespace zeco
