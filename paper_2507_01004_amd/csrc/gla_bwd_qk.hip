// Backward of the chunkwise GLA forward for the two gated operands (App. A.4): dQ and dK, and the
// gate gradient dG.  bf16 inputs and outputs, bf16 MFMA operands, fp32 accumulation and states.
//
// Both gradients have the shape of the forward output pass with the operands in other roles.  With
// Lambda the in-chunk cumulative decay, gamma the chunk decay, S the forward state entering a chunk,
// dS the state gradient entering it from the later chunks, dA = mask(dO V^T) (shared by both):
//   dQ_t = Lambda_t   .* [ dO_t S^T                    + sum_{s<=t} dA_ts (K_s / Lambda_s) ]      forward over chunks
//   dK_s = 1/Lambda_s .* [ V_s ((gamma^T 1) .* dS)^T   + sum_{t>=s} dA_ts (Q_t .* Lambda_t) ]    backward over chunks
// i.e.  out_r = F_r .* [ X_r W + sum_{r'<=r} (X_r . Y_r') Z~_r' ]  with
//   dQ: X = dO, Y = V, Z~ = K / Lambda, F = Lambda,     W = S^T,   W <- (W + Y^T Z~) .* gamma (columns)
//   dK: X = V, Y = dO, Z~ = Q .* Lambda, F = 1/Lambda,  W = dS^T,  W <- gamma .* W first, then W += Y^T Z~
// (as built, Lambda is counted from HALF the chunk's total log decay and gamma is applied as two factors
// sqrt(gamma), one before the chunk's products and one after its update: the same products with half the
// range of exponents)
// where for dK the chunks are visited last to first and token t of a chunk sits at tile row 63 - t,
// which turns "t >= s" into the causal mask of the forward pass.  W (d_v x d_k, the transposed state)
// stays in MFMA accumulators; wave w owns the 16 output channels [16w, 16w+16).  The gated dimension
// d_k is the OUTPUT dimension here, so the decay acts on the columns of W (one scalar per lane) and
// the factor F must be applied to the finished tile element by element: the gate pass leaves it in
// LDS in fp32.
//
// One workgroup of d_k/16 waves owns a (batch, segment, head) stream; all waves take part in the gate
// pass and in the matrix products of a chunk, one after the other, on single-buffered LDS tiles; the
// raw inputs of the next chunk are fetched into registers while the current one is processed.
//
// dG (last line of the backward listing of App. A.4): dG_t = sum over later tokens s >= t of
// (Q_s .* dQ_s - K_s .* dK_s).  Inside one segment this is a reverse cumulative sum; what the later
// segments contribute is the constant row_sum(dS_end .* S_end) of the segment's final state and its
// gradient, which follows from unrolling the recurrence of dS one step past the segment boundary.
// The two products nearly cancel term by term (the sum stays of the size of one term), so they are
// formed from the fp32 gradients before those are rounded to bf16: summing rounded terms over
// thousands of tokens is a random walk that reaches several percent of dG.  The dQ pass leaves
// Q .* dQ (fp32) in the dG array; the dK pass, which walks the tokens from the last to the first
// anyway, subtracts K .* dK, accumulates and overwrites the array with dG.  Both do this one chunk
// late, from the fp32 result tile left in LDS, in the gate pass's thread layout (coalesced rows).
//
// Re-anchoring.  What is left in that running sum is the rounding noise of the bf16 MFMA operands, a random
// walk that grows with the square root of the tokens summed (about 1 % of max|dG| after 512 tokens, 4 % after
// 8192).  At every chunk boundary the exact value of the sum is known: the contribution of all later tokens
// to dG is row_sum(dS .* S) of the forward state at the boundary and its gradient.  The dQ pass holds that
// state in its accumulators and the dK pass holds the gradient, so with a checkpoint array (S_ck) the dQ
// pass stores the state entering every kAnchor-th chunk and the dK pass, when it arrives at the same
// boundary from the other side, replaces its running value by the exact one.  For that the two passes
// must cut a segment at the same tokens: with S_ck the dQ pass puts the short chunk of a length that is no
// multiple of 64 at the segment's END (short_last), where the dK pass has it.
//
// State gradient of a segment as a by-product of the dQ pass (EMIT).  What a segment sends back to the
// state entering it is  dS_loc = scale * sum_t (Q_t .* exp(G_t))^T dO_t  with G_t the log decay from
// the segment's first token through t: the first loop of the backward listing run from dS = 0.  The
// listing walks the chunks backwards; the sum itself has no order, so the dQ pass, which reads q, g
// and dO anyway, accumulates it in a second set of accumulators (transposed like W) from two more
// tiles, dO^T and (Q .* exp(G))^T, and the separate pass over q, g, dO is not needed.
#include "zeco_device.h"
#include "zeco_internal.h"

namespace zeco {

template <int DK, int DV, bool EMIT = false> struct QKCfg {
    static constexpr int NW = DK / 16;             // waves, 16 output channels each
    static constexpr int NT = 64 * NW;
    static constexpr int NIT = DV / 16;            // row tiles of W per wave
    // gate pass over the gated operand: 4 channels x TPT consecutive tokens per thread
    static constexpr int CQ = DK / 4;
    static constexpr int GW = 64 / CQ;             // token groups inside one wave
    static constexpr int TG = NT / CQ;             // token groups
    static constexpr int TPT = 64 / TG;
    // copy pass over X and Y: 4 channels x TPTV consecutive tokens per thread
    static constexpr int VQ = DV / 4;
    static constexpr int TPTV = 64 / (NT / VQ);
    // LDS (bytes)
    static constexpr int XS = DV * 2 + 16;         // row stride of Xs, Ys (token-major)
    static constexpr int TS = 64 * 2 + 16;         // row stride of Yt, Zt, Ps (64 tokens per row)
    static constexpr int FS = DK * 4 + 16;         // row stride of Fs (fp32)
    static constexpr int kOffX = 0;
    static constexpr int kOffY = kOffX + 64 * XS;
    static constexpr int kOffYT = kOffY + 64 * XS;
    static constexpr int kOffZT = kOffYT + DV * TS;
    static constexpr int kOffP = kOffZT + DK * TS;
    static constexpr int kOffF = kOffP + 64 * TS;
    static constexpr int kOffTot = kOffF + 64 * FS;
    static constexpr int kOffGam = kOffTot + NW * DK * 4;
    static constexpr int kOffTot2 = kOffGam + DK * 4;        // [wave][channel] sums of the dG terms
    static constexpr int kOffCarry = kOffTot2 + NW * DK * 4; // [channel] dG contribution of later segments
    static constexpr int kOffAnchor = kOffCarry + DK * 4;    // [channel] exact dG contribution at the last checkpoint passed
    static constexpr int kOffXT = kOffAnchor + DK * 4;       // EMIT: X^T (channel-major) and (Q .* exp(G))^T
    static constexpr int kOffQT = kOffXT + (EMIT ? DV * TS : 0);
    static constexpr int kBytes = kOffQT + (EMIT ? DK * TS : 0);

    // LDS position of contraction channel j inside an Xs / Ys row.  A lane of a 16x16 accumulator
    // tile owns rows 4 kg .. 4 kg + 3; the rows it owns in two adjacent tiles of W serve as its eight
    // k-slots of the 16x16x32 MFMA, so channel 16 q + 4 kg + m of a block of 32 sits at 8 kg + 4 q + m.
    __device__ static __forceinline__ constexpr int pos_of_channel(int j) {
        const int jl = j % 32;
        return (j - jl) + 8 * ((jl / 4) % 4) + 4 * (jl / 16) + (jl % 4);
    }
};

constexpr int kAnchor = 8;   // chunks between two checkpoints of the forward state (512 tokens)

__device__ __forceinline__ bf16x8 pack2x4(f32x4 a, f32x4 b) {
    u32x4 w = {pack_bf16(a[0], a[1]), pack_bf16(a[2], a[3]), pack_bf16(b[0], b[1]),
               pack_bf16(b[2], b[3])};
    return __builtin_bit_cast(bf16x8, w);
}

// REV = false: dQ (x = dO, y = v, z = k, W_init = forward states; the query scale multiplies the
// output).  REV = true: dK (x = v, y = dO, z = q, W_init = state gradients entering each segment's
// final state; the query scale rides on Q .* Lambda, so that the running dS is the true gradient).
// EMIT (dQ pass only): also accumulate the segment's state gradient dS_loc and emit it (and, when asked,
// the segment's total log decay).
template <int DK, int DV, bool REV, int GM, bool EMIT>
__global__ __launch_bounds__(DK * 4) void gla_bwd_qk_kernel(BwdQKParams p) {
    static_assert(!(REV && EMIT), "the state gradient is a by-product of the forward-direction pass");
    typedef QKCfg<DK, DV, EMIT> Cfg;
    typedef Mma<16> M;
    typedef GateVal<GM> GV;
    constexpr int XS = Cfg::XS, TS = Cfg::TS, FS = Cfg::FS, NW = Cfg::NW, NT = Cfg::NT;
    constexpr int TPT = Cfg::TPT, TPTV = Cfg::TPTV, CQ = Cfg::CQ, GW = Cfg::GW;
    constexpr int GB = GM == kGateBF16 ? 2 : 4;
    constexpr bool GH = GM == kGateHead;
    constexpr float kLog2e = 1.4426950408889634f;
    constexpr float SZ = REV ? 1.f : -1.f;   // exponent sign of the operand Z~; the factor F takes the other
    extern __shared__ __align__(16) unsigned char lds[];
    unsigned char *Xs = lds + Cfg::kOffX, *Ys = lds + Cfg::kOffY, *Yt = lds + Cfg::kOffYT;
    unsigned char *Zt = lds + Cfg::kOffZT, *Ps = lds + Cfg::kOffP, *Fs = lds + Cfg::kOffF;
    float *wtot = reinterpret_cast<float *>(lds + Cfg::kOffTot);   // [wave][channel] gate sums
    float *gam = reinterpret_cast<float *>(lds + Cfg::kOffGam);    // e^(total / 2) of the chunk [channel]
    float *wtot2 = reinterpret_cast<float *>(lds + Cfg::kOffTot2);
    float *carry0 = reinterpret_cast<float *>(lds + Cfg::kOffCarry);
    float *anchor = reinterpret_cast<float *>(lds + Cfg::kOffAnchor);
    unsigned char *Xt = lds + Cfg::kOffXT, *Qt = lds + Cfg::kOffQT;

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, kg = lane >> 4;
    int N = p.n_chunks, pad = p.pad;   // (per segment when the segments differ in length, see below)
    auto chunk_of = [&](int m) { return REV ? N - 1 - m : m; };
    auto pos_of = [](int t) { return REV ? 63 - t : t; };
    // When L is no multiple of 64 the chunk processed FIRST is the short one, 64 - pad tokens: the segment's
    // first tokens in the dQ pass, its last ones in the dK pass.  It is loaded as a full window inside the
    // segment, [0, 64) or [L - 64, L); the gated operand, the log decays and the dG terms of the window's
    // surplus rows are taken as zero - they then touch no state, no decay and no other row - and their
    // gradient rows are not stored.
    // (With checkpoints the dQ pass cuts like the dK pass: the short chunk is the segment's last one.)
    const bool short_last = REV || p.short_last;
    auto cstart = [&](int c) {
        return short_last ? (long long)c * 64 - (c == N - 1 ? pad : 0) : (c ? (long long)c * 64 - pad : 0ll);
    };
    auto dead = [&](int t) { return short_last ? t < pad : t >= 64 - pad; };
    auto is_short = [&](int c) { return c == (short_last ? N - 1 : 0); };   // chunk c is the short one (if any is)

    // workgroup -> stream, dealt so that consecutive streams land on different XCDs
    const size_t sbh = blockIdx.x;                  // (seg * B + b) * H + h
    int sidx = blockIdx.x;
    const int h = sidx % p.H;
    sidx /= p.H;
    const int b = sidx % p.B, seg = sidx / p.B;
    long long tok0 = (long long)seg * p.L, T = (long long)p.P * p.L;   // first token; tokens per batch entry
    if (p.seg_start) {
        // segments of unequal length: this one's bounds from the table; a segment that cannot be taken (under
        // 64 tokens, over the bound L, outside the tensor) is left alone: the whole workgroup leaves
        tok0 = p.seg_start[seg];
        T = p.T;
        const long long len = p.seg_start[seg + 1] - tok0;
        if (tok0 < 0 || len < 64 || len > p.L || tok0 > T - len) return;   // (in this order: no sum can overflow)
        N = (int)((len + 63) >> 6);
        pad = 64 * N - (int)len;
    }
    const long long kbase = b * p.sb + tok0 * p.st + h * p.sh;
    const long long vbase = b * p.vb + tok0 * p.vt + h * p.vh;
    const unsigned char *xb = (const unsigned char *)p.x + vbase * 2;
    const unsigned char *yb = (const unsigned char *)p.y + vbase * 2;
    const unsigned char *zb = (const unsigned char *)p.z + kbase * 2;
    const long long hbase = ((long long)b * T + tok0) * p.H + h;   // per-head arrays [B,T,H]
    const unsigned char *gb = (const unsigned char *)p.g + (GH ? hbase : kbase) * GB;
    const long long gst = GH ? (long long)p.H : p.st;                       // gate elements between tokens
    const unsigned char *z2b = (const unsigned char *)p.z2 + kbase * 2;
    unsigned char *ob = (unsigned char *)p.out + kbase * 2;
    const long long st = p.st, vt = p.vt;
    float *dgb = p.dg + hbase * (GH ? 1 : DK);   // [B,T,H,d_k] contiguous ([B,T,H] with per-head gates)
    const long long gcs = (long long)p.H * (GH ? 1 : DK);

    // gate-pass coordinates (z, g) and copy-pass coordinates (x, y)
    const int cq = lane % CQ, gl = lane / CQ, tq = w * GW + gl;
    const int vq = tid % Cfg::VQ, tv = tid / Cfg::VQ;
    const int xpos = Cfg::pos_of_channel(4 * vq);

    // W^T tile init: Sacc[it][rr] = W[row 16 it + 4 kg + rr][col 16 w + l16] = W_init[col][row]
    f32x4 Sacc[Cfg::NIT];
    {
        const float *Wi = p.W_init + sbh * DK * DV + (size_t)(w * 16 + l16) * DV + 4 * kg;
#pragma unroll
        for (int it = 0; it < Cfg::NIT; ++it) Sacc[it] = *reinterpret_cast<const f32x4 *>(Wi + it * 16);
    }

    // EMIT: dS_loc^T in the layout of W, and the log decay of the chunks done so far (this thread's channels)
    f32x4 Dacc[EMIT ? Cfg::NIT : 1];
    f32x4 gpre = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int it = 0; it < (EMIT ? Cfg::NIT : 1); ++it) Dacc[it] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Score tiles above the diagonal are never computed: zero them once.
    for (int e = tid; e < 64 * TS / 16; e += NT)
        *reinterpret_cast<u32x4 *>(Ps + e * 16) = u32x4{0u, 0u, 0u, 0u};

    // dG carried in from the later segments: c[i] = sum_j dS_end[i][j] S_end[i][j]  (4 threads per row)
    f32x4 carry = {0.f, 0.f, 0.f, 0.f};
    if constexpr (REV) {
        const float *A = p.W_init + sbh * DK * DV;
        const float *Bm = (seg + 1 < p.P) ? p.S_init + (sbh + (size_t)p.B * p.H) * DK * DV
                                          : p.S_last + ((size_t)b * p.H + h) * DK * DV;
        const int i = tid >> 2, part = tid & 3;
        float acc = 0.f;
        for (int j = part * 4; j < DV; j += 16) {
            const f32x4 x = *reinterpret_cast<const f32x4 *>(A + (size_t)i * DV + j);
            const f32x4 y = *reinterpret_cast<const f32x4 *>(Bm + (size_t)i * DV + j);
            acc += x[0] * y[0] + x[1] * y[1] + x[2] * y[2] + x[3] * y[3];
        }
        acc += __shfl_xor(acc, 1, 64);
        acc += __shfl_xor(acc, 2, 64);
        if (part == 0) carry0[i] = acc;
        __syncthreads();
        carry = *reinterpret_cast<const f32x4 *>(carry0 + 4 * (lane % CQ));
    }

    // raw inputs of the chunk worked on next
    u32x2 rx[TPTV], ry[TPTV], rz[TPT];
    u32x2 rq[EMIT ? TPT : 1];   // EMIT: q of the chunk worked on next (otherwise q is fetched late, for dG only)
    typename GV::raw_t rg[TPT];
    {
        const long long c0 = cstart(chunk_of(0));
#pragma unroll
        for (int u = 0; u < TPT; ++u) {
            if constexpr (EMIT) rq[u] = *reinterpret_cast<const u32x2 *>(z2b + ((c0 + tq * TPT + u) * st + 4 * cq) * 2);
            rz[u] = *reinterpret_cast<const u32x2 *>(zb + ((c0 + tq * TPT + u) * st + 4 * cq) * 2);
            rg[u] = *reinterpret_cast<const typename GV::raw_t *>(gb + ((c0 + tq * TPT + u) * gst + (GH ? 0 : 4 * cq)) * GB);
        }
#pragma unroll
        for (int u = 0; u < TPTV; ++u) {
            rx[u] = *reinterpret_cast<const u32x2 *>(xb + ((c0 + tv * TPTV + u) * vt + 4 * vq) * 2);
            ry[u] = *reinterpret_cast<const u32x2 *>(yb + ((c0 + tv * TPTV + u) * vt + 4 * vq) * 2);
        }
    }

    // sum over the d_k channels of a token: the 4 of this thread, then the CQ lanes that share the token
    auto channel_sum = [&](f32x4 x) __attribute__((always_inline)) {
        float tot = (x[0] + x[1]) + (x[2] + x[3]);
#pragma unroll
        for (int d = 1; d < CQ; d <<= 1) tot += __shfl_xor(tot, d, 64);
        return tot;
    };
    // dG bookkeeping of the chunk finished last: raw z2 (q for dQ, k for dK) and, for dK, the Q .* dQ terms
    u32x2 rz2[TPT];
    f32x4 rqd[TPT], dterm[TPT];
    f32x4 later_in_wave = {0.f, 0.f, 0.f, 0.f};

    // first half: the finished chunk's gradient rows go to HBM, and the dG terms are formed from the fp32
    // result tile in Fs; dQ stores them, dK starts the reverse sums
    auto dg_first = [&](long long tc, bool first) __attribute__((always_inline)) {
        float *row = dgb + (tc + tq * TPT) * gcs + (GH ? 0 : 4 * cq);
        f32x4 run = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = TPT - 1; u >= 0; --u) {
            if (first && dead(tq * TPT + u)) {   // surplus row: nothing stored, no dG term
                if constexpr (REV) dterm[u] = run;
                continue;
            }
            const f32x4 val = *reinterpret_cast<const f32x4 *>(Fs + pos_of(tq * TPT + u) * FS + 16 * cq);
            // the gradient itself: 32 lanes write one contiguous row (the accumulator layout of the
            // products would give 32-byte pieces)
            __builtin_nontemporal_store(u32x2{pack_bf16(val[0], val[1]), pack_bf16(val[2], val[3])},
                                        reinterpret_cast<u32x2 *>(ob + ((tc + tq * TPT + u) * st + 4 * cq) * 2));
            const u32x2 zw = rz2[u];
            const f32x4 pr = {bf16_lo(zw[0]) * val[0], bf16_hi(zw[0]) * val[1],
                              bf16_lo(zw[1]) * val[2], bf16_hi(zw[1]) * val[3]};
            if constexpr (!REV && GH) {
                const float tot = channel_sum(pr);
                if (cq == 0) row[u * gcs] = tot;
            } else if constexpr (!REV) {
                *reinterpret_cast<f32x4 *>(row + u * gcs) = pr;
            } else {
#pragma unroll
                for (int a = 0; a < 4; ++a) run[a] += rqd[u][a] - pr[a];
                dterm[u] = run;   // sum over this thread's tokens >= u
            }
        }
        if constexpr (REV) {
            f32x4 inc = run;   // inclusive suffix scan over the wave's token groups
#pragma unroll
            for (int s = 1; s < GW; s <<= 1) {
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const float dn = __shfl_down(inc[a], s * CQ, 64);
                    if (gl + s < GW) inc[a] += dn;
                }
            }
#pragma unroll
            for (int a = 0; a < 4; ++a) later_in_wave[a] = inc[a] - run[a];
            if (gl == 0) *reinterpret_cast<f32x4 *>(wtot2 + w * DK + 4 * cq) = inc;
        }
    };
    // second half (dK, after a barrier): add the later waves and the later chunks, store dG
    auto dg_second = [&](long long tc, bool first, int c) __attribute__((always_inline)) {
        float *row = dgb + (tc + tq * TPT) * gcs + (GH ? 0 : 4 * cq);
        // chunk c ends at a checkpoint: what the later tokens contribute is known exactly (left in `anchor`
        // when the pass crossed that boundary, two iterations ago)
        if (p.S_ck && (c + 1) % kAnchor == 0 && c + 1 < N) carry = *reinterpret_cast<const f32x4 *>(anchor + 4 * cq);
        f32x4 later = carry, total = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int a = 0; a < 4; ++a) later[a] += later_in_wave[a];
#pragma unroll
        for (int u = 0; u < NW; ++u) {
            const f32x4 x = *reinterpret_cast<const f32x4 *>(wtot2 + u * DK + 4 * cq);
            const float sel = (u > w) ? 1.f : 0.f;   // wave-uniform
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                later[a] = __builtin_fmaf(sel, x[a], later[a]);
                total[a] += x[a];
            }
        }
#pragma unroll
        for (int u = 0; u < TPT; ++u) {
            if (first && dead(tq * TPT + u)) continue;
            f32x4 o;
#pragma unroll
            for (int a = 0; a < 4; ++a) o[a] = dterm[u][a] + later[a];
            if constexpr (GH) {
                const float tot = channel_sum(o);
                if (cq == 0) row[u * gcs] = tot;
            } else {
                __builtin_nontemporal_store(o, reinterpret_cast<f32x4 *>(row + u * gcs));
            }
        }
#pragma unroll
        for (int a = 0; a < 4; ++a) carry[a] += total[a];
    };

    for (int n = 0; n < N; ++n) {
        const long long t0 = cstart(chunk_of(n));                          // this chunk
        const long long t1 = cstart(chunk_of((n + 1 < N) ? n + 1 : n));    // chunk fetched meanwhile
        const long long tp = cstart(chunk_of((n > 0) ? n - 1 : 0));        // chunk finished last
        const bool first = is_short(chunk_of(n));                          // the short chunk, if there is one
        if (n > 0) dg_first(tp, is_short(chunk_of(n - 1)));
        if constexpr (!REV) {
            // checkpoint: the forward state entering this chunk, for the dK pass to re-anchor dG with
            if (p.S_ck && n > 0 && n % kAnchor == 0) {
                float *ck = p.S_ck + (sbh * p.n_ck + (n / kAnchor - 1)) * DK * DV + (size_t)(w * 16 + l16) * DV + 4 * kg;
#pragma unroll
                for (int it = 0; it < Cfg::NIT; ++it) *reinterpret_cast<f32x4 *>(ck + it * 16) = Sacc[it];
            }
        }

        // ---- gate pass, part 1: per-thread cumulative sums of g; X, Y, Y^T -> LDS -----------------
        f32x4 cs[TPT];
        f32x4 excl = {0.f, 0.f, 0.f, 0.f};
        {
            f32x4 run = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < TPT; ++u) {
                f32x4 gv = GV::get(rg[u]);
                if (first && dead(tq * TPT + u)) gv = f32x4{0.f, 0.f, 0.f, 0.f};
                rg[u] = *reinterpret_cast<const typename GV::raw_t *>(gb + ((t1 + tq * TPT + u) * gst + (GH ? 0 : 4 * cq)) * GB);
#pragma unroll
                for (int a = 0; a < 4; ++a) run[a] += gv[a];
                cs[u] = run;
            }
            f32x4 inc = run;   // inclusive scan of the group sums over the wave's GW token groups
#pragma unroll
            for (int d = 1; d < GW; d <<= 1) {
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const float up = __shfl_up(inc[a], d * CQ, 64);
                    if (gl >= d) inc[a] += up;
                }
            }
#pragma unroll
            for (int a = 0; a < 4; ++a) excl[a] = inc[a] - run[a];
            if (gl == GW - 1) *reinterpret_cast<f32x4 *>(wtot + w * DK + 4 * cq) = inc;
        }
        {
            TokenRun<TPTV> ch[4];
#pragma unroll
            for (int u = 0; u < TPTV; ++u) {
                const int r = pos_of(tv * TPTV + u);
                *reinterpret_cast<u32x2 *>(Xs + r * XS + xpos * 2) = rx[u];
                *reinterpret_cast<u32x2 *>(Ys + r * XS + xpos * 2) = ry[u];
            }
            if constexpr (EMIT) {   // X^T, channel-major (forward direction: tokens in order)
                TokenRun<TPTV> cx[4];
#pragma unroll
                for (int m = 0; m < TPTV / 2; ++m) {
                    cx[0].w[m] = pair_lo(rx[2 * m][0], rx[2 * m + 1][0]);
                    cx[1].w[m] = pair_hi(rx[2 * m][0], rx[2 * m + 1][0]);
                    cx[2].w[m] = pair_lo(rx[2 * m][1], rx[2 * m + 1][1]);
                    cx[3].w[m] = pair_hi(rx[2 * m][1], rx[2 * m + 1][1]);
                }
#pragma unroll
                for (int a = 0; a < 4; ++a) cx[a].store(Xt + (4 * vq + a) * TS + tv * TPTV * 2);
            }
#pragma unroll
            for (int m = 0; m < TPTV / 2; ++m) {
                // tokens (2m, 2m+1) of the run share a word; reversed, the run is written back to front
                const u32x2 a0 = REV ? ry[2 * m + 1] : ry[2 * m], a1 = REV ? ry[2 * m] : ry[2 * m + 1];
                const int wd = REV ? TPTV / 2 - 1 - m : m;
                ch[0].w[wd] = pair_lo(a0[0], a1[0]);
                ch[1].w[wd] = pair_hi(a0[0], a1[0]);
                ch[2].w[wd] = pair_lo(a0[1], a1[1]);
                ch[3].w[wd] = pair_hi(a0[1], a1[1]);
            }
#pragma unroll
            for (int u = 0; u < TPTV; ++u) {
                rx[u] = *reinterpret_cast<const u32x2 *>(xb + ((t1 + tv * TPTV + u) * vt + 4 * vq) * 2);
                ry[u] = *reinterpret_cast<const u32x2 *>(yb + ((t1 + tv * TPTV + u) * vt + 4 * vq) * 2);
            }
            const int c0 = REV ? 64 - (tv + 1) * TPTV : tv * TPTV;
#pragma unroll
            for (int a = 0; a < 4; ++a) ch[a].store(Yt + (4 * vq + a) * TS + c0 * 2);
        }
        __syncthreads();
        if constexpr (REV) {
            if (n > 0) dg_second(tp, is_short(chunk_of(n - 1)), chunk_of(n - 1));
        }

        // ---- gate pass, part 2: stitch waves; Z~^T and the factor tile -> LDS ----------------------
        {
            // The decay factors of Z~ and F are taken relative to half the chunk's total log decay, as in the forward
            // kernel: no exponent then exceeds |total| / 2.  W is decayed in two equal steps to match: by e^(total/2)
            // before the chunk's products and again after its update.
            f32x4 pre = excl, total = {0.f, 0.f, 0.f, 0.f}, mid;
#pragma unroll
            for (int u = 0; u < NW; ++u) {
                const f32x4 x = *reinterpret_cast<const f32x4 *>(wtot + u * DK + 4 * cq);
                const float sel = (u < w) ? 1.f : 0.f;   // wave-uniform
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    pre[a] = __builtin_fmaf(sel, x[a], pre[a]);
                    total[a] += x[a];
                }
            }
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                mid[a] = 0.5f * total[a];
                pre[a] -= mid[a];
            }
            TokenRun<TPT> zt[4];
            u32x2 zprev = {0u, 0u};
            TokenRun<TPT> qt[EMIT ? 4 : 1];
            u32x2 qprev = {0u, 0u};
            f32x4 epre = {0.f, 0.f, 0.f, 0.f};   // EMIT: scale * decay of the earlier chunks of the segment
            if constexpr (EMIT) {
#pragma unroll
                for (int a = 0; a < 4; ++a) epre[a] = __builtin_amdgcn_exp2f((gpre[GH ? 0 : a] + mid[GH ? 0 : a]) * kLog2e) * p.qscale;
            }
#pragma unroll
            for (int u = 0; u < TPT; ++u) {
                const int t = tq * TPT + u;
                f32x4 ez, ef;
                if constexpr (GH) {   // one decay per token: one pair of exponentials for the four channels
                    const float y = (cs[u][0] + pre[0]) * kLog2e;
                    const float z = __builtin_amdgcn_exp2f(SZ * y) * p.zscale, f = __builtin_amdgcn_exp2f(-SZ * y);
                    ez = f32x4{z, z, z, z};
                    ef = f32x4{f, f, f, f};
                } else {
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        const float y = (cs[u][a] + pre[a]) * kLog2e;   // in-chunk cumulative log2 decay
                        ez[a] = __builtin_amdgcn_exp2f(SZ * y) * p.zscale;
                        ef[a] = __builtin_amdgcn_exp2f(-SZ * y);
                    }
                }
                u32x2 zw = rz[u];
                if (first && dead(t)) zw = u32x2{0u, 0u};
                rz[u] = *reinterpret_cast<const u32x2 *>(zb + ((t1 + t) * st + 4 * cq) * 2);
                const u32x2 zq = {pack_bf16(bf16_lo(zw[0]) * ez[0], bf16_hi(zw[0]) * ez[1]),
                                  pack_bf16(bf16_lo(zw[1]) * ez[2], bf16_hi(zw[1]) * ez[3])};
                *reinterpret_cast<f32x4 *>(Fs + pos_of(t) * FS + 16 * cq) = ef;
                if constexpr (EMIT) {   // (Q .* exp(G))^T: F = Lambda here, times the earlier chunks' decay
                    u32x2 qw = rq[u];
                    if (first && dead(t)) qw = u32x2{0u, 0u};
                    rq[u] = *reinterpret_cast<const u32x2 *>(z2b + ((t1 + t) * st + 4 * cq) * 2);
                    rz2[u] = qw;   // kept for this chunk's dG terms
                    const u32x2 qh = {pack_bf16(bf16_lo(qw[0]) * ef[0] * epre[0], bf16_hi(qw[0]) * ef[1] * epre[1]),
                                      pack_bf16(bf16_lo(qw[1]) * ef[2] * epre[2], bf16_hi(qw[1]) * ef[3] * epre[3])};
                    if (u % 2 == 1) {
                        qt[0].w[u / 2] = pair_lo(qprev[0], qh[0]);
                        qt[1].w[u / 2] = pair_hi(qprev[0], qh[0]);
                        qt[2].w[u / 2] = pair_lo(qprev[1], qh[1]);
                        qt[3].w[u / 2] = pair_hi(qprev[1], qh[1]);
                    }
                    qprev = qh;
                }
                if (u % 2 == 1) {
                    const u32x2 a0 = REV ? zq : zprev, a1 = REV ? zprev : zq;
                    const int wd = REV ? (TPT - 1 - u) / 2 : u / 2;
                    zt[0].w[wd] = pair_lo(a0[0], a1[0]);
                    zt[1].w[wd] = pair_hi(a0[0], a1[0]);
                    zt[2].w[wd] = pair_lo(a0[1], a1[1]);
                    zt[3].w[wd] = pair_hi(a0[1], a1[1]);
                }
                zprev = zq;
            }
            const int c0 = REV ? 64 - (tq + 1) * TPT : tq * TPT;
#pragma unroll
            for (int a = 0; a < 4; ++a) zt[a].store(Zt + (4 * cq + a) * TS + c0 * 2);
            if constexpr (EMIT) {
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    qt[a].store(Qt + (4 * cq + a) * TS + c0 * 2);
                    gpre[a] += total[a];
                }
            }
            if (tq == 0) {
                f32x4 gh;
#pragma unroll
                for (int a = 0; a < 4; ++a) gh[a] = __builtin_amdgcn_exp2f(mid[a] * kLog2e);
                *reinterpret_cast<f32x4 *>(gam + 4 * cq) = gh;
            }
        }
        __syncthreads();

        // operands of this chunk's dG terms, consumed one iteration later
#pragma unroll
        for (int u = 0; u < TPT; ++u) {
            if constexpr (!EMIT) rz2[u] = *reinterpret_cast<const u32x2 *>(z2b + ((t0 + tq * TPT + u) * st + 4 * cq) * 2);
            if constexpr (REV && GH) {   // the channel sum of q .* dq, booked on the first channel
                const float x = dgb[(t0 + tq * TPT + u) * gcs];
                rqd[u] = f32x4{cq == 0 ? x : 0.f, 0.f, 0.f, 0.f};
            } else if constexpr (REV) {
                rqd[u] = *reinterpret_cast<const f32x4 *>(dgb + (t0 + tq * TPT + u) * gcs + 4 * cq);
            }
        }

        // ---- scores: P^T tiles (r' <= r), 16x16x32 over the d_v channels -----------------------------
        // half the decay of this lane's column of W: once before the chunk's products, once after its update
        const float gcol = gam[w * 16 + l16];
#pragma unroll
        for (int it = 0; it < Cfg::NIT; ++it)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) Sacc[it][rr] *= gcol;
#pragma unroll
        for (int i = 0; i < (10 + NW - 1) / NW; ++i) {
            const int idx = w + NW * i;   // wave-uniform
            if (idx < 10) {
                const int tt = (idx >= 6) ? 3 : (idx >= 3) ? 2 : (idx >= 1) ? 1 : 0;
                const int ts = idx - tt * (tt + 1) / 2;
                const unsigned char *ya = Ys + (16 * ts + l16) * XS + 16 * kg;
                const unsigned char *xf = Xs + (16 * tt + l16) * XS + 16 * kg;
                bf16x8 fa[DV / 32], fb[DV / 32];
#pragma unroll
                for (int ks = 0; ks < DV / 32; ++ks) {
                    fa[ks] = lds_frag(ya, 64 * ks);
                    fb[ks] = lds_frag(xf, 64 * ks);
                }
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < DV / 32; ++ks) acc = M::run(fa[ks], fb[ks], acc);
                if (ts == tt) {
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr)
                        if (4 * kg + rr > l16) acc[rr] = 0.f;
                }
                *reinterpret_cast<u32x2 *>(Ps + (16 * tt + l16) * TS + (16 * ts + 4 * kg) * 2) =
                    u32x2{pack_bf16(acc[0], acc[1]), pack_bf16(acc[2], acc[3])};
            }
        }
        // ---- inter: O^T = W^T X^T with W fed from the accumulators -----------------------------------
        f32x4 Oacc[4];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) Oacc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < DV / 32; ++ks) {
            const bf16x8 sf = pack2x4(Sacc[2 * ks], Sacc[2 * ks + 1]);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
                Oacc[mt] = M::run(sf, lds_frag(Xs, (mt * 16 + l16) * XS + (ks * 32 + 8 * kg) * 2), Oacc[mt]);
        }
        __syncthreads();

        // ---- intra: O^T += Zt Ps^T over the causal range; factor, scale, store ------------------------
        bf16x8 zf[2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) zf[ks] = lds_frag(Zt, (w * 16 + l16) * TS + (ks * 32 + 8 * kg) * 2);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
            for (int ks = 0; ks <= mt / 2; ++ks)
                Oacc[mt] = M::run(zf[ks], lds_frag(Ps, (mt * 16 + l16) * TS + (ks * 32 + 8 * kg) * 2), Oacc[mt]);
            const int r = mt * 16 + l16;
            float *fr = reinterpret_cast<float *>(Fs + r * FS + (w * 16 + 4 * kg) * 4);
            const f32x4 f = *reinterpret_cast<const f32x4 *>(fr);
            const f32x4 val = {Oacc[mt][0] * f[0] * p.oscale, Oacc[mt][1] * f[1] * p.oscale,
                               Oacc[mt][2] * f[2] * p.oscale, Oacc[mt][3] * f[3] * p.oscale};
            *reinterpret_cast<f32x4 *>(fr) = val;   // fp32 gradient; stored and used for dG one chunk later
        }
        // ---- state: W += Yt Zt^T (then the column decay in the forward direction) ---------------------
#pragma unroll
        for (int it = 0; it < Cfg::NIT; ++it) {
            f32x4 acc = Sacc[it];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
                acc = M::run(lds_frag(Yt, (it * 16 + l16) * TS + (ks * 32 + 8 * kg) * 2), zf[ks], acc);
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) acc[rr] *= gcol;
            Sacc[it] = acc;
        }
        if constexpr (REV) {
            // W is now the gradient of the state entering this chunk.  At a checkpoint: the exact dG
            // contribution of this chunk and everything after it to the earlier tokens, row_sum(dS .* S)
            const int c = chunk_of(n);
            if (p.S_ck && c > 0 && c % kAnchor == 0) {
                const float *ck = p.S_ck + (sbh * p.n_ck + (c / kAnchor - 1)) * DK * DV + (size_t)(w * 16 + l16) * DV + 4 * kg;
                float acc = 0.f;
#pragma unroll
                for (int it = 0; it < Cfg::NIT; ++it) {
                    const f32x4 x = *reinterpret_cast<const f32x4 *>(ck + it * 16);
                    acc += (Sacc[it][0] * x[0] + Sacc[it][1] * x[1]) + (Sacc[it][2] * x[2] + Sacc[it][3] * x[3]);
                }
                acc += __shfl_xor(acc, 16, 64);
                acc += __shfl_xor(acc, 32, 64);
                if (kg == 0) anchor[w * 16 + l16] = acc;
            }
        }
        if constexpr (EMIT) {   // dS_loc^T += X^T (Q .* exp(G))
            bf16x8 qf[2];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) qf[ks] = lds_frag(Qt, (w * 16 + l16) * TS + (ks * 32 + 8 * kg) * 2);
#pragma unroll
            for (int it = 0; it < Cfg::NIT; ++it)
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
                    Dacc[it] = M::run(lds_frag(Xt, (it * 16 + l16) * TS + (ks * 32 + 8 * kg) * 2), qf[ks], Dacc[it]);
        }
        __syncthreads();
    }
    if constexpr (EMIT) {
        float *Dl = p.dS_loc + sbh * DK * DV + (size_t)(w * 16 + l16) * DV + 4 * kg;
#pragma unroll
        for (int it = 0; it < Cfg::NIT; ++it) *reinterpret_cast<f32x4 *>(Dl + it * 16) = Dacc[it];
        if (p.G_tot_out && tq == 0) {   // total log decay of the segment
            if constexpr (GH) {
                if (cq == 0) p.G_tot_out[sbh] = gpre[0];
            } else {
                *reinterpret_cast<f32x4 *>(p.G_tot_out + sbh * DK + 4 * cq) = gpre;
            }
        }
    }
    // dG terms of the last chunk processed
    const long long tl = cstart(chunk_of(N - 1));
    dg_first(tl, is_short(chunk_of(N - 1)));
    if constexpr (REV) {
        __syncthreads();
        dg_second(tl, is_short(chunk_of(N - 1)), chunk_of(N - 1));
    }
}

template <int DK, int DV, bool REV, int GM, bool EMIT>
static hipError_t launch_qk2(const BwdQKParams &p, hipStream_t s) {
    typedef QKCfg<DK, DV, EMIT> Cfg;
    auto kern = gla_bwd_qk_kernel<DK, DV, REV, GM, EMIT>;
    static LdsLimit limit;   // one per instantiation
    hipError_t e = limit.raise((const void *)kern, Cfg::kBytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(p.B * p.P * p.H), dim3(Cfg::NT), Cfg::kBytes, s, p);
    return hipGetLastError();
}
template <int DK, int DV, bool REV, int GM>
static hipError_t launch_qk(const BwdQKParams &p, hipStream_t s) {
    if constexpr (!REV) {
        if (p.dS_loc) return launch_qk2<DK, DV, false, GM, true>(p, s);
    }
    return launch_qk2<DK, DV, REV, GM, false>(p, s);
}

template <bool REV, int GM>
static hipError_t dispatch_qk(const BwdQKParams &p, int d_k, int d_v, hipStream_t s) {
    if (d_k == 64 && d_v == 64) return launch_qk<64, 64, REV, GM>(p, s);
    if (d_k == 128 && d_v == 64) return launch_qk<128, 64, REV, GM>(p, s);
    if (d_k == 64 && d_v == 128) return launch_qk<64, 128, REV, GM>(p, s);
    if (d_k == 128 && d_v == 128) return launch_qk<128, 128, REV, GM>(p, s);
    return hipErrorInvalidValue;
}

hipError_t launch_bwd_qk(const BwdQKParams &p, int d_k, int d_v, int gate_mode, bool reverse, hipStream_t s) {
    if (gate_mode == kGateBF16)
        return reverse ? dispatch_qk<true, kGateBF16>(p, d_k, d_v, s) : dispatch_qk<false, kGateBF16>(p, d_k, d_v, s);
    if (gate_mode == kGateHead)
        return reverse ? dispatch_qk<true, kGateHead>(p, d_k, d_v, s) : dispatch_qk<false, kGateHead>(p, d_k, d_v, s);
    return reverse ? dispatch_qk<true, kGateF32>(p, d_k, d_v, s) : dispatch_qk<false, kGateF32>(p, d_k, d_v, s);
}

}  // namespace zeco
