// Chunkwise GLA forward of a segment, fp32 inputs, fp32 MFMA (16x16x4), chunk length C = 16, 32 or 64.
//
// One workgroup per (batch, segment, head) walks the N = ceil(L/C) chunks in order (Sec. 3.1, local
// state recurrence) and, per chunk, evaluates the chunk equations of Sec. 2.1 with the intra-chunk
// scores of Alg. 1 (Q .* Lambda)(K / Lambda)^T under the causal mask (diagonal included):
//     O   = (Q .* Lambda) S  +  [scores .* M] V
//     S  <- (gamma^T 1) .* S + (K .* Gamma)^T V
// The d_k x d_v state lives in MFMA accumulators for the whole segment: wave w owns columns
// [16w, 16w+16) of S, and because an accumulator register of lane l holds S[16*it + 4*(l/16) + r]
// [l%16], that register IS the B operand of the 16x16x4 step whose four k-slots are the channels
// 16*it + 4*kg + r (kg = 0..3) - the inter-chunk product reads S without leaving the registers.
// This is the accuracy path (relative error <= 1e-4 against the fp64 oracle); the bf16 kernel is
// the throughput path.  The chunk length is a template parameter here (Sec. 2.1 leaves C free): a
// shorter chunk does less masked work per token and, since K / Lambda spans the decay of one chunk,
// takes proportionally stronger gates (the sum of |g| over a chunk must stay below 160: the factors
// are counted from half the chunk's total log decay).
//
// MODE (the phases of Alg. 1, as in the bf16 kernel): kF32Local the local pass from the zero state
// (o, S_loc, G_cum, G_tot); kF32States only the final state and total decay of each segment (S_loc,
// G_tot; q is not read); kF32Output the output pass from given initial states S_init (o only).
//
// Two more modes run the same equations over the REVERSED sequence for the backward pass (App. A.4):
//   kF32DState  dS <- (gamma^T 1) .* dS + (Q .* Lambda)^T dO from zero; S_loc receives the gradient the
//               segment sends to the state entering it (called with k := q, v := dO)
//   kF32DV      dV = (K / Lambda)((gamma^T 1) .* dS) + (intra-chunk scores)^T dO with dS started from
//               S_init, the gradient entering the segment's final state (called with q := k, k := q,
//               v := dO, o := dV)
// With rho = L - 1 - t both are the forward recurrence in rho, except that the decay between two tokens
// then covers the gate of the one in the key role and not of the one in the query role: the cumulative
// sum of g over a chunk is taken EXCLUSIVE of a token's own gate.  The query scale rides on the operand in
// the key role (p.kscale), so that the running dS is the true gradient.
//
// A segment length that is no multiple of C makes the FIRST chunk the short one: it covers the
// tokens [0, r), r = L - C (N - 1), is loaded as the window [0, C) (inside the segment, L >= C)
// with g, k, v of the rows >= r taken as zero - such rows leave the state, the decay and the other
// rows' outputs untouched - and stores only its first r rows; chunk n >= 1 starts at token r + C (n - 1).
#include "zeco_device.h"
#include "zeco_internal.h"

namespace zeco {

enum F32Mode { kF32Local = 0, kF32States = 1, kF32Output = 2, kF32DState = 3, kF32DV = 4 };

template <int DK, int DV, int C> struct F32Cfg {
    static constexpr int kWaves = DV / 16;
    static constexpr int kThreads = 64 * kWaves;
    static constexpr int kTG = kThreads / DK;       // token groups in the gate pass
    static constexpr int kTPT = C / kTG;            // tokens per thread in the gate pass
    static constexpr int kNT = C / 16;              // 16-token tiles per chunk
    static constexpr int kTiles = kNT * (kNT + 1) / 2;   // score tiles on and below the diagonal
    static constexpr int kQS = DK + 4;              // row strides (floats), chosen bank-conflict free
    static constexpr int kKT = DK + 16;
    static constexpr int kVS = DV + 16;
    static constexpr int kPS = C + 4;
    static constexpr int kOffQ = 0;
    static constexpr int kOffK = kOffQ + C * kQS;
    static constexpr int kOffKT = kOffK + C * kQS;
    static constexpr int kOffV = kOffKT + C * kKT;
    static constexpr int kOffP = kOffV + C * kVS;
    static constexpr int kOffTot = kOffP + C * kPS;
    static constexpr int kOffGam = kOffTot + kTG * DK;
    static constexpr int kOffMid = kOffGam + DK;
    static constexpr int kFloats = kOffMid + DK;
    static constexpr size_t kBytes = sizeof(float) * kFloats;
    static_assert(kTPT >= 1 && C % 16 == 0, "chunk length");
};

template <int DK, int DV, int C, int MODE>
__global__ __launch_bounds__(DV * 4) void gla_chunk_f32_kernel(ChunkParams p) {
    typedef F32Cfg<DK, DV, C> Cfg;
    constexpr bool REV = MODE == kF32DState || MODE == kF32DV;       // the sequence reversed
    constexpr bool NOQ = MODE == kF32States || MODE == kF32DState;   // only the state is computed
    constexpr bool FROM_INIT = MODE == kF32Output || MODE == kF32DV; // start from S_init, emit o only
    constexpr bool EMIT_G = MODE == kF32Local;
    extern __shared__ __align__(16) float lds[];
    float *Qs = lds + Cfg::kOffQ;    // Q .* Lambda * scale      [t][i]
    float *Ks = lds + Cfg::kOffK;    // K / Lambda               [s][i]
    float *Kt = lds + Cfg::kOffKT;   // K .* Gamma               [s][i]
    float *Vs = lds + Cfg::kOffV;    // V                        [s][j]
    float *Ps = lds + Cfg::kOffP;    // masked scores            [t][s]
    float *tot = lds + Cfg::kOffTot; // per token-group gate sums [tg][i]
    float *gam = lds + Cfg::kOffGam; // chunk decay gamma         [i]
    float *emid = lds + Cfg::kOffMid; // sqrt(gamma)               [i]

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int l16 = lane & 15, kg = lane >> 4;

    int sidx = blockIdx.x;                       // stream index = (b * P + p) * H + h
    const int h = sidx % p.H;
    sidx /= p.H;
    const int seg = sidx % p.P, b = sidx / p.P;
    long long tok0 = (long long)seg * p.L, T = (long long)p.P * p.L;   // first token; tokens per batch entry
    int n_chunks = p.n_chunks, pad = p.pad;
    long long len = p.L;
    if (p.seg_start) {
        // segments of unequal length: this one's bounds from the table; a segment that cannot be taken (under
        // 64 tokens, over the bound L, outside the tensor) is left alone
        tok0 = p.seg_start[seg];
        T = p.T;
        len = p.seg_start[seg + 1] - tok0;
        if (tok0 < 0 || len < 64 || len > p.L || tok0 > T - len) return;   // (in this order: no sum can overflow)
        n_chunks = (int)((len + C - 1) / C);
        pad = C * n_chunks - (int)len;
    }
    const float *q = (const float *)p.q + b * p.sb + tok0 * p.st + h * p.sh;
    const float *k = (const float *)p.k + b * p.sb + tok0 * p.st + h * p.sh;
    const float *g = (const float *)p.g + b * p.sb + tok0 * p.st + h * p.sh;
    const float *v = (const float *)p.v + b * p.vb + tok0 * p.vt + h * p.vh;
    float *o = (float *)p.o + b * p.vb + tok0 * p.vt + h * p.vh;
    float *Gc = p.G_cum + (((long long)b * T + tok0) * p.H + h) * DK;
    const long long gcs = (long long)p.H * DK;
    const size_t sbh = ((size_t)seg * p.B + b) * p.H + h;

    f32x4 Sacc[DK / 16];
#pragma unroll
    for (int it = 0; it < DK / 16; ++it) {
        if constexpr (FROM_INIT) {
            const float *Si = p.S_init + sbh * DK * DV;
#pragma unroll
            for (int r = 0; r < 4; ++r) Sacc[it][r] = Si[(16 * it + 4 * kg + r) * DV + 16 * w + l16];
        } else {
            Sacc[it] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }

    const int gc = tid % DK, tg = tid / DK;      // gate pass: channel and token group
    // position in the segment of the token that sits at place x of the order the chunks are walked in
    auto at = [&](long long x) { return REV ? len - 1 - x : x; };
    double seg_prefix = 0.0;                     // log decay accumulated over previous chunks

    for (int n = 0; n < n_chunks; ++n) {
        const long long t0 = n ? (long long)n * C - pad : 0;
        const int rows = n ? C : C - pad;        // real tokens of this chunk
        // ---- gate pass: inclusive cumulative sum of g over the chunk, per channel -------------
        float cs[Cfg::kTPT];
        {
            float run = 0.f;
#pragma unroll
            for (int u = 0; u < Cfg::kTPT; ++u) {
                const int t = tg * Cfg::kTPT + u;
                if constexpr (REV) cs[u] = run;   // without the token's own gate
                run += t < rows ? g[at(t0 + t) * p.st + gc] : 0.f;
                if constexpr (!REV) cs[u] = run;
            }
            tot[tg * DK + gc] = run;
        }
        for (int e = tid; e < C * DV; e += Cfg::kThreads) {
            const int t = e / DV, j = e % DV;
            Vs[t * Cfg::kVS + j] = t < rows ? v[at(t0 + t) * p.vt + j] : 0.f;
        }
        __syncthreads();
        // The factors of Qs and Ks are taken relative to half the chunk's total log decay (mid = total / 2): the
        // same products e^(c_t - c_s) with no exponent beyond |total| / 2; the inter-chunk product makes up for it
        // with e^mid on the state's rows.
        float pre = 0.f, total = 0.f;
#pragma unroll
        for (int u = 0; u < Cfg::kTG; ++u) {
            const float x = tot[u * DK + gc];
            if (u < tg) pre += x;
            total += x;
        }
        const float mid = 0.5f * total;
#pragma unroll
        for (int u = 0; u < Cfg::kTPT; ++u) {
            const int t = tg * Cfg::kTPT + u;
            const float c = pre + cs[u];
            float kv = t < rows ? k[at(t0 + t) * p.st + gc] : 0.f;
            if constexpr (REV) kv *= p.kscale;
            if constexpr (!NOQ) {
                Qs[t * Cfg::kQS + gc] = q[at(t0 + t) * p.st + gc] * fast_exp(c - mid) * p.scale;
                Ks[t * Cfg::kQS + gc] = kv * fast_exp(mid - c);
            }
            Kt[t * Cfg::kKT + gc] = kv * fast_exp(total - c);
            if constexpr (EMIT_G) {
                if (t < rows) Gc[(t0 + t) * gcs + gc] = (float)(seg_prefix + (double)c);
            }
        }
        if (tg == 0) {
            gam[gc] = fast_exp(total);
            emid[gc] = fast_exp(mid);
        }
        seg_prefix += (double)total;
        __syncthreads();

        f32x4 Oacc[Cfg::kNT];
        if constexpr (!NOQ) {
            // ---- intra-chunk scores on the lower-triangular 16x16 tiles ------------------------------
            for (int idx = w; idx < Cfg::kTiles; idx += Cfg::kWaves) {
                int tt = 0, rem = idx;
                while (rem > tt) { rem -= tt + 1; ++tt; }
                const int ts = rem;
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                const float *qa = Qs + (16 * tt + l16) * Cfg::kQS + kg;
                const float *kb = Ks + (16 * ts + l16) * Cfg::kQS + kg;
#pragma unroll 8
                for (int ks = 0; ks < DK / 4; ++ks) acc = mma_f32(qa[4 * ks], kb[4 * ks], acc);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int t = 16 * tt + 4 * kg + r, s = 16 * ts + l16;
                    Ps[t * Cfg::kPS + s] = (s <= t) ? acc[r] : 0.f;
                }
            }

            // ---- inter-chunk product with the state held in the accumulators ------------------------
#pragma unroll
            for (int mt = 0; mt < Cfg::kNT; ++mt) Oacc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int it = 0; it < DK / 16; ++it) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float bval = Sacc[it][r] * emid[16 * it + 4 * kg + r];
#pragma unroll
                    for (int mt = 0; mt < Cfg::kNT; ++mt) {
                        const float a = Qs[(16 * mt + l16) * Cfg::kQS + 16 * it + 4 * kg + r];
                        Oacc[mt] = mma_f32(a, bval, Oacc[mt]);
                    }
                }
            }
            __syncthreads();

            // ---- intra-chunk output P V (causal: only s < 16 (mt + 1)) ------------------------------
#pragma unroll
            for (int mt = 0; mt < Cfg::kNT; ++mt) {
                for (int ks = 0; ks < 4 * (mt + 1); ++ks) {
                    const float a = Ps[(16 * mt + l16) * Cfg::kPS + 4 * ks + kg];
                    const float bv = Vs[(4 * ks + kg) * Cfg::kVS + 16 * w + l16];
                    Oacc[mt] = mma_f32(a, bv, Oacc[mt]);
                }
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (16 * mt + 4 * kg + r < rows) o[at(t0 + 16 * mt + 4 * kg + r) * p.vt + 16 * w + l16] = Oacc[mt][r];
            }
        }

        // ---- state update S <- gamma .* S + (K .* Gamma)^T V -------------------------------------
#pragma unroll
        for (int it = 0; it < DK / 16; ++it) {
            f32x4 acc = Sacc[it];
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r] *= gam[16 * it + 4 * kg + r];
#pragma unroll 4
            for (int ks = 0; ks < C / 4; ++ks) {
                const float a = Kt[(4 * ks + kg) * Cfg::kKT + 16 * it + l16];
                const float bv = Vs[(4 * ks + kg) * Cfg::kVS + 16 * w + l16];
                acc = mma_f32(a, bv, acc);
            }
            Sacc[it] = acc;
        }
        __syncthreads();
    }

    if constexpr (!FROM_INIT) {
        float *Sl = p.S_loc + sbh * DK * DV;
#pragma unroll
        for (int it = 0; it < DK / 16; ++it)
#pragma unroll
            for (int r = 0; r < 4; ++r) Sl[(16 * it + 4 * kg + r) * DV + 16 * w + l16] = Sacc[it][r];
        if (tg == 0 && (!REV || p.G_tot)) p.G_tot[sbh * DK + gc] = (float)seg_prefix;
    }
}

template <int DK, int DV, int C, int MODE> static hipError_t launch_f32(const ChunkParams &p, hipStream_t s) {
    typedef F32Cfg<DK, DV, C> Cfg;
    auto kern = gla_chunk_f32_kernel<DK, DV, C, MODE>;
    static LdsLimit limit;   // one per instantiation
    hipError_t e = limit.raise((const void *)kern, (int)Cfg::kBytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(p.B * p.P * p.H), dim3(Cfg::kThreads), Cfg::kBytes, s, p);
    return hipGetLastError();
}

template <int DK, int DV, int C> static hipError_t dispatch_f32_mode(const ChunkParams &p, int mode, hipStream_t s) {
    if (mode == kF32States) return launch_f32<DK, DV, C, kF32States>(p, s);
    if (mode == kF32Output) return launch_f32<DK, DV, C, kF32Output>(p, s);
    if (mode == kF32DState) return launch_f32<DK, DV, C, kF32DState>(p, s);
    if (mode == kF32DV) return launch_f32<DK, DV, C, kF32DV>(p, s);
    return launch_f32<DK, DV, C, kF32Local>(p, s);
}

template <int DK, int DV> static hipError_t dispatch_f32_chunk(const ChunkParams &p, int C, int mode, hipStream_t s) {
    if (C == 16) return dispatch_f32_mode<DK, DV, 16>(p, mode, s);
    if (C == 32) return dispatch_f32_mode<DK, DV, 32>(p, mode, s);
    if (C == 64) return dispatch_f32_mode<DK, DV, 64>(p, mode, s);
    return hipErrorInvalidValue;
}

// mode: 0 local pass, 1 states only, 2 output pass from S_init, 3 backward state pass, 4 dV pass (the same
// numbering as the bf16 kernel's);
// p.n_chunks and p.pad count chunks of C tokens
hipError_t launch_chunk_f32(const ChunkParams &p, int d_k, int d_v, int C, int mode, hipStream_t s) {
    if (d_k == 64 && d_v == 64) return dispatch_f32_chunk<64, 64>(p, C, mode, s);
    if (d_k == 64 && d_v == 128) return dispatch_f32_chunk<64, 128>(p, C, mode, s);
    if (d_k == 128 && d_v == 64) return dispatch_f32_chunk<128, 64>(p, C, mode, s);
    if (d_k == 128 && d_v == 128) return dispatch_f32_chunk<128, 128>(p, C, mode, s);
    return hipErrorInvalidValue;
}

}  // namespace zeco
