// Chunkwise GLA forward of a segment from the zero state: bf16 inputs, bf16 MFMA operands,
// fp32 accumulation, fp32 state.  The throughput path.
//
// Work decomposition.  A (batch, segment, head) stream is a serial recurrence over N = L/64
// chunks (Sec. 3.1).  One workgroup of NW = d_v/16 waves owns a stream; wave w owns columns
// [16w, 16w+16) of the d_k x d_v state, which stays in MFMA accumulators for the whole segment.
// With d_v = 128 that is 8 waves, two per SIMD, so that one wave's LDS / transcendental / memory
// latencies are covered by the other's issue slots.
//
// Per chunk (chunk equations of Sec. 2.1, scores as in Alg. 1):
//   gate pass   each thread owns 4 channels x TPT consecutive tokens: serial cumsum in registers,
//               token groups stitched by lane shuffles inside a wave and through LDS across waves:
//               cs = inclusive cumsum of g, Lambda = e^cs.
//               writes  Qs = Q .* Lambda, Ks = K / Lambda  (token-major, bf16)
//                       Kt = (K / Lambda)^T, Vt = V^T       (channel-major, bf16)
//   scores      P^T = Ks Qs^T on the 10 lower-triangular 16x16 tiles, causal select, -> Ps (bf16)
//   inter       O^T += S^T Qs^T   with S fed straight from the accumulators (see below)
//   intra       O^T += Vt Ps^T    (causal k-range); O * scale stored to HBM
//   state       S <- (gamma^T 1) .* (S + Kt Vt^T)
// The last line is Eq. (3) with K .* Gamma = (gamma^T 1)-scaled K / Lambda (Gamma = gamma / Lambda),
// so one scaled copy of K serves both the scores and the state update.
//
// Accumulator-as-operand.  Lane l of a 16x16 accumulator tile holds column l%16 and rows
// 4*(l/16) .. +3.  The MFMA operand layout wants, from the same lane, row (column) l%16 and eight
// k-slots.  Summation over k is order-free, so the eight state rows a lane owns in two adjacent
// tiles are used as its eight k-slots, and Qs is stored in LDS with its channels permuted to
// match (pos_of_channel); Ks uses the same permutation so the scores are unaffected.
//
// Memory pipeline.  One register set holds the raw q, k, g, v of the current chunk; each piece
// is reloaded with the next chunk's data right after its last use, so the global loads are spread
// over the gate pass and stay in flight for a whole iteration.
#include "zeco_device.h"
#include "zeco_internal.h"

namespace zeco {

#ifdef ZECO_PHASE_TIMING
// Development aid: cycle-counter stamps of workgroup 0, chunks 64..67, 12 points per chunk and wave.
unsigned long long *g_phase_dbg = nullptr;
#define ZPT(pt)                                                                                  \
    if (p.dbg && blockIdx.x == 0 && lane == 0 && n >= 64 && n < 68)                              \
    p.dbg[((w * 4 + (n - 64)) * 12) + (pt)] = __builtin_readcyclecounter()
#else
#define ZPT(pt)
#endif

template <int DK, int DV> struct B16Cfg {
    static constexpr int NW = DV / 16;             // waves per workgroup, 16 state columns each
    static constexpr int NT = 64 * NW;
    static constexpr int NIT = DK / 16;            // state row tiles per wave
    static constexpr int NKS_D = DK / 32;          // MFMA k-steps across channels
    // gate pass thread mapping: 4 channels x TPT tokens per thread
    static constexpr int CQ = DK / 4;              // channel quads
    static constexpr int GW = 64 / CQ;             // token groups inside one wave (2 or 4)
    static constexpr int TG = NT / CQ;             // token groups
    static constexpr int TPT = 64 / TG;            // consecutive tokens per thread (8, 4 or 2)
    static constexpr int VQ = DV / 4;
    static constexpr int TPTV = 64 / (NT / VQ);    // = 4
    // LDS (bytes)
    static constexpr int QS = DK * 2 + 16;         // row stride of Qs, Ks
    static constexpr int TS = 64 * 2 + 16;         // row stride of Kt, Vt, Ps
    static constexpr int kOffQ = 0;
    static constexpr int kOffK = kOffQ + 64 * QS;
    static constexpr int kOffKT = kOffK + 64 * QS;
    static constexpr int kOffVT = kOffKT + DK * TS;
    static constexpr int kOffP = kOffVT + DV * TS;
    static constexpr int kOffTot = kOffP + 64 * TS;
    static constexpr int kOffGam = kOffTot + NW * DK * 4;
    static constexpr int kBytes = kOffGam + DK * 4;

    // LDS position of channel i inside a Qs/Ks row (see "Accumulator-as-operand"): within each
    // block of 32 channels, channel 16 q + 4 kg + m sits at 8 kg + 4 q + m.
    __device__ static __forceinline__ constexpr int pos_of_channel(int i) {
        const int il = i % 32;
        return (i - il) + 8 * ((il / 4) % 4) + 4 * (il / 16) + (il % 4);
    }
};

__device__ __forceinline__ bf16x8 pack8(f32x4 a, f32x4 b) {
    u32x4 w = {pack_bf16(a[0], a[1]), pack_bf16(a[2], a[3]), pack_bf16(b[0], b[1]),
               pack_bf16(b[2], b[3])};
    return __builtin_bit_cast(bf16x8, w);
}

// Four consecutive gate values of one token, as loaded and as floats.
template <bool GBF16> struct GateVal;
template <> struct GateVal<false> {
    typedef f32x4 raw_t;
    __device__ static __forceinline__ raw_t load(const void *g, long long elem) {
        return *reinterpret_cast<const f32x4 *>((const float *)g + elem);
    }
    __device__ static __forceinline__ f32x4 get(raw_t r) { return r; }
};
template <> struct GateVal<true> {
    typedef u32x2 raw_t;
    __device__ static __forceinline__ raw_t load(const void *g, long long elem) {
        return *reinterpret_cast<const u32x2 *>((const uint16_t *)g + elem);
    }
    __device__ static __forceinline__ f32x4 get(raw_t r) {
        return f32x4{bf16_lo(r[0]), bf16_hi(r[0]), bf16_lo(r[1]), bf16_hi(r[1])};
    }
};

// N consecutive bf16 values (two per word) stored as one LDS write.
template <int N> struct TokenRun;
template <> struct TokenRun<8> {
    uint32_t w[4];
    __device__ __forceinline__ void store(unsigned char *dst) const {
        *reinterpret_cast<u32x4 *>(dst) = u32x4{w[0], w[1], w[2], w[3]};
    }
};
template <> struct TokenRun<4> {
    uint32_t w[2];
    __device__ __forceinline__ void store(unsigned char *dst) const {
        *reinterpret_cast<u32x2 *>(dst) = u32x2{w[0], w[1]};
    }
};
template <> struct TokenRun<2> {
    uint32_t w[1];
    __device__ __forceinline__ void store(unsigned char *dst) const {
        *reinterpret_cast<uint32_t *>(dst) = w[0];
    }
};

// Low halves / high halves of two packed bf16 pairs: (x.lo, y.lo) and (x.hi, y.hi).
__device__ __forceinline__ uint32_t pair_lo(uint32_t x, uint32_t y) {
    return __builtin_amdgcn_perm(y, x, 0x05040100u);
}
__device__ __forceinline__ uint32_t pair_hi(uint32_t x, uint32_t y) {
    return __builtin_amdgcn_perm(y, x, 0x07060302u);
}

template <int DK, int DV, bool GBF16>
__global__ __launch_bounds__(DV * 4) void gla_chunk_bf16_kernel(ChunkParams p) {
    typedef B16Cfg<DK, DV> Cfg;
    typedef Mma<16> M;
    typedef GateVal<GBF16> GV;
    constexpr int QS = Cfg::QS, TS = Cfg::TS, NW = Cfg::NW, NT = Cfg::NT;
    constexpr int TPT = Cfg::TPT, TPTV = Cfg::TPTV, CQ = Cfg::CQ, GW = Cfg::GW;
    constexpr float kLog2e = 1.4426950408889634f;
    extern __shared__ __align__(16) unsigned char lds[];
    unsigned char *Qs = lds + Cfg::kOffQ, *Ks = lds + Cfg::kOffK, *Kt = lds + Cfg::kOffKT;
    unsigned char *Vt = lds + Cfg::kOffVT, *Ps = lds + Cfg::kOffP;
    float *wtot = reinterpret_cast<float *>(lds + Cfg::kOffTot);   // [wave][channel] gate sums
    float *gam = reinterpret_cast<float *>(lds + Cfg::kOffGam);    // chunk decay gamma [channel]

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave index, known uniform
    const int l16 = lane & 15, kg = lane >> 4;                // MFMA lane coordinates

    const size_t sbh = blockIdx.x;                  // (seg * B + b) * H + h  (S_loc / G_tot order)
    int sidx = blockIdx.x;
    const int h = sidx % p.H;
    sidx /= p.H;
    const int b = sidx % p.B, seg = sidx / p.B;
    const long long tok0 = (long long)seg * p.L;
    const long long kbase = b * p.sb + tok0 * p.st + h * p.sh;
    const long long vbase = b * p.vb + tok0 * p.vt + h * p.vh;
    const uint16_t *qp = (const uint16_t *)p.q + kbase;
    const uint16_t *kp = (const uint16_t *)p.k + kbase;
    const uint16_t *vp = (const uint16_t *)p.v + vbase;
    uint16_t *op = (uint16_t *)p.o + vbase;
    const long long T = (long long)p.P * p.L;
    float *Gc = p.G_cum + (((long long)b * T + tok0) * p.H + h) * DK;
    const long long gcs = (long long)p.H * DK;

    // gate-pass coordinates: channel quad and token group (q, k, g), column quad and token group (v)
    const int cq = lane % CQ, gl = lane / CQ, tq = w * GW + gl;
    const int vq = tid % Cfg::VQ, tv = tid / Cfg::VQ;
    const int qpos = Cfg::pos_of_channel(4 * cq);

    f32x4 Sacc[Cfg::NIT];
#pragma unroll
    for (int it = 0; it < Cfg::NIT; ++it) Sacc[it] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Score tiles above the diagonal are never computed: zero them once.
    for (int e = tid; e < 64 * TS / 16; e += NT)
        *reinterpret_cast<u32x4 *>(Ps + e * 16) = u32x4{0u, 0u, 0u, 0u};

    struct Raw {
        u32x2 q[TPT], k[TPT];
        typename GV::raw_t g[TPT];
        u32x2 v[TPTV];
    };
    auto q_off = [&](int n, int u) { return ((long long)n * 64 + tq * TPT + u) * p.st + 4 * cq; };
    auto v_off = [&](int n, int u) { return ((long long)n * 64 + tv * TPTV + u) * p.vt + 4 * vq; };
    Raw r;
#pragma unroll
    for (int u = 0; u < TPT; ++u) {
        r.q[u] = *reinterpret_cast<const u32x2 *>(qp + q_off(0, u));
        r.k[u] = *reinterpret_cast<const u32x2 *>(kp + q_off(0, u));
        r.g[u] = GV::load(p.g, kbase + q_off(0, u));
    }
#pragma unroll
    for (int u = 0; u < TPTV; ++u) r.v[u] = *reinterpret_cast<const u32x2 *>(vp + v_off(0, u));

    // Log decay of the previous chunks for this thread's 4 channels, as an unevaluated sum hi + lo.
    f32x4 seg_hi = {0.f, 0.f, 0.f, 0.f}, seg_lo = {0.f, 0.f, 0.f, 0.f};

    for (int n = 0; n < p.n_chunks; ++n) {
        const long long t0 = (long long)n * 64;
        // Chunk whose data is fetched during this iteration; the last iteration refetches its own.
        const int nn = (n + 1 < p.n_chunks) ? n + 1 : n;
        ZPT(0);

        // ---- gate pass, part 1: per-thread cumulative sums, V^T ---------------------------------
        f32x4 cs[TPT];
        f32x4 excl = {0.f, 0.f, 0.f, 0.f};   // sum over the wave's earlier token groups
        {
            f32x4 run = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < TPT; ++u) {
                const f32x4 gv = GV::get(r.g[u]);
                r.g[u] = GV::load(p.g, kbase + q_off(nn, u));
#pragma unroll
                for (int a = 0; a < 4; ++a) run[a] += gv[a];
                cs[u] = run;
            }
            // inclusive scan of the group sums over the GW token groups of this wave
            f32x4 inc = run;
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
        ZPT(1);
        {
            TokenRun<TPTV> ch[4];
#pragma unroll
            for (int m = 0; m < TPTV / 2; ++m) {
                const u32x2 x = r.v[2 * m], y = r.v[2 * m + 1];
                ch[0].w[m] = pair_lo(x[0], y[0]);
                ch[1].w[m] = pair_hi(x[0], y[0]);
                ch[2].w[m] = pair_lo(x[1], y[1]);
                ch[3].w[m] = pair_hi(x[1], y[1]);
            }
#pragma unroll
            for (int u = 0; u < TPTV; ++u) r.v[u] = *reinterpret_cast<const u32x2 *>(vp + v_off(nn, u));
#pragma unroll
            for (int a = 0; a < 4; ++a) ch[a].store(Vt + (4 * vq + a) * TS + tv * TPTV * 2);
        }
        ZPT(2);
        __syncthreads();
        ZPT(3);

        // ---- gate pass, part 2: stitch waves, scale q and k -------------------------------------
        f32x4 pre = excl, total = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < NW; ++u) {
            const f32x4 x = *reinterpret_cast<const f32x4 *>(wtot + u * DK + 4 * cq);
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                if (u < w) pre[a] += x[a];
                total[a] += x[a];
            }
        }
        {
            // c = pre + cs is the in-chunk cumulative log decay; exp(c) = exp2(cs*log2e + pre*log2e);
            // G_cum = (segment prefix + pre) + cs with the prefix folded once per channel.
            f32x4 pre2, gbase;
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                pre2[a] = pre[a] * kLog2e;
                gbase[a] = seg_hi[a] + (pre[a] + seg_lo[a]);
            }
            TokenRun<TPT> kt[4];
            u32x2 kprev = {0u, 0u};
#pragma unroll
            for (int u = 0; u < TPT; ++u) {
                const int t = tq * TPT + u;
                f32x4 lam, ilam, gout;
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const float y = __builtin_fmaf(cs[u][a], kLog2e, pre2[a]);
                    lam[a] = __builtin_amdgcn_exp2f(y);
                    ilam[a] = __builtin_amdgcn_exp2f(-y);
                    gout[a] = gbase[a] + cs[u][a];
                }
                const u32x2 qw = r.q[u], kw = r.k[u];
                r.q[u] = *reinterpret_cast<const u32x2 *>(qp + q_off(nn, u));
                r.k[u] = *reinterpret_cast<const u32x2 *>(kp + q_off(nn, u));
                *reinterpret_cast<u32x2 *>(Qs + t * QS + qpos * 2) =
                    u32x2{pack_bf16(bf16_lo(qw[0]) * lam[0], bf16_hi(qw[0]) * lam[1]),
                          pack_bf16(bf16_lo(qw[1]) * lam[2], bf16_hi(qw[1]) * lam[3])};
                const u32x2 kq = {pack_bf16(bf16_lo(kw[0]) * ilam[0], bf16_hi(kw[0]) * ilam[1]),
                                  pack_bf16(bf16_lo(kw[1]) * ilam[2], bf16_hi(kw[1]) * ilam[3])};
                *reinterpret_cast<u32x2 *>(Ks + t * QS + qpos * 2) = kq;
                if (u % 2 == 1) {   // transpose: tokens (u-1, u) of each channel share a word
                    kt[0].w[u / 2] = pair_lo(kprev[0], kq[0]);
                    kt[1].w[u / 2] = pair_hi(kprev[0], kq[0]);
                    kt[2].w[u / 2] = pair_lo(kprev[1], kq[1]);
                    kt[3].w[u / 2] = pair_hi(kprev[1], kq[1]);
                }
                kprev = kq;
                *reinterpret_cast<f32x4 *>(Gc + (t0 + t) * gcs + 4 * cq) = gout;
            }
#pragma unroll
            for (int a = 0; a < 4; ++a) kt[a].store(Kt + (4 * cq + a) * TS + tq * TPT * 2);
        }
        if (tq == 0) {
            f32x4 gm;
#pragma unroll
            for (int a = 0; a < 4; ++a) gm[a] = __builtin_amdgcn_exp2f(total[a] * kLog2e);
            *reinterpret_cast<f32x4 *>(gam + 4 * cq) = gm;
        }
#pragma unroll
        for (int a = 0; a < 4; ++a) {   // (hi, lo) += total, error-free transformation
            const float x = total[a] + seg_lo[a];
            const float s = seg_hi[a] + x;
            const float bb = s - seg_hi[a];
            seg_lo[a] = (seg_hi[a] - (s - bb)) + (x - bb);
            seg_hi[a] = s;
        }
        ZPT(4);
        __syncthreads();
        ZPT(5);

        // ---- scores: P^T tiles (ts <= tt), 16x16x32; all operand reads of a tile issued up front ---
#pragma unroll
        for (int i = 0; i < (10 + NW - 1) / NW; ++i) {
            const int idx = w + NW * i;   // wave-uniform
            if (idx < 10) {
                const int tt = (idx >= 6) ? 3 : (idx >= 3) ? 2 : (idx >= 1) ? 1 : 0;
                const int ts = idx - tt * (tt + 1) / 2;
                const unsigned char *ka = Ks + (16 * ts + l16) * QS + 16 * kg;
                const unsigned char *qb = Qs + (16 * tt + l16) * QS + 16 * kg;
                bf16x8 fa[DK / 32], fb[DK / 32];
#pragma unroll
                for (int ks = 0; ks < DK / 32; ++ks) {
                    fa[ks] = lds_frag(ka, 64 * ks);
                    fb[ks] = lds_frag(qb, 64 * ks);
                }
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < DK / 32; ++ks) acc = M::run(fa[ks], fb[ks], acc);
                if (ts == tt) {
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr)
                        if (4 * kg + rr > l16) acc[rr] = 0.f;
                }
                *reinterpret_cast<u32x2 *>(Ps + (16 * tt + l16) * TS + (16 * ts + 4 * kg) * 2) =
                    u32x2{pack_bf16(acc[0], acc[1]), pack_bf16(acc[2], acc[3])};
            }
        }

        ZPT(6);
        // ---- inter: O^T += S^T Qs^T --------------------------------------------------------------
        f32x4 Oacc[4];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) Oacc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < Cfg::NKS_D; ++ks) {
            const bf16x8 sf = pack8(Sacc[2 * ks], Sacc[2 * ks + 1]);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
                Oacc[mt] = M::run(sf, lds_frag(Qs, (mt * 16 + l16) * QS + (ks * 32 + 8 * kg) * 2), Oacc[mt]);
        }
        ZPT(7);
        __syncthreads();
        ZPT(8);

        // ---- intra: O^T += Vt Ps^T, causal k-range; store O ---------------------------------------
        bf16x8 vf[2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) vf[ks] = lds_frag(Vt, (w * 16 + l16) * TS + (ks * 32 + 8 * kg) * 2);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
            for (int ks = 0; ks <= mt / 2; ++ks)   // tokens s < 16 (mt + 1) only
                Oacc[mt] = M::run(vf[ks], lds_frag(Ps, (mt * 16 + l16) * TS + (ks * 32 + 8 * kg) * 2), Oacc[mt]);
            uint16_t *orow = op + (t0 + mt * 16 + l16) * p.vt + w * 16 + 4 * kg;
            *reinterpret_cast<u32x2 *>(orow) =
                u32x2{pack_bf16(Oacc[mt][0] * p.scale, Oacc[mt][1] * p.scale),
                      pack_bf16(Oacc[mt][2] * p.scale, Oacc[mt][3] * p.scale)};
        }

        ZPT(9);
        // ---- state: S <- gamma .* (S + Kt Vt^T) ----------------------------------------------------
#pragma unroll
        for (int it = 0; it < Cfg::NIT; ++it) {
            f32x4 acc = Sacc[it];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
                acc = M::run(lds_frag(Kt, (it * 16 + l16) * TS + (ks * 32 + 8 * kg) * 2), vf[ks], acc);
            const f32x4 gm = *reinterpret_cast<const f32x4 *>(gam + it * 16 + 4 * kg);
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) acc[rr] *= gm[rr];
            Sacc[it] = acc;
        }
        ZPT(10);
        __syncthreads();
        ZPT(11);
    }

    float *Sl = p.S_loc + sbh * DK * DV + w * 16 + l16;
#pragma unroll
    for (int it = 0; it < Cfg::NIT; ++it)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) Sl[(size_t)(it * 16 + 4 * kg + rr) * DV] = Sacc[it][rr];
    if (tq == 0) {
        f32x4 gt;
#pragma unroll
        for (int a = 0; a < 4; ++a) gt[a] = seg_hi[a] + seg_lo[a];
        *reinterpret_cast<f32x4 *>(p.G_tot + sbh * DK + 4 * cq) = gt;
    }
}

template <int DK, int DV, bool GBF16>
static hipError_t launch_b16(const ChunkParams &p, hipStream_t s) {
    typedef B16Cfg<DK, DV> Cfg;
    auto kern = gla_chunk_bf16_kernel<DK, DV, GBF16>;
    hipError_t e = hipFuncSetAttribute((const void *)kern,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kBytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(p.B * p.P * p.H), dim3(Cfg::NT), Cfg::kBytes, s, p);
    return hipGetLastError();
}

template <bool GBF16>
static hipError_t dispatch_b16(const ChunkParams &p, int d_k, int d_v, hipStream_t s) {
    if (d_k == 64 && d_v == 64) return launch_b16<64, 64, GBF16>(p, s);
    if (d_k == 128 && d_v == 64) return launch_b16<128, 64, GBF16>(p, s);
    if (d_k == 64 && d_v == 128) return launch_b16<64, 128, GBF16>(p, s);
    if (d_k == 128 && d_v == 128) return launch_b16<128, 128, GBF16>(p, s);
    return hipErrorInvalidValue;
}

hipError_t launch_chunk_bf16(const ChunkParams &p, int d_k, int d_v, bool g_bf16, hipStream_t s) {
    return g_bf16 ? dispatch_b16<true>(p, d_k, d_v, s) : dispatch_b16<false>(p, d_k, d_v, s);
}

}  // namespace zeco
