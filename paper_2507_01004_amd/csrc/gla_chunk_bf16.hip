// Chunkwise GLA forward of a segment from the zero state: bf16 inputs, bf16 MFMA operands,
// fp32 accumulation, fp32 state.  The throughput path.
//
// Work decomposition.  A (batch, segment, head) stream is a serial recurrence over N = L/64
// chunks (Sec. 3.1).  A workgroup of 4 waves owns one stream and a slice of DVW columns of d_v
// (DVW = d_v: one workgroup per stream; DVW = d_v/2: two sibling workgroups per stream, placed
// on the same XCD so that their common q, k, g traffic is served by that XCD's L2).  Wave w owns
// TILE = DVW/4 columns of the state; the state stays in MFMA accumulators for the whole segment.
//
// Per chunk (chunk equations of Sec. 2.1, scores as in Alg. 1):
//   gate pass   lane = channel pair, each thread scans its tokens serially, groups are stitched
//               through LDS: cs = inclusive cumsum of g;  Lambda = e^cs, 1/Lambda, Gamma = e^(cs_C-cs)
//               writes  Qs = Q.*Lambda*scale, Ks = K/Lambda   (token-major, bf16)
//                       Kt = (K.*Gamma)^T,  Vt = V^T           (channel-major, bf16)
//   scores      P^T = Ks Qs^T on the 10 lower-triangular 16x16 tiles, causal select, -> Ps (bf16)
//   inter       O^T += S^T Qs^T   with S fed straight from the accumulators (see below)
//   intra       O^T += Vt Ps^T    (causal k-range), O stored to HBM
//   state       S <- (gamma^T 1) .* S + Kt Vt^T
//
// Accumulator-as-operand.  Lane l of an accumulator tile holds column l%TILE and, with
// kg = l/TILE, a fixed set of rows.  The MFMA operand layout wants, from the same lane, row
// (column) l%TILE and eight k-slots.  Summation over k is order-free, so the eight state rows a
// lane already owns are used as its eight k-slots, and Qs is stored in LDS with its channels
// permuted to match (pos_of_channel); Ks uses the same permutation so the scores are unaffected.
#include "zeco_device.h"
#include "zeco_internal.h"

namespace zeco {

template <int DK, int DVW> struct B16Cfg {
    static constexpr int TILE = DVW / 4;
    static constexpr int NKG = 64 / TILE;          // lane groups along k: 4 (TILE 16) or 2 (TILE 32)
    static constexpr int KS = 8 * NKG;             // k extent of one MFMA: 32 or 16
    static constexpr int ACC = TILE * TILE / 64;   // accumulator registers per tile
    static constexpr int NIT = DK / TILE;          // state row tiles
    static constexpr int NMT = 64 / TILE;          // token tiles
    static constexpr int NKS_C = 64 / KS;          // k-steps across the tokens of a chunk
    static constexpr int NKS_D = DK / KS;          // k-steps across channels
    // gate pass thread mapping
    static constexpr int LPR = DK / 2;             // lanes per token row (2 channels per lane)
    static constexpr int TG = 4 * (64 / LPR);      // token groups
    static constexpr int TPT = 64 / TG;            // consecutive tokens per thread
    static constexpr int LPRV = DVW / 2;
    static constexpr int TGV = 4 * (64 / LPRV);
    static constexpr int TPTV = 64 / TGV;
    // LDS (bytes)
    static constexpr int QS = DK * 2 + 16;         // row stride of Qs, Ks
    static constexpr int TS = 64 * 2 + 16;         // row stride of Kt, Vt, Ps
    static constexpr int kOffQ = 0;
    static constexpr int kOffK = kOffQ + 64 * QS;
    static constexpr int kOffKT = kOffK + 64 * QS;
    static constexpr int kOffVT = kOffKT + DK * TS;
    static constexpr int kOffP = kOffVT + DVW * TS;
    static constexpr int kOffTot = kOffP + 64 * TS;
    static constexpr int kOffGam = kOffTot + TG * DK * 4;
    static constexpr int kBytes = kOffGam + DK * 4;

    // LDS position of channel i inside a Qs/Ks row (see "Accumulator-as-operand").
    __device__ static __forceinline__ constexpr int pos_of_channel(int i) {
        const int il = i % KS;
        return (i - il) + 8 * ((il / 4) % NKG) + 4 * (il / (4 * NKG)) + (il % 4);
    }
};

__device__ __forceinline__ bf16x8 pack8(float a0, float a1, float a2, float a3, float a4, float a5,
                                        float a6, float a7) {
    u32x4 w = {pack_bf16(a0, a1), pack_bf16(a2, a3), pack_bf16(a4, a5), pack_bf16(a6, a7)};
    return __builtin_bit_cast(bf16x8, w);
}

// Eight state rows owned by this lane for channel k-step ks, as an MFMA operand.
template <int TILE, int NIT>
__device__ __forceinline__ bf16x8 state_frag(const typename Mma<TILE>::acc_t (&S)[NIT], int ks) {
    if constexpr (TILE == 16) {
        const f32x4 a = S[2 * ks], b = S[2 * ks + 1];
        return pack8(a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]);
    } else {
        const f32x16 a = S[ks / 2];
        if (ks % 2 == 0) return pack8(a[0], a[1], a[2], a[3], a[4], a[5], a[6], a[7]);
        return pack8(a[8], a[9], a[10], a[11], a[12], a[13], a[14], a[15]);
    }
}

template <bool GBF16> struct GateVal;
template <> struct GateVal<false> {
    typedef f32x2 raw_t;
    __device__ static __forceinline__ raw_t load(const void *g, long long elem) {
        return *reinterpret_cast<const f32x2 *>((const float *)g + elem);
    }
    __device__ static __forceinline__ float lo(raw_t r) { return r[0]; }
    __device__ static __forceinline__ float hi(raw_t r) { return r[1]; }
};
template <> struct GateVal<true> {
    typedef uint32_t raw_t;
    __device__ static __forceinline__ raw_t load(const void *g, long long elem) {
        return *reinterpret_cast<const uint32_t *>((const uint16_t *)g + elem);
    }
    __device__ static __forceinline__ float lo(raw_t r) { return bf16_lo(r); }
    __device__ static __forceinline__ float hi(raw_t r) { return bf16_hi(r); }
};

template <int DK, int DVW, bool GBF16>
__global__ __launch_bounds__(256) void gla_chunk_bf16_kernel(ChunkParams p) {
    typedef B16Cfg<DK, DVW> Cfg;
    typedef Mma<Cfg::TILE> M;
    typedef GateVal<GBF16> GV;
    constexpr int TILE = Cfg::TILE, KS = Cfg::KS, QS = Cfg::QS, TS = Cfg::TS;
    extern __shared__ __align__(16) unsigned char lds[];
    unsigned char *Qs = lds + Cfg::kOffQ, *Ks = lds + Cfg::kOffK, *Kt = lds + Cfg::kOffKT;
    unsigned char *Vt = lds + Cfg::kOffVT, *Ps = lds + Cfg::kOffP;
    float *tot = reinterpret_cast<float *>(lds + Cfg::kOffTot);
    float *gam = reinterpret_cast<float *>(lds + Cfg::kOffGam);

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int lt = lane % TILE, kg = lane / TILE;   // lane coordinates for the TILE-shaped MFMA
    const int l16 = lane & 15, kg16 = lane >> 4;    // and for the 16x16x32 score tiles

    // Workgroup -> (stream, slice).  Workgroup ids are dealt round-robin to the 8 XCDs, so sibling
    // slices of a stream take consecutive slots of one XCD.
    const int streams = p.B * p.P * p.H;
    const int NS = p.n_slices;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    int sidx = (slot / NS) * 8 + xcd;
    const int slice = slot % NS;
    if (sidx >= streams) return;
    const size_t sbh = sidx;                        // (seg * B + b) * H + h  (S_loc / G_tot order)
    const int h = sidx % p.H;
    sidx /= p.H;
    const int b = sidx % p.B, seg = sidx / p.B;
    const long long tok0 = (long long)seg * p.L;
    const long long kbase = b * p.sb + tok0 * p.st + h * p.sh;
    const long long vbase = b * p.vb + tok0 * p.vt + h * p.vh + slice * DVW;
    const uint16_t *qp = (const uint16_t *)p.q + kbase;
    const uint16_t *kp = (const uint16_t *)p.k + kbase;
    const uint16_t *vp = (const uint16_t *)p.v + vbase;
    uint16_t *op = (uint16_t *)p.o + vbase;
    const long long T = (long long)p.P * p.L;
    float *Gc = p.G_cum + (((long long)b * T + tok0) * p.H + h) * DK;
    const long long gcs = (long long)p.H * DK;

    // gate-pass coordinates
    const int c2 = lane % Cfg::LPR, tg = w * (64 / Cfg::LPR) + lane / Cfg::LPR;
    const int c2v = lane % Cfg::LPRV, tgv = w * (64 / Cfg::LPRV) + lane / Cfg::LPRV;
    const int qpos = Cfg::pos_of_channel(2 * c2);

    typename M::acc_t Sacc[Cfg::NIT];
#pragma unroll
    for (int it = 0; it < Cfg::NIT; ++it)
#pragma unroll
        for (int r = 0; r < Cfg::ACC; ++r) Sacc[it][r] = 0.f;

    // Score tiles above the diagonal are never computed: zero them once.
    for (int e = tid; e < 64 * TS / 16; e += 256)
        *reinterpret_cast<u32x4 *>(Ps + e * 16) = u32x4{0u, 0u, 0u, 0u};

    struct Raw {
        uint32_t q[Cfg::TPT], k[Cfg::TPT];
        typename GV::raw_t g[Cfg::TPT];
        uint32_t v[Cfg::TPTV];
    };
    auto load_raw = [&](int n, Raw &r) {
        const long long t0 = (long long)n * 64;
#pragma unroll
        for (int u = 0; u < Cfg::TPT; ++u) {
            const long long e = (t0 + tg * Cfg::TPT + u) * p.st + 2 * c2;
            r.q[u] = *reinterpret_cast<const uint32_t *>(qp + e);
            r.k[u] = *reinterpret_cast<const uint32_t *>(kp + e);
            r.g[u] = GV::load(p.g, kbase + e);
        }
#pragma unroll
        for (int u = 0; u < Cfg::TPTV; ++u)
            r.v[u] = *reinterpret_cast<const uint32_t *>(
                vp + (t0 + tgv * Cfg::TPTV + u) * p.vt + 2 * c2v);
    };

    double seg0 = 0.0, seg1 = 0.0;   // log decay of the previous chunks, channels 2*c2, 2*c2+1
    Raw nxt;
    load_raw(0, nxt);

    for (int n = 0; n < p.n_chunks; ++n) {
        const long long t0 = (long long)n * 64;
        Raw cur = nxt;

        // ---- gate pass ---------------------------------------------------------------------------
        float cs0[Cfg::TPT], cs1[Cfg::TPT];
        {
            float r0 = 0.f, r1 = 0.f;
#pragma unroll
            for (int u = 0; u < Cfg::TPT; ++u) {
                r0 += GV::lo(cur.g[u]);
                r1 += GV::hi(cur.g[u]);
                cs0[u] = r0;
                cs1[u] = r1;
            }
            *reinterpret_cast<f32x2 *>(tot + tg * DK + 2 * c2) = f32x2{r0, r1};
        }
        // V^T: each thread owns TPTV consecutive tokens of two columns.
        {
#pragma unroll
            for (int pc = 0; pc < Cfg::TPTV / 8; ++pc) {
                u32x4 a, bq;
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const uint32_t x = cur.v[8 * pc + 2 * m], y = cur.v[8 * pc + 2 * m + 1];
                    a[m] = (x & 0xffffu) | (y << 16);
                    bq[m] = (x >> 16) | (y & 0xffff0000u);
                }
                const int off = (tgv * Cfg::TPTV + 8 * pc) * 2;
                *reinterpret_cast<u32x4 *>(Vt + (2 * c2v) * TS + off) = a;
                *reinterpret_cast<u32x4 *>(Vt + (2 * c2v + 1) * TS + off) = bq;
            }
        }
        __syncthreads();
        float pre0 = 0.f, pre1 = 0.f, tot0 = 0.f, tot1 = 0.f;
#pragma unroll
        for (int u = 0; u < Cfg::TG; ++u) {
            const f32x2 x = *reinterpret_cast<const f32x2 *>(tot + u * DK + 2 * c2);
            if (u < tg) { pre0 += x[0]; pre1 += x[1]; }
            tot0 += x[0];
            tot1 += x[1];
        }
        {
            float kt0[Cfg::TPT], kt1[Cfg::TPT];
#pragma unroll
            for (int u = 0; u < Cfg::TPT; ++u) {
                const int t = tg * Cfg::TPT + u;
                const float a0 = pre0 + cs0[u], a1 = pre1 + cs1[u];
                const float q0 = bf16_lo(cur.q[u]), q1 = bf16_hi(cur.q[u]);
                const float k0 = bf16_lo(cur.k[u]), k1 = bf16_hi(cur.k[u]);
                *reinterpret_cast<uint32_t *>(Qs + t * QS + qpos * 2) =
                    pack_bf16(q0 * fast_exp(a0) * p.scale, q1 * fast_exp(a1) * p.scale);
                *reinterpret_cast<uint32_t *>(Ks + t * QS + qpos * 2) =
                    pack_bf16(k0 * fast_exp(-a0), k1 * fast_exp(-a1));
                kt0[u] = k0 * fast_exp(tot0 - a0);
                kt1[u] = k1 * fast_exp(tot1 - a1);
                if ((u % NS) == slice)   // sibling slices share the G_cum rows between them
                    *reinterpret_cast<f32x2 *>(Gc + (t0 + t) * gcs + 2 * c2) =
                        f32x2{(float)(seg0 + (double)a0), (float)(seg1 + (double)a1)};
            }
#pragma unroll
            for (int pc = 0; pc < Cfg::TPT / 8; ++pc) {
                u32x4 a, bq;
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    a[m] = pack_bf16(kt0[8 * pc + 2 * m], kt0[8 * pc + 2 * m + 1]);
                    bq[m] = pack_bf16(kt1[8 * pc + 2 * m], kt1[8 * pc + 2 * m + 1]);
                }
                const int off = (tg * Cfg::TPT + 8 * pc) * 2;
                *reinterpret_cast<u32x4 *>(Kt + (2 * c2) * TS + off) = a;
                *reinterpret_cast<u32x4 *>(Kt + (2 * c2 + 1) * TS + off) = bq;
            }
        }
        if (tg == 0) *reinterpret_cast<f32x2 *>(gam + 2 * c2) = f32x2{fast_exp(tot0), fast_exp(tot1)};
        seg0 += (double)tot0;
        seg1 += (double)tot1;
        if (n + 1 < p.n_chunks) load_raw(n + 1, nxt);   // in flight during the MFMA phases
        __syncthreads();

        // ---- scores: P^T tiles (ts <= tt), 16x16x32 ----------------------------------------------
        for (int idx = w; idx < 10; idx += 4) {
            int tt = 0, rem = idx;
            while (rem > tt) { rem -= tt + 1; ++tt; }
            const int ts = rem;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            const unsigned char *ka = Ks + (16 * ts + l16) * QS + 16 * kg16;
            const unsigned char *qb = Qs + (16 * tt + l16) * QS + 16 * kg16;
#pragma unroll
            for (int ks = 0; ks < DK / 32; ++ks)
                acc = Mma<16>::run(lds_frag(ka, 64 * ks), lds_frag(qb, 64 * ks), acc);
            if (ts == tt) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (4 * kg16 + r > l16) acc[r] = 0.f;
            }
            *reinterpret_cast<u32x2 *>(Ps + (16 * tt + l16) * TS + (16 * ts + 4 * kg16) * 2) =
                u32x2{pack_bf16(acc[0], acc[1]), pack_bf16(acc[2], acc[3])};
        }

        // ---- inter: O^T += S^T Qs^T --------------------------------------------------------------
        typename M::acc_t Oacc[Cfg::NMT];
#pragma unroll
        for (int mt = 0; mt < Cfg::NMT; ++mt)
#pragma unroll
            for (int r = 0; r < Cfg::ACC; ++r) Oacc[mt][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < Cfg::NKS_D; ++ks) {
            const bf16x8 sf = state_frag<TILE, Cfg::NIT>(Sacc, ks);
#pragma unroll
            for (int mt = 0; mt < Cfg::NMT; ++mt)
                Oacc[mt] = M::run(sf, lds_frag(Qs, (mt * TILE + lt) * QS + (ks * KS + 8 * kg) * 2),
                                  Oacc[mt]);
        }
        __syncthreads();

        // ---- intra: O^T += Vt Ps^T, causal k-range; store O ---------------------------------------
        bf16x8 vf[Cfg::NKS_C];
#pragma unroll
        for (int ks = 0; ks < Cfg::NKS_C; ++ks)
            vf[ks] = lds_frag(Vt, (w * TILE + lt) * TS + (ks * KS + 8 * kg) * 2);
#pragma unroll
        for (int mt = 0; mt < Cfg::NMT; ++mt) {
            const int nks = ((mt + 1) * TILE + KS - 1) / KS;
#pragma unroll
            for (int ks = 0; ks < Cfg::NKS_C; ++ks)
                if (ks < nks)
                    Oacc[mt] = M::run(vf[ks],
                                      lds_frag(Ps, (mt * TILE + lt) * TS + (ks * KS + 8 * kg) * 2),
                                      Oacc[mt]);
            uint16_t *orow = op + (t0 + mt * TILE + lt) * p.vt + w * TILE;
#pragma unroll
            for (int qd = 0; qd < Cfg::ACC / 4; ++qd) {
                const int j = M::row(4 * qd, kg);
                *reinterpret_cast<u32x2 *>(orow + j) =
                    u32x2{pack_bf16(Oacc[mt][4 * qd], Oacc[mt][4 * qd + 1]),
                          pack_bf16(Oacc[mt][4 * qd + 2], Oacc[mt][4 * qd + 3])};
            }
        }

        // ---- state: S <- gamma .* S + Kt Vt^T ------------------------------------------------------
#pragma unroll
        for (int it = 0; it < Cfg::NIT; ++it) {
            typename M::acc_t acc = Sacc[it];
#pragma unroll
            for (int r = 0; r < Cfg::ACC; ++r) acc[r] *= gam[it * TILE + M::row(r, kg)];
#pragma unroll
            for (int ks = 0; ks < Cfg::NKS_C; ++ks)
                acc = M::run(lds_frag(Kt, (it * TILE + lt) * TS + (ks * KS + 8 * kg) * 2), vf[ks],
                             acc);
            Sacc[it] = acc;
        }
        __syncthreads();
    }

    float *Sl = p.S_loc + sbh * DK * (DVW * NS) + slice * DVW + w * TILE + lt;
#pragma unroll
    for (int it = 0; it < Cfg::NIT; ++it)
#pragma unroll
        for (int r = 0; r < Cfg::ACC; ++r)
            Sl[(size_t)(it * TILE + M::row(r, kg)) * (DVW * NS)] = Sacc[it][r];
    if (tg == 0 && slice == 0)
        *reinterpret_cast<f32x2 *>(p.G_tot + sbh * DK + 2 * c2) = f32x2{(float)seg0, (float)seg1};
}

int chunk_bf16_slices(int streams, int d_v) {
    // Two sibling workgroups per stream while one per stream would leave compute units idle.
    return (d_v == 128 && streams < 256) ? 2 : 1;
}

template <int DK, int DVW, bool GBF16>
static hipError_t launch_b16(const ChunkParams &p, hipStream_t s) {
    typedef B16Cfg<DK, DVW> Cfg;
    auto kern = gla_chunk_bf16_kernel<DK, DVW, GBF16>;
    hipError_t e = hipFuncSetAttribute((const void *)kern,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kBytes);
    if (e != hipSuccess) return e;
    const int streams = p.B * p.P * p.H;
    const int grid = ((streams + 7) / 8) * 8 * p.n_slices;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), Cfg::kBytes, s, p);
    return hipGetLastError();
}

template <bool GBF16>
static hipError_t dispatch_b16(const ChunkParams &p, int d_k, int dvw, hipStream_t s) {
    if (d_k == 64 && dvw == 64) return launch_b16<64, 64, GBF16>(p, s);
    if (d_k == 64 && dvw == 128) return launch_b16<64, 128, GBF16>(p, s);
    if (d_k == 128 && dvw == 64) return launch_b16<128, 64, GBF16>(p, s);
    if (d_k == 128 && dvw == 128) return launch_b16<128, 128, GBF16>(p, s);
    return hipErrorInvalidValue;
}

hipError_t launch_chunk_bf16(const ChunkParams &p, int d_k, int d_v, bool g_bf16, hipStream_t s) {
    const int dvw = d_v / p.n_slices;
    return g_bf16 ? dispatch_b16<true>(p, d_k, dvw, s) : dispatch_b16<false>(p, d_k, dvw, s);
}

}  // namespace zeco
