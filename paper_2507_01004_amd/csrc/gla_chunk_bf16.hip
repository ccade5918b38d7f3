// Chunkwise GLA forward of a segment from the zero state: bf16 inputs, bf16 MFMA operands,
// fp32 accumulation, fp32 state.  The throughput path.
//
// Work decomposition.  A (batch, segment, head) stream is a serial recurrence over N = L/64
// chunks (Sec. 3.1).  One workgroup owns a stream and is split into two kinds of waves that run
// concurrently on the same SIMDs and use different execution resources:
//   * 4 gate waves (VALU, transcendentals, global memory): for chunk n+1 they load q, k, g, v,
//     compute the in-chunk cumulative log decay and write the scaled operand tiles to LDS;
//   * d_v/32 MFMA waves (matrix cores, LDS reads): for chunk n they compute scores, outputs and the
//     state update; wave j owns columns [32j, 32j+32) of the d_k x d_v state, which stays in MFMA
//     accumulators for the whole segment.
// The LDS tiles are double buffered and the two kinds meet at two workgroup barriers per chunk.
//
// Per chunk (chunk equations of Sec. 2.1, scores as in Alg. 1):
//   gate, part 1   each thread owns 4 channels x TPT consecutive tokens: serial cumsum of g in
//                  registers, token groups stitched by lane shuffles inside a wave and one LDS
//                  exchange across the gate waves;  Vs = V -> LDS as it comes (token-major)
//   gate, part 2   cs = inclusive cumsum of g, Lambda = e^cs;  Qs = Q .* Lambda, Ks = K / Lambda
//                  (token-major) -> LDS;  G_cum -> HBM
//   MFMA, part 1   P^T = Ks Qs^T on the 10 lower-triangular 16x16 tiles, causal select -> Ps (bf16);
//                  O^T  = S^T Qs^T   with S fed straight from the accumulators (see below)
//   MFMA, part 2   O^T += V^T Ps^T (causal k-range), O * scale -> HBM;
//                  S <- (gamma^T 1) .* (S + (K / Lambda)^T V)
// The last line is Eq. (3) with K .* Gamma = (gamma^T 1)-scaled K / Lambda (Gamma = gamma / Lambda),
// so one scaled copy of K serves both the scores and the state update.
//
// Transposed operands.  The two products of part 2 contract over tokens, so they need V^T and
// (K / Lambda)^T fragments (lane = channel, k-slots = tokens).  The matrix waves take them from the
// token-major tiles with gfx950's transposing LDS read (lds_frag_tr below); the gate waves never
// transpose anything.  (Channel-major copies written by the gate waves cost them two permutes per
// token pair and stores whose rows sit four apart per lane, 8-way bank conflicts: 5-6 % of the
// local pass where the gate waves set the pace, 10-16 % with per-head gates.)
//
// Accumulator-as-operand.  Lane l of a 32x32 accumulator tile holds column l%32 and, with
// kg = l/32, rows 8q + 4kg + m (q < 4, m < 4).  The MFMA operand layout wants, from the same lane,
// row (column) l%32 and eight k-slots.  Summation over k is order-free, so the eight state rows a
// lane owns in half a tile are used as its eight k-slots, and Qs is stored in LDS with its
// channels permuted to match (pos_of_channel); Ks uses the same permutation, so the scores are
// unaffected.
//
// Memory pipeline.  One register set holds the raw q, k, g, v of the chunk the gate waves work on;
// each piece is reloaded with the following chunk's data right after its last use, so the global
// loads are spread out and stay in flight for a whole iteration.
#include "zeco_device.h"
#include "zeco_internal.h"

namespace zeco {


template <int DK, int DV, int NWG_, int NWI_ = 0> struct B16Cfg {
    static constexpr int NWM = DV / 32;            // MFMA waves, 32 state columns each
    static constexpr int NWG = NWG_;               // gate waves
    static constexpr int NWI = NWI_;               // idle waves (placement only, see idle_waves)
    static constexpr int NT = 64 * (NWM + NWG + NWI);
    static constexpr int NIT = DK / 32;            // state row tiles per MFMA wave
    // gate pass thread mapping over the 256 gate threads: 4 channels x TPT tokens per thread
    static constexpr int CQ = DK / 4;              // channel quads
    static constexpr int GW = 64 / CQ;             // token groups inside one wave (2 or 4)
    static constexpr int TPT = 64 / (NWG * GW);    // consecutive tokens per thread (8 or 4)
    static constexpr int VQ = DV / 4;
    static constexpr int TPTV = 64 / (64 * NWG / VQ);   // 8, 4 or 2
    // LDS (bytes).  The scaled tiles are double buffered.
    static constexpr int QS = DK * 2 + 16;         // row stride of Qs, Ks
    static constexpr int TS = 64 * 2 + 16;         // row stride of Ps
    // row stride of Vs: 16 dwords past a multiple of 64 banks, so that the 32 lanes of a transposing read
    // (4 rows x 4 quads x 2 groups of 16 lanes) fall on 64 different banks
    static constexpr int VS = DV * 2 + 64;
    static constexpr int kOffQ = 0;                // offsets inside one tile buffer
    static constexpr int kOffK = kOffQ + 64 * QS;
    static constexpr int kOffV = kOffK + 64 * QS;
    static constexpr int kOffO2 = kOffV + 64 * VS; // staged output columns beyond d_k (only when d_v > d_k)
    static constexpr int kTileBytes = kOffO2 + (DV > DK ? 64 * QS : 0);
    static constexpr int kOffP = 2 * kTileBytes;
    static constexpr int kOffTot = kOffP + 64 * TS;
    static constexpr int kOffGam = kOffTot + NWG * DK * 4;
    static constexpr int kBytes = kOffGam + 2 * DK * 4;

    // LDS position of channel i inside a Qs/Ks row (see "Accumulator-as-operand"): within each
    // block of 16 channels, channel 8 q + 4 kg + m sits at 8 kg + 4 q + m.
    __device__ static __forceinline__ constexpr int pos_of_channel(int i) {
        const int il = i % 16;
        return (i - il) + 8 * ((il / 4) % 2) + 4 * (il / 8) + (il % 4);
    }
};

__device__ __forceinline__ bf16x8 pack8(const f32x16 &a, int base) {
    u32x4 w = {pack_bf16(a[base + 0], a[base + 1]), pack_bf16(a[base + 2], a[base + 3]),
               pack_bf16(a[base + 4], a[base + 5]), pack_bf16(a[base + 6], a[base + 7])};
    return __builtin_bit_cast(bf16x8, w);
}

// DV is the number of state columns this workgroup owns: d_v, or d_v / NS when NS sibling workgroups
// share a stream (each recomputes the gate pass and takes its own slice of v, o and the state).
// MODE selects what a launch computes:
//   kLocal   the local pass from the zero state: o, S_loc, G_cum, G_tot          (Sec. 3.1)
//   kStates  only the final local state and total decay of each segment: S_loc, G_tot
//            (Alg. 1's chunk-state loop; q is not read, nothing per token is written)
//   kOutput  the output pass from given initial states S_init[p]: o only
//            (Alg. 1's output pass, the incoming state folded into the running state)
//   kLocalCD the local pass with the cumulative decay kept per chunk, as Alg. 1 stores it (the list of
//            gamma~_[n]): o, S_loc, G_tot and G_chunk[n] = log gamma~_[n-1], the log decay from the segment's
//            first token up to the start of chunk n; no per-token G_cum is written
//   kLocalInit  the output pass that also emits the per-token cumulative log decay, counted from the
//            given offsets G_off[p]: o, G_cum (second pass of the local pass when a segment is cut
//            into sub-segments; S_init[p] and G_off[p] then hold what precedes sub-segment p inside
//            its segment)
// and two passes of the backward (App. A.4), which walk the chunks of a segment from the last to the
// first and keep dS, the gradient of the running state, in the accumulators:
//   kDState  dS <- (gamma^T 1) .* dS + (Q .* Lambda)^T dO from zero; S_loc receives the gradient that
//            leaves the segment towards the state entering it (first loop of the backward listing)
//   kDV      dV = (K / Lambda) ((gamma^T 1) .* dS) + (intra-chunk scores)^T dO, with dS started from
//            S_init[p] = the gradient entering the segment's final state
// The backward modes are called with the tensors in other roles (kDState: k := q, v := dO;
// kDV: q := k, k := q, v := dO, o := dV), flip the sign of the decay exponents, apply gamma before the
// chunk's products instead of after, and store token t of a chunk at tile row 63 - t, so that the
// causal structure of the tiles is the one of the forward pass.
enum ChunkMode { kLocal = 0, kStates = 1, kOutput = 2, kDState = 3, kDV = 4, kLocalInit = 5, kLocalCD = 6 };

// Gate waves per workgroup: 4, one per SIMD beside an MFMA wave; 8 in the local pass with per-channel
// gates at d_k = 128, which moves the most bytes per chunk and gains 2-3 % from the second set of
// loads in flight (the other modes lose as much).
constexpr int gate_waves(int dk, int gm, int mode) {
    return (dk == 128 && (mode == kLocal || mode == kLocalInit) && gm != kGateHead) ? 8 : 4;
}
// Waves of a workgroup go round the four SIMDs of the compute unit in order.  With two matrix waves and eight
// gate waves that puts each matrix wave on a SIMD with two gate waves and leaves two SIMDs with two gate waves
// only - and the matrix waves are the longer side of both phases (cycle stamps: they reach the barriers last,
// the gate waves wait there for a quarter of the chunk).  Two waves that do nothing but keep the barriers
// (wave slots 4 and 5) shift the placement: a matrix wave then shares its SIMD with one gate wave, the other
// two SIMDs carry three gate waves each.  With four gate waves the matrix waves then have their SIMDs to
// themselves (2-3 % on the sibling configurations of the other modes).
constexpr int idle_waves(int dk, int dv, int gm, int mode) { return (dv / 32 == 2) ? 2 : 0; }
constexpr int chunk_threads(int dk, int dv, int gm, int mode) {
    return 64 * (dv / 32 + gate_waves(dk, gm, mode) + idle_waves(dk, dv, gm, mode));
}

//
// WIDE selects the reference point of the decay factors in the operand tiles.  With c the in-chunk cumulative
// log decay and total its value at the chunk's end, the tiles hold Q .* e^(c - ref) and K .* e^(ref - c); any
// ref per channel gives the same products e^(c_t - c_s).
//   WIDE = false: ref = 0, the chunk's start, as in Alg. 1.  The state takes one factor per chunk, e^total
//            (gamma), and the tiles span e^(+-|total|): |total| has to stay below 80 for bf16 operands.
//   WIDE = true:  ref = total / 2.  No exponent exceeds |total| / 2 wherever in the chunk the decay happens,
//            so |total| may reach 160.  The state takes e^(total/2) twice, before the chunk's products with
//            it and after its update (in either walking direction), which costs the MFMA waves a second
//            multiplication of the state per chunk: about 3 % of the local pass.
template <int DK, int DV, int NS, int GM, int MODE, bool WIDE>
__global__ __launch_bounds__(chunk_threads(DK, DV, GM, MODE)) void gla_chunk_bf16_kernel(ChunkParams p) {
    typedef B16Cfg<DK, DV, gate_waves(DK, GM, MODE), idle_waves(DK, DV, GM, MODE)> Cfg;
    typedef Mma<32> M;
    typedef GateVal<GM> GV;
    constexpr int QS = Cfg::QS, TS = Cfg::TS, VS = Cfg::VS, NWM = Cfg::NWM, NT = Cfg::NT;
    constexpr int TPT = Cfg::TPT, TPTV = Cfg::TPTV, CQ = Cfg::CQ, GW = Cfg::GW;
    constexpr int GB = GM == kGateBF16 ? 2 : 4;   // bytes per gate element
    constexpr bool GH = GM == kGateHead;
    constexpr bool REV = MODE == kDState || MODE == kDV;          // chunks and tokens in reverse
    constexpr bool NOQ = MODE == kStates || MODE == kDState;      // only the state is computed
    constexpr bool FROM_INIT = MODE == kOutput || MODE == kDV || MODE == kLocalInit;   // start from S_init, emit no state
    constexpr bool EMIT_G = MODE == kLocal || MODE == kLocalInit;  // per-token cumulative log decay
    constexpr float SGN = REV ? -1.f : 1.f;                       // sign of the decay exponents
    constexpr float kLog2e = 1.4426950408889634f;
    extern __shared__ __align__(16) unsigned char lds[];
    unsigned char *Ps = lds + Cfg::kOffP;
    float *wtot = reinterpret_cast<float *>(lds + Cfg::kOffTot);   // [gate wave][channel] gate sums
    float *gam = reinterpret_cast<float *>(lds + Cfg::kOffGam);    // [buffer][channel] chunk decay e^total (WIDE: e^(total/2))

    const int tid = threadIdx.x, lane = tid & 63;
    const int pw = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave slot, known uniform
    // role: w < NWM matrix wave w, NWM <= w < NWM + NWG gate wave w - NWM, beyond that idle (slots 4, 5)
    const int w = Cfg::NWI == 0 ? pw : (pw < NWM ? pw : (pw == 4 || pw == 5) ? NWM + Cfg::NWG + (pw - 4)
                                                                              : NWM + (pw < 4 ? pw - 2 : pw - 4));
    int N = p.n_chunks, pad = p.pad;   // (per segment when the segments differ in length, see below)
    auto chunk_of = [&](int m) { return REV ? N - 1 - m : m; };   // m-th chunk in processing order
    // First token of chunk n.  When L is no multiple of 64 the chunk processed FIRST is the short one,
    // 64 - pad tokens: the segment's first tokens in the forward modes, its last ones in the reverse modes.
    // It is loaded as a full window inside the segment - [0, 64), or [L - 64, L) - with g, k, v of the
    // window's surplus rows (the far end, or the near end) taken as zero, which leaves state, decay and the
    // real rows' outputs untouched, and stores only its real rows; all other chunks are full.
    auto cstart = [&](int n) {
        if constexpr (REV) return (long long)n * 64 - (n == N - 1 ? pad : 0);
        else return n ? (long long)n * 64 - pad : 0ll;
    };
    auto dead = [&](int t) { return REV ? t < pad : t >= 64 - pad; };   // surplus row of the short chunk
    auto pos_of = [](int t) { return REV ? 63 - t : t; };         // tile row of token t of a chunk

    // Workgroup -> (stream, slice).  Workgroup ids are dealt round-robin to the 8 XCDs, so sibling
    // slices of a stream take consecutive slots of one XCD and share its L2 for q, k, g.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    int sidx = (slot / NS) * 8 + xcd;
    const int slice = slot % NS;
    if (sidx >= p.B * p.P * p.H) return;
    const size_t sbh = sidx;                        // (seg * B + b) * H + h  (S_loc / G_tot order)
    const int h = sidx % p.H;
    sidx /= p.H;
    const int b = sidx % p.B, seg = sidx / p.B;
    long long tok0 = (long long)seg * p.L, T = (long long)p.P * p.L;   // first token; tokens per batch entry
    if constexpr (MODE != kLocalInit && MODE != kLocalCD) {
        if (p.seg_start) {
            // segments of unequal length: this one's bounds from the table.  A segment the kernel cannot take
            // (under 64 tokens, over the bound L, outside the tensor) is left alone: the whole workgroup leaves.
            tok0 = p.seg_start[seg];
            T = p.T;
            const long long len = p.seg_start[seg + 1] - tok0;
            if (tok0 < 0 || len < 64 || len > p.L || tok0 > T - len) return;   // (in this order: no sum can overflow)
            N = (int)((len + 63) >> 6);
            pad = 64 * N - (int)len;
        }
    }
    const long long kbase = b * p.sb + tok0 * p.st + h * p.sh;
    const long long vbase = b * p.vb + tok0 * p.vt + h * p.vh + slice * DV;
    const unsigned st = (unsigned)p.st, vt = (unsigned)p.vt;

    // Score tiles above the diagonal are never computed: zero them once.
    for (int e = tid; e < 64 * TS / 16; e += NT)
        *reinterpret_cast<u32x4 *>(Ps + e * 16) = u32x4{0u, 0u, 0u, 0u};

    if (w >= NWM + Cfg::NWG) {
        // idle waves: the barriers of the other waves, nothing else (2 before the loop, 2 per chunk)
        for (int i = 0; i < 2 * N + 2; ++i) __syncthreads();
    } else if (w >= NWM) {
        // ================================ gate waves ===========================================
        const int gw = w - NWM, gtid = gw * 64 + lane;
        // Uniform byte pointers to the stream's first token; per-thread 32-bit offsets on top.
        const unsigned char *qb = (const unsigned char *)p.q + kbase * 2;
        const unsigned char *kb = (const unsigned char *)p.k + kbase * 2;
        const long long hbase = ((long long)b * T + tok0) * p.H + h;   // per-head gates: [B,T,H]
        const unsigned char *gb = (const unsigned char *)p.g + (GH ? hbase : kbase) * GB;
        const unsigned gst = GH ? (unsigned)p.H : st;                          // gate elements between tokens
        const unsigned char *vb = (const unsigned char *)p.v + vbase * 2;
        const long long c0 = cstart(chunk_of(0));   // first token of the first chunk processed
        unsigned char *Gb = (unsigned char *)(p.G_cum + (((long long)b * T + tok0) * p.H + h) * (GH ? 1 : DK));
        const unsigned gcs = (unsigned)(p.H * (GH ? 1 : DK));

        // channel quad and token group (q, k, g); column quad and token group (v)
        const int cq = lane % CQ, gl = lane / CQ, tq = gw * GW + gl;
        const int vq = gtid % Cfg::VQ, tv = gtid / Cfg::VQ;
        const int qpos = Cfg::pos_of_channel(4 * cq);
        // Per-thread byte offsets of its first token inside a chunk; token u and the chunk are added
        // to the uniform base pointer, so one offset register serves every access of a tensor.
        const unsigned q_b0 = ((unsigned)(tq * TPT) * st + 4 * cq) * 2;
        const unsigned g_in_b0 = ((unsigned)(tq * TPT) * gst + (GH ? 0 : 4 * cq)) * GB;
        const unsigned v_b0 = ((unsigned)(tv * TPTV) * vt + 4 * vq) * 2;
        const unsigned g_b0 = ((unsigned)(tq * TPT) * gcs + (GH ? 0 : 4 * cq)) * 4;   // G_cum: contiguous [.., H, d_k]

        // Reloads of the streamed inputs: read once by this workgroup, so non-temporal - unless sibling
        // workgroups share them through the XCD's L2 (NS = 2), where the hint would cost HBM re-reads.
        auto stream_load = [](auto *ptr) __attribute__((always_inline)) {
            if constexpr (NS == 1) return __builtin_nontemporal_load(ptr);
            else return *ptr;
        };

        // Raw q, k, g, v of the chunk worked on next; each piece is reloaded with the following
        // chunk's data right after its last use (clamped to the last chunk).
        u32x2 rq[TPT], rk[TPT], rv[TPTV];
        typename GV::raw_t rg[TPT];
#pragma unroll
        for (int u = 0; u < TPT; ++u) {
            if constexpr (!NOQ) rq[u] = *reinterpret_cast<const u32x2 *>(qb + (c0 + u) * st * 2 + q_b0);
            rk[u] = *reinterpret_cast<const u32x2 *>(kb + (c0 + u) * st * 2 + q_b0);
            rg[u] = *reinterpret_cast<const typename GV::raw_t *>(gb + (c0 + u) * gst * GB + g_in_b0);
        }
#pragma unroll
        for (int u = 0; u < TPTV; ++u) rv[u] = *reinterpret_cast<const u32x2 *>(vb + (c0 + u) * vt * 2 + v_b0);

        // Log decay of the previous chunks for this thread's 4 channels, as an unevaluated sum.
        f32x4 seg_hi = {0.f, 0.f, 0.f, 0.f}, seg_lo = {0.f, 0.f, 0.f, 0.f};
        if constexpr (MODE == kLocalInit) {
            if constexpr (GH) {
                const float x = p.G_off[sbh];   // one log decay per head
                seg_hi = f32x4{x, x, x, x};
            } else {
                seg_hi = *reinterpret_cast<const f32x4 *>(p.G_off + sbh * DK + 4 * cq);
            }
        }
        f32x4 cs[TPT];                          // in-thread inclusive cumsum of g (part 1 -> part 2)
        f32x4 excl = {0.f, 0.f, 0.f, 0.f};      // sum over the wave's earlier token groups

        // part 1 of chunk m: per-thread cumulative sums and gate sums
        // (first: the short chunk; the literal `false` of the loop's calls folds the masks away)
        auto gate_a = [&](int m, bool first) __attribute__((always_inline)) {
            const int nn = chunk_of((m + 1 < N) ? m + 1 : N - 1);
            const unsigned char *gn = gb + cstart(nn) * gst * GB;   // uniform
            f32x4 run = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < TPT; ++u) {
                f32x4 gv = GV::get(rg[u]);
                if (first && dead(tq * TPT + u)) gv = f32x4{0.f, 0.f, 0.f, 0.f};
                rg[u] = stream_load(reinterpret_cast<const typename GV::raw_t *>(gn + (size_t)(u * gst) * GB + g_in_b0));
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
            if (gl == GW - 1) *reinterpret_cast<f32x4 *>(wtot + gw * DK + 4 * cq) = inc;
        };
        // V of chunk m -> tile buffer, token-major as it comes (the matrix waves read it transposed)
        auto vt_store = [&](int m, unsigned char *tile, bool first) __attribute__((always_inline)) {
            const int nn = chunk_of((m + 1 < N) ? m + 1 : N - 1);
            const unsigned char *vn = vb + cstart(nn) * vt * 2;   // uniform
#pragma unroll
            for (int u = 0; u < TPTV; ++u) {
                if (first && dead(tv * TPTV + u)) rv[u] = u32x2{0u, 0u};
                *reinterpret_cast<u32x2 *>(tile + Cfg::kOffV + pos_of(tv * TPTV + u) * VS + 8 * vq) = rv[u];
                rv[u] = stream_load(reinterpret_cast<const u32x2 *>(vn + (size_t)(u * vt) * 2 + v_b0));
            }
        };

        // Output rows.  The MFMA waves leave the finished O tile of chunk c (bf16, token-major) in the Qs
        // (and, when d_v > d_k, Ks) tile of the buffer chunk c used, which nobody reads after the scores
        // and the inter-chunk product.  The gate waves copy it to HBM just before they overwrite the same
        // bytes with the tiles of chunk c+2: a thread moves exactly the 8 bytes per row it is about to
        // reuse, and the 32 lanes that share a token write one contiguous row (the accumulator layout
        // itself would give 16-byte pieces, which cost about twice their share of the traffic).  The rows
        // (and the G_cum rows) are streamed out with non-temporal stores: nothing reads them back in
        // this kernel, and the local pass at 1024 streams runs 6 % faster for it.
        unsigned char *og = (unsigned char *)p.o + vbase * 2;
        auto flush_o = [&](int c, unsigned char *tile, int u0, int u1) __attribute__((always_inline)) {
            if constexpr (!NOQ) {
                unsigned char *oc = og + cstart(chunk_of(c)) * vt * 2;   // uniform
#pragma unroll
                for (int u = u0; u < u1; ++u) {
                    const int t = tq * TPT + u;
                    if (c == 0 && dead(t)) continue;
                    if (qpos < DV)
                        __builtin_nontemporal_store(*reinterpret_cast<const u32x2 *>(tile + Cfg::kOffQ + pos_of(t) * QS + qpos * 2),
                            reinterpret_cast<u32x2 *>(oc + ((size_t)t * vt + qpos) * 2));
                    if constexpr (DV > DK)
                        __builtin_nontemporal_store(*reinterpret_cast<const u32x2 *>(tile + Cfg::kOffO2 + pos_of(t) * QS + qpos * 2),
                            reinterpret_cast<u32x2 *>(oc + ((size_t)t * vt + DK + qpos) * 2));
                }
            }
        };

        // part 2 of chunk m: stitch waves (setup), scale q and k -> tile buffer and G_cum -> HBM in two
        // token halves, then gamma and the segment prefix (finish)
        f32x4 pre2, gbase, total;
        auto gate_b_setup = [&]() __attribute__((always_inline)) {
            f32x4 pre = excl;
            total = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < Cfg::NWG; ++u) {
                const f32x4 x = *reinterpret_cast<const f32x4 *>(wtot + u * DK + 4 * cq);
                const float sel = (u < gw) ? 1.f : 0.f;   // wave-uniform
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    pre[a] = __builtin_fmaf(sel, x[a], pre[a]);
                    total[a] += x[a];
                }
            }
            // c = pre + cs is the in-chunk cumulative log decay; exp(c - ref) = exp2(cs*log2e + (pre - ref)*log2e);
            // G_cum = (segment prefix + pre) + cs with the prefix folded once per channel.
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                pre2[a] = (WIDE ? __builtin_fmaf(-0.5f, total[a], pre[a]) : pre[a]) * kLog2e;
                gbase[a] = seg_hi[a] + (pre[a] + seg_lo[a]);
            }
        };
        auto gate_b_half = [&](int m, int half, unsigned char *tile, bool first) __attribute__((always_inline)) {
            constexpr int HT = TPT / 2;
            unsigned char *Qs = tile + Cfg::kOffQ, *Ks = tile + Cfg::kOffK;
            const int nn = chunk_of((m + 1 < N) ? m + 1 : N - 1);
            const unsigned char *qn = qb + cstart(nn) * st * 2;   // uniform
            const unsigned char *kn = kb + cstart(nn) * st * 2;
            unsigned char *Gm = Gb + cstart(m) * gcs * 4;
            if (m >= 2) flush_o(m - 2, tile, half * HT, half * HT + HT);   // before these rows are rewritten
#pragma unroll
            for (int uu = 0; uu < HT; ++uu) {
                const int u = half * HT + uu;
                const int t = tq * TPT + u;
                f32x4 yv, ilam;
                if constexpr (GH) {   // one decay per token: one exponential serves the four channels
                    const float y = __builtin_fmaf(cs[u][0], kLog2e, pre2[0]);
                    float il = __builtin_amdgcn_exp2f(-SGN * y);
                    if constexpr (REV) il *= p.kscale;
                    yv = f32x4{y, y, y, y};
                    ilam = f32x4{il, il, il, il};
                } else {
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        yv[a] = __builtin_fmaf(cs[u][a], kLog2e, pre2[a]);
                        ilam[a] = __builtin_amdgcn_exp2f(-SGN * yv[a]);
                        if constexpr (REV) ilam[a] *= p.kscale;   // the query scale rides on Q .* Lambda
                    }
                }
                u32x2 kw = rk[u];
                if (first && dead(t)) kw = u32x2{0u, 0u};
                rk[u] = stream_load(reinterpret_cast<const u32x2 *>(kn + (size_t)(u * st) * 2 + q_b0));
                const u32x2 kq = {pack_bf16(bf16_lo(kw[0]) * ilam[0], bf16_hi(kw[0]) * ilam[1]),
                                  pack_bf16(bf16_lo(kw[1]) * ilam[2], bf16_hi(kw[1]) * ilam[3])};
                if constexpr (!NOQ) {   // scores and outputs need Q .* Lambda
                    f32x4 lam;
                    if constexpr (GH) {
                        const float l = __builtin_amdgcn_exp2f(SGN * yv[0]);
                        lam = f32x4{l, l, l, l};
                    } else {
#pragma unroll
                        for (int a = 0; a < 4; ++a) lam[a] = __builtin_amdgcn_exp2f(SGN * yv[a]);
                    }
                    const u32x2 qw = rq[u];
                    rq[u] = stream_load(reinterpret_cast<const u32x2 *>(qn + (size_t)(u * st) * 2 + q_b0));
                    *reinterpret_cast<u32x2 *>(Qs + pos_of(t) * QS + qpos * 2) =
                        u32x2{pack_bf16(bf16_lo(qw[0]) * lam[0], bf16_hi(qw[0]) * lam[1]),
                              pack_bf16(bf16_lo(qw[1]) * lam[2], bf16_hi(qw[1]) * lam[3])};
                }
                *reinterpret_cast<u32x2 *>(Ks + pos_of(t) * QS + qpos * 2) = kq;
                if constexpr (EMIT_G) if (!(first && dead(t))) {
                    f32x4 gout;
#pragma unroll
                    for (int a = 0; a < 4; ++a) gout[a] = gbase[a] + cs[u][a];
                    if constexpr (GH) {
                        if (u % NS == slice && cq == 0)
                            *reinterpret_cast<float *>(Gm + (size_t)(u * gcs) * 4 + g_b0) = gout[0];
                    } else if (u % NS == slice) {   // sibling slices share the G_cum rows between them
                        __builtin_nontemporal_store(gout, reinterpret_cast<f32x4 *>(Gm + (size_t)(u * gcs) * 4 + g_b0));
                    }
                }
            }
        };
        auto gate_b_finish = [&](int m, float *gam_m) __attribute__((always_inline)) {
            if (tq == 0) {
                f32x4 gm;
#pragma unroll
                for (int a = 0; a < 4; ++a) gm[a] = __builtin_amdgcn_exp2f(total[a] * (WIDE ? 0.5f * kLog2e : kLog2e));
                *reinterpret_cast<f32x4 *>(gam_m + 4 * cq) = gm;
            }
            // decay outputs: the local pass and the two state passes (the backward one emits G_tot when
            // asked, so that the reverse scan does not need the forward state pass)
            if constexpr (MODE == kOutput || MODE == kDV) return;
            if constexpr (MODE == kDState) {
                if (!p.G_tot) return;
            }
            if constexpr (MODE == kLocalCD) {   // log gamma~ before this chunk
                if (tq == 0 && slice == 0) {
                    f32x4 gp;
#pragma unroll
                    for (int a = 0; a < 4; ++a) gp[a] = seg_hi[a] + seg_lo[a];
                    *reinterpret_cast<f32x4 *>(p.G_chunk + ((((long long)b * p.P + seg) * N + m) * p.H + h) * DK + 4 * cq) = gp;
                }
            }
#pragma unroll
            for (int a = 0; a < 4; ++a) {   // (hi, lo) += total, error-free transformation
                const float x = total[a] + seg_lo[a];
                const float s = seg_hi[a] + x;
                const float bb = s - seg_hi[a];
                seg_lo[a] = (seg_hi[a] - (s - bb)) + (x - bb);
                seg_hi[a] = s;
            }
            if constexpr (MODE == kLocalInit) return;
            if (m == N - 1 && tq == 0 && slice == 0) {   // segment total: log of gamma~_[N]
                f32x4 gt;
#pragma unroll
                for (int a = 0; a < 4; ++a) gt[a] = seg_hi[a] + seg_lo[a];
                if constexpr (GH) {
                    if (cq == 0) p.G_tot[sbh] = gt[0];
                } else {
                    *reinterpret_cast<f32x4 *>(p.G_tot + sbh * DK + 4 * cq) = gt;
                }
            }
        };

        // Schedule (the MFMA waves run part 1 of chunk n in phase X(n) and part 2 in phase Y(n)):
        //   X(n): V^T(n+1) -> LDS, setup and first token half of part 2 of chunk n+1
        //   Y(n): second token half and finish of chunk n+1, then part 1 of chunk n+2
        // so that both phases carry a similar amount of gate work.  The loop bodies are free of
        // branches (a conditional around the passes would force the reloaded registers through
        // merge copies, and with them a wait for every load in flight); the tail is peeled.
        gate_a(0, true);
        vt_store(0, lds, true);
        __syncthreads();
        gate_b_setup();
        gate_b_half(0, 0, lds, true);
        gate_b_half(0, 1, lds, true);
        gate_b_finish(0, gam);
        if (N > 1) gate_a(1, false);
        __syncthreads();
        int n = 0;
        for (; n + 2 < N; ++n) {
            unsigned char *nxt = lds + ((n + 1) & 1) * Cfg::kTileBytes;
            vt_store(n + 1, nxt, false);
            gate_b_setup();
            gate_b_half(n + 1, 0, nxt, false);
            __syncthreads();   // Ps of chunk n visible to the MFMA waves
            gate_b_half(n + 1, 1, nxt, false);
            gate_b_finish(n + 1, gam + ((n + 1) & 1) * DK);
            gate_a(n + 2, false);
            __syncthreads();   // tiles of chunk n+1 and gate sums of chunk n+2 complete
        }
        if (N > 1) {   // n = N-2: produce the last chunk
            unsigned char *nxt = lds + ((n + 1) & 1) * Cfg::kTileBytes;
            vt_store(n + 1, nxt, false);
            gate_b_setup();
            gate_b_half(n + 1, 0, nxt, false);
            __syncthreads();
            gate_b_half(n + 1, 1, nxt, false);
            gate_b_finish(n + 1, gam + ((n + 1) & 1) * DK);
            __syncthreads();
        }
        // n = N-1: nothing left to produce; the output rows of the last two chunks are still in LDS
        if (N > 1) flush_o(N - 2, lds + ((N - 2) & 1) * Cfg::kTileBytes, 0, TPT);
        __syncthreads();
        __syncthreads();
        flush_o(N - 1, lds + ((N - 1) & 1) * Cfg::kTileBytes, 0, TPT);
    } else {
        // ================================ MFMA waves ===========================================
        const int lt = lane & 31, kg = lane >> 5;       // 32x32x16 lane coordinates
        const int l16 = lane & 15, kg16 = lane >> 4;    // 16x16x32 lane coordinates (score tiles)
        // this lane's 8-byte slots in the staged O tile: row lt (+32 mt), columns 32 w + 8 qd + 4 kg ..+3;
        // columns beyond d_k continue in the Ks tile
        const int o_col = w * 32 + 4 * kg;
        const unsigned o_s0 = (o_col < DK ? Cfg::kOffQ : Cfg::kOffO2 - DK * 2) + lt * QS + o_col * 2;
        // Transposing reads: this lane's address inside its group of 16 (row k = (lane % 16) / 4 of the
        // group's 4 rows, element quad r = lane % 4), for the tokens 8 kg .. 8 kg + 7 of a 16-token step.
        const int tr_k = (lane & 15) >> 2, tr_r = lane & 3, tr_h = lt >> 4;
        // V: columns w*32 + 16 tr_h + 4 r .. of the token-major tile
        const unsigned v_tr0 = Cfg::kOffV + (8 * kg + tr_k) * VS + (w * 32 + 16 * tr_h + 4 * tr_r) * 2;
        // K / Lambda: channel 32 it + 16 tr_h + 4 r sits at position 8 (r % 2) + 4 (r / 2) of its block of
        // 16 (the Ks rows keep the stride that suits the 16-byte reads of the score products, so these reads
        // see some two-way bank conflicts; an order of the k-slots that avoids them needs a second set of
        // V fragments and measured 2 % slower)
        const unsigned k_tr0 = Cfg::kOffK + (8 * kg + tr_k) * QS + (16 * tr_h + 8 * (tr_r & 1) + 4 * (tr_r >> 1)) * 2;

        f32x16 Sacc[Cfg::NIT], Oacc[2];
        float *Sl = p.S_loc + sbh * DK * (DV * NS) + slice * DV + w * 32 + lt;   // this lane's state column
        const float *Si = p.S_init + sbh * DK * (DV * NS) + slice * DV + w * 32 + lt;
#pragma unroll
        for (int it = 0; it < Cfg::NIT; ++it)
#pragma unroll
            for (int rr = 0; rr < 16; ++rr)
                Sacc[it][rr] = FROM_INIT ? Si[(size_t)(it * 32 + M::row(rr, kg)) * (DV * NS)] : 0.f;

        // rows of the state scaled by the chunk decay
        auto decay_state = [&](const float *gam_n) __attribute__((always_inline)) {
#pragma unroll
            for (int it = 0; it < Cfg::NIT; ++it)
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    const f32x4 gm = *reinterpret_cast<const f32x4 *>(gam_n + it * 32 + 8 * qd + 4 * kg);
#pragma unroll
                    for (int mm = 0; mm < 4; ++mm) Sacc[it][4 * qd + mm] *= gm[mm];
                }
        };

        // part 1: scores -> Ps, inter-chunk product -> Oacc
        auto mfma_a = [&](const unsigned char *tile, const float *gam_n) __attribute__((always_inline)) {
            const unsigned char *Qs = tile + Cfg::kOffQ, *Ks = tile + Cfg::kOffK;
            if constexpr (MODE == kDV || (WIDE && !REV)) decay_state(gam_n);
            // P^T tiles (ts <= tt), 16x16x32; all operand reads of a tile are issued up front
#pragma unroll
            for (int i = 0; i < (10 + NWM - 1) / NWM; ++i) {
                const int idx = w + NWM * i;   // wave-uniform
                if (idx < 10) {
                    const int tt = (idx >= 6) ? 3 : (idx >= 3) ? 2 : (idx >= 1) ? 1 : 0;
                    const int ts = idx - tt * (tt + 1) / 2;
                    const unsigned char *ka = Ks + (16 * ts + l16) * QS + 16 * kg16;
                    const unsigned char *qf = Qs + (16 * tt + l16) * QS + 16 * kg16;
                    bf16x8 fa[DK / 32], fb[DK / 32];
#pragma unroll
                    for (int ks = 0; ks < DK / 32; ++ks) {
                        fa[ks] = lds_frag(ka, 64 * ks);
                        fb[ks] = lds_frag(qf, 64 * ks);
                    }
                    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < DK / 32; ++ks) acc = Mma<16>::run(fa[ks], fb[ks], acc);
                    if (ts == tt) {
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr)
                            if (4 * kg16 + rr > l16) acc[rr] = 0.f;
                    }
                    *reinterpret_cast<u32x2 *>(Ps + (16 * tt + l16) * TS + (16 * ts + 4 * kg16) * 2) =
                        u32x2{pack_bf16(acc[0], acc[1]), pack_bf16(acc[2], acc[3])};
                }
            }
            // O^T = S^T Qs^T
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int rr = 0; rr < 16; ++rr) Oacc[mt][rr] = 0.f;
#pragma unroll
            for (int ks = 0; ks < DK / 16; ++ks) {
                const bf16x8 sf = pack8(Sacc[ks / 2], 8 * (ks % 2));
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
                    Oacc[mt] = M::run(sf, lds_frag(Qs, (mt * 32 + lt) * QS + (ks * 16 + 8 * kg) * 2), Oacc[mt]);
            }
        };

        // part 2 of chunk n: intra-chunk output, O store, state update
        auto mfma_b = [&](int n, const unsigned char *tile, const float *gam_n) __attribute__((always_inline)) {
            unsigned char *os = const_cast<unsigned char *>(tile) + o_s0;
            if constexpr (MODE == kDState || (WIDE && MODE == kStates)) decay_state(gam_n);
            bf16x8 vf[4];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) vf[ks] = lds_frag_tr(tile + v_tr0 + ks * 16 * VS, 4 * VS);
            // O^T += Vt Ps^T over the causal k-range (tokens s < 32 (mt + 1))
#pragma unroll
            for (int mt = 0; mt < (NOQ ? 0 : 2); ++mt) {
#pragma unroll
                for (int ks = 0; ks < 2 * (mt + 1); ++ks)
                    Oacc[mt] = M::run(vf[ks], lds_frag(Ps, (mt * 32 + lt) * TS + (ks * 16 + 8 * kg) * 2), Oacc[mt]);
#pragma unroll
                for (int qd = 0; qd < 4; ++qd)
                    *reinterpret_cast<u32x2 *>(os + mt * 32 * QS + 8 * qd * 2) =
                        u32x2{pack_bf16(Oacc[mt][4 * qd] * p.scale, Oacc[mt][4 * qd + 1] * p.scale),
                              pack_bf16(Oacc[mt][4 * qd + 2] * p.scale, Oacc[mt][4 * qd + 3] * p.scale)};
            }
            // S <- gamma .* (S + Kt Vt^T)
#pragma unroll
            for (int it = 0; it < Cfg::NIT; ++it) {
                f32x16 acc = Sacc[it];
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    acc = M::run(lds_frag_tr(tile + k_tr0 + ks * 16 * QS + it * 64, 4 * QS), vf[ks], acc);
                if constexpr (!REV || WIDE) {
#pragma unroll
                    for (int qd = 0; qd < 4; ++qd) {
                        const f32x4 gm = *reinterpret_cast<const f32x4 *>(gam_n + it * 32 + 8 * qd + 4 * kg);
#pragma unroll
                        for (int mm = 0; mm < 4; ++mm) acc[4 * qd + mm] *= gm[mm];
                    }
                }
                Sacc[it] = acc;
            }
        };

        __syncthreads();
        __syncthreads();
        for (int n = 0; n < N; ++n) {
            const unsigned char *cur = lds + (n & 1) * Cfg::kTileBytes;
            if constexpr (!NOQ) mfma_a(cur, gam + (n & 1) * DK);
            __syncthreads();
            mfma_b(n, cur, gam + (n & 1) * DK);
            __syncthreads();
        }

        if constexpr (!FROM_INIT) {
#pragma unroll
            for (int it = 0; it < Cfg::NIT; ++it)
#pragma unroll
                for (int rr = 0; rr < 16; ++rr)
                    Sl[(size_t)(it * 32 + M::row(rr, kg)) * (DV * NS)] = Sacc[it][rr];
        }
    }
}

template <int DK, int DV, int NS, int GM, int MODE, bool WIDE>
static hipError_t launch_b16(const ChunkParams &p, hipStream_t s) {
    typedef B16Cfg<DK, DV, gate_waves(DK, GM, MODE), idle_waves(DK, DV, GM, MODE)> Cfg;
    auto kern = gla_chunk_bf16_kernel<DK, DV, NS, GM, MODE, WIDE>;
    static LdsLimit limit;   // one per instantiation
    hipError_t e = limit.raise((const void *)kern, Cfg::kBytes);
    if (e != hipSuccess) return e;
    const int streams = p.B * p.P * p.H;
    const int grid = ((streams + 7) / 8) * 8 * NS;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(Cfg::NT), Cfg::kBytes, s, p);
    return hipGetLastError();
}

template <int GM, int MODE, bool WIDE>
static hipError_t dispatch_dims(const ChunkParams &p, int d_k, int d_v, hipStream_t s) {
    // With at most half as many streams as compute units, two sibling workgroups split d_v = 128 so that
    // more compute units stream memory; the gate pass is then computed twice.  Between 128 and 256 streams
    // one workgroup per stream on part of the chip is faster than two rounds of siblings (192 streams:
    // 1.21 ms against 1.58 ms for the local pass of 16384 tokens).
    const bool split = d_v == 128 && p.B * p.P * p.H * 2 <= 256;
    if (d_k == 64 && d_v == 64) return launch_b16<64, 64, 1, GM, MODE, WIDE>(p, s);
    if (d_k == 128 && d_v == 64) return launch_b16<128, 64, 1, GM, MODE, WIDE>(p, s);
    if (d_k == 64 && d_v == 128)
        return split ? launch_b16<64, 64, 2, GM, MODE, WIDE>(p, s) : launch_b16<64, 128, 1, GM, MODE, WIDE>(p, s);
    if (d_k == 128 && d_v == 128)
        return split ? launch_b16<128, 64, 2, GM, MODE, WIDE>(p, s) : launch_b16<128, 128, 1, GM, MODE, WIDE>(p, s);
    return hipErrorInvalidValue;
}

template <int GM, int MODE>
static hipError_t dispatch_b16(const ChunkParams &p, int d_k, int d_v, bool wide, hipStream_t s) {
    return wide ? dispatch_dims<GM, MODE, true>(p, d_k, d_v, s) : dispatch_dims<GM, MODE, false>(p, d_k, d_v, s);
}

template <int MODE>
static hipError_t dispatch_gate(const ChunkParams &p, int d_k, int d_v, int gate_mode, hipStream_t s) {
    const bool wide = (gate_mode & kGateWide) != 0;
    const int layout = gate_mode & ~kGateWide;
    if (layout == kGateBF16) return dispatch_b16<kGateBF16, MODE>(p, d_k, d_v, wide, s);
    if (layout == kGateHead) {
        if constexpr (MODE == kLocalCD) return hipErrorInvalidValue;   // per-channel gates only
        else return dispatch_b16<kGateHead, MODE>(p, d_k, d_v, wide, s);
    }
    return dispatch_b16<kGateF32, MODE>(p, d_k, d_v, wide, s);
}

hipError_t launch_chunk_bf16(const ChunkParams &p, int d_k, int d_v, int gate_mode, int mode, hipStream_t s) {
    if (mode == kStates) return dispatch_gate<kStates>(p, d_k, d_v, gate_mode, s);
    if (mode == kOutput) return dispatch_gate<kOutput>(p, d_k, d_v, gate_mode, s);
    if (mode == kDState) return dispatch_gate<kDState>(p, d_k, d_v, gate_mode, s);
    if (mode == kDV) return dispatch_gate<kDV>(p, d_k, d_v, gate_mode, s);
    if (mode == kLocalInit) return dispatch_gate<kLocalInit>(p, d_k, d_v, gate_mode, s);
    if (mode == kLocalCD) return dispatch_gate<kLocalCD>(p, d_k, d_v, gate_mode, s);
    return dispatch_gate<kLocal>(p, d_k, d_v, gate_mode, s);
}

}  // namespace zeco
