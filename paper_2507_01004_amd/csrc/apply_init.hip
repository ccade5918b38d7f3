// Initial-state correction  o_t += (scale * q_t .* exp(G_cum[t])) S_init[p]  (Eq. (global-correction)
// carried to the output; the term Alg. 1's output pass adds to S_[n-1]).
//
// A skinny GEMM (tokens x d_k)(d_k x d_v) that must stay HBM-bound: q, G_cum and o are streamed
// once, S_init[p] is loaded once per workgroup and kept in registers as an MFMA operand, and the
// contraction runs on the matrix cores (at 25.6 flop/byte it would be ALU-bound on plain FMAs).
// A workgroup takes `tokens_per_wg` consecutive tokens of one (batch, segment, head).
//
// Vanished decay.  The log decay is <= 0, so G_cum never increases along a segment.  Once every
// channel of a token has G_cum < kVanish, exp(G_cum) is exactly 0 in fp32 for that token and all
// later ones of the segment (2^-151 rounds to zero even with denormals), the product above is an
// exact zero and o keeps its value: the kernel stops there instead of streaming q, G_cum and o
// through to add nothing.  With the decays of a trained GLA layer (e-folding length of tens to
// hundreds of tokens) that is all but the first few thousand tokens of a long segment.  `dense`
// switches the test off (measurement of the full-traffic kernel, equality tests).
//
// Segment lengths that are no multiple of 64 follow the chunk kernels' convention: the first 64-token
// block of a segment is the short one, holding the tokens [0, 64 - pad); it is loaded and computed as the
// window [0, 64) (inside the segment), only its real rows are stored, and block c >= 1 starts at token
// 64 c - pad.  The last workgroup of a segment may have fewer blocks than the others.
#include "zeco_device.h"
#include "zeco_internal.h"

namespace zeco {

constexpr float kVanish = -105.f;   // exp2(-105 log2(e)) = 2^-151.5 rounds to 0 in fp32

// q, G_cum and o are read with ordinary loads and o is written back with non-temporal stores.  Measured
// (dense call, c3 / c4): that combination 5.3 TB/s, ordinary loads and stores 5.1-5.2, non-temporal loads with
// ordinary stores 4.3-4.4, both non-temporal 4.7.  A plain streaming kernel with this kernel's traffic (three
// token-major streams read, one of them rewritten in place) reaches 5.0-5.5 TB/s whatever the length of the
// contiguous pieces a workgroup takes (256 bytes of a token's row up to the whole 4 KiB row): the in-place
// rewrite, not the row length, sets the rate.
// q, G_cum (or g) and o are streamed once.  Non-temporal loads together with non-temporal stores of o give the
// dense call 5.7 TB/s against 5.3 with ordinary loads (c3, c4) - provided nothing is loaded twice: with the
// prefetch of the block after a workgroup's last one clamped to that last block, the second fetch of its rows hit
// the cache with ordinary loads and went to HBM again with non-temporal ones (4.3-4.7 TB/s), so the prefetch
// is skipped there instead.  The hint costs latency, though: where the call stops at the vanished decay and
// few workgroups find work (c3: about 340 of them, fewer than the chip has slots) it is 20 % slower, so the
// launcher asks for it only in dense calls and in launches with more streams than workgroup slots.
// (Other combinations, dense call: ordinary loads and stores 5.1-5.2 TB/s, non-temporal loads with ordinary
// stores 4.3-5.2.  The order of the workgroups - token blocks of a stream together, heads of a token block
// together, a linear sweep through memory - moves the figure by 2 % at most.)
template <bool NT, typename T> __device__ __forceinline__ T apply_ld(const T *p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <typename T> __device__ __forceinline__ void apply_st(T v, T *p) { __builtin_nontemporal_store(v, p); }

// ------------------------------------------------------------------------------------------ bf16
template <int DK, int DV> struct ApplyCfg {
    static constexpr int TILE = DV / 4;
    static constexpr int NKG = 64 / TILE;
    static constexpr int KS = 8 * NKG;
    static constexpr int ACC = TILE * TILE / 64;
    static constexpr int NMT = 64 / TILE;
    static constexpr int NKS = DK / KS;
    static constexpr int QS = DK * 2 + 16;          // LDS row stride (bytes)
    static constexpr int ITEMS = 64 * DK / 8 / 256; // 8-channel groups per thread per 64 tokens
    static constexpr int OITEMS = 64 * DV / 8 / 256; // 8-column pieces of o per thread per 64 tokens
    static constexpr int CS = DV + 4;               // row stride (floats) of the fp32 staging tile
    static constexpr int kBytes = 64 * QS + 64 * CS * 4;
};

// Segments a launch corrects: p0, p0 + seg_step, .. below P.
__host__ __device__ __forceinline__ int apply_segments(const ApplyParams &p) { return (p.P - p.p0 + p.seg_step - 1) / p.seg_step; }

// Workgroup id -> (stream, token block), a stream being a (segment, batch, head); returns the stream's
// index over (segment - p0, batch, head) and sets tb.
// Order: (group of 128 streams, token block, stream in the group).  Inside a group the early token
// blocks of every stream come first - the ones with work left once the decay has vanished - and
// spread evenly over the XCDs, which take workgroup ids round-robin; a stream stays on one XCD (128 is
// a multiple of 8), and a group's S_init states (8 MiB at d = 128) stay in the L2s while its token
// blocks are worked through.
__device__ __forceinline__ int apply_stream_of_workgroup(const ApplyParams &p, int &tb) {
    constexpr int kGroup = 128;
    const int blocks_per_seg = p.wgs_per_seg, streams = apply_segments(p) * p.B * p.H;
    const int grp = blockIdx.x / (kGroup * blocks_per_seg), r = blockIdx.x % (kGroup * blocks_per_seg);
    const int gsz = min(kGroup, streams - grp * kGroup);
    const int j = r % gsz;
    tb = r / gsz;
    // position j of a row -> stream: rotated inside each aligned block of 8 by the block's index, so that
    // the streams of one head (which share a decay speed, hence an amount of work) do not all fall on the
    // same XCD when H is a multiple of 8
    return grp * kGroup + (((j | 7) < gsz) ? (j & ~7) + ((j - (j >> 3)) & 7) : j);
}

// First token (inside its segment) of 64-token block c, and the number of rows of it to store.
// (pad = 64 ceil(L / 64) - L of the segment: block 0 is the short one)
__device__ __forceinline__ long long apply_block_start(int pad, int c) { return c ? (long long)c * 64 - pad : 0ll; }
__device__ __forceinline__ int apply_block_rows(int pad, int c) { return c ? 64 : 64 - pad; }

// Workgroup-wide AND of `mine` through the four flags in LDS; ends with a barrier.  Calls must be
// separated by at least one other barrier.
__device__ __forceinline__ bool apply_all(bool mine, int *flags) {
    const bool wave_all = __ballot(mine) == ~0ull;
    if ((threadIdx.x & 63) == 0) flags[threadIdx.x >> 6] = wave_all;
    __syncthreads();
    return (flags[0] & flags[1] & flags[2] & flags[3]) != 0;
}

// S_init[p] columns [w*TILE, (w+1)*TILE) as the A operand of O^T = S^T Qh^T: lane holds column lt
// and, for k-step ks, channels ks*KS + 8*kg .. +7.
template <int DK, int DV>
__device__ __forceinline__ void apply_load_state(const float *S, bf16x8 (&sf)[ApplyCfg<DK, DV>::NKS]) {
    typedef ApplyCfg<DK, DV> Cfg;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int lt = lane % Cfg::TILE, kg = lane / Cfg::TILE;
#pragma unroll
    for (int ks = 0; ks < Cfg::NKS; ++ks) {
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = S[(size_t)(ks * Cfg::KS + 8 * kg + e) * DV + w * Cfg::TILE + lt];
        u32x4 wv = {pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3]), pack_bf16(x[4], x[5]),
                    pack_bf16(x[6], x[7])};
        sf[ks] = __builtin_bit_cast(bf16x8, wv);
    }
}

// o is read-modified-written in 16-byte pieces (8 columns of one token per item).
template <int DV, bool NT>
__device__ __forceinline__ void apply_load_o(const uint16_t *o_blk, long long vt, u32x4 (&ro)[64 * DV / 8 / 256]) {
#pragma unroll
    for (int m = 0; m < 64 * DV / 8 / 256; ++m) {
        const int item = threadIdx.x + 256 * m, t = item / (DV / 8), cg = item % (DV / 8);
        ro[m] = apply_ld<NT>(reinterpret_cast<const u32x4 *>(o_blk + t * vt + 8 * cg));
    }
}

// One 64-token block, after a barrier has made the tile Qh (scale * q .* exp(G), bf16, token-major)
// complete: the product on the matrix cores, through an fp32 staging tile in LDS (so that o is
// written in coalesced 16-byte pieces), added to the old rows `ocur`.  Contains one barrier; the
// caller's next barrier separates the reads of the staging tile from the next block's products.
template <int DK, int DV>
__device__ __forceinline__ void apply_block(const bf16x8 (&sf)[ApplyCfg<DK, DV>::NKS], const unsigned char *Qh,
                                            float *Cs, uint16_t *o_blk, long long vt,
                                            const u32x4 (&ocur)[ApplyCfg<DK, DV>::OITEMS], int rows) {
    typedef ApplyCfg<DK, DV> Cfg;
    typedef Mma<Cfg::TILE> M;
    constexpr int TILE = Cfg::TILE, KS = Cfg::KS, QS = Cfg::QS;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int lt = lane % TILE, kg = lane / TILE;
#pragma unroll
    for (int mt = 0; mt < Cfg::NMT; ++mt) {
        typename M::acc_t acc;
#pragma unroll
        for (int r = 0; r < Cfg::ACC; ++r) acc[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < Cfg::NKS; ++ks)
            acc = M::run(sf[ks], lds_frag(Qh, (mt * TILE + lt) * QS + (ks * KS + 8 * kg) * 2), acc);
#pragma unroll
        for (int qd = 0; qd < Cfg::ACC / 4; ++qd)   // lane holds 4 consecutive columns of token lt
            *reinterpret_cast<f32x4 *>(Cs + (mt * TILE + lt) * Cfg::CS + w * TILE + M::row(4 * qd, kg)) =
                f32x4{acc[4 * qd], acc[4 * qd + 1], acc[4 * qd + 2], acc[4 * qd + 3]};
    }
    __syncthreads();   // staging tile complete; Qh free for the next block
#pragma unroll
    for (int m = 0; m < Cfg::OITEMS; ++m) {
        const int item = tid + 256 * m, t = item / (DV / 8), cg = item % (DV / 8);
        const f32x4 c0 = *reinterpret_cast<const f32x4 *>(Cs + t * Cfg::CS + 8 * cg);
        const f32x4 c1 = *reinterpret_cast<const f32x4 *>(Cs + t * Cfg::CS + 8 * cg + 4);
        const u32x4 old = ocur[m];
        if (t < rows) apply_st(
            u32x4{pack_bf16(bf16_lo(old[0]) + c0[0], bf16_hi(old[0]) + c0[1]),
                  pack_bf16(bf16_lo(old[1]) + c0[2], bf16_hi(old[1]) + c0[3]),
                  pack_bf16(bf16_lo(old[2]) + c1[0], bf16_hi(old[2]) + c1[1]),
                  pack_bf16(bf16_lo(old[3]) + c1[2], bf16_hi(old[3]) + c1[3])},
            reinterpret_cast<u32x4 *>(o_blk + t * vt + 8 * cg));
    }
}

// GH: the cumulative log decay is one value per (token, head), G_cum [B,T,H].
// NT: non-temporal loads of the streamed rows (see above).
template <int DK, int DV, bool GH, bool NT>
__global__ __launch_bounds__(256) void apply_init_bf16_kernel(ApplyParams p) {
    typedef ApplyCfg<DK, DV> Cfg;
    constexpr int QS = Cfg::QS;
    __shared__ __align__(16) unsigned char lds[Cfg::kBytes];
    __shared__ int gone[4];
    unsigned char *Qh = lds;                                      // scale * q .* exp(G_cum), bf16
    float *Cs = reinterpret_cast<float *>(lds + 64 * QS);         // correction tile, fp32

    const int tid = threadIdx.x;
    int tb;
    int id = apply_stream_of_workgroup(p, tb);
    const int h = id % p.H;
    id /= p.H;
    const int b = id % p.B, seg = p.p0 + p.seg_step * (id / p.B);
    long long tok0 = (long long)seg * p.L;                       // the segment's first token
    long long T = (long long)p.P * p.L;                          // tokens per batch entry
    int n_chunks = p.n_chunks, pad = p.pad;
    const int c0 = tb * (p.tokens_per_wg / 64);                  // this workgroup's first block
    if (p.seg_start) {
        // segments of unequal length: bounds from the table; the grid is sized for the longest segment allowed,
        // so workgroups past this segment's end leave, and so do those of a segment that cannot be taken
        tok0 = p.seg_start[seg];
        T = p.T;
        const long long len = p.seg_start[seg + 1] - tok0;
        if (tok0 < 0 || len < 64 || len > p.L || tok0 > T - len) return;   // (in this order: no sum can overflow)
        n_chunks = (int)((len + 63) >> 6);
        pad = 64 * n_chunks - (int)len;
        if (c0 >= n_chunks) return;
    }
    const int nblk = min(p.tokens_per_wg / 64, n_chunks - c0);
    const uint16_t *qp = (const uint16_t *)p.q + b * p.sb + tok0 * p.st + h * p.sh;
    uint16_t *op = (uint16_t *)p.o + b * p.vb + tok0 * p.vt + h * p.vh;
    const float *Gc = p.G_cum + (((long long)b * T + tok0) * p.H + h) * (GH ? 1 : DK);
    const long long gcs = (long long)p.H * (GH ? 1 : DK);
    const float *S = p.S_init + (((size_t)seg * p.B + b) * p.H + h) * DK * DV;

    // Nothing to add from this workgroup's first token on?
    const bool may_stop = !p.dense;
    if (may_stop && apply_all(Gc[apply_block_start(pad, c0) * gcs + (GH ? 0 : tid % DK)] < kVanish, gone)) return;

    bf16x8 sf[Cfg::NKS];
    apply_load_state<DK, DV>(S, sf);

    struct Raw {
        u32x4 q[Cfg::ITEMS];
        f32x4 g0[Cfg::ITEMS], g1[Cfg::ITEMS];
    };
    auto load_raw = [&](int blk, Raw &r) {
#pragma unroll
        for (int m = 0; m < Cfg::ITEMS; ++m) {
            const int item = tid + 256 * m, t = item / (DK / 8), cg = item % (DK / 8);
            const long long tt = apply_block_start(pad, c0 + blk) + t;
            r.q[m] = apply_ld<NT>(reinterpret_cast<const u32x4 *>(qp + tt * p.st + 8 * cg));
            if constexpr (GH) {
                const float x = Gc[tt * gcs];
                r.g0[m] = r.g1[m] = f32x4{x, x, x, x};
            } else {
                r.g0[m] = apply_ld<NT>(reinterpret_cast<const f32x4 *>(Gc + tt * gcs + 8 * cg));
                r.g1[m] = apply_ld<NT>(reinterpret_cast<const f32x4 *>(Gc + tt * gcs + 8 * cg + 4));
            }
        }
    };

    Raw nxt;
    u32x4 onx[Cfg::OITEMS];
    load_raw(0, nxt);
    apply_load_o<DV, NT>(op + apply_block_start(pad, c0) * p.vt, p.vt, onx);
    for (int blk = 0; blk < nblk; ++blk) {
        const Raw cur = nxt;
        u32x4 ocur[Cfg::OITEMS];
#pragma unroll
        for (int m = 0; m < Cfg::OITEMS; ++m) ocur[m] = onx[m];
        if (may_stop && blk > 0) {   // first token of this block: item 0 of the threads tid < DK/8
            bool mine = true;
            if (tid < DK / 8) {
#pragma unroll
                for (int e = 0; e < 4; ++e) mine = mine && cur.g0[0][e] < kVanish && cur.g1[0][e] < kVanish;
            }
            if (apply_all(mine, gone)) break;
        }
#pragma unroll
        for (int m = 0; m < Cfg::ITEMS; ++m) {
            const int item = tid + 256 * m, t = item / (DK / 8), cg = item % (DK / 8);
            u32x4 out;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float ga = e < 2 ? cur.g0[m][2 * e] : cur.g1[m][2 * e - 4];
                const float gb = e < 2 ? cur.g0[m][2 * e + 1] : cur.g1[m][2 * e - 3];
                out[e] = pack_bf16(bf16_lo(cur.q[m][e]) * fast_exp(ga) * p.scale,
                                   bf16_hi(cur.q[m][e]) * fast_exp(gb) * p.scale);
            }
            *reinterpret_cast<u32x4 *>(Qh + t * QS + 16 * cg) = out;
        }
        if (blk + 1 < nblk) {   // (uniform) the next block's rows; nothing is fetched twice
            load_raw(blk + 1, nxt);
            apply_load_o<DV, NT>(op + apply_block_start(pad, c0 + blk + 1) * p.vt, p.vt, onx);
        }
        __syncthreads();   // Qh complete; every thread is done with the staging tile of the last block
        apply_block<DK, DV>(sf, Qh, Cs, op + apply_block_start(pad, c0 + blk) * p.vt, p.vt, ocur, apply_block_rows(pad, c0 + blk));
    }
}

// The same correction from the per-chunk cumulative decay (Alg. 1's list of gamma~_[n]) and the log
// decays themselves:  exp(G_t) with  G_t = G_chunk[n] + sum of g over the chunk's tokens up to t,
// the in-chunk factor Lambda_t of Sec. 2.1 times gamma~_[n-1].  A thread owns 4 channels and TPT
// consecutive tokens of the 64-token block: cumulative sum in registers, the token groups stitched
// through LDS.  Stops where G_chunk[n] < kVanish in every channel (see "Vanished decay").
template <int DK, int DV, int GM, bool NT>
__global__ __launch_bounds__(256) void apply_init_cd_bf16_kernel(ApplyParams p) {
    typedef ApplyCfg<DK, DV> Cfg;
    typedef GateVal<GM> GV;
    constexpr int QS = Cfg::QS;
    constexpr int CQ = DK / 4, NG = 256 / CQ, TPT = 64 / NG;   // channel quads, token groups, tokens per thread
    constexpr int GB = GM == kGateBF16 ? 2 : 4;
    __shared__ __align__(16) unsigned char lds[Cfg::kBytes];
    __shared__ __align__(16) float tot[NG * DK];
    __shared__ int gone[4];
    unsigned char *Qh = lds;
    float *Cs = reinterpret_cast<float *>(lds + 64 * QS);

    const int tid = threadIdx.x, cq = tid % CQ, tg = tid / CQ;
    int tb;
    int id = apply_stream_of_workgroup(p, tb);
    const int h = id % p.H;
    id /= p.H;
    const int b = id % p.B, seg = p.p0 + p.seg_step * (id / p.B);
    const long long tok0 = (long long)seg * p.L;                 // the segment's first token
    const int c0 = tb * (p.tokens_per_wg / 64);                  // this workgroup's first block (= chunk)
    const int nblk = min(p.tokens_per_wg / 64, p.n_chunks - c0);
    const long long kb = b * p.sb + tok0 * p.st + h * p.sh;
    const uint16_t *qp = (const uint16_t *)p.q + kb + (long long)(tg * TPT) * p.st + 4 * cq;
    const unsigned char *gp = (const unsigned char *)p.g + (kb + (long long)(tg * TPT) * p.st + 4 * cq) * GB;
    uint16_t *op = (uint16_t *)p.o + b * p.vb + tok0 * p.vt + h * p.vh;
    const long long NC = (long long)p.P * p.n_chunks;           // chunks per batch entry
    const float *Gk = p.G_chunk + ((b * NC + (long long)seg * p.n_chunks + c0) * p.H + h) * DK + 4 * cq;
    const long long gks = (long long)p.H * DK;                  // floats between chunks
    const float *S = p.S_init + (((size_t)seg * p.B + b) * p.H + h) * DK * DV;

    auto vanished = [](const f32x4 &x) { return x[0] < kVanish && x[1] < kVanish && x[2] < kVanish && x[3] < kVanish; };
    const bool may_stop = !p.dense;
    f32x4 pre_n = *reinterpret_cast<const f32x4 *>(Gk);
    if (may_stop && apply_all(vanished(pre_n), gone)) return;

    bf16x8 sf[Cfg::NKS];
    apply_load_state<DK, DV>(S, sf);

    u32x2 qn[TPT];
    typename GV::raw_t gn[TPT];
    u32x4 onx[Cfg::OITEMS];
    auto load_raw = [&](int blk) {
#pragma unroll
        for (int u = 0; u < TPT; ++u) {
            const long long tt = apply_block_start(p.pad, c0 + blk) + u;
            qn[u] = apply_ld<NT>(reinterpret_cast<const u32x2 *>(qp + tt * p.st));
            gn[u] = apply_ld<NT>(reinterpret_cast<const typename GV::raw_t *>(gp + tt * p.st * GB));
        }
    };
    load_raw(0);
    apply_load_o<DV, NT>(op + apply_block_start(p.pad, c0) * p.vt, p.vt, onx);
    for (int blk = 0; blk < nblk; ++blk) {
        const f32x4 pre = pre_n;
        u32x2 qc[TPT];
        f32x4 cs[TPT];
        u32x4 ocur[Cfg::OITEMS];
#pragma unroll
        for (int m = 0; m < Cfg::OITEMS; ++m) ocur[m] = onx[m];
        if (may_stop && blk > 0 && apply_all(vanished(pre), gone)) break;
        f32x4 run = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < TPT; ++u) {
            qc[u] = qn[u];
            run += GV::get(gn[u]);
            cs[u] = run;
        }
        *reinterpret_cast<f32x4 *>(tot + tg * DK + 4 * cq) = run;
        if (blk + 1 < nblk) {   // (uniform) the next block's rows; nothing is fetched twice
            load_raw(blk + 1);
            apply_load_o<DV, NT>(op + apply_block_start(p.pad, c0 + blk + 1) * p.vt, p.vt, onx);
            pre_n = *reinterpret_cast<const f32x4 *>(Gk + (long long)(blk + 1) * gks);
        }
        __syncthreads();   // group sums visible; every thread is done with the staging tile of the last block
        f32x4 base = pre;
#pragma unroll
        for (int r = 0; r < NG; ++r) {
            const f32x4 x = *reinterpret_cast<const f32x4 *>(tot + r * DK + 4 * cq);
            const float sel = r < tg ? 1.f : 0.f;
#pragma unroll
            for (int a = 0; a < 4; ++a) base[a] = __builtin_fmaf(sel, x[a], base[a]);
        }
#pragma unroll
        for (int u = 0; u < TPT; ++u) {
            const f32x4 G = base + cs[u];
            *reinterpret_cast<u32x2 *>(Qh + (tg * TPT + u) * QS + 8 * cq) =
                u32x2{pack_bf16(bf16_lo(qc[u][0]) * fast_exp(G[0]) * p.scale, bf16_hi(qc[u][0]) * fast_exp(G[1]) * p.scale),
                      pack_bf16(bf16_lo(qc[u][1]) * fast_exp(G[2]) * p.scale, bf16_hi(qc[u][1]) * fast_exp(G[3]) * p.scale)};
        }
        __syncthreads();   // Qh complete
        apply_block<DK, DV>(sf, Qh, Cs, op + apply_block_start(p.pad, c0 + blk) * p.vt, p.vt, ocur, apply_block_rows(p.pad, c0 + blk));
    }
}

// ------------------------------------------------------------------------------------------ fp32
template <int DK, int DV>
__global__ __launch_bounds__(DV * 4) void apply_init_f32_kernel(ApplyParams p) {
    constexpr int NT = DV * 4, QS = DK + 4;
    __shared__ __align__(16) float Qh[64 * QS];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int l16 = lane & 15, kg = lane >> 4;

    // Workgroup id -> (group of 128 streams, token block, stream in the group), a stream being a
    // (segment, batch, head).  Inside a group the early token blocks of every stream come first - the
    // ones with work left once the decay has vanished - and spread evenly over the XCDs, which take
    // workgroup ids round-robin; a stream stays on one XCD (128 is a multiple of 8), and a group's
    // S_init states (8 MiB at d = 128) stay in the L2s while its token blocks are worked through.
    constexpr int kGroup = 128;
    const int blocks_per_seg = p.wgs_per_seg, streams = apply_segments(p) * p.B * p.H;
    const int grp = blockIdx.x / (kGroup * blocks_per_seg), r = blockIdx.x % (kGroup * blocks_per_seg);
    const int gsz = min(kGroup, streams - grp * kGroup);
    const int tb = r / gsz, j = r % gsz;
    // position j of a row -> stream: rotated inside each aligned block of 8 by the block's index, so that
    // the streams of one head (which share a decay speed, hence an amount of work) do not all fall on the
    // same XCD when H is a multiple of 8
    int id = grp * kGroup + (((j | 7) < gsz) ? (j & ~7) + ((j - (j >> 3)) & 7) : j);
    const int h = id % p.H;
    id /= p.H;
    const int b = id % p.B, seg = p.p0 + p.seg_step * (id / p.B);
    long long tok0 = (long long)seg * p.L;                       // the segment's first token
    long long T = (long long)p.P * p.L;                          // tokens per batch entry
    int n_chunks = p.n_chunks, pad = p.pad;
    const int c0 = tb * (p.tokens_per_wg / 64);                  // this workgroup's first block
    if (p.seg_start) {   // segments of unequal length, as in the bf16 kernel
        tok0 = p.seg_start[seg];
        T = p.T;
        const long long len = p.seg_start[seg + 1] - tok0;
        if (tok0 < 0 || len < 64 || len > p.L || tok0 > T - len) return;   // (in this order: no sum can overflow)
        n_chunks = (int)((len + 63) >> 6);
        pad = 64 * n_chunks - (int)len;
        if (c0 >= n_chunks) return;
    }
    const int nblk = min(p.tokens_per_wg / 64, n_chunks - c0);
    const float *qp = (const float *)p.q + b * p.sb + tok0 * p.st + h * p.sh;
    float *op = (float *)p.o + b * p.vb + tok0 * p.vt + h * p.vh;
    const float *Gc = p.G_cum + (((long long)b * T + tok0) * p.H + h) * DK;
    const long long gcs = (long long)p.H * DK;
    const float *S = p.S_init + (((size_t)seg * p.B + b) * p.H + h) * DK * DV;

    if (!p.dense && __syncthreads_and(Gc[apply_block_start(pad, c0) * gcs + tid % DK] < kVanish)) return;   // see "Vanished decay"

    f32x4 Sreg[DK / 16];   // B operand: register r of tile it = S[16 it + 4 kg + r][16 w + l16]
#pragma unroll
    for (int it = 0; it < DK / 16; ++it)
#pragma unroll
        for (int r = 0; r < 4; ++r) Sreg[it][r] = S[(size_t)(16 * it + 4 * kg + r) * DV + 16 * w + l16];

    for (int blk = 0; blk < nblk; ++blk) {
        const long long t0 = apply_block_start(pad, c0 + blk);
        const int rows = apply_block_rows(pad, c0 + blk);
        for (int e = tid; e < 64 * DK; e += NT) {
            const int t = e / DK, c = e % DK;
            const long long tt = t0 + t;
            Qh[t * QS + c] = qp[tt * p.st + c] * fast_exp(Gc[tt * gcs + c]) * p.scale;
        }
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int it = 0; it < DK / 16; ++it)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc = mma_f32(Qh[(16 * mt + l16) * QS + 16 * it + 4 * kg + r], Sreg[it][r], acc);
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (16 * mt + 4 * kg + r < rows) op[(t0 + 16 * mt + 4 * kg + r) * p.vt + 16 * w + l16] += acc[r];
        }
        __syncthreads();
    }
}

template <int DK, int DV> static hipError_t launch_ab16(const ApplyParams &p, hipStream_t s) {
    const long long wgs = (long long)apply_segments(p) * p.B * p.H * p.wgs_per_seg;
    if (wgs > 0x7fffffffll) return hipErrorInvalidValue;   // beyond the grid's x dimension
    const int grid = (int)wgs;
    // non-temporal loads: dense calls, and launches with more streams than the chip has workgroup slots
    const bool nt = p.dense || (long long)apply_segments(p) * p.B * p.H >= 768;
    if (p.gate_per_head) {
        if (nt) hipLaunchKernelGGL((apply_init_bf16_kernel<DK, DV, true, true>), dim3(grid), dim3(256), 0, s, p);
        else hipLaunchKernelGGL((apply_init_bf16_kernel<DK, DV, true, false>), dim3(grid), dim3(256), 0, s, p);
    } else {
        if (nt) hipLaunchKernelGGL((apply_init_bf16_kernel<DK, DV, false, true>), dim3(grid), dim3(256), 0, s, p);
        else hipLaunchKernelGGL((apply_init_bf16_kernel<DK, DV, false, false>), dim3(grid), dim3(256), 0, s, p);
    }
    return hipGetLastError();
}
template <int DK, int DV> static hipError_t launch_acd(const ApplyParams &p, hipStream_t s) {
    const long long wgs = (long long)apply_segments(p) * p.B * p.H * p.wgs_per_seg;
    if (wgs > 0x7fffffffll) return hipErrorInvalidValue;   // beyond the grid's x dimension
    const int grid = (int)wgs;
    const bool nt = p.dense || (long long)apply_segments(p) * p.B * p.H >= 768;   // as in launch_ab16
    if (p.g_bf16) {
        if (nt) hipLaunchKernelGGL((apply_init_cd_bf16_kernel<DK, DV, kGateBF16, true>), dim3(grid), dim3(256), 0, s, p);
        else hipLaunchKernelGGL((apply_init_cd_bf16_kernel<DK, DV, kGateBF16, false>), dim3(grid), dim3(256), 0, s, p);
    } else {
        if (nt) hipLaunchKernelGGL((apply_init_cd_bf16_kernel<DK, DV, kGateF32, true>), dim3(grid), dim3(256), 0, s, p);
        else hipLaunchKernelGGL((apply_init_cd_bf16_kernel<DK, DV, kGateF32, false>), dim3(grid), dim3(256), 0, s, p);
    }
    return hipGetLastError();
}
template <int DK, int DV> static hipError_t launch_af32(const ApplyParams &p, hipStream_t s) {
    const long long wgs = (long long)apply_segments(p) * p.B * p.H * p.wgs_per_seg;
    if (wgs > 0x7fffffffll) return hipErrorInvalidValue;   // beyond the grid's x dimension
    const int grid = (int)wgs;
    hipLaunchKernelGGL((apply_init_f32_kernel<DK, DV>), dim3(grid), dim3(DV * 4), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_apply_bf16(const ApplyParams &p, int d_k, int d_v, hipStream_t s) {
    if (apply_segments(p) <= 0) return hipSuccess;
    if (d_k == 64 && d_v == 64) return launch_ab16<64, 64>(p, s);
    if (d_k == 64 && d_v == 128) return launch_ab16<64, 128>(p, s);
    if (d_k == 128 && d_v == 64) return launch_ab16<128, 64>(p, s);
    if (d_k == 128 && d_v == 128) return launch_ab16<128, 128>(p, s);
    return hipErrorInvalidValue;
}
hipError_t launch_apply_cd_bf16(const ApplyParams &p, int d_k, int d_v, hipStream_t s) {
    if (apply_segments(p) <= 0) return hipSuccess;
    if (d_k == 64 && d_v == 64) return launch_acd<64, 64>(p, s);
    if (d_k == 64 && d_v == 128) return launch_acd<64, 128>(p, s);
    if (d_k == 128 && d_v == 64) return launch_acd<128, 64>(p, s);
    if (d_k == 128 && d_v == 128) return launch_acd<128, 128>(p, s);
    return hipErrorInvalidValue;
}
hipError_t launch_apply_f32(const ApplyParams &p, int d_k, int d_v, hipStream_t s) {
    if (apply_segments(p) <= 0) return hipSuccess;
    if (d_k == 64 && d_v == 64) return launch_af32<64, 64>(p, s);
    if (d_k == 64 && d_v == 128) return launch_af32<64, 128>(p, s);
    if (d_k == 128 && d_v == 64) return launch_af32<128, 64>(p, s);
    if (d_k == 128 && d_v == 128) return launch_af32<128, 128>(p, s);
    return hipErrorInvalidValue;
}

}  // namespace zeco
