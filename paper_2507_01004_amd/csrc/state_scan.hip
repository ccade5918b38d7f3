// Segment-state scan: S_init[p+1] = (exp(G_tot[p])^T 1) .* S_init[p] + S_loc[p]  (Sec. 3.2 block
// update, applied along the chain of segments resident on one GPU).  With `reverse` the chain runs
// from the last segment to the first (the backward direction of Alg. 2): S_init[p] is then what
// enters segment p from segment p+1, and the end value is what leaves segment 0.
//
// Pure streaming: every state element is an independent serial chain of length P, so one thread
// owns a few consecutive floats of a (head, d_k-row-block) slab and walks p = 0..P-1.  The loads of
// the following segments do not depend on the chain and are issued ahead of the FMAs that consume them,
// which is what keeps HBM busy (the on-device analogue of the block pipeline of Sec. 3.2:
// all row blocks advance concurrently, each block's chain is latency-bound on its own).
// One fused multiply-add per element per segment, in segment order: bitwise reproducible and
// independent of how rows are grouped into blocks.
#include "zeco_device.h"
#include "zeco_internal.h"

namespace zeco {

// V floats of a state row per thread, D segments of loads in flight per thread.
template <int V> struct alignas(4 * V) ScanVec { float v[V]; };
template <int V> struct ScanRaw;
template <> struct ScanRaw<4> { typedef f32x4 t; };
template <> struct ScanRaw<2> { typedef f32x2 t; };
template <> struct ScanRaw<1> { typedef float t; };
// S_loc is read once and never again by this kernel: non-temporal loads.  They change nothing when the
// inputs stream from HBM with clean caches (5.3 TB/s either way at 64 x 16 and 256 x 8 states of 128 x 128) and
// help when the caches are full of another kernel's dirty lines (3.5 -> 4.9 TB/s after a 512 MiB fill); with the
// working set in the Infinity Cache ordinary loads are the faster ones (6.3 against 5.7 TB/s).  S_init is
// stored with ordinary stores: the correction reads it next.
template <int V> __device__ __forceinline__ ScanVec<V> scan_load(const float *ptr) {
    typedef typename ScanRaw<V>::t raw_t;
    return __builtin_bit_cast(ScanVec<V>, __builtin_nontemporal_load(reinterpret_cast<const raw_t *>(ptr)));
}
template <int V> __device__ __forceinline__ void scan_store(float *ptr, const ScanVec<V> &x) {
    typedef typename ScanRaw<V>::t raw_t;
    *reinterpret_cast<raw_t *>(ptr) = __builtin_bit_cast(raw_t, x);
}

// Grid: x = (head, row block, part of the block's slab), y = chain.  A thread owns V consecutive floats of
// one state row and walks the chain; its loads run D segments ahead of the multiply-adds in a ring of
// registers (the slot a step has just consumed is refilled with the step D further on), so that D loads per
// thread are in flight at every moment, not only at the start of a batch: with BH * d_k * d_v / V threads
// and a DRAM latency of 1-2 us that product is what decides how much of the HBM rate the kernel sees.
// The steady-state loop is free of branches (a branch makes the compiler wait for all outstanding loads at
// the join): STORE (S_init is written) and BYP (the by-products G_pre / G_sum are wanted) are template
// flags, and the rounds whose refills would run past the chain's end are peeled off into a guarded tail.
// Loads, the gate loads and the stores all count against the 63 memory operations a wave can have
// outstanding, so D beyond 20 buys nothing.
template <int V, int D, bool STORE, bool BYP>
__global__ __launch_bounds__(256) void state_scan_kernel(ScanParams p, int parts) {
    typedef ScanVec<V> vec_t;
    const int blocks_per_head = p.d_k / p.rows_per_block;
    const int part = blockIdx.x % parts, rb = blockIdx.x / parts;
    const int bh = rb / blocks_per_head;
    const int row0 = (rb % blocks_per_head) * p.rows_per_block;
    const int dvv = p.d_v / V;                               // threads per state row
    const int slab = p.rows_per_block * dvv;                 // threads' worth of work in a row block
    const size_t state = (size_t)p.d_k * p.d_v;
    const size_t seg_stride = (size_t)p.BH * state;         // floats between segments
    const size_t gdim = p.gate_per_head ? 1 : p.d_k;        // log decays per (segment, head)
    const size_t g_stride = (size_t)p.BH * gdim;
    const size_t grp = blockIdx.y;                          // chain (group of P segments)
    const int P = p.P;

    const int e = part * 256 + threadIdx.x;
    if (e >= slab) return;
    const int row = row0 + e / dvv;
    const size_t off = (size_t)bh * state + (size_t)row * p.d_v + (size_t)(e % dvv) * V;
    const float *loc = p.S_loc + grp * P * seg_stride + off;
    const float *gt = p.G_tot + grp * P * g_stride + (size_t)bh * gdim + (p.gate_per_head ? 0 : row);
    float *init = STORE ? p.S_init + grp * P * seg_stride + off : nullptr;
    vec_t s;
#pragma unroll
    for (int i = 0; i < V; ++i) s.v[i] = 0.f;
    if (p.S0) s = *reinterpret_cast<const vec_t *>(p.S0 + grp * seg_stride + off);
    // optional by-products: the log decay preceding each segment of the chain (forward chains) and the
    // chain's total, kept by the thread that owns the first columns of a row (of the head's first row
    // when the head has one decay)
    const bool prefix = BYP && e % dvv == 0 && (!p.gate_per_head || row == 0);
    const size_t gcol = (size_t)bh * gdim + (p.gate_per_head ? 0 : row);
    float *gpre = (prefix && p.G_pre) ? p.G_pre + grp * P * g_stride + gcol : nullptr;
    float gsum = 0.f;

    // running pointers: of the next step to fetch, of the next step to consume (chain order, either direction)
    const long long first = p.reverse ? P - 1 : 0, dir = p.reverse ? -1 : 1;
    const long long sstep = dir * (long long)seg_stride, gstep = dir * (long long)g_stride;
    const float *lf = loc + first * (long long)seg_stride, *gf = gt + first * (long long)g_stride;
    float *sp = STORE ? init + first * (long long)seg_stride : nullptr;
    float *gp = gpre ? gpre + first * (long long)g_stride : nullptr;
    vec_t x[D];
    float a[D];
    auto fetch = [&](int u) {
        x[u] = scan_load<V>(lf);
        a[u] = *gf;
        lf += sstep;
        gf += gstep;
    };
    auto consume = [&](int u) {
        if (STORE) {
            scan_store<V>(sp, s);
            sp += sstep;
        }
        if (BYP) {
            if (gp) {
                *gp = gsum;
                gp += gstep;
            }
            gsum += a[u];
        }
        const float d = fast_exp(a[u]);
#pragma unroll
        for (int i = 0; i < V; ++i) s.v[i] = __builtin_fmaf(d, s.v[i], x[u].v[i]);
    };
    int p0 = 0;
    if (P >= 2 * D) {
        // long chain: unconditional prologue, then rounds in which every step and its refill are in the chain
#pragma unroll
        for (int u = 0; u < D; ++u) {
            fetch(u);
            __builtin_amdgcn_sched_barrier(0);   // in ring order: the waits below count the loads issued since
        }
        for (; p0 + 2 * D <= P; p0 += D) {
#pragma unroll
            for (int u = 0; u < D; ++u) {
                consume(u);
                // (the refill must not be scheduled above the last use of the slot it overwrites: the slot
                // would then need a second register and a copy at the loop's head, which waits for every load)
                __builtin_amdgcn_sched_barrier(0);
                fetch(u);
            }
        }
    } else {
#pragma unroll
        for (int u = 0; u < D; ++u)
            if (u < P) fetch(u);
    }
    for (; p0 < P; p0 += D) {              // the last one or two rounds (all of a short chain)
#pragma unroll
        for (int u = 0; u < D; ++u) {
            if (p0 + u < P) {
                consume(u);
                if (p0 + u + D < P) fetch(u);
            }
        }
    }
    if (p.S_last) *reinterpret_cast<vec_t *>(p.S_last + grp * seg_stride + off) = s;
    if (prefix && p.G_sum) p.G_sum[grp * g_stride + gcol] = gsum;
}

template <int V, int D> static hipError_t launch_scan_vd(const ScanParams &p, hipStream_t s) {
    const int slab = p.rows_per_block * (p.d_v / V);
    const int parts = (slab + 255) / 256;
    int threads = ((slab + 63) / 64) * 64;
    if (threads > 256) threads = 256;
    const long long blocks = (long long)p.BH * (p.d_k / p.rows_per_block) * parts;
    if (blocks > 0x7fffffffll) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks, p.groups), block(threads);
    const bool byp = p.G_pre || p.G_sum;
    if (p.S_init) {
        if (byp) hipLaunchKernelGGL((state_scan_kernel<V, D, true, true>), grid, block, 0, s, p, parts);
        else hipLaunchKernelGGL((state_scan_kernel<V, D, true, false>), grid, block, 0, s, p, parts);
    } else {
        if (byp) hipLaunchKernelGGL((state_scan_kernel<V, D, false, true>), grid, block, 0, s, p, parts);
        else hipLaunchKernelGGL((state_scan_kernel<V, D, false, false>), grid, block, 0, s, p, parts);
    }
    return hipGetLastError();
}

// Floats per thread and ring depth, measured on MI355X at d_k = d_v = 128 with inputs not in any cache:
// 16 heads (65536 threads at four floats each) run best with 16-byte accesses and 8 segments in flight
// (5.2 TB/s; deeper rings are 5-10 % slower); 8 heads fill the chip only at two floats per thread (256 x 8:
// 4.5 -> 5.3 TB/s with 16 in flight); a single head at one float per thread (1024 x 1: 1.5 -> 2.3 TB/s).
hipError_t launch_scan(const ScanParams &p, hipStream_t s) {
    const long long quads = (long long)p.groups * p.BH * p.d_k * p.d_v / 4;   // (d_v is a multiple of 4)
    if (quads >= 65536) return launch_scan_vd<4, 8>(p, s);
    if (quads >= 32768) return launch_scan_vd<2, 16>(p, s);
    return launch_scan_vd<1, 16>(p, s);
}

// G_cum[b, t, h] += G_pre[piece of t, b, h] for per-head log decays (G_cum [B,T,H], G_pre [pieces,B,H], pieces
// of `len` tokens counted over the whole sequence): rebases the cumulative decay of pieces that were run
// from their own first token onto the segment's first token.
__global__ __launch_bounds__(256) void gate_offset_head_kernel(float *G_cum, const float *G_pre, int B, long long T, int H, int len) {
    const long long n = (long long)B * T * H;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) {
        const int h = (int)(i % H);
        const long long bt = i / H, t = bt % T, b = bt / T;
        G_cum[i] += G_pre[((t / len) * B + b) * H + h];
    }
}

hipError_t launch_gate_offset_head(float *G_cum, const float *G_pre, int B, long long T, int H, int len, hipStream_t s) {
    const long long n = (long long)B * T * H;
    long long blocks = (n + 255) / 256;
    if (blocks > 256 * 8) blocks = 256 * 8;
    if (blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(gate_offset_head_kernel, dim3((unsigned)blocks), dim3(256), 0, s, G_cum, G_pre, B, T, H, len);
    return hipGetLastError();
}

// Plain copy used to calibrate the profiler's HBM byte counters and the achievable bandwidth.
__global__ __launch_bounds__(256) void hbm_copy_kernel(u32x4 *dst, const u32x4 *src, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

hipError_t launch_copy(void *dst, const void *src, size_t bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(hbm_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (u32x4 *)dst,
                       (const u32x4 *)src, n16);
    return hipGetLastError();
}

// Calibration of the achievable HBM rate for a given mix of traffic: every thread reads one 16-byte word from
// each of R source arrays and writes one to each of W destination arrays per step (the arrays are consecutive
// slices of n16 words of src and dst).  A workgroup takes one contiguous piece of 16 KiB of every stream, the
// pieces in workgroup order; loads are non-temporal, stores ordinary.  Of the plain patterns measured this is
// the fastest (one read per write: 6.9-7.0 TB/s, against 5.1-5.7 for a grid-stride loop with either kind of
// load and store); dst may be one of the source slices (a stream rewritten in place).
constexpr int kMixPiece = 1024;   // 16-byte words per workgroup and stream
template <int R, int W>
__global__ __launch_bounds__(256) void hbm_mix_kernel(u32x4 *dst, const u32x4 *src, size_t n16) {
    const size_t i0 = (size_t)blockIdx.x * kMixPiece;
    u32x4 keep = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int it = 0; it < kMixPiece / 256; ++it) {
        const size_t i = i0 + it * 256 + threadIdx.x;
        if (i < n16) {
            u32x4 x = {(uint32_t)i, 1u, 2u, 3u};
#pragma unroll
            for (int r = 0; r < R; ++r) x ^= __builtin_nontemporal_load(src + r * n16 + i);
#pragma unroll
            for (int w = 0; w < W; ++w) dst[w * n16 + i] = x;
            if (W == 0) keep ^= x;
        }
    }
    // (a read-only run must still use what it read: one word per thread, written only if it is the rare value)
    if (W == 0 && (keep[0] ^ keep[1] ^ keep[2] ^ keep[3]) == 0x9e3779b9u) dst[0] = keep;
}

template <int R, int W> static hipError_t launch_mix_rw(void *dst, const void *src, size_t n16, hipStream_t s) {
    const size_t blocks = (n16 + kMixPiece - 1) / kMixPiece;
    if (blocks > 0x7fffffffull) return hipErrorInvalidValue;
    hipLaunchKernelGGL((hbm_mix_kernel<R, W>), dim3((unsigned)blocks), dim3(256), 0, s, (u32x4 *)dst, (const u32x4 *)src, n16);
    return hipGetLastError();
}

hipError_t launch_mix(void *dst, const void *src, size_t slice_bytes, int reads, int writes, hipStream_t s) {
    const size_t n16 = slice_bytes / 16;
    if (n16 == 0) return hipSuccess;
    switch (reads * 4 + writes) {
        case 1 * 4 + 0: return launch_mix_rw<1, 0>(dst, src, n16, s);
        case 0 * 4 + 1: return launch_mix_rw<0, 1>(dst, src, n16, s);
        case 1 * 4 + 1: return launch_mix_rw<1, 1>(dst, src, n16, s);
        case 2 * 4 + 1: return launch_mix_rw<2, 1>(dst, src, n16, s);
        case 3 * 4 + 1: return launch_mix_rw<3, 1>(dst, src, n16, s);
        case 4 * 4 + 1: return launch_mix_rw<4, 1>(dst, src, n16, s);
        case 5 * 4 + 3: return launch_mix_rw<5, 3>(dst, src, n16, s);
        case 3 * 4 + 2: return launch_mix_rw<3, 2>(dst, src, n16, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace zeco
