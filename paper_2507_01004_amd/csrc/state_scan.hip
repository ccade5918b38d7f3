// Segment-state scan: S_init[p+1] = (exp(G_tot[p])^T 1) .* S_init[p] + S_loc[p]  (Sec. 3.2 block
// update, applied along the chain of segments resident on one GPU).  With `reverse` the chain runs
// from the last segment to the first (the backward direction of Alg. 2): S_init[p] is then what
// enters segment p from segment p+1, and the end value is what leaves segment 0.
//
// Pure streaming: every state element is an independent serial chain of length P, so one thread
// owns one float4 of a (head, d_k-row-block) slab and walks p = 0..P-1.  The loads of the next
// kDepth segments do not depend on the chain and are issued ahead of the FMAs that consume them,
// which is what keeps HBM busy (the on-device analogue of the block pipeline of Sec. 3.2:
// all row blocks advance concurrently, each block's chain is latency-bound on its own).
// One fused multiply-add per element per segment, in segment order: bitwise reproducible and
// independent of how rows are grouped into blocks.
#include "zeco_device.h"
#include "zeco_internal.h"

namespace zeco {

constexpr int kScanDepth = 8;

__global__ __launch_bounds__(256) void state_scan_kernel(ScanParams p) {
    const int blocks_per_head = p.d_k / p.rows_per_block;
    const int bh = blockIdx.x / blocks_per_head;
    const int row0 = (blockIdx.x % blocks_per_head) * p.rows_per_block;
    const int dv4 = p.d_v >> 2;
    const int slab4 = p.rows_per_block * dv4;
    const size_t state = (size_t)p.d_k * p.d_v;
    const size_t seg_stride = (size_t)p.BH * state;         // floats between segments
    const size_t gdim = p.gate_per_head ? 1 : p.d_k;        // log decays per (segment, head)
    const size_t g_stride = (size_t)p.BH * gdim;
    const size_t grp = blockIdx.y;                          // chain (group of P segments)

    for (int e = threadIdx.x; e < slab4; e += blockDim.x) {
        const int row = row0 + e / dv4;
        const size_t off = (size_t)bh * state + (size_t)row * p.d_v + (size_t)(e % dv4) * 4;
        const float *loc = p.S_loc + grp * p.P * seg_stride + off;
        const float *gt = p.G_tot + grp * p.P * g_stride + (size_t)bh * gdim + (p.gate_per_head ? 0 : row);
        float *init = p.S_init ? p.S_init + grp * p.P * seg_stride + off : nullptr;   // null: end values only
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
        if (p.S0) s = *reinterpret_cast<const f32x4 *>(p.S0 + grp * seg_stride + off);
        // optional by-products: the log decay preceding each segment of the chain (forward chains) and the
        // chain's total, kept by the thread that owns the first columns of a row (of the head's first row
        // when the head has one decay)
        const bool prefix = (p.G_pre || p.G_sum) && e % dv4 == 0 && (!p.gate_per_head || row == 0);
        const size_t gcol = (size_t)bh * gdim + (p.gate_per_head ? 0 : row);
        float *gpre = (prefix && p.G_pre) ? p.G_pre + grp * p.P * g_stride + gcol : nullptr;
        float gsum = 0.f;

        for (int p0 = 0; p0 < p.P; p0 += kScanDepth) {
            f32x4 x[kScanDepth];
            float a[kScanDepth];
#pragma unroll
            for (int u = 0; u < kScanDepth; ++u) {
                if (p0 + u < p.P) {
                    const size_t sg = p.reverse ? p.P - 1 - (p0 + u) : p0 + u;   // segment of this step
                    x[u] = *reinterpret_cast<const f32x4 *>(loc + sg * seg_stride);
                    a[u] = gt[sg * g_stride];
                }
            }
#pragma unroll
            for (int u = 0; u < kScanDepth; ++u) {
                if (p0 + u < p.P) {
                    const size_t sg = p.reverse ? p.P - 1 - (p0 + u) : p0 + u;
                    if (init) *reinterpret_cast<f32x4 *>(init + sg * seg_stride) = s;
                    if (prefix) {
                        if (gpre) gpre[sg * g_stride] = gsum;
                        gsum += a[u];
                    }
                    const float d = fast_exp(a[u]);
                    s[0] = __builtin_fmaf(d, s[0], x[u][0]);
                    s[1] = __builtin_fmaf(d, s[1], x[u][1]);
                    s[2] = __builtin_fmaf(d, s[2], x[u][2]);
                    s[3] = __builtin_fmaf(d, s[3], x[u][3]);
                }
            }
        }
        if (p.S_last) *reinterpret_cast<f32x4 *>(p.S_last + grp * seg_stride + off) = s;
        if (prefix && p.G_sum) p.G_sum[grp * g_stride + gcol] = gsum;
    }
}

hipError_t launch_scan(const ScanParams &p, hipStream_t s) {
    const int blocks = p.BH * (p.d_k / p.rows_per_block);
    const int slab4 = p.rows_per_block * (p.d_v / 4);
    int threads = ((slab4 + 63) / 64) * 64;
    if (threads > 256) threads = 256;
    hipLaunchKernelGGL(state_scan_kernel, dim3(blocks, p.groups), dim3(threads), 0, s, p);
    return hipGetLastError();
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

}  // namespace zeco
