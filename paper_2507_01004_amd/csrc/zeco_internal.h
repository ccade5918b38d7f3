// Host-side launcher interface between the C ABI (zeco_api.hip) and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace zeco {

// Gate layouts: kGateF32 / kGateBF16 = one log decay per (token, head, channel); kGateHead = one fp32
// log decay per (token, head), shared by all channels (g, G_cum [B,T,H] contiguous; G_tot [P,B,H]).
enum GateMode { kGateF32 = 0, kGateBF16 = 1, kGateHead = 2 };
// added to the gate layout handed to launch_chunk_bf16: decay factors of the tiles counted from half the chunk's
// total log decay (twice the range of gates, one more multiplication of the state per chunk)
constexpr int kGateWide = 4;

struct ChunkParams {
    const void *q, *k, *v, *g;
    void *o;
    float *S_loc, *G_cum, *G_tot;
    const float *S_init;       // [P,B,H,d_k,d_v] initial states (modes that start from a given state)
    const float *G_off = nullptr;   // [P,B,H,d_k] ([P,B,H] per-head) log decay preceding each segment (mode 5 only)
    float *G_chunk = nullptr;       // [B,P,n_chunks,H,d_k] log decay from the segment start to each chunk's start (mode 6 only)
    int B, P, H, L;
    int n_chunks;              // ceil(L / 64)
    int pad = 0;               // 64 n_chunks - L: the first chunk processed holds 64 - pad tokens
    // Segments of unequal length (modes 0 to 4 of the bf16 kernel, and the fp32 kernel): segment p covers tokens
    // [seg_start[p], seg_start[p+1]) of the T tokens of every batch entry; L is then the upper bound of the
    // lengths, n_chunks and pad are unused.
    const long long *seg_start = nullptr;
    long long T = 0;
    float scale;
    float kscale;              // backward modes: multiplier carried by the operand in the k role
    long long sb, st, sh;      // q/k/g element strides
    long long vb, vt, vh;      // v/o element strides
};

struct ApplyParams {
    const void *q;
    const float *G_cum = nullptr;    // [B,T,H,d_k] per-token cumulative log decay, or
    const float *G_chunk = nullptr;  // [B,P,n_chunks,H,d_k] per-chunk one, together with
    const void *g = nullptr;         //   the log decays themselves (layout of q)
    int g_bf16 = 0;                  //   stored as bf16 (1) or fp32 (0)
    const float *S_init;
    void *o;
    int B, P, H, L;
    int p0;                    // first segment to correct
    int seg_step = 1;          // ... and every seg_step-th one after it
    int tokens_per_wg;         // multiple of 64
    int n_chunks, pad;         // 64-token blocks per segment, ceil(L / 64), and 64 n_chunks - L: the first block is the short one
    int wgs_per_seg;           // workgroups per segment, ceil(64 n_chunks / tokens_per_wg)
    const long long *seg_start = nullptr;   // segments of unequal length (the kernels that read G_cum):
    long long T = 0;                        //   as in ChunkParams; n_chunks, pad, wgs_per_seg describe the bound L
    int gate_per_head = 0;     // 1: G_cum [B,T,H] (bf16 kernel only)
    int dense = 0;             // 1: stream every token, also where exp(G_cum) has vanished
    float scale;
    long long sb, st, sh, vb, vt, vh;
};

// `groups` independent chains of P segments each: S_loc, S_init [groups*P, BH, d_k, d_v],
// G_tot [groups*P, BH, d_k], S0 and S_last [groups, BH, d_k, d_v].
struct ScanParams {
    const float *S_loc, *G_tot, *S0;
    float *S_init, *S_last;      // either may be null (not stored)
    int P, BH, d_k, d_v, rows_per_block, groups;
    int reverse = 0;             // 1: chain runs from segment P-1 down to 0
    // optional, each on its own: G_pre [groups*P, BH, d_k] = sum of G_tot over the earlier segments of the
    // chain (forward chains only), G_sum [groups, BH, d_k] = sum over all of them ([.., BH] with one decay per head)
    float *G_pre = nullptr, *G_sum = nullptr;
    int gate_per_head = 0;       // 1: G_tot [groups*P, BH], one log decay per head
};

// dQ / dK pass (gla_bwd_qk.hip).  x, y: [B,T,H,d_v] operands (strides vb, vt, vh); z, z2, g, out:
// [B,T,H,d_k] (strides sb, st, sh); W_init [P,B,H,d_k,d_v] fp32; dg [B,T,H,d_k] fp32 contiguous (the dQ
// pass leaves q .* dq there, the dK pass turns it into dG); S_init, S_last: forward states (dK pass).
// With per-head gates g and dg are [B,T,H] and the channel sums are taken before anything is stored.
struct BwdQKParams {
    const void *x, *y, *z, *z2, *g;
    void *out;
    float *dg;
    const float *W_init, *S_init, *S_last;
    int B, P, H, L, n_chunks;    // n_chunks = ceil(L / 64)
    int pad = 0;                 // 64 n_chunks - L: the first chunk processed holds 64 - pad tokens
    const long long *seg_start = nullptr;   // segments of unequal length, as in ChunkParams (L = bound on the
    long long T = 0;                        //   lengths, T = tokens per batch entry)
    float zscale, oscale;        // multipliers of the gated operand and of the output
    // dQ pass only, optional: also emit each segment's state gradient from dS = 0,
    // dS_loc [P,B,H,d_k,d_v] = qscale * sum_t (q_t .* exp(G_t))^T x_t, and its total log decay G_tot_out
    float *dS_loc = nullptr, *G_tot_out = nullptr;
    float qscale = 1.f;
    // optional checkpoints that re-anchor dG: S_ck [B*P*H, n_ck, d_k, d_v], the forward state entering every
    // 8th chunk (chunks 8, 16, ..) of each segment; written by the dQ pass, read by the dK pass.  With it the dQ
    // pass must be launched with short_last = 1 (the short chunk of a ragged length at the segment's end).
    float *S_ck = nullptr;
    int n_ck = 0, short_last = 0;
    long long sb, st, sh, vb, vt, vh;
};

// A kernel that uses more dynamic LDS than the default limit has the limit raised once per device (the
// attribute belongs to the function on that device), not at every launch.  One static object per kernel
// instantiation; devices beyond the 64 the mask covers are simply set every time.
struct LdsLimit {
    std::atomic<unsigned long long> done{0};
    hipError_t raise(const void *kernel, int bytes) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        const unsigned long long bit = (dev >= 0 && dev < 64) ? 1ull << dev : 0ull;
        if (bit && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e == hipSuccess && bit) done.fetch_or(bit, std::memory_order_release);
        return e;
    }
};

// Each returns hipSuccess or the launch error.  d_k, d_v in {64,128}.
// fp32 kernel: chunk length C in {16, 32, 64} (p.n_chunks, p.pad count chunks of C tokens); mode 0 local pass,
// 1 states only, 2 output pass from S_init, 3 backward state pass, 4 dV pass (as in the bf16 kernel below)
hipError_t launch_chunk_f32(const ChunkParams &p, int d_k, int d_v, int C, int mode, hipStream_t s);
// mode: 0 local pass (o, S_loc, G_cum, G_tot), 1 states only (S_loc, G_tot), 2 output pass from S_init (o),
// 3 backward state pass (k := q, v := dO; S_loc := dS leaving the segment), 4 dV pass (q := k, k := q,
// v := dO, S_init := dS entering the segment's final state, o := dV), 5 output pass from S_init that also
// writes G_cum counted from G_off (o, G_cum), 6 local pass with the cumulative decay
// per chunk instead of per token (o, S_loc, G_chunk, G_tot; per-channel gates only)
hipError_t launch_chunk_bf16(const ChunkParams &p, int d_k, int d_v, int gate_mode, int mode, hipStream_t s);
hipError_t launch_apply_f32(const ApplyParams &p, int d_k, int d_v, hipStream_t s);
hipError_t launch_apply_bf16(const ApplyParams &p, int d_k, int d_v, hipStream_t s);
// from (g, G_chunk) instead of G_cum; per-channel gates
hipError_t launch_apply_cd_bf16(const ApplyParams &p, int d_k, int d_v, hipStream_t s);
hipError_t launch_scan(const ScanParams &p, hipStream_t s);
// reverse = false: dQ (x = dO, y = v, z = k, z2 = q, W_init = forward states); true: dK (x = v, y = dO,
// z = q, z2 = k, W_init = state gradients; must run after the dQ pass, whose q .* dq it consumes)
hipError_t launch_bwd_qk(const BwdQKParams &p, int d_k, int d_v, int gate_mode, bool reverse, hipStream_t s);
// the same two passes on fp32 tensors (gla_bwd_f32.hip), chunk length C in {16, 32, 64}; no by-products
hipError_t launch_bwd_qk_f32(const BwdQKParams &p, int d_k, int d_v, int C, bool reverse, hipStream_t s);
// per-head log decays: G_cum [B,T,H] += G_pre [T/len, B, H] of the piece each token lies in
hipError_t launch_gate_offset_head(float *G_cum, const float *G_pre, int B, long long T, int H, int len, hipStream_t s);
hipError_t launch_copy(void *dst, const void *src, size_t bytes, hipStream_t s);
// reads x writes 16-byte streams over slices of slice_bytes each (calibration of the HBM rate of a traffic mix)
hipError_t launch_mix(void *dst, const void *src, size_t slice_bytes, int reads, int writes, hipStream_t s);

}  // namespace zeco
