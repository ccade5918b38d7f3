// Host-side launcher interface between the C ABI (zeco_api.hip) and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace zeco {

struct ChunkParams {
    const void *q, *k, *v, *g;
    void *o;
    float *S_loc, *G_cum, *G_tot;
    int B, P, H, L;
    int n_chunks;              // L / 64
    float scale;
    long long sb, st, sh;      // q/k/g element strides
    long long vb, vt, vh;      // v/o element strides
#ifdef ZECO_PHASE_TIMING
    unsigned long long *dbg;   // development builds only: cycle stamps of workgroup 0
#endif
};
#ifdef ZECO_PHASE_TIMING
extern unsigned long long *g_phase_dbg;
#endif

struct ApplyParams {
    const void *q;
    const float *G_cum, *S_init;
    void *o;
    int B, P, H, L;
    int p0;                    // first segment to correct
    int tokens_per_wg;         // multiple of 64 dividing L
    float scale;
    long long sb, st, sh, vb, vt, vh;
};

struct ScanParams {
    const float *S_loc, *G_tot, *S0;
    float *S_init, *S_last;
    int P, BH, d_k, d_v, rows_per_block;
};

// Each returns hipSuccess or the launch error.  d_k, d_v in {64,128}.
hipError_t launch_chunk_f32(const ChunkParams &p, int d_k, int d_v, hipStream_t s);
hipError_t launch_chunk_bf16(const ChunkParams &p, int d_k, int d_v, bool g_bf16, hipStream_t s);
hipError_t launch_apply_f32(const ApplyParams &p, int d_k, int d_v, hipStream_t s);
hipError_t launch_apply_bf16(const ApplyParams &p, int d_k, int d_v, hipStream_t s);
hipError_t launch_scan(const ScanParams &p, hipStream_t s);
hipError_t launch_copy(void *dst, const void *src, size_t bytes, hipStream_t s);

}  // namespace zeco
