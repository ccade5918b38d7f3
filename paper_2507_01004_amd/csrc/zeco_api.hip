// C ABI of the ZeCO hot path (declared in include/zeco.h): argument validation and dispatch to
// the gfx950 kernels.  Validation happens before any HIP call so that the error paths can be
// exercised on a host without a GPU.
#include "../../include/zeco.h"
#include "zeco_internal.h"

#include <atomic>

// Scratch of zeco_state_scan_tree_static, the entry point for callers that cannot allocate: a fixed array in
// the library's device image, one copy per GPU the library runs on, held until the process ends.  In host
// code this name only identifies the symbol - it is not a device address; the address on the current GPU
// comes from hipGetSymbolAddress (static_scratch() below) and that pointer is what the launches are given.
constexpr size_t kStaticScratchBytes = (size_t)33 << 20;
static __device__ __align__(256) unsigned char zeco_static_scratch[kStaticScratchBytes];

namespace {

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool dim_ok(int d) { return d == 64 || d == 128; }

// ZECO_OK when the descriptor is well formed and supported.  `any_length`: the entry point takes segment
// lengths that are no multiple of the chunk size (the forward entry points do, from 64 tokens on).
zeco_status check_desc(const zeco_gla_desc *d, bool any_length = false) {
    if (!d) return ZECO_ERR_INVALID_ARG;
    if (d->B < 0 || d->P <= 0 || d->H <= 0 || d->L <= 0 || d->d_k <= 0 || d->d_v <= 0 || d->C <= 0)
        return ZECO_ERR_INVALID_ARG;   // (B = 0, an empty batch, is valid: every entry point returns at once)
    if (d->io_dtype != ZECO_F32 && d->io_dtype != ZECO_BF16) return ZECO_ERR_INVALID_ARG;
    if (d->g_dtype != ZECO_F32 && d->g_dtype != ZECO_BF16) return ZECO_ERR_INVALID_ARG;
    if (!(d->scale == d->scale)) return ZECO_ERR_INVALID_ARG;
    if ((int64_t)d->P * d->L > (int64_t)1 << 40 || d->L > (1 << 30)) return ZECO_ERR_INVALID_ARG;
    const int64_t s[6] = {d->stride_b, d->stride_t, d->stride_h, d->vstride_b, d->vstride_t, d->vstride_h};
    for (int i = 0; i < 6; ++i)
        if (s[i] < 0 || s[i] % 8 != 0) return ZECO_ERR_INVALID_ARG;
    if (d->stride_h < d->d_k || d->vstride_h < d->d_v) return ZECO_ERR_INVALID_ARG;
    if (d->stride_t < d->d_k || d->vstride_t < d->d_v) return ZECO_ERR_INVALID_ARG;
    // the kernels keep in-chunk offsets (64 tokens x stride_t elements) in 32 bits
    if (d->stride_t > ((int64_t)1 << 24) || d->vstride_t > ((int64_t)1 << 24)) return ZECO_ERR_UNSUPPORTED;
    if ((int64_t)d->B * d->P * d->H > (int64_t)1 << 24) return ZECO_ERR_INVALID_ARG;
    // chunk length: 64 for bf16 (one token per lane of a wavefront); the fp32 kernel also takes 16 and 32
    const bool chunk_ok = d->C == 64 || (d->io_dtype == ZECO_F32 && (d->C == 16 || d->C == 32));
    if (!chunk_ok || !dim_ok(d->d_k) || !dim_ok(d->d_v)) return ZECO_ERR_UNSUPPORTED;
    if (d->L % d->C != 0 && !any_length) return ZECO_ERR_UNSUPPORTED;
    if (d->L < 64) return ZECO_ERR_UNSUPPORTED;   // (the correction works on windows of 64 tokens inside a segment)
    if (d->io_dtype == ZECO_F32 && d->g_dtype != ZECO_F32) return ZECO_ERR_UNSUPPORTED;
    if (d->g_per_head != 0 && d->g_per_head != 1) return ZECO_ERR_INVALID_ARG;
    if (d->g_per_head && (d->io_dtype != ZECO_BF16 || d->g_dtype != ZECO_F32)) return ZECO_ERR_UNSUPPORTED;
    if (d->wide_gates != 0 && d->wide_gates != 1) return ZECO_ERR_INVALID_ARG;
    return ZECO_OK;
}

int gate_mode(const zeco_gla_desc *d) {
    if (d->g_per_head) return zeco::kGateHead;
    return d->g_dtype == ZECO_BF16 ? zeco::kGateBF16 : zeco::kGateF32;
}

// the same with the descriptor's choice of range, for the bf16 chunk kernel
int chunk_gate(const zeco_gla_desc *d) { return gate_mode(d) | (d->wide_gates ? zeco::kGateWide : 0); }

zeco_status from_hip(hipError_t e) { return e == hipSuccess ? ZECO_OK : ZECO_ERR_HIP; }

int chunks_of(int L) { return (L + 63) / 64; }

// Segment length of a chunk-kernel launch: chunks, and how far the first one falls short of 64 tokens.
void set_length(zeco::ChunkParams &p, int L) {
    p.L = L; p.n_chunks = chunks_of(L); p.pad = 64 * p.n_chunks - L;
}
// The same in chunks of C tokens (the fp32 kernel).
void set_length_c(zeco::ChunkParams &p, int L, int C) {
    p.L = L; p.n_chunks = (L + C - 1) / C; p.pad = C * p.n_chunks - L;
}

int gate_mode(const zeco_gla_desc *d);
int chunk_gate(const zeco_gla_desc *d);
// One of the phases both precisions have (0 local pass, 1 states only, 2 output pass from S_init, 3 backward
// state pass, 4 dV pass), on the segments p describes (p.L tokens each, or the table p.seg_start).
hipError_t launch_phase(zeco::ChunkParams &p, const zeco_gla_desc *d, int mode, hipStream_t s) {
    if (d->io_dtype == ZECO_F32) {
        set_length_c(p, p.L, d->C);
        return zeco::launch_chunk_f32(p, d->d_k, d->d_v, d->C, mode, s);
    }
    return zeco::launch_chunk_bf16(p, d->d_k, d->d_v, chunk_gate(d), mode, s);
}

// Segments per group of the two-level scan: the divisor g of P that minimises the length of the serial
// work, 2 g + P / g (two passes inside the groups, one over the groups).  Returns P when no proper divisor helps.
int tree_group(int P) {
    int best = P;
    long long cost = P;                       // the plain chain
    auto consider = [&](int g) {
        const long long c = 2ll * g + P / g;
        if (c < cost || (c == cost && g < best)) { cost = c; best = g; }
    };
    for (int a = 2; (long long)a * a <= P; ++a) {   // divisor pairs (a, P / a)
        if (P % a) continue;
        consider(a);
        consider(P / a);
    }
    return best;
}

// Floats of scratch the two-level scan of a chain of P segments needs (0: the chain is not split).
size_t tree_floats(int P, int BH, int d_k, int d_v, int gate_per_head) {
    const int g = tree_group(P);
    if (g == P) return 0;
    const size_t J = P / g, state = (size_t)BH * d_k * d_v;
    return 2 * J * state + J * (size_t)BH * (gate_per_head ? 1 : d_k);
}

// The two-level scan of one chain (sp.groups == 1, sp.P segments): every group of g segments from the zero
// state (end state and total log decay), the chain over the groups, every group again from the state
// entering it.  `scratch`: tree_floats() floats.
hipError_t launch_scan_tree(zeco::ScanParams sp, float *scratch, hipStream_t s) {
    const int P = sp.P, g = tree_group(P), J = P / g;
    const size_t state = (size_t)sp.BH * sp.d_k * sp.d_v;
    float *T = scratch, *I = T + J * state, *Gt = I + J * state;
    zeco::ScanParams p = sp;
    p.G_pre = nullptr;
    p.S0 = nullptr; p.S_init = nullptr; p.S_last = T; p.G_sum = Gt; p.P = g; p.groups = J;
    hipError_t e = zeco::launch_scan(p, s);
    if (e != hipSuccess) return e;
    p.S_loc = T; p.G_tot = Gt; p.S0 = sp.S0; p.S_init = I; p.S_last = sp.S_last; p.G_sum = nullptr;
    p.P = J; p.groups = 1;
    if ((e = zeco::launch_scan(p, s)) != hipSuccess) return e;
    p.S_loc = sp.S_loc; p.G_tot = sp.G_tot; p.S0 = I; p.S_init = sp.S_init; p.S_last = nullptr;
    p.P = g; p.groups = J;
    return zeco::launch_scan(p, s);
}

// Inside the fused calls: is the chain of P pieces better scanned as a tree?  Only for a single head: its
// serial chain (16384 threads at one float each) is bound by the latency of a step, 1024 segments take
// 0.057 ms against 0.044 ms as a tree, 4096 take 0.227 against 0.198 ms; at 256 segments the two are even,
// and from two heads on the serial scan is the faster one at every length (1024 x 2: 0.060 against 0.077 ms).
bool chain_wants_tree(int P, int BH) {
    if (!(BH == 1 && P >= 512)) return false;
    const int g = tree_group(P);
    return g != P && P / g <= 65535;          // (the groups are the y dimension of the launch)
}
size_t chain_scratch_floats(int P, int BH, int d_k, int d_v, int gate_per_head) {
    return chain_wants_tree(P, BH) ? tree_floats(P, BH, d_k, d_v, gate_per_head) : 0;
}
hipError_t launch_scan_chain(const zeco::ScanParams &sp, float *scratch, hipStream_t s) {
    return chain_wants_tree(sp.P, sp.BH) ? launch_scan_tree(sp, scratch, s) : zeco::launch_scan(sp, s);
}

// Device address of zeco_static_scratch on the current GPU.  Every GPU has its own copy of the array at its
// own address, so the address is looked up once per device, with that device current, and kept.  (Two
// threads that make a device's first call together both look up the same address; no lock is needed.)
constexpr int kMaxDevices = 64;
std::atomic<void *> g_static_scratch[kMaxDevices];
hipError_t static_scratch(void **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void *ptr = g_static_scratch[dev].load(std::memory_order_acquire);
    if (!ptr) {
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(zeco_static_scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_static_scratch[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return hipSuccess;
}

}  // namespace

extern "C" {

// Can the S equal pieces of a segment of L tokens be halved once more?  Pieces of whole chunks stay pieces of
// whole chunks; a length that is no multiple of 64 is cut into equal pieces wherever it divides, each
// piece then starting with a short chunk of its own.
static bool halves_evenly(int L, int S) { return L % 64 == 0 ? L % (2 * S * 64) == 0 : L % (2 * S) == 0; }

// Number of sub-segments each segment is split into inside zeco_gla_local_fwd (1 = none).  A stream is
// a serial chain over chunks, so with few (batch, segment, head) streams most compute units would
// idle; the local pass then applies the method to itself: sub-segment states from the zero state, a scan
// of them inside each segment, and the output pass of every sub-segment from its scanned state.
static int subsegments(const zeco_gla_desc *d) {
    if (d->io_dtype != ZECO_BF16) return 1;
    const long long streams = (long long)d->B * d->P * d->H;
    if (streams > 64) return 1;
    int S = 1;   // as many workgroups as fit the 256 compute units in one round, not more
    while (streams * S * 2 <= 256 && halves_evenly(d->L, S) && d->L / (2 * S) >= 256) S *= 2;
    return S;
}

// With one decay per head and between 65 and 128 streams the local pass runs every segment as two halves
// from the zero state on whole workgroups (256 streams), then corrects the second halves' outputs with the
// first halves' end states where their decay has not vanished, and rebases the second halves' G_cum, which
// costs 4 bytes per token and head in this layout: sibling workgroups on 128 streams leave the kernel bound
// by its own pipeline (3.3 TB/s at c3), whole workgroups on 256 streams move 5.4 TB/s.
static bool halves_with_correction(const zeco_gla_desc *d) {
    if (d->io_dtype != ZECO_BF16 || !d->g_per_head || d->d_v != 128) return false;
    const long long streams = (long long)d->B * d->P * d->H;
    return streams > 64 && streams <= 128 && d->L % 128 == 0 && d->L / 2 >= 4096;
}

struct SubLayout {          // workspace carve-up, in floats
    size_t states, gates;   // elements of one state array / one gate array over all sub-segments
    size_t off_Ssub, off_Sinit, off_Gtot, off_Gpre, total;
};
static SubLayout sub_layout(const zeco_gla_desc *d, int S) {
    SubLayout w;
    const size_t n = (size_t)d->P * S * d->B * d->H;
    w.states = n * d->d_k * d->d_v;
    w.gates = n * d->d_k;
    w.off_Ssub = 0;
    w.off_Sinit = w.off_Ssub + w.states;
    w.off_Gtot = w.off_Sinit + w.states;
    w.off_Gpre = w.off_Gtot + w.gates;
    w.total = w.off_Gpre + w.gates;
    return w;
}

static void fill_apply_params(zeco::ApplyParams &p, const zeco_gla_desc *d, int P, int L);

size_t zeco_gla_local_fwd_workspace(const zeco_gla_desc *desc) {
    if (check_desc(desc, true) != ZECO_OK) return 0;
    if (halves_with_correction(desc)) return sub_layout(desc, 2).total * sizeof(float);
    const int S = subsegments(desc);
    return S > 1 ? sub_layout(desc, S).total * sizeof(float) : 0;
}

zeco_status zeco_gla_local_fwd(const zeco_gla_desc *d, const void *q, const void *k, const void *v,
                               const void *g, void *o, float *S_loc, float *G_cum, float *G_tot,
                               void *workspace, size_t workspace_bytes, void *stream) {
    const zeco_status st = check_desc(d, true);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    if (!q || !k || !v || !g || !o || !S_loc || !G_cum || !G_tot) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g) || !aligned16(o) ||
        !aligned16(S_loc) || !aligned16(G_cum) || !aligned16(G_tot))
        return ZECO_ERR_INVALID_ARG;
    const size_t need = zeco_gla_local_fwd_workspace(d);
    if (workspace_bytes < need) return ZECO_ERR_WORKSPACE;
    if (need && (!workspace || !aligned16(workspace))) return ZECO_ERR_INVALID_ARG;
    const int S = subsegments(d);
    hipStream_t s = static_cast<hipStream_t>(stream);

    zeco::ChunkParams p;
    p.q = q; p.k = k; p.v = v; p.g = g; p.o = o;
    p.S_loc = S_loc; p.G_cum = G_cum; p.G_tot = G_tot; p.S_init = nullptr;
    p.B = d->B; p.P = d->P; p.H = d->H;
    set_length(p, d->L);
    p.scale = d->scale; p.kscale = 1.f;
    p.sb = d->stride_b; p.st = d->stride_t; p.sh = d->stride_h;
    p.vb = d->vstride_b; p.vt = d->vstride_t; p.vh = d->vstride_h;
    if (d->io_dtype == ZECO_F32) return from_hip(launch_phase(p, d, 0, s));
    if (halves_with_correction(d)) {
        const SubLayout w = sub_layout(d, 2);
        float *ws = static_cast<float *>(workspace);
        float *Ssub = ws + w.off_Ssub, *Sinit = ws + w.off_Sinit, *Gtot = ws + w.off_Gtot, *Gpre = ws + w.off_Gpre;
        // the halves from the zero state: o, G_cum counted from each half's first token, end states
        p.P = d->P * 2; set_length(p, d->L / 2);
        p.S_loc = Ssub; p.G_tot = Gtot;
        if (zeco::launch_chunk_bf16(p, d->d_k, d->d_v, chunk_gate(d), 0, s) != hipSuccess) return ZECO_ERR_HIP;
        // chain of the two halves of every segment: the state and the log decay entering the second half,
        // the segment's end state and total
        zeco::ScanParams sp;
        sp.S_loc = Ssub; sp.G_tot = Gtot; sp.S0 = nullptr; sp.S_init = Sinit; sp.S_last = S_loc;
        sp.P = 2; sp.groups = d->P; sp.BH = d->B * d->H; sp.d_k = d->d_k; sp.d_v = d->d_v;
        sp.rows_per_block = d->d_k / 16; sp.gate_per_head = 1;
        sp.G_pre = Gpre; sp.G_sum = G_tot;
        if (zeco::launch_scan(sp, s) != hipSuccess) return ZECO_ERR_HIP;
        // second halves (every other piece): o += (scale q .* exp(G_cum)) S_entering, with G_cum still counted
        // from the half's first token
        zeco::ApplyParams ap;
        fill_apply_params(ap, d, d->P * 2, d->L / 2);
        ap.q = q; ap.G_cum = G_cum; ap.S_init = Sinit; ap.o = o; ap.p0 = 1; ap.seg_step = 2;
        if (zeco::launch_apply_bf16(ap, d->d_k, d->d_v, s) != hipSuccess) return ZECO_ERR_HIP;
        return from_hip(zeco::launch_gate_offset_head(G_cum, Gpre, d->B, (long long)d->P * d->L, d->H, d->L / 2, s));
    }
    if (S == 1) return from_hip(zeco::launch_chunk_bf16(p, d->d_k, d->d_v, chunk_gate(d), 0, s));

    // Few streams: P*S sub-segments of L/S tokens, Alg. 1's schedule applied inside each segment: the
    // sub-segments' end states and total decays from the zero state, their scan inside the segment,
    // then the output pass of every sub-segment from its scanned state, which also writes G_cum counted
    // from the segment's first token.
    const SubLayout w = sub_layout(d, S);
    float *ws = static_cast<float *>(workspace);
    float *Ssub = ws + w.off_Ssub, *Sinit = ws + w.off_Sinit, *Gtot = ws + w.off_Gtot, *Gpre = ws + w.off_Gpre;
    p.P = d->P * S; set_length(p, d->L / S);
    p.S_loc = Ssub; p.G_tot = Gtot;
    hipError_t e = zeco::launch_chunk_bf16(p, d->d_k, d->d_v, chunk_gate(d), 1, s);
    if (e != hipSuccess) return ZECO_ERR_HIP;

    zeco::ScanParams sp;   // one chain of S sub-segments per segment; its end state is the segment's S_loc
    sp.S_loc = Ssub; sp.G_tot = Gtot; sp.S0 = nullptr; sp.S_init = Sinit; sp.S_last = S_loc;
    sp.P = S; sp.groups = d->P; sp.BH = d->B * d->H; sp.d_k = d->d_k; sp.d_v = d->d_v;
    sp.rows_per_block = d->d_k / 16; sp.gate_per_head = d->g_per_head;
    sp.G_pre = Gpre; sp.G_sum = G_tot;   // log decay preceding each sub-segment; the segment's total
    if ((e = zeco::launch_scan(sp, s)) != hipSuccess) return ZECO_ERR_HIP;

    p.S_loc = nullptr; p.G_tot = nullptr; p.S_init = Sinit; p.G_off = Gpre;
    return from_hip(zeco::launch_chunk_bf16(p, d->d_k, d->d_v, chunk_gate(d), 5, s));
}

// ---- two-phase forward ------------------------------------------------------------------------------
static void fill_chunk_params(zeco::ChunkParams &p, const zeco_gla_desc *d) {
    p.q = p.k = p.v = p.g = nullptr; p.o = nullptr;
    p.S_loc = p.G_cum = p.G_tot = nullptr; p.S_init = nullptr;
    p.B = d->B; p.P = d->P; p.H = d->H;
    set_length(p, d->L);
    p.scale = d->scale; p.kscale = 1.f;
    p.sb = d->stride_b; p.st = d->stride_t; p.sh = d->stride_h;
    p.vb = d->vstride_b; p.vt = d->vstride_t; p.vh = d->vstride_h;
}

// Tokens per workgroup of the correction: the largest of cap..64 (powers of two) that divides L, or, when the
// segments need not divide evenly (a ragged L, unequal segments), that is not above L - the last workgroup
// of a segment then has fewer blocks.  1024 where the call stops at the vanished decay (fewer workgroups
// that find nothing to do), 256 where it streams every token (measured 4 % faster there).
static void set_apply_share(zeco::ApplyParams &p, int L, int cap, bool divide) {
    int tpw = cap;
    if (divide) {
        while (tpw > 64 && L % tpw != 0) tpw >>= 1;
    } else {
        while (tpw > 64 && tpw > L) tpw >>= 1;
    }
    p.tokens_per_wg = tpw;
    p.wgs_per_seg = (64 * p.n_chunks + tpw - 1) / tpw;
}

// Correction over P segments of L tokens each (the caller's, or the pieces of a fused call).
static void fill_apply_params(zeco::ApplyParams &p, const zeco_gla_desc *d, int P, int L) {
    p.B = d->B; p.P = P; p.H = d->H; p.L = L;
    p.p0 = 0; p.gate_per_head = d->g_per_head; p.dense = 0;
    p.n_chunks = chunks_of(L); p.pad = 64 * p.n_chunks - L;
    set_apply_share(p, L, 1024, p.pad == 0);
    p.scale = d->scale;
    p.sb = d->stride_b; p.st = d->stride_t; p.sh = d->stride_h;
    p.vb = d->vstride_b; p.vt = d->vstride_t; p.vh = d->vstride_h;
}

zeco_status zeco_gla_local_state(const zeco_gla_desc *d, const void *k, const void *v, const void *g,
                                 float *S_loc, float *G_tot, void *stream) {
    const zeco_status st = check_desc(d, true);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    if (!k || !v || !g || !S_loc || !G_tot) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(k) || !aligned16(v) || !aligned16(g) || !aligned16(S_loc) || !aligned16(G_tot))
        return ZECO_ERR_INVALID_ARG;
    zeco::ChunkParams p;
    fill_chunk_params(p, d);
    p.k = k; p.v = v; p.g = g; p.S_loc = S_loc; p.G_tot = G_tot;
    return from_hip(launch_phase(p, d, 1, static_cast<hipStream_t>(stream)));
}

zeco_status zeco_gla_fwd_from_state(const zeco_gla_desc *d, const void *q, const void *k, const void *v,
                                    const void *g, const float *S_init, void *o, void *stream) {
    const zeco_status st = check_desc(d, true);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    if (!q || !k || !v || !g || !S_init || !o) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g) || !aligned16(S_init) ||
        !aligned16(o))
        return ZECO_ERR_INVALID_ARG;
    zeco::ChunkParams p;
    fill_chunk_params(p, d);
    p.q = q; p.k = k; p.v = v; p.g = g; p.o = o; p.S_init = S_init;
    return from_hip(launch_phase(p, d, 2, static_cast<hipStream_t>(stream)));
}

// Pieces each segment is cut into by zeco_gla_fused_fwd: up to 256 streams, at least 256 tokens each.
static int fused_pieces(const zeco_gla_desc *d) {
    const long long streams = (long long)d->B * d->P * d->H;
    // as many workgroups as fit the 256 compute units in one round, not more; the fp32 kernels' tiles shrink
    // with the chunk length, and 64 / C of their workgroups share a compute unit
    const long long slots = 256 * (d->io_dtype == ZECO_F32 ? 64 / d->C : 1);
    int S = 1;
    while (streams * S * 2 <= slots && halves_evenly(d->L, S) && d->L / (2 * S) >= 256) S *= 2;
    return S;
}

static int bwd_pieces(const zeco_gla_desc *d);

// Workspace of zeco_gla_fused_fwd, in floats: piece states S_loc [n], S_init [n], their G_tot [n], the
// cumulative decay of the CORRECT schedule (per chunk and channel, or per token with per-head gates), and
// the scratch of the piece scan where it runs as a tree.
struct FwdLayout {
    size_t n, states, off_Sinit, off_Gtot, off_decay, off_tree, total;
};
static FwdLayout fwd_layout(const zeco_gla_desc *d, int S) {
    FwdLayout w;
    const size_t gd = d->g_per_head ? 1 : d->d_k;
    w.n = (size_t)d->P * S * d->B * d->H;
    w.states = w.n * d->d_k * d->d_v;
    w.off_Sinit = w.states;
    w.off_Gtot = 2 * w.states;
    w.off_decay = w.off_Gtot + ((w.n * gd + 3) & ~(size_t)3);
    const size_t decay = d->g_per_head ? (size_t)d->B * d->P * d->L * d->H
                                       : (size_t)d->B * d->P * S * chunks_of(d->L / S) * d->H * d->d_k;
    w.off_tree = w.off_decay + ((decay + 3) & ~(size_t)3);
    w.total = w.off_tree + chain_scratch_floats(d->P * S, d->B * d->H, d->d_k, d->d_v, d->g_per_head);
    return w;
}

size_t zeco_gla_fused_fwd_workspace(const zeco_gla_desc *desc) {
    if (check_desc(desc, true) != ZECO_OK) return 0;
    return fwd_layout(desc, fused_pieces(desc)).total * sizeof(float);
}

zeco_status zeco_gla_fused_fwd(const zeco_gla_desc *d, const void *q, const void *k, const void *v,
                               const void *g, const float *S0, void *o, float *S_last, float *S_save,
                               int32_t schedule, void *workspace, size_t workspace_bytes, void *stream) {
    const zeco_status st = check_desc(d, true);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    if (!q || !k || !v || !g || !o || !workspace) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g) || !aligned16(o) ||
        !aligned16(S0) || !aligned16(S_last) || !aligned16(S_save) || !aligned16(workspace))
        return ZECO_ERR_INVALID_ARG;
    if (schedule != ZECO_SCHEDULE_AUTO && schedule != ZECO_SCHEDULE_TWO_PHASE && schedule != ZECO_SCHEDULE_CORRECT)
        return ZECO_ERR_INVALID_ARG;
    // fp32: the two phases of Alg. 1 only (no chunk-decay correction, no states saved for a backward)
    if (d->io_dtype != ZECO_BF16 && S_save) return ZECO_ERR_UNSUPPORTED;
    const bool can_correct = d->io_dtype == ZECO_BF16;
    if (schedule == ZECO_SCHEDULE_CORRECT && !can_correct) return ZECO_ERR_UNSUPPORTED;
    if (workspace_bytes < zeco_gla_fused_fwd_workspace(d)) return ZECO_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int S = fused_pieces(d);
    const FwdLayout w = fwd_layout(d, S);
    float *Sloc = static_cast<float *>(workspace), *Sinit = Sloc + w.off_Sinit, *Gtot = Sloc + w.off_Gtot;
    float *Gchunk = Sloc + w.off_decay, *tree = Sloc + w.off_tree;
    // With S_save the scan writes the states entering the pieces, and the end state after them, straight into
    // it: the backward works on the same pieces and reads them there (S_save [n pieces + 1 slot per (b, h)]).
    if (S_save) Sinit = S_save;
    float *save_last = S_save ? S_save + w.states : nullptr;

    zeco::ChunkParams p;
    fill_chunk_params(p, d);
    p.P = d->P * S; set_length(p, d->L / S);
    const bool correct = schedule == ZECO_SCHEDULE_CORRECT || (schedule == ZECO_SCHEDULE_AUTO && can_correct && p.L >= 4096);

    // first pass: the pieces from the zero state - with their local outputs and the cumulative decay per chunk
    // (per token with per-head gates, whose G_cum is 4 bytes per token and head), or their end states only
    p.k = k; p.v = v; p.g = g; p.S_loc = Sloc; p.G_tot = Gtot;
    hipError_t e;
    if (correct) {
        p.q = q; p.o = o;
        if (d->g_per_head) p.G_cum = Gchunk; else p.G_chunk = Gchunk;
        e = zeco::launch_chunk_bf16(p, d->d_k, d->d_v, chunk_gate(d), d->g_per_head ? 0 : 6, s);
    } else {
        e = launch_phase(p, d, 1, s);
    }
    if (e != hipSuccess) return ZECO_ERR_HIP;

    zeco::ScanParams sp;
    sp.S_loc = Sloc; sp.G_tot = Gtot; sp.S0 = S0; sp.S_init = Sinit; sp.S_last = S_save ? save_last : S_last;
    sp.P = p.P; sp.groups = 1; sp.BH = d->B * d->H; sp.d_k = d->d_k; sp.d_v = d->d_v;
    sp.rows_per_block = d->d_k / 16; sp.gate_per_head = d->g_per_head;
    if ((e = launch_scan_chain(sp, tree, s)) != hipSuccess) return ZECO_ERR_HIP;
    if (S_save && S_last) {
        e = zeco::launch_copy(S_last, save_last, (size_t)d->B * d->H * d->d_k * d->d_v * sizeof(float), s);
        if (e != hipSuccess) return ZECO_ERR_HIP;
    }

    if (correct) {   // correction of the pieces' heads
        zeco::ApplyParams ap;
        fill_apply_params(ap, d, p.P, p.L);
        ap.q = q; ap.S_init = Sinit; ap.o = o;
        ap.p0 = S0 ? 0 : 1;
        if (d->g_per_head) {
            ap.G_cum = Gchunk;
            return from_hip(zeco::launch_apply_bf16(ap, d->d_k, d->d_v, s));
        }
        ap.g = g; ap.g_bf16 = d->g_dtype == ZECO_BF16; ap.G_chunk = Gchunk;
        return from_hip(zeco::launch_apply_cd_bf16(ap, d->d_k, d->d_v, s));
    }
    p.q = q; p.o = o; p.S_init = Sinit; p.S_loc = nullptr; p.G_tot = nullptr;   // output pass from the scanned states
    return from_hip(launch_phase(p, d, 2, s));
}

// ---- backward (App. A.4) ------------------------------------------------------------------------------
// The gradient passes over `P` pieces of `L` tokens.  dQ from the forward states; with `dS_loc` it also
// emits every piece's state gradient from dS = 0 (and with `G_tot_out` its total log decay), which is
// what the reverse scan chains into dS_in.
static void fill_bwd_params(zeco::BwdQKParams &b, const zeco_gla_desc *d, int P, int L, const void *g,
                            float *dg, const float *S_init, const float *S_last) {
    b.g = g; b.B = d->B; b.P = P; b.H = d->H; b.L = L; b.n_chunks = chunks_of(L); b.pad = 64 * b.n_chunks - L;
    b.sb = d->stride_b; b.st = d->stride_t; b.sh = d->stride_h;
    b.vb = d->vstride_b; b.vt = d->vstride_t; b.vh = d->vstride_h;
    b.dg = dg; b.S_init = S_init; b.S_last = S_last;
}

// Checkpoints of the forward state per (batch, segment, head) that re-anchor dG: one at every 8th chunk
// boundary inside a segment of (at most) L tokens.
static int bwd_checkpoints(int L) { return (chunks_of(L) - 1) / 8; }
static size_t bwd_checkpoint_floats(const zeco_gla_desc *d, int P, int L) {
    return (size_t)d->B * P * d->H * bwd_checkpoints(L) * d->d_k * d->d_v;
}

static zeco_status bwd_dq_pass(const zeco_gla_desc *d, int P, int L, const void *q, const void *k,
                               const void *v, const void *g, const void *dO, const float *S_init,
                               const float *S_last, void *dq, float *dg, float *dS_loc, float *G_tot_out,
                               float *S_ck, hipStream_t s, const int64_t *seg_start = nullptr, int64_t T = 0) {
    zeco::BwdQKParams b;
    fill_bwd_params(b, d, P, L, g, dg, S_init, S_last);
    if (S_ck && bwd_checkpoints(L) > 0) { b.S_ck = S_ck; b.n_ck = bwd_checkpoints(L); b.short_last = 1; }
    b.seg_start = reinterpret_cast<const long long *>(seg_start); b.T = T;
    b.x = dO; b.y = v; b.z = k; b.z2 = q; b.out = dq; b.W_init = S_init; b.zscale = 1.f; b.oscale = d->scale;
    if (d->io_dtype == ZECO_F32) {
        // the fp32 kernels: dQ, and the segments' state gradients from dS = 0 as a pass of their own
        if (zeco::launch_bwd_qk_f32(b, d->d_k, d->d_v, d->C, false, s) != hipSuccess) return ZECO_ERR_HIP;
        if (!dS_loc) return ZECO_OK;
        zeco::ChunkParams c;
        fill_chunk_params(c, d);
        c.P = P; set_length_c(c, L, d->C);
        c.seg_start = reinterpret_cast<const long long *>(seg_start); c.T = T;
        c.k = q; c.v = dO; c.g = g; c.S_loc = dS_loc; c.G_tot = G_tot_out; c.scale = 1.f; c.kscale = d->scale;
        return from_hip(zeco::launch_chunk_f32(c, d->d_k, d->d_v, d->C, 3, s));
    }
    b.dS_loc = dS_loc; b.G_tot_out = G_tot_out; b.qscale = d->scale;
    return from_hip(zeco::launch_bwd_qk(b, d->d_k, d->d_v, gate_mode(d), false, s));
}

// dV and dK from the state gradients entering the pieces, dG from all of them (after the dQ pass, whose
// q .* dq left in dg the dK pass consumes).
static zeco_status bwd_dv_dk_passes(const zeco_gla_desc *d, int P, int L, const void *q, const void *k,
                                    const void *v, const void *g, const void *dO, const float *S_init,
                                    const float *S_last, const float *dS_in, void *dk, void *dv,
                                    float *dg, float *S_ck, hipStream_t s, const int64_t *seg_start = nullptr,
                                    int64_t T = 0) {
    const int gb = gate_mode(d);
    zeco::ChunkParams c;
    fill_chunk_params(c, d);
    c.P = P; set_length(c, L);
    c.seg_start = reinterpret_cast<const long long *>(seg_start); c.T = T;
    c.q = k; c.k = q; c.v = dO; c.g = g; c.o = dv; c.S_init = dS_in; c.scale = 1.f; c.kscale = d->scale;
    if (launch_phase(c, d, 4, s) != hipSuccess) return ZECO_ERR_HIP;

    zeco::BwdQKParams b;
    fill_bwd_params(b, d, P, L, g, dg, S_init, S_last);
    b.seg_start = reinterpret_cast<const long long *>(seg_start); b.T = T;
    b.x = v; b.y = dO; b.z = q; b.z2 = k; b.out = dk; b.W_init = dS_in; b.zscale = d->scale; b.oscale = 1.f;
    if (S_ck && bwd_checkpoints(L) > 0) { b.S_ck = S_ck; b.n_ck = bwd_checkpoints(L); }
    if (d->io_dtype == ZECO_F32) return from_hip(zeco::launch_bwd_qk_f32(b, d->d_k, d->d_v, d->C, true, s));
    return from_hip(zeco::launch_bwd_qk(b, d->d_k, d->d_v, gb, true, s));
}

zeco_status zeco_gla_bwd_dstate(const zeco_gla_desc *d, const void *q, const void *g, const void *dO,
                                float *dS_loc, void *stream) {
    const zeco_status st = check_desc(d, true);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    if (!q || !g || !dO || !dS_loc) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(g) || !aligned16(dO) || !aligned16(dS_loc)) return ZECO_ERR_INVALID_ARG;
    zeco::ChunkParams p;
    fill_chunk_params(p, d);
    p.k = q; p.v = dO; p.g = g; p.S_loc = dS_loc; p.kscale = d->scale;
    return from_hip(launch_phase(p, d, 3, static_cast<hipStream_t>(stream)));
}

size_t zeco_gla_bwd_from_state_workspace(const zeco_gla_desc *desc) {
    if (check_desc(desc, true) != ZECO_OK) return 0;
    return bwd_checkpoint_floats(desc, desc->P, desc->L) * sizeof(float);
}

zeco_status zeco_gla_bwd_from_state(const zeco_gla_desc *d, const void *q, const void *k, const void *v,
                                    const void *g, const void *dO, const float *S_init, const float *S_last,
                                    const float *dS_in, void *dq, void *dk, void *dv, float *dg,
                                    void *workspace, size_t workspace_bytes, void *stream) {
    const zeco_status st = check_desc(d, true);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    const size_t need = zeco_gla_bwd_from_state_workspace(d);
    if (workspace_bytes < need) return ZECO_ERR_WORKSPACE;
    if (need && (!workspace || !aligned16(workspace))) return ZECO_ERR_INVALID_ARG;
    if (!q || !k || !v || !g || !dO || !S_init || !S_last || !dS_in || !dq || !dk || !dv || !dg)
        return ZECO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g) || !aligned16(dO) ||
        !aligned16(S_init) || !aligned16(S_last) || !aligned16(dS_in) || !aligned16(dq) || !aligned16(dk) ||
        !aligned16(dv) || !aligned16(dg))
        return ZECO_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *S_ck = need ? static_cast<float *>(workspace) : nullptr;
    const zeco_status sq = bwd_dq_pass(d, d->P, d->L, q, k, v, g, dO, S_init, S_last, dq, dg, nullptr, nullptr, S_ck, s);
    if (sq != ZECO_OK) return sq;
    return bwd_dv_dk_passes(d, d->P, d->L, q, k, v, g, dO, S_init, S_last, dS_in, dk, dv, dg, S_ck, s);
}

// Pieces each segment is cut into by zeco_gla_fused_bwd: the forward's (as many streams as fill the compute units
// once, whole chunks or equal ragged pieces).  The gate gradient, a running sum of nearly cancelling terms whose
// bf16 rounding noise grows with the square root of the run length, is re-anchored every 512 tokens inside a
// piece from the forward-state checkpoints of the dQ pass, so the pieces need not be short for its sake: cut
// down to 512 tokens each (as this call once did) the same passes spend 12-20 % more time on pipeline prologues,
// on the states of 64 times as many pieces and on scans over them (c3 3.58 -> 3.12 ms, c4 28.2 -> 22.6 ms,
// c5 113 -> 93.5 ms).
static int bwd_pieces(const zeco_gla_desc *d) { return fused_pieces(d); }

// Workspace of zeco_gla_fused_bwd, in floats: forward piece states S_loc [n], S_init [n + one more
// slot per (b,h) for the final state], their G_tot [n]; state gradients dS_loc [n], dS_in [n].
struct BwdLayout {
    size_t n, state, off_Sloc, off_Sinit, off_Gtot, off_dSloc, off_dSin, off_tree, off_ck, total;
};
static BwdLayout bwd_layout(const zeco_gla_desc *d, int S) {
    BwdLayout w;
    const size_t bh = (size_t)d->B * d->H;
    w.n = (size_t)d->P * S * bh;
    w.state = (size_t)d->d_k * d->d_v;
    w.off_Sloc = 0;
    w.off_Sinit = w.off_Sloc + w.n * w.state;
    w.off_Gtot = w.off_Sinit + (w.n + bh) * w.state;
    w.off_dSloc = w.off_Gtot + w.n * d->d_k;
    w.off_dSin = w.off_dSloc + w.n * w.state;
    w.off_tree = w.off_dSin + w.n * w.state;   // scratch of the two piece scans where they run as trees
    // checkpoints inside pieces that could not be cut down to 512 tokens (a chunk count without a fitting factor)
    w.off_ck = w.off_tree + chain_scratch_floats(d->P * S, d->B * d->H, d->d_k, d->d_v, d->g_per_head);
    w.total = w.off_ck + bwd_checkpoint_floats(d, d->P * S, d->L / S);
    return w;
}

size_t zeco_gla_saved_states_bytes(const zeco_gla_desc *desc) {
    if (check_desc(desc, true) != ZECO_OK || desc->io_dtype != ZECO_BF16) return 0;
    const BwdLayout w = bwd_layout(desc, bwd_pieces(desc));
    return (w.n + (size_t)desc->B * desc->H) * w.state * sizeof(float);
}

size_t zeco_gla_fused_bwd_workspace(const zeco_gla_desc *desc) {
    if (check_desc(desc, true) != ZECO_OK) return 0;
    return bwd_layout(desc, bwd_pieces(desc)).total * sizeof(float);
}

zeco_status zeco_gla_fused_bwd(const zeco_gla_desc *d, const void *q, const void *k, const void *v,
                               const void *g, const void *dO, const float *S0, const float *dS_T,
                               const float *S_saved, void *dq, void *dk, void *dv, float *dg, float *dS0,
                               void *workspace, size_t workspace_bytes, void *stream) {
    const zeco_status st = check_desc(d, true);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    if (!q || !k || !v || !g || !dO || !dq || !dk || !dv || !dg || !workspace) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g) || !aligned16(dO) ||
        !aligned16(S0) || !aligned16(dS_T) || !aligned16(S_saved) || !aligned16(dq) || !aligned16(dk) || !aligned16(dv) ||
        !aligned16(dg) || !aligned16(dS0) || !aligned16(workspace))
        return ZECO_ERR_INVALID_ARG;
    if (d->io_dtype != ZECO_BF16 && S_saved) return ZECO_ERR_UNSUPPORTED;   // (the fp32 forward saves no states)
    if (workspace_bytes < zeco_gla_fused_bwd_workspace(d)) return ZECO_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int S = bwd_pieces(d);
    const BwdLayout w = bwd_layout(d, S);
    float *ws = static_cast<float *>(workspace);
    float *Sloc = ws + w.off_Sloc, *Sinit = ws + w.off_Sinit, *Gtot = ws + w.off_Gtot;
    float *dSloc = ws + w.off_dSloc, *dSin = ws + w.off_dSin;
    float *Slast = Sinit + w.n * w.state;
    const int gb = gate_mode(d);
    const int P = d->P * S, L = d->L / S;

    zeco::ChunkParams p;
    fill_chunk_params(p, d);
    p.P = P; set_length(p, L);
    zeco::ScanParams sp;
    sp.P = P; sp.groups = 1; sp.BH = d->B * d->H; sp.d_k = d->d_k; sp.d_v = d->d_v;
    sp.rows_per_block = d->d_k / 16; sp.gate_per_head = d->g_per_head;
    hipError_t e;
    const float *Sin = Sinit, *Sl = Slast;
    if (S_saved) {
        // forward states at the piece boundaries as the forward left them
        Sin = S_saved; Sl = S_saved + w.n * w.state;
    } else {
        // recomputed: phase 1 of the forward and its scan
        p.k = k; p.v = v; p.g = g; p.S_loc = Sloc; p.G_tot = Gtot;
        if ((e = launch_phase(p, d, 1, s)) != hipSuccess) return ZECO_ERR_HIP;
        sp.S_loc = Sloc; sp.G_tot = Gtot; sp.S0 = S0; sp.S_init = Sinit; sp.S_last = Slast;
        if ((e = launch_scan_chain(sp, ws + w.off_tree, s)) != hipSuccess) return ZECO_ERR_HIP;
    }

    // dQ from the forward states; the same pass leaves every piece's state gradient from dS = 0 (and
    // the pieces' total decays when the forward state pass did not run), which the reverse scan chains
    // from the last piece to the first
    float *S_ck = bwd_checkpoints(L) > 0 ? ws + w.off_ck : nullptr;
    zeco_status zs = bwd_dq_pass(d, P, L, q, k, v, g, dO, Sin, Sl, dq, dg, dSloc, S_saved ? Gtot : nullptr, S_ck, s);
    if (zs != ZECO_OK) return zs;
    sp.S_loc = dSloc; sp.G_tot = Gtot; sp.S0 = dS_T; sp.S_init = dSin; sp.S_last = dS0; sp.reverse = 1;
    if ((e = launch_scan_chain(sp, ws + w.off_tree, s)) != hipSuccess) return ZECO_ERR_HIP;

    return bwd_dv_dk_passes(d, P, L, q, k, v, g, dO, Sin, Sl, dSin, dk, dv, dg, S_ck, s);
}

zeco_status zeco_state_scan(int32_t P, int32_t BH, int32_t d_k, int32_t d_v, int32_t K_blocks,
                            const float *S_loc, const float *G_tot, const float *S0, float *S_init,
                            float *S_last, int32_t direction, int32_t gate_per_head, void *stream) {
    if (P <= 0 || BH < 0 || d_k <= 0 || d_v <= 0 || K_blocks <= 0) return ZECO_ERR_INVALID_ARG;
    if (d_k % K_blocks != 0) return ZECO_ERR_INVALID_ARG;
    if (direction != 0 && direction != 1) return ZECO_ERR_INVALID_ARG;
    if (gate_per_head != 0 && gate_per_head != 1) return ZECO_ERR_INVALID_ARG;
    if (BH == 0) return ZECO_OK;   // empty batch: nothing to do
    if (!S_loc || !G_tot || !S_init) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(S_loc) || !aligned16(S_init) || !aligned16(S0) || !aligned16(S_last) ||
        (reinterpret_cast<uintptr_t>(G_tot) & 3u))
        return ZECO_ERR_INVALID_ARG;
    if ((int64_t)BH * K_blocks > (int64_t)1 << 30) return ZECO_ERR_INVALID_ARG;
    if (d_v % 4 != 0) return ZECO_ERR_UNSUPPORTED;

    zeco::ScanParams p;
    p.reverse = direction; p.gate_per_head = gate_per_head;
    p.S_loc = S_loc; p.G_tot = G_tot; p.S0 = S0; p.S_init = S_init; p.S_last = S_last;
    p.P = P; p.BH = BH; p.d_k = d_k; p.d_v = d_v; p.rows_per_block = d_k / K_blocks; p.groups = 1;
    return from_hip(zeco::launch_scan(p, static_cast<hipStream_t>(stream)));
}

// ---- two-level (tree of depth two) scan ----------------------------------------------------------------
size_t zeco_state_scan_tree_workspace(int32_t P, int32_t BH, int32_t d_k, int32_t d_v, int32_t gate_per_head) {
    if (P <= 0 || BH <= 0 || d_k <= 0 || d_v <= 0) return 0;
    return tree_floats(P, BH, d_k, d_v, gate_per_head) * sizeof(float);
}

zeco_status zeco_state_scan_tree(int32_t P, int32_t BH, int32_t d_k, int32_t d_v, const float *S_loc,
                                 const float *G_tot, const float *S0, float *S_init, float *S_last,
                                 int32_t direction, int32_t gate_per_head, void *workspace,
                                 size_t workspace_bytes, void *stream) {
    const int g = P > 0 ? tree_group(P) : 0;
    if (P <= 0 || g == P || BH <= 0)   // nothing to split (or an argument the plain scan reports)
        return zeco_state_scan(P, BH, d_k, d_v, d_k >= 16 && d_k % 16 == 0 ? 16 : 1, S_loc, G_tot, S0, S_init, S_last,
                               direction, gate_per_head, stream);
    if (d_k <= 0 || d_v <= 0 || d_k % 16 != 0) return ZECO_ERR_INVALID_ARG;
    if (direction != 0 && direction != 1) return ZECO_ERR_INVALID_ARG;
    if (gate_per_head != 0 && gate_per_head != 1) return ZECO_ERR_INVALID_ARG;
    if (!S_loc || !G_tot || !S_init) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(S_loc) || !aligned16(S_init) || !aligned16(S0) || !aligned16(S_last) ||
        (reinterpret_cast<uintptr_t>(G_tot) & 3u))
        return ZECO_ERR_INVALID_ARG;
    if ((int64_t)BH * 16 > (int64_t)1 << 30 || P / g > 65535) return ZECO_ERR_INVALID_ARG;
    if (d_v % 4 != 0) return ZECO_ERR_UNSUPPORTED;
    if (workspace_bytes < zeco_state_scan_tree_workspace(P, BH, d_k, d_v, gate_per_head)) return ZECO_ERR_WORKSPACE;
    if (!workspace || !aligned16(workspace)) return ZECO_ERR_INVALID_ARG;

    zeco::ScanParams p;
    p.reverse = direction; p.gate_per_head = gate_per_head;
    p.BH = BH; p.d_k = d_k; p.d_v = d_v; p.rows_per_block = d_k / 16;
    p.S_loc = S_loc; p.G_tot = G_tot; p.S0 = S0; p.S_init = S_init; p.S_last = S_last;
    p.P = P; p.groups = 1;
    return from_hip(launch_scan_tree(p, static_cast<float *>(workspace), static_cast<hipStream_t>(stream)));
}

size_t zeco_state_scan_tree_static_limit(void) { return kStaticScratchBytes; }

zeco_status zeco_state_scan_tree_static(int32_t P, int32_t BH, int32_t d_k, int32_t d_v, const float *S_loc,
                                        const float *G_tot, const float *S0, float *S_init, float *S_last,
                                        int32_t direction, int32_t gate_per_head, void *stream) {
    // the size check comes first: it needs nothing but the four sizes
    const size_t need = zeco_state_scan_tree_workspace(P, BH, d_k, d_v, gate_per_head);
    if (need > kStaticScratchBytes) return ZECO_ERR_SCRATCH_LIMIT;
    if (need == 0)   // the chain is not split (or an argument is bad, which the workspace variant reports)
        return zeco_state_scan_tree(P, BH, d_k, d_v, S_loc, G_tot, S0, S_init, S_last, direction, gate_per_head,
                                    nullptr, 0, stream);
    // Validate what zeco_state_scan_tree validates before the first HIP call (the lookup below is one).
    if (d_k % 16 != 0 || (direction != 0 && direction != 1) || (gate_per_head != 0 && gate_per_head != 1))
        return ZECO_ERR_INVALID_ARG;
    if (!S_loc || !G_tot || !S_init) return ZECO_ERR_INVALID_ARG;
    void *scratch = nullptr;
    if (static_scratch(&scratch) != hipSuccess) return ZECO_ERR_HIP;
    // The three passes write every byte of the scratch they later read (group end states and decay sums, then
    // the states entering the groups), so whatever an earlier call left there does not matter.
    return zeco_state_scan_tree(P, BH, d_k, d_v, S_loc, G_tot, S0, S_init, S_last, direction, gate_per_head,
                                scratch, kStaticScratchBytes, stream);
}

zeco_status zeco_apply_init_state(const zeco_gla_desc *d, const void *q, const float *G_cum,
                                  const float *S_init, void *o, int32_t flags, void *stream) {
    const zeco_status st = check_desc(d, true);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    if (!q || !G_cum || !S_init || !o) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(G_cum) || !aligned16(S_init) || !aligned16(o))
        return ZECO_ERR_INVALID_ARG;
    if (flags & ~(ZECO_APPLY_FIRST_SEGMENT_ZERO | ZECO_APPLY_DENSE)) return ZECO_ERR_INVALID_ARG;

    zeco::ApplyParams p;
    fill_apply_params(p, d, d->P, d->L);
    p.q = q; p.G_cum = G_cum; p.S_init = S_init; p.o = o;
    p.p0 = (flags & ZECO_APPLY_FIRST_SEGMENT_ZERO) ? 1 : 0;
    p.dense = (flags & ZECO_APPLY_DENSE) ? 1 : 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (d->io_dtype == ZECO_F32) return from_hip(zeco::launch_apply_f32(p, d->d_k, d->d_v, s));
    if (p.dense) set_apply_share(p, d->L, 256, p.pad == 0);
    return from_hip(zeco::launch_apply_bf16(p, d->d_k, d->d_v, s));
}

// ---- segments of unequal length ---------------------------------------------------------------------------
static zeco_status check_varlen(const zeco_gla_desc *d, const int64_t *seg_start, int64_t T) {
    const zeco_status st = check_desc(d, true);
    if (st != ZECO_OK) return st;
    if (T < (int64_t)d->P * d->C || T > (int64_t)1 << 40) return ZECO_ERR_INVALID_ARG;
    if (d->B == 0) return ZECO_OK;
    if (!seg_start || (reinterpret_cast<uintptr_t>(seg_start) & 7u)) return ZECO_ERR_INVALID_ARG;
    return ZECO_OK;
}

zeco_status zeco_gla_local_fwd_varlen(const zeco_gla_desc *d, const int64_t *seg_start, int64_t T,
                                      const void *q, const void *k, const void *v, const void *g, void *o,
                                      float *S_loc, float *G_cum, float *G_tot, void *stream) {
    const zeco_status st = check_varlen(d, seg_start, T);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    if (!q || !k || !v || !g || !o || !S_loc || !G_cum || !G_tot) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g) || !aligned16(o) ||
        !aligned16(S_loc) || !aligned16(G_cum) || !aligned16(G_tot))
        return ZECO_ERR_INVALID_ARG;
    static_assert(sizeof(long long) == sizeof(int64_t), "the kernels read the table as long long");
    zeco::ChunkParams p;
    fill_chunk_params(p, d);
    p.q = q; p.k = k; p.v = v; p.g = g; p.o = o;
    p.S_loc = S_loc; p.G_cum = G_cum; p.G_tot = G_tot;
    p.seg_start = reinterpret_cast<const long long *>(seg_start); p.T = T;
    hipStream_t s = static_cast<hipStream_t>(stream);
    return from_hip(launch_phase(p, d, 0, s));
}

zeco_status zeco_apply_init_state_varlen(const zeco_gla_desc *d, const int64_t *seg_start, int64_t T,
                                         const void *q, const float *G_cum, const float *S_init, void *o,
                                         int32_t flags, void *stream) {
    const zeco_status st = check_varlen(d, seg_start, T);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    if (!q || !G_cum || !S_init || !o) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(G_cum) || !aligned16(S_init) || !aligned16(o))
        return ZECO_ERR_INVALID_ARG;
    if (flags & ~(ZECO_APPLY_FIRST_SEGMENT_ZERO | ZECO_APPLY_DENSE)) return ZECO_ERR_INVALID_ARG;
    zeco::ApplyParams p;
    fill_apply_params(p, d, d->P, d->L);
    p.dense = (flags & ZECO_APPLY_DENSE) ? 1 : 0;
    // a launch sized for the longest segment allowed; the lengths need not divide into the workgroups' shares
    set_apply_share(p, d->L, (p.dense && d->io_dtype == ZECO_BF16) ? 256 : 1024, false);
    p.q = q; p.G_cum = G_cum; p.S_init = S_init; p.o = o;
    p.seg_start = reinterpret_cast<const long long *>(seg_start); p.T = T;
    p.p0 = (flags & ZECO_APPLY_FIRST_SEGMENT_ZERO) ? 1 : 0;
    p.dense = (flags & ZECO_APPLY_DENSE) ? 1 : 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (d->io_dtype == ZECO_F32) return from_hip(zeco::launch_apply_f32(p, d->d_k, d->d_v, s));
    return from_hip(zeco::launch_apply_bf16(p, d->d_k, d->d_v, s));
}

// The two phases of Alg. 1's own schedule over the same table (bf16 only, like the equal-length calls).
zeco_status zeco_gla_local_state_varlen(const zeco_gla_desc *d, const int64_t *seg_start, int64_t T,
                                        const void *k, const void *v, const void *g, float *S_loc,
                                        float *G_tot, void *stream) {
    const zeco_status st = check_varlen(d, seg_start, T);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    if (!k || !v || !g || !S_loc || !G_tot) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(k) || !aligned16(v) || !aligned16(g) || !aligned16(S_loc) || !aligned16(G_tot))
        return ZECO_ERR_INVALID_ARG;
    zeco::ChunkParams p;
    fill_chunk_params(p, d);
    p.k = k; p.v = v; p.g = g; p.S_loc = S_loc; p.G_tot = G_tot;
    p.seg_start = reinterpret_cast<const long long *>(seg_start); p.T = T;
    return from_hip(launch_phase(p, d, 1, static_cast<hipStream_t>(stream)));
}

zeco_status zeco_gla_fwd_from_state_varlen(const zeco_gla_desc *d, const int64_t *seg_start, int64_t T,
                                           const void *q, const void *k, const void *v, const void *g,
                                           const float *S_init, void *o, void *stream) {
    const zeco_status st = check_varlen(d, seg_start, T);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    if (!q || !k || !v || !g || !S_init || !o) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g) || !aligned16(S_init) || !aligned16(o))
        return ZECO_ERR_INVALID_ARG;
    zeco::ChunkParams p;
    fill_chunk_params(p, d);
    p.q = q; p.k = k; p.v = v; p.g = g; p.o = o; p.S_init = S_init;
    p.seg_start = reinterpret_cast<const long long *>(seg_start); p.T = T;
    return from_hip(launch_phase(p, d, 2, static_cast<hipStream_t>(stream)));
}

// The backward's building blocks over the same table (bf16 only, like the equal-length calls).
zeco_status zeco_gla_bwd_dstate_varlen(const zeco_gla_desc *d, const int64_t *seg_start, int64_t T,
                                       const void *q, const void *g, const void *dO, float *dS_loc,
                                       void *stream) {
    const zeco_status st = check_varlen(d, seg_start, T);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    if (!q || !g || !dO || !dS_loc) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(g) || !aligned16(dO) || !aligned16(dS_loc)) return ZECO_ERR_INVALID_ARG;
    zeco::ChunkParams p;
    fill_chunk_params(p, d);
    p.k = q; p.v = dO; p.g = g; p.S_loc = dS_loc; p.kscale = d->scale;
    p.seg_start = reinterpret_cast<const long long *>(seg_start); p.T = T;
    return from_hip(launch_phase(p, d, 3, static_cast<hipStream_t>(stream)));
}

zeco_status zeco_gla_bwd_from_state_varlen(const zeco_gla_desc *d, const int64_t *seg_start, int64_t T,
                                           const void *q, const void *k, const void *v, const void *g,
                                           const void *dO, const float *S_init, const float *S_last,
                                           const float *dS_in, void *dq, void *dk, void *dv, float *dg,
                                           void *workspace, size_t workspace_bytes, void *stream) {
    const zeco_status st = check_varlen(d, seg_start, T);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    const size_t need = zeco_gla_bwd_from_state_workspace(d);   // sized for the bound on the lengths
    if (workspace_bytes < need) return ZECO_ERR_WORKSPACE;
    if (need && (!workspace || !aligned16(workspace))) return ZECO_ERR_INVALID_ARG;
    if (!q || !k || !v || !g || !dO || !S_init || !S_last || !dS_in || !dq || !dk || !dv || !dg)
        return ZECO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g) || !aligned16(dO) ||
        !aligned16(S_init) || !aligned16(S_last) || !aligned16(dS_in) || !aligned16(dq) || !aligned16(dk) ||
        !aligned16(dv) || !aligned16(dg))
        return ZECO_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *S_ck = need ? static_cast<float *>(workspace) : nullptr;
    const zeco_status sq = bwd_dq_pass(d, d->P, d->L, q, k, v, g, dO, S_init, S_last, dq, dg, nullptr, nullptr, S_ck, s,
                                       seg_start, T);
    if (sq != ZECO_OK) return sq;
    return bwd_dv_dk_passes(d, d->P, d->L, q, k, v, g, dO, S_init, S_last, dS_in, dk, dv, dg, S_ck, s, seg_start, T);
}

// The whole forward and the whole backward over the same table, each in one call: the phases of Alg. 1 (states,
// scan, output pass) and of the backward (forward states and their scan, dQ pass with the segments' state
// gradients, reverse scan, dV and dK passes) on the segments as given.
struct VarlenLayout {   // workspace carve-up, in floats
    size_t state, off_Sinit, off_Gtot, off_dSloc, off_dSin, off_ck, total;
};
static VarlenLayout varlen_layout(const zeco_gla_desc *d, bool backward) {
    VarlenLayout w;
    const size_t n = (size_t)d->P * d->B * d->H, bh = (size_t)d->B * d->H;
    w.state = (size_t)d->d_k * d->d_v;
    w.off_Sinit = n * w.state;                          // S_loc [n] first
    w.off_Gtot = w.off_Sinit + (n + bh) * w.state;      // S_init [n] and one more slot: the final state
    w.off_dSloc = w.off_Gtot + ((n * (d->g_per_head ? 1 : d->d_k) + 3) & ~(size_t)3);
    if (!backward) { w.off_dSin = w.off_ck = w.total = w.off_dSloc; return w; }
    w.off_dSin = w.off_dSloc + n * w.state;
    w.off_ck = w.off_dSin + n * w.state;
    w.total = w.off_ck + bwd_checkpoint_floats(d, d->P, d->L);
    return w;
}

size_t zeco_gla_fused_fwd_varlen_workspace(const zeco_gla_desc *desc) {
    if (check_desc(desc, true) != ZECO_OK) return 0;
    return varlen_layout(desc, false).total * sizeof(float);
}
size_t zeco_gla_fused_bwd_varlen_workspace(const zeco_gla_desc *desc) {
    if (check_desc(desc, true) != ZECO_OK) return 0;
    return varlen_layout(desc, true).total * sizeof(float);
}

zeco_status zeco_gla_fused_fwd_varlen(const zeco_gla_desc *d, const int64_t *seg_start, int64_t T, const void *q,
                                      const void *k, const void *v, const void *g, const float *S0, void *o,
                                      float *S_last, void *workspace, size_t workspace_bytes, void *stream) {
    const zeco_status st = check_varlen(d, seg_start, T);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    if (!q || !k || !v || !g || !o || !workspace) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g) || !aligned16(o) || !aligned16(S0) ||
        !aligned16(S_last) || !aligned16(workspace))
        return ZECO_ERR_INVALID_ARG;
    if (workspace_bytes < zeco_gla_fused_fwd_varlen_workspace(d)) return ZECO_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const VarlenLayout w = varlen_layout(d, false);
    float *Sloc = static_cast<float *>(workspace), *Sinit = Sloc + w.off_Sinit, *Gtot = Sloc + w.off_Gtot;
    zeco::ChunkParams p;
    fill_chunk_params(p, d);
    p.seg_start = reinterpret_cast<const long long *>(seg_start); p.T = T;
    p.k = k; p.v = v; p.g = g; p.S_loc = Sloc; p.G_tot = Gtot;
    if (launch_phase(p, d, 1, s) != hipSuccess) return ZECO_ERR_HIP;
    zeco::ScanParams sp;
    sp.S_loc = Sloc; sp.G_tot = Gtot; sp.S0 = S0; sp.S_init = Sinit; sp.S_last = S_last;
    sp.P = d->P; sp.groups = 1; sp.BH = d->B * d->H; sp.d_k = d->d_k; sp.d_v = d->d_v;
    sp.rows_per_block = d->d_k / 16; sp.gate_per_head = d->g_per_head;
    if (zeco::launch_scan(sp, s) != hipSuccess) return ZECO_ERR_HIP;
    p.q = q; p.o = o; p.S_init = Sinit; p.S_loc = nullptr; p.G_tot = nullptr;
    return from_hip(launch_phase(p, d, 2, s));
}

zeco_status zeco_gla_fused_bwd_varlen(const zeco_gla_desc *d, const int64_t *seg_start, int64_t T, const void *q,
                                      const void *k, const void *v, const void *g, const void *dO,
                                      const float *S0, const float *dS_T, void *dq, void *dk, void *dv, float *dg,
                                      float *dS0, void *workspace, size_t workspace_bytes, void *stream) {
    const zeco_status st = check_varlen(d, seg_start, T);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    if (!q || !k || !v || !g || !dO || !dq || !dk || !dv || !dg || !workspace) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g) || !aligned16(dO) || !aligned16(S0) ||
        !aligned16(dS_T) || !aligned16(dq) || !aligned16(dk) || !aligned16(dv) || !aligned16(dg) || !aligned16(dS0) ||
        !aligned16(workspace))
        return ZECO_ERR_INVALID_ARG;
    if (workspace_bytes < zeco_gla_fused_bwd_varlen_workspace(d)) return ZECO_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const VarlenLayout w = varlen_layout(d, true);
    const size_t n = (size_t)d->P * d->B * d->H;
    float *ws = static_cast<float *>(workspace);
    float *Sloc = ws, *Sinit = ws + w.off_Sinit, *Slast = Sinit + n * w.state, *Gtot = ws + w.off_Gtot;
    float *dSloc = ws + w.off_dSloc, *dSin = ws + w.off_dSin;
    float *S_ck = bwd_checkpoints(d->L) > 0 ? ws + w.off_ck : nullptr;
    zeco::ChunkParams p;
    fill_chunk_params(p, d);
    p.seg_start = reinterpret_cast<const long long *>(seg_start); p.T = T;
    p.k = k; p.v = v; p.g = g; p.S_loc = Sloc; p.G_tot = Gtot;
    if (launch_phase(p, d, 1, s) != hipSuccess) return ZECO_ERR_HIP;
    zeco::ScanParams sp;
    sp.S_loc = Sloc; sp.G_tot = Gtot; sp.S0 = S0; sp.S_init = Sinit; sp.S_last = Slast;
    sp.P = d->P; sp.groups = 1; sp.BH = d->B * d->H; sp.d_k = d->d_k; sp.d_v = d->d_v;
    sp.rows_per_block = d->d_k / 16; sp.gate_per_head = d->g_per_head;
    if (zeco::launch_scan(sp, s) != hipSuccess) return ZECO_ERR_HIP;
    zeco_status zs = bwd_dq_pass(d, d->P, d->L, q, k, v, g, dO, Sinit, Slast, dq, dg, dSloc, nullptr, S_ck, s, seg_start, T);
    if (zs != ZECO_OK) return zs;
    sp.S_loc = dSloc; sp.S0 = dS_T; sp.S_init = dSin; sp.S_last = dS0; sp.reverse = 1;
    if (zeco::launch_scan(sp, s) != hipSuccess) return ZECO_ERR_HIP;
    return bwd_dv_dk_passes(d, d->P, d->L, q, k, v, g, dO, Sinit, Slast, dSin, dk, dv, dg, S_ck, s, seg_start, T);
}

// ---- chunk-decay form of the local pass and the correction ---------------------------------------------
zeco_status zeco_gla_local_fwd_chunk_decay(const zeco_gla_desc *d, const void *q, const void *k,
                                           const void *v, const void *g, void *o, float *S_loc,
                                           float *G_chunk, float *G_tot, void *stream) {
    const zeco_status st = check_desc(d, true);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    if (!q || !k || !v || !g || !o || !S_loc || !G_chunk || !G_tot) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g) || !aligned16(o) ||
        !aligned16(S_loc) || !aligned16(G_chunk) || !aligned16(G_tot))
        return ZECO_ERR_INVALID_ARG;
    if (d->io_dtype != ZECO_BF16 || d->g_per_head) return ZECO_ERR_UNSUPPORTED;
    zeco::ChunkParams p;
    fill_chunk_params(p, d);
    p.q = q; p.k = k; p.v = v; p.g = g; p.o = o; p.S_loc = S_loc; p.G_tot = G_tot; p.G_chunk = G_chunk;
    return from_hip(zeco::launch_chunk_bf16(p, d->d_k, d->d_v, chunk_gate(d), 6,
                                            static_cast<hipStream_t>(stream)));
}

zeco_status zeco_apply_init_state_chunk_decay(const zeco_gla_desc *d, const void *q, const void *g,
                                              const float *G_chunk, const float *S_init, void *o,
                                              int32_t flags, void *stream) {
    const zeco_status st = check_desc(d, true);
    if (st != ZECO_OK) return st;
    if (d->B == 0) return ZECO_OK;   // empty batch: nothing to do
    if (!q || !g || !G_chunk || !S_init || !o) return ZECO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(g) || !aligned16(G_chunk) || !aligned16(S_init) || !aligned16(o))
        return ZECO_ERR_INVALID_ARG;
    if (flags & ~(ZECO_APPLY_FIRST_SEGMENT_ZERO | ZECO_APPLY_DENSE)) return ZECO_ERR_INVALID_ARG;
    if (d->io_dtype != ZECO_BF16 || d->g_per_head) return ZECO_ERR_UNSUPPORTED;
    zeco::ApplyParams p;
    fill_apply_params(p, d, d->P, d->L);
    p.q = q; p.g = g; p.g_bf16 = d->g_dtype == ZECO_BF16; p.G_chunk = G_chunk; p.S_init = S_init; p.o = o;
    p.p0 = (flags & ZECO_APPLY_FIRST_SEGMENT_ZERO) ? 1 : 0;
    p.dense = (flags & ZECO_APPLY_DENSE) ? 1 : 0;
    return from_hip(zeco::launch_apply_cd_bf16(p, d->d_k, d->d_v, static_cast<hipStream_t>(stream)));
}

zeco_status zeco_hbm_copy(void *dst, const void *src, size_t bytes, void *stream) {
    if (!dst || !src || !aligned16(dst) || !aligned16(src) || bytes % 16 != 0) return ZECO_ERR_INVALID_ARG;
    return from_hip(zeco::launch_copy(dst, src, bytes, static_cast<hipStream_t>(stream)));
}

zeco_status zeco_hbm_mix(void *dst, const void *src, size_t slice_bytes, int32_t reads, int32_t writes, void *stream) {
    if (!dst || !src || !aligned16(dst) || !aligned16(src) || slice_bytes % 16 != 0) return ZECO_ERR_INVALID_ARG;
    const int ok[][2] = {{1, 0}, {0, 1}, {1, 1}, {2, 1}, {3, 1}, {4, 1}, {5, 3}, {3, 2}};
    bool found = false;
    for (auto &m : ok) found = found || (m[0] == reads && m[1] == writes);
    if (!found) return ZECO_ERR_UNSUPPORTED;
    return from_hip(zeco::launch_mix(dst, src, slice_bytes, reads, writes, static_cast<hipStream_t>(stream)));
}

const char *zeco_status_string(int32_t status) {
    switch (status) {
        case ZECO_OK: return "ok";
        case ZECO_ERR_INVALID_ARG: return "invalid argument";
        case ZECO_ERR_UNSUPPORTED: return "unsupported configuration";
        case ZECO_ERR_WORKSPACE: return "workspace too small";
        case ZECO_ERR_HIP: return "HIP runtime error";
        case ZECO_ERR_SCRATCH_LIMIT: return "problem needs more than the library's static scratch";
        default: return "unknown status";
    }
}

int32_t zeco_version(void) { return 100; }

}  // extern "C"
