/*
 * zeco.h - C ABI of the MI355X (gfx950) ZeCO hot path: chunkwise gated-linear-attention (GLA)
 * segment forward, segment-state scan (the arithmetic of All-Scan) and initial-state correction.
 *
 * Conventions for every entry point
 *   - Tensor pointers are DEVICE pointers owned by the caller, 16-byte aligned.  The library never
 *     allocates, frees or synchronises; all work is enqueued on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream).
 *   - Arguments are validated before any HIP call: ZECO_ERR_INVALID_ARG, _UNSUPPORTED, _WORKSPACE and
 *     _SCRATCH_LIMIT mean that nothing was launched and no output was touched.  ZECO_ERR_HIP means that the
 *     runtime refused a launch (or a kernel attribute); entry points that launch several kernels may then
 *     have enqueued the earlier ones, and the outputs are unspecified.
 *   - Results are deterministic (no atomics) and independent of launch-shape heuristics.
 *   - Notation: B batch, P segments (the paper's devices), L tokens per segment, T = P*L, H heads,
 *     C chunk length, g = log(alpha) <= 0 the LOG decay of Eq. (1), scale multiplies q
 *     (1.0 reproduces the paper).  Decay scales row i (the d_k index) of a d_k x d_v state.
 */
#ifndef ZECO_H
#define ZECO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ZECO_OK = 0,
    ZECO_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, misaligned pointer, bad stride */
    ZECO_ERR_UNSUPPORTED = 2, /* valid but not implemented: C not 64 (bf16) or 16/32/64 (fp32), d not in {64,128}, dtype mix, L < 64 */
    ZECO_ERR_WORKSPACE = 3,   /* workspace smaller than the entry point's own *_workspace() query says */
    ZECO_ERR_HIP = 4,         /* HIP runtime refused a launch / attribute */
    ZECO_ERR_SCRATCH_LIMIT = 5 /* zeco_state_scan_tree_static: the problem needs more than the library's static scratch */
} zeco_status;

typedef enum { ZECO_F32 = 0, ZECO_BF16 = 1 } zeco_dtype;

/* Problem descriptor (Alg. 1 inputs: Q, K in R^{L x d_k}, V in R^{L x d_v}, G, chunk size C,
 * number of devices P - here P segments resident on one GPU).
 * q, k, g are addressed as  base + b*stride_b + t*stride_t + h*stride_h + i   (i < d_k, t < T)
 * v, o as                   base + b*vstride_b + t*vstride_t + h*vstride_h + j (j < d_v)
 * in ELEMENTS; the innermost dimension is contiguous.  Strides must be multiples of 8 elements, the token
 * strides at most 2^24 elements (ZECO_ERR_UNSUPPORTED beyond). */
typedef struct {
    int32_t B, P, H, L;        /* B = 0 (an empty batch; BH = 0 in zeco_state_scan) is valid: the entry points
                                * return ZECO_OK at once, touch no pointer and launch nothing.  Limits
                                * (ZECO_ERR_INVALID_ARG beyond): B*P*H <= 2^24, L <= 2^30, P*L <= 2^40 */
    int32_t d_k, d_v, C;       /* supported: d_k and d_v in {64, 128}; C = 64, and with fp32 q/k/v also 16 and 32 (the
                                * result does not depend on C beyond rounding; the sum of |g| over a chunk is limited,
                                * see wide_gates, so a shorter chunk takes stronger gates); any L >= 64.  When L % C != 0
                                * one chunk of every segment is short, L - C*(ceil(L/C) - 1) tokens (the
                                * first one in the passes that walk a segment forwards, the last one in
                                * those that walk it backwards; chunking changes rounding, not the result). */
    int32_t io_dtype;          /* zeco_dtype of q, k, v, o */
    int32_t g_dtype;           /* zeco_dtype of g */
    float scale;
    int64_t stride_b, stride_t, stride_h;
    int64_t vstride_b, vstride_t, vstride_h;
    int32_t g_per_head;        /* 0: one log decay per (token, head, channel), g as described above.
                                * 1: one log decay per (token, head) shared by all d_k channels (the
                                *    scalar-decay members of the family, Sec. 2.1): g, G_cum and dg are
                                *    contiguous [B,T,H] fp32, G_tot is [P,B,H]; bf16 q/k/v only. */
    int32_t wide_gates;        /* Range of the gates with bf16 q/k/v (fp32 q/k/v always have the wide range).
                                * The intra-chunk scores use Q .* Lambda and K / Lambda as in Alg. 1, whose
                                * factors grow with the chunk's total log decay; per chunk and channel the sum
                                * of |g| over the chunk's tokens must stay
                                * 0: below 80 (log Lambda counted from the chunk's start, as in Alg. 1:
                                *    mean decays alpha > 0.29 per token at C = 64),
                                * 1: below 160 (log Lambda counted from half the chunk's total, however the
                                *    decay is spread over the chunk: alpha > 0.08 per token), at about 3 % more
                                *    time in the chunk kernels.
                                * No call can check this: beyond the range the factors overflow and the
                                * outputs come out as inf / NaN while the status is still ZECO_OK. */
} zeco_gla_desc;

/* Bytes of device workspace zeco_gla_local_fwd needs for this descriptor (may be 0).
 * Non-zero when the problem has few (batch, segment, head) streams (bf16, B*P*H <= 64; with one decay per
 * head up to 128, where every segment is run as two halves and the second half corrected): the local pass
 * then splits every segment into sub-segments and runs Alg. 1's own schedule inside each segment (end
 * states of the sub-segments from the zero state, their scan, the output pass of every sub-segment from
 * its scanned state), and keeps the sub-segment states in the workspace (device memory, 16-byte aligned,
 * caller-owned, contents unspecified afterwards).
 * Returns 0 for an invalid descriptor. */
size_t zeco_gla_local_fwd_workspace(const zeco_gla_desc *desc);

/* Local pass (Sec. 3.1 "Local State Computation", Alg. 1 chunk loop and output pass with a zero
 * incoming state; chunk equations of Sec. 2.1): every segment p runs the chunkwise GLA forward
 * from the ZERO state.
 *   in   q, k, v, g   device, layouts per the descriptor (io_dtype / g_dtype)
 *   out  o      [B,T,H,d_v] (descriptor strides), io_dtype: local output
 *   out  S_loc  [P,B,H,d_k,d_v] fp32 contiguous: final local state S_[N] of each segment
 *   out  G_cum  [B,T,H,d_k] fp32 contiguous: per token, sum of g from the segment's first token
 *               through that token (log of Lambda_t .* gamma~_[n-1]; Eq. (gamma) kept per token)
 *   out  G_tot  [P,B,H,d_k] fp32 contiguous: G_cum at each segment's last token (log gamma~_[N])
 * bf16 io: bf16 MFMA operands, fp32 accumulation and fp32 state.  fp32 io: fp32 MFMA throughout.
 * Precondition: the gates stay inside the range the descriptor's wide_gates selects; so for every forward and
 * backward entry point below. */
zeco_status zeco_gla_local_fwd(const zeco_gla_desc *desc, const void *q, const void *k,
                               const void *v, const void *g, void *o, float *S_loc, float *G_cum,
                               float *G_tot, void *workspace, size_t workspace_bytes,
                               void *stream);

/* Segment-state scan: the block update of Sec. 3.2 ("Pipelined State Scan") applied along the
 * chain of segments on one device; Alg. 2 returns (S_recv, S_send) = (S_init[p], S_init[p+1]).
 *   S_init[0] = S0 (zeros if NULL),  S_init[p+1] = (exp(G_tot[p])^T 1) .* S_init[p] + S_loc[p]
 *   in   S_loc  [P,BH,d_k,d_v] fp32,  G_tot [P,BH,d_k] fp32,  S0 [BH,d_k,d_v] fp32 or NULL
 *   out  S_init [P,BH,d_k,d_v] fp32,  S_last [BH,d_k,d_v] fp32 or NULL (= state after segment P-1)
 * K_blocks: number of contiguous d_k-row blocks the state is split into (d_k % K_blocks == 0);
 * each block is an independent slab and the result is bitwise independent of K_blocks.
 * gate_per_head: 0 = G_tot [P,BH,d_k]; 1 = G_tot [P,BH], one log decay per head (see zeco_gla_desc).
 * direction: 0 = forward chain.  1 = the backward direction of Alg. 2: the chain runs from the last
 *   segment to the first, S_init[p] = what enters segment p from segment p+1 (S0 enters the last
 *   segment), S_last = what leaves segment 0; used for the state gradients of App. A.4.
 * d_v % 4 == 0 required; any d_k >= 1. */
zeco_status zeco_state_scan(int32_t P, int32_t BH, int32_t d_k, int32_t d_v, int32_t K_blocks,
                            const float *S_loc, const float *G_tot, const float *S0,
                            float *S_init, float *S_last, int32_t direction, int32_t gate_per_head,
                            void *stream);

/* The same scan as a tree of depth two (the conclusion's outlook names a tree-like All-Scan): the chain of
 * P segments is cut into P/g groups of g segments; (1) every group is scanned on its own from the zero
 * state (its end state and total log decay), (2) the chain over the groups gives the state entering each
 * group and S_last, (3) every group is scanned again from the state entering it, which writes S_init.
 * The serial depth drops from P to about 2 g + P/g (g is chosen to minimise it over the divisors of P)
 * for one more read of S_loc: it pays where a single chain is latency-bound, i.e. one head and 512 segments
 * or more; from two heads on zeco_state_scan has enough chains in flight and is the faster one.
 * Same arguments and conventions as zeco_state_scan; the result differs from it by rounding only (the
 * groups re-associate the sums), it is deterministic; d_k % 16 == 0.  When P has no divisor that
 * shortens the chain (P prime, P <= 4) the call is zeco_state_scan and needs no workspace.
 * workspace: device memory of zeco_state_scan_tree_workspace() bytes (may be 0), 16-byte aligned,
 * caller-owned, contents unspecified afterwards; ZECO_ERR_WORKSPACE when too small. */
size_t zeco_state_scan_tree_workspace(int32_t P, int32_t BH, int32_t d_k, int32_t d_v, int32_t gate_per_head);
zeco_status zeco_state_scan_tree(int32_t P, int32_t BH, int32_t d_k, int32_t d_v, const float *S_loc,
                                 const float *G_tot, const float *S0, float *S_init, float *S_last,
                                 int32_t direction, int32_t gate_per_head, void *workspace,
                                 size_t workspace_bytes, void *stream);

/* zeco_state_scan_tree for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, conventions and results (bitwise) as
 * zeco_state_scan_tree, without the workspace: the group states live in a fixed array inside the library's
 * device image, zeco_state_scan_tree_static_limit() bytes (33 MiB) on every GPU the library runs on, held
 * until the process ends.  The call allocates and frees nothing.
 *   - A problem whose zeco_state_scan_tree_workspace() exceeds the limit returns ZECO_ERR_SCRATCH_LIMIT and
 *     launches nothing (33 MiB covers 1024 segments of up to 4 heads, or 16384 segments of one head, at
 *     d_k = d_v = 128; the tree is the faster scan only for few heads).
 *   - The first call on a device looks up the array's address on that device (hipGetSymbolAddress, no
 *     allocation, no synchronisation); make that call with the device current, as for every other call.
 *   - All calls on one GPU share that GPU's array.  Nothing in it has to start at zero and nothing is kept
 *     from call to call (each call writes every byte it later reads), but two calls that overlap on one GPU
 *     - on different streams, or from different threads - race on it: order them on one stream. */
size_t zeco_state_scan_tree_static_limit(void);
zeco_status zeco_state_scan_tree_static(int32_t P, int32_t BH, int32_t d_k, int32_t d_v, const float *S_loc,
                                        const float *G_tot, const float *S0, float *S_init, float *S_last,
                                        int32_t direction, int32_t gate_per_head, void *stream);

/* Initial-state correction (Eq. (global-correction) carried to the output; the highlighted term
 * of Alg. 1's output pass, with Lambda_t .* gamma~_[n-1] = exp(G_cum[t])):
 *   o_t += (scale * q_t .* exp(G_cum[t])) S_init[p]      for every token t of segment p
 *   in     q (descriptor layout), G_cum [B,T,H,d_k] fp32, S_init [P,B,H,d_k,d_v] fp32 (finite values)
 *   in/out o (descriptor layout)
 * flags: bit set of
 *   ZECO_APPLY_FIRST_SEGMENT_ZERO  segment 0 is skipped (its incoming state is known to be zero)
 *   ZECO_APPLY_DENSE               stream every token.  Without it the call stops, per (batch, segment,
 *                                  head) and at 64-token granularity, at the first token whose G_cum is
 *                                  below -105 in every channel: exp() of that is exactly zero in fp32,
 *                                  and because g <= 0 makes G_cum non-increasing along a segment the same
 *                                  holds for all later tokens, whose o the update would leave unchanged.
 *                                  Both settings give the same o (a -0 may come out as +0 when dense). */
enum { ZECO_APPLY_FIRST_SEGMENT_ZERO = 1, ZECO_APPLY_DENSE = 2 };
zeco_status zeco_apply_init_state(const zeco_gla_desc *desc, const void *q, const float *G_cum,
                                  const float *S_init, void *o, int32_t flags, void *stream);

/* ---- The local pass and the correction with the cumulative decay kept per chunk, as Alg. 1 stores it
 * (the list of gamma~_[n], one d_k vector per chunk) instead of per token: the local pass then writes
 * 8 instead of 512 bytes of decay per token and head (d_k = 128), and the correction rebuilds the
 * in-chunk factor Lambda_t (Sec. 2.1) from g for the tokens it works on.  bf16 q/k/v/o and per-channel
 * gates only (otherwise ZECO_ERR_UNSUPPORTED).  Same conventions as above. ----------------------------- */

/* Local pass: as zeco_gla_local_fwd, with
 *   out  G_chunk [B,P,N,H,d_k] fp32 contiguous, N = ceil(L/C) (= [B,T/C,H,d_k] when L % C == 0): for chunk
 *        n of a segment (n = 0 .. N-1), the sum of g from the segment's first token to the last token
 *        BEFORE the chunk (log gamma~_[n], zero for the segment's first chunk)
 * in place of G_cum.  Uses no workspace (with few (batch, segment, head) streams it is not split further). */
zeco_status zeco_gla_local_fwd_chunk_decay(const zeco_gla_desc *desc, const void *q, const void *k,
                                           const void *v, const void *g, void *o, float *S_loc,
                                           float *G_chunk, float *G_tot, void *stream);

/* Correction: as zeco_apply_init_state, with exp(G_cum[t]) formed as
 *   exp(G_chunk[n] + sum of g over the tokens of chunk n up to and including t).
 * Without ZECO_APPLY_DENSE it stops, per (batch, segment, head), at the first chunk whose G_chunk is
 * below -105 in every channel. */
zeco_status zeco_apply_init_state_chunk_decay(const zeco_gla_desc *desc, const void *q, const void *g,
                                              const float *G_chunk, const float *S_init, void *o,
                                              int32_t flags, void *stream);

/* ---- The local pass and the correction over segments of unequal length.  Sec. 3.1 cuts the sequence into
 * P equal segments; nothing in its local pass, in the state recurrence of Sec. 3.2 or in the correction
 * depends on that, only the token range each segment covers does.  Here segment p covers the tokens
 *   [seg_start[p], seg_start[p+1])   of the T tokens of EVERY batch entry,
 * with seg_start a DEVICE array of P+1 int64 (8-byte aligned), read by the kernels, never by the host.
 *   desc->L          upper bound of the segment lengths (any value >= C; it sizes the correction's launch)
 *   T                tokens per batch entry of q, k, v, g, o and G_cum ([B,T,H,..]); P * C <= T <= 2^40
 *   every segment    C <= seg_start[p+1] - seg_start[p] <= desc->L, inside [0, T]; tokens before seg_start[0]
 *                    and from seg_start[P] on belong to no segment and are neither read nor written
 * A segment that breaks these rules is skipped by the kernels (nothing of it is read or written, its S_loc
 * and G_tot stay as they were); the host cannot see that, so the call still returns ZECO_OK.
 * Outputs as in zeco_gla_local_fwd and zeco_apply_init_state, G_cum counted from each segment's own first
 * token; the scan between the two calls is zeco_state_scan, unchanged.  No workspace: the segments are not
 * split further.  All dtypes and gate layouts of the ordinary calls. ------------- */
zeco_status zeco_gla_local_fwd_varlen(const zeco_gla_desc *desc, const int64_t *seg_start, int64_t T,
                                      const void *q, const void *k, const void *v, const void *g, void *o,
                                      float *S_loc, float *G_cum, float *G_tot, void *stream);
zeco_status zeco_apply_init_state_varlen(const zeco_gla_desc *desc, const int64_t *seg_start, int64_t T,
                                         const void *q, const float *G_cum, const float *S_init, void *o,
                                         int32_t flags, void *stream);

/* The two phases of Alg. 1's own schedule (zeco_gla_local_state, zeco_gla_fwd_from_state below) over the same
 * table: end state and total log decay of every segment from the zero state; then, after zeco_state_scan,
 * the forward of every segment from the state entering it, which writes the final o.  No o from the zero
 * state and no G_cum are ever stored.  bf16 and fp32 q/k/v/o. */
zeco_status zeco_gla_local_state_varlen(const zeco_gla_desc *desc, const int64_t *seg_start, int64_t T,
                                        const void *k, const void *v, const void *g, float *S_loc,
                                        float *G_tot, void *stream);
zeco_status zeco_gla_fwd_from_state_varlen(const zeco_gla_desc *desc, const int64_t *seg_start, int64_t T,
                                           const void *q, const void *k, const void *v, const void *g,
                                           const float *S_init, void *o, void *stream);

/* The backward's building blocks (zeco_gla_bwd_dstate, zeco_gla_bwd_from_state below) over the same table:
 * every segment's state gradient from dS = 0; then, after the reverse zeco_state_scan, dq, dk, dv, dg of
 * every segment.  Arguments as in the equal-length calls; the workspace is
 * zeco_gla_bwd_from_state_workspace(desc) bytes, sized for the bound desc->L on the lengths. */
zeco_status zeco_gla_bwd_dstate_varlen(const zeco_gla_desc *desc, const int64_t *seg_start, int64_t T,
                                       const void *q, const void *g, const void *dO, float *dS_loc,
                                       void *stream);
zeco_status zeco_gla_bwd_from_state_varlen(const zeco_gla_desc *desc, const int64_t *seg_start, int64_t T,
                                           const void *q, const void *k, const void *v, const void *g,
                                           const void *dO, const float *S_init, const float *S_last,
                                           const float *dS_in, void *dq, void *dk, void *dv, float *dg,
                                           void *workspace, size_t workspace_bytes, void *stream);

/* The whole forward and the whole backward over the same table, each in one call, on the segments as given
 * (they are not cut into shorter pieces: the longest segment sets a pass's duration): the three phases of
 * Alg. 1 - states from the zero state, their scan from S0, output pass - and, for the backward (App. A.4),
 * the forward states and their scan again, the dQ pass, which also leaves every segment's state gradient, the
 * reverse scan from dS_T, and the dV and dK passes; dg is re-anchored every 512 tokens as in
 * zeco_gla_bwd_from_state.  Arguments as in zeco_gla_fused_fwd / zeco_gla_fused_bwd (no saved states, no
 * schedule); workspace sizes from the *_workspace queries, sized for the bound desc->L.  Both take bf16 and
 * fp32 q/k/v. */
size_t zeco_gla_fused_fwd_varlen_workspace(const zeco_gla_desc *desc);
zeco_status zeco_gla_fused_fwd_varlen(const zeco_gla_desc *desc, const int64_t *seg_start, int64_t T,
                                      const void *q, const void *k, const void *v, const void *g,
                                      const float *S0, void *o, float *S_last, void *workspace,
                                      size_t workspace_bytes, void *stream);
size_t zeco_gla_fused_bwd_varlen_workspace(const zeco_gla_desc *desc);
zeco_status zeco_gla_fused_bwd_varlen(const zeco_gla_desc *desc, const int64_t *seg_start, int64_t T,
                                      const void *q, const void *k, const void *v, const void *g,
                                      const void *dO, const float *S0, const float *dS_T, void *dq, void *dk,
                                      void *dv, float *dg, float *dS0, void *workspace,
                                      size_t workspace_bytes, void *stream);

/* ---- Two-phase forward: Alg. 1's own schedule (chunk-state loop, All-Scan, output pass), which never
 * materialises the local output or the per-token cumulative decay.  bf16 and fp32 q/k/v/o (fp32: no saved
 * states, no ZECO_SCHEDULE_CORRECT).  Same conventions as above. ------------------------------------- */

/* Phase 1 (Alg. 1 chunk-state loop, Eq. (local-recurrence) and Eq. (gamma)): final local state and
 * total log decay of every segment from the zero state.  Reads k, v, g only.
 *   out  S_loc [P,B,H,d_k,d_v] fp32,  G_tot [P,B,H,d_k] fp32 */
zeco_status zeco_gla_local_state(const zeco_gla_desc *desc, const void *k, const void *v,
                                 const void *g, float *S_loc, float *G_tot, void *stream);

/* Phase 2 (Alg. 1 output pass with the incoming state, Eq. (global-correction)): chunkwise forward of
 * every segment p started from S_init[p] (as produced by zeco_state_scan); writes the final output.
 *   in   S_init [P,B,H,d_k,d_v] fp32      out  o (descriptor layout, io_dtype) */
zeco_status zeco_gla_fwd_from_state(const zeco_gla_desc *desc, const void *q, const void *k,
                                    const void *v, const void *g, const float *S_init, void *o,
                                    void *stream);

/* The whole forward in one call, for all P segments resident on this device.  The library may cut the
 * segments further (more, shorter segments keep every compute unit busy); the states of those pieces
 * live in the workspace.
 *   in   S0 [B,H,d_k,d_v] fp32 or NULL: state entering the first segment
 *   out  o;  S_last [B,H,d_k,d_v] fp32 or NULL: state after the last token
 *   out  S_save: NULL, or zeco_gla_saved_states_bytes(desc) bytes of device memory that receive the
 *        forward states entering the pieces the backward works on (the forward's own pieces), and the
 *        end state; handing it to zeco_gla_fused_bwd spares that call the recomputation of the forward
 *        states.  Contents are private to the library.  bf16 only.
 *   schedule:
 *     ZECO_SCHEDULE_TWO_PHASE  Alg. 1's: chunk-state pass (k, v, g), scan, output pass from the scanned
 *                              states.  Traffic does not depend on the data.
 *     ZECO_SCHEDULE_CORRECT    local pass from the zero state (chunk-decay form), scan, correction.  The
 *                              correction stops where the decay factor has vanished, so with decays whose
 *                              e-folding length is far below the piece length k, v, g are read once
 *                              instead of twice; with decays near 1 it moves about 10 % more than
 *                              two-phase (measured 15 - 20 % more time: ask for TWO_PHASE with such data).
 *     ZECO_SCHEDULE_AUTO       CORRECT when it is available and the pieces are at least 4096 tokens long,
 *                              else TWO_PHASE.
 * workspace: zeco_gla_fused_fwd_workspace(desc) bytes of device memory, 16-byte aligned (enough for
 * either schedule). */
enum { ZECO_SCHEDULE_AUTO = 0, ZECO_SCHEDULE_TWO_PHASE = 1, ZECO_SCHEDULE_CORRECT = 2 };
size_t zeco_gla_fused_fwd_workspace(const zeco_gla_desc *desc);
size_t zeco_gla_saved_states_bytes(const zeco_gla_desc *desc);
zeco_status zeco_gla_fused_fwd(const zeco_gla_desc *desc, const void *q, const void *k, const void *v,
                               const void *g, const float *S0, void *o, float *S_last, float *S_save,
                               int32_t schedule, void *workspace, size_t workspace_bytes, void *stream);

/* ---- Backward pass (App. A.4): gradients of  sum_t <o_t, dO_t> + <S_T, dS_T>  for the forward above.
 * q/k/v/dO and the gradients dq, dk, dv share one dtype, bf16 (bf16 MFMA operands, fp32 accumulation and
 * states: the throughput path) or fp32 (fp32 MFMA throughout, chunk length desc->C: the accuracy path, about
 * 7 times slower).  dO, dv use the layout of v;
 * dq, dk the layout of q; dg [B,T,H,d_k] fp32 contiguous; all state arrays fp32.  The state gradients
 * are true gradients (they include `scale`). --------------------------------------------------------- */

/* First loop of the backward listing: per segment, from dS = 0, last chunk to first,
 *   dS <- (gamma^T 1) .* dS + (Q .* Lambda)^T dO * scale
 * and what is left after the segment's first token, decayed past it: the gradient this segment sends
 * to the final state of the segment before it.
 *   out  dS_loc [P,B,H,d_k,d_v] fp32.
 * Chained by zeco_state_scan(direction = 1) with the same G_tot as the forward chain. */
zeco_status zeco_gla_bwd_dstate(const zeco_gla_desc *desc, const void *q, const void *g, const void *dO,
                                float *dS_loc, void *stream);

/* The remaining loops of the backward listing, for every segment p, given the forward state S_init[p]
 * entering it, the forward state after the last segment (S_last), and dS_in[p], the gradient entering
 * its final state (zeco_state_scan, direction = 1):
 *   dq, dk, dv as in App. A.4 (the chunk states S_[n], dS_[n] are recomputed on chip, never stored);
 *   dg_t = sum over the segment's tokens s >= t of (q_s .* dq_s - k_s .* dk_s)
 *          + row sums of dS_in[p] .* S_end[p],  S_end[p] = S_init[p+1] (S_last for the last segment):
 *          the reverse cumulative sum of the listing's last line, carried across segments.
 * The two products of that sum nearly cancel, and what is left of it after thousands of tokens is mostly the
 * rounding noise of the bf16 matrix operands.  The sum is therefore restarted every 512 tokens from its
 * exactly known value there, the row sums of (gradient of the state) .* (forward state) at that token:
 * the dQ pass leaves the forward states at those tokens in the workspace, the dK pass reads them back.
 * workspace: zeco_gla_bwd_from_state_workspace(desc) bytes of device memory (a d_k x d_v fp32 state per 512
 * tokens and head; 0 for segments of up to 512 tokens), 16-byte aligned, caller-owned, contents unspecified
 * afterwards; ZECO_ERR_WORKSPACE when too small. */
size_t zeco_gla_bwd_from_state_workspace(const zeco_gla_desc *desc);
zeco_status zeco_gla_bwd_from_state(const zeco_gla_desc *desc, const void *q, const void *k,
                                    const void *v, const void *g, const void *dO, const float *S_init,
                                    const float *S_last, const float *dS_in, void *dq, void *dk,
                                    void *dv, float *dg, void *workspace, size_t workspace_bytes,
                                    void *stream);

/* The whole backward in one call: recomputes the forward segment states (phase 1 and its scan, from
 * S0), runs the state-gradient pass and its reverse scan (from dS_T), then the gradient passes.  Like
 * zeco_gla_fused_fwd it may cut the segments into shorter pieces.
 *   in   S0, dS_T [B,H,d_k,d_v] fp32 or NULL (zero)
 *   in   S_saved: NULL, or what zeco_gla_fused_fwd left in S_save for the same descriptor and inputs
 *        (S0 is then not read: it is already part of the saved states)
 *   out  dq, dk, dv, dg;  dS0 [B,H,d_k,d_v] fp32 or NULL: gradient of the state entering the first segment
 * workspace: zeco_gla_fused_bwd_workspace(desc) bytes of device memory, 16-byte aligned. */
size_t zeco_gla_fused_bwd_workspace(const zeco_gla_desc *desc);
zeco_status zeco_gla_fused_bwd(const zeco_gla_desc *desc, const void *q, const void *k, const void *v,
                               const void *g, const void *dO, const float *S0, const float *dS_T,
                               const float *S_saved, void *dq, void *dk, void *dv, float *dg, float *dS0,
                               void *workspace, size_t workspace_bytes, void *stream);

/* Bandwidth calibration utility (not part of the method): copies `bytes` (a multiple of 16) from
 * src to dst with a plain grid-stride kernel of 16-byte accesses.  Used to scale the HBM byte
 * counters of the profiler and to quote the achievable copy bandwidth beside the nominal peak.
 * Both pointers are device pointers, 16-byte aligned, non-overlapping. */
zeco_status zeco_hbm_copy(void *dst, const void *src, size_t bytes, void *stream);

/* The same for a mix of traffic: `reads` source streams and `writes` destination streams of slice_bytes each
 * (src holds reads * slice_bytes bytes, dst writes * slice_bytes; a read-only run needs 16 bytes of dst), one
 * 16-byte word of every stream per thread and step.  Gives the rate the memory system reaches for a kernel's
 * ratio of reads to writes, to quote beside that kernel's own figure.  Mixes built: 1:0, 0:1, 1:1, 2:1, 3:1,
 * 4:1 (the correction), 3:2, 5:3 (the local pass); others return ZECO_ERR_UNSUPPORTED. */
zeco_status zeco_hbm_mix(void *dst, const void *src, size_t slice_bytes, int32_t reads, int32_t writes,
                         void *stream);

const char *zeco_status_string(int32_t status);
int32_t zeco_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ZECO_H */
