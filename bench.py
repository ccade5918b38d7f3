#!/usr/bin/env python3
"""Benchmark of the ZeCO hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input already resident in HBM:
zeco_gla_local_fwd -> zeco_state_scan -> zeco_apply_init_state.  Prints ONE JSON line with the
whole-job throughput (tokens/s), the roofline of the dominant kernel (the chunk kernel of the
local pass) measured live with HIP events on the launch stream, and the CPU oracle timed on a
bounded sample of the same workload.

The default workload is c5 (H = 8, 256 segments x 32768 tokens = 8.4 M tokens, 128 GiB of tensors), the largest
configuration that fits one GPU; the same legs at c3 and the single-segment case c2 are appended under
`other_workloads`.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5|c4|c3|c2] [--g-dtype f32|bf16]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
MFMA_BF16_PEAK_TF = 2500.0  # dense bf16

# HBM bytes per launch of the chunk kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# (profiles/pipeline_kernels_c2_c3_c4_c5.md gives the commands and the copy-kernel calibration); None = not measured.
# c5: not measured (the counter pass of that workload ended in the profiler before any kernel ran and is not
# repeated); c4 runs the same instantiation of the chunk kernel, one workgroup per stream.
MEASURED_TRAFFIC = {("c3", "f32"): 4305900000, ("c4", "f32"): 34469000000}   # profiles/pipeline_kernels_c2_c3_c4_c5.md


def algorithmic_bytes(c, g_in, g_cum):
    """Algorithmic HBM bytes per launch of each kernel (per token-head figures x units).
    g_in, g_cum: bytes of g and of G_cum per token-head."""
    B, H, P, L, dk, dv = c["B"], c["H"], c["P"], c["L"], c["d_k"], c["d_v"]
    io = 2 if c["io"] == "bf16" else 4
    th = B * P * L * H                                  # token-heads per launch
    streams = B * P * H
    local = th * (2 * dk * io + dv * io + g_in           # read q, k, v, g
                  + dv * io + g_cum)                      # write o, G_cum
    local += streams * (dk * dv * 4 + dk * 4)            # S_loc, G_tot
    scan = streams * (2 * dk * dv * 4 + dk * 4) + B * H * dk * dv * 4
    th_c = B * (P - 1) * L * H                           # segment 0 needs no correction
    apply_ = th_c * (dk * io + g_cum + 2 * dv * io) + B * (P - 1) * H * dk * dv * 4
    return dict(local=local, scan=scan, apply=apply_)


def algorithmic_flops(c):
    B, H, P, L, dk, dv, C = c["B"], c["H"], c["P"], c["L"], c["d_k"], c["d_v"], c["C"]
    th = B * P * L * H
    local = th * (2 * C * dk + 2 * C * dv + 2 * dk * dv + 2 * dk * dv)   # dense count, Sec. 2.1
    apply_ = B * (P - 1) * L * H * 2 * dk * dv
    return dict(local=local, apply=apply_)


def cpu_baseline(inp, c, sample_tokens):
    """The oracle as it stands, on the first `sample_tokens` tokens of every head."""
    from oracle import oracle
    from paper_2507_01004_amd import synth
    h = {n: synth.to_f64(t[:, :sample_tokens]) for n, t in inp.items()}
    t0 = time.perf_counter()
    oracle.gla_recurrent(h["q"], h["k"], h["v"], h["g"])
    dt = time.perf_counter() - t0
    model = ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return {"value": c["B"] * sample_tokens / dt, "unit": "tokens/s", "cores": oracle.num_threads(),
            "cpu_model": model,
            "kind": "oracle", "seconds": round(dt, 3),
            "sample": "fp64 token recurrence (Eq. 1) over the first %d tokens of all %d heads of "
                      "the same inputs, OpenMP over heads" % (sample_tokens, c["H"])}


def single_segment_case(args):
    """configs[1] (one segment of 16384 tokens, H = 16: the local pass alone) timed beside the headline
    workload: the three calls (scan and correction have nothing to do at P = 1) and the fused forward."""
    import torch
    from paper_2507_01004_amd import synth, zeco
    inp, c = synth.config_inputs("c2", device="cuda:0", g=args.g_dtype, per_head_gate=args.gate == "head")
    q, k, v, g = inp["q"], inp["k"], inp["v"], inp["g"]
    B, T, H, dk = q.shape
    dv, P = v.shape[-1], c["P"]
    gdim = (dk,) if args.gate == "channel" else ()
    outs = (torch.empty_like(v), torch.empty(P, B, H, dk, dv, dtype=torch.float32, device="cuda:0"),
            torch.empty((B, T, H) + gdim, dtype=torch.float32, device="cuda:0"),
            torch.empty((P, B, H) + gdim, dtype=torch.float32, device="cuda:0"))
    S_init, S_last = torch.empty_like(outs[1]), torch.empty(B, H, dk, dv, dtype=torch.float32, device="cuda:0")
    nws = zeco.local_fwd_workspace_bytes(q, v, g, P)
    ws = torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda:0") if nws else None
    wsf = torch.empty(max(zeco.fused_workspace_bytes(q, v, g, P), 16), dtype=torch.uint8, device="cuda:0")

    def step():
        zeco.gla_local_fwd(q, k, v, g, P, out=outs, workspace=ws)
        zeco.state_scan(outs[1], outs[3], K_blocks=args.k_blocks, out=(S_init, S_last))
        zeco.apply_init_state(q, g, outs[2], S_init, outs[0], P, first_segment_is_zero=True)

    res = {}
    for name, fn in (("three_call", step), ("local_fwd", lambda: zeco.gla_local_fwd(q, k, v, g, P, out=outs, workspace=ws)),
                     ("fused_fwd", lambda: zeco.gla_fused_fwd(q, k, v, g, P, out=(outs[0], S_last), workspace=wsf))):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        res[name] = e0.elapsed_time(e1) / args.steps
    g_in = (dk * (4 if args.g_dtype == "f32" else 2)) if args.gate == "channel" else 4
    ab = algorithmic_bytes(c, g_in, dk * 4 if args.gate == "channel" else 4)["local"]
    return {"workload": "c2: B=%d H=%d P=%d x L=%d, d_k=d_v=%d" % (B, H, P, c["L"], dk),
            "ms_per_step": round(res["three_call"], 4), "tokens_per_s": round(B * T / (res["three_call"] * 1e-3), 1),
            "local_fwd_ms": round(res["local_fwd"], 4), "local_fwd_alg_bytes": ab,
            "local_fwd_hbm_frac": round(ab / res["local_fwd"] / 1e6 / HBM_PEAK_GBS, 4),
            "fused_fwd_ms": round(res["fused_fwd"], 4),
            "fused_fwd_tokens_per_s": round(B * T / (res["fused_fwd"] * 1e-3), 1)}


def scan_variants_case(args):
    """The segment-state scan alone where one chain is latency-bound (few heads, many segments) and where
    it streams (many heads): zeco_state_scan against zeco_state_scan_tree, d_k = d_v = 128."""
    import torch
    from paper_2507_01004_amd import zeco
    rows = []
    for P, BH in ((128, 1), (256, 1), (1024, 1), (4096, 1), (256, 2), (1024, 2), (4096, 2), (1024, 4), (256, 8), (64, 16)):
        gen = torch.Generator(device="cuda:0").manual_seed(P + BH)
        S_loc = torch.randn(P, BH, 128, 128, device="cuda:0", generator=gen)
        G_tot = -torch.rand(P, BH, 128, device="cuda:0", generator=gen)
        out = (torch.empty_like(S_loc), torch.empty(BH, 128, 128, device="cuda:0"))
        ws = torch.empty(max(16, int(zeco.lib().zeco_state_scan_tree_workspace(P, BH, 128, 128, 0))),
                         dtype=torch.uint8, device="cuda:0")
        ms = {}
        for name, fn in (("serial", lambda: zeco.state_scan(S_loc, G_tot, K_blocks=args.k_blocks, out=out)),
                         ("tree", lambda: zeco.state_scan_tree(S_loc, G_tot, out=out, workspace=ws))):
            for _ in range(args.warmup):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ms[name] = e0.elapsed_time(e1) / args.steps
        by = 2 * S_loc.numel() * 4
        rows.append({"P": P, "BH": BH, "serial_ms": round(ms["serial"], 4), "tree_ms": round(ms["tree"], 4),
                     "serial_GBps": round(by / ms["serial"] / 1e6, 1), "alg_bytes": by})
    return rows


def unequal_segments_case(args, inp, P, T):
    """The local pass and the correction over P segments of unequal length summing to the workload's T
    tokens (zeco_gla_local_fwd_varlen, zeco_apply_init_state_varlen): equal lengths, lengths within an
    eighth of the mean, and lengths from a quarter to seven quarters of the mean."""
    import torch
    from paper_2507_01004_amd import zeco
    q, k, v, g = (inp[n] for n in ("q", "k", "v", "g"))
    L = T // P
    spreads = {"equal": [0] * P, "mild": [((-1) ** i) * (L // 8) * ((i // 2) % 2 + 1) // 2 for i in range(P)],
               "wide": [((-1) ** i) * (L // 4) * ((i // 2) % 3 + 1) for i in range(P)]}
    rows = []
    for name, delta in spreads.items():
        lengths = [L + d for d in delta]
        lengths[-1] += T - sum(lengths)          # whatever the pattern leaves over goes to the last segment
        if min(lengths) < 64:
            continue
        start = [0]
        for n in lengths:
            start.append(start[-1] + n)
        seg = torch.tensor(start, dtype=torch.int64, device="cuda:0")
        bound = max(lengths)
        out = zeco.gla_local_fwd_varlen(q, k, v, g, seg, bound)
        o, S_loc, G_cum, G_tot = out
        S_init, _ = zeco.state_scan(S_loc, G_tot)
        ms = {}
        for leg, fn in (("local", lambda: zeco.gla_local_fwd_varlen(q, k, v, g, seg, bound, out=out)),
                        ("apply", lambda: zeco.apply_init_state_varlen(q, g, G_cum, S_init, o, seg, bound))):
            for _ in range(args.warmup):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ms[leg] = e0.elapsed_time(e1) / args.steps
        rows.append({"lengths": name, "min": min(lengths), "max": bound, "local_ms": round(ms["local"], 4),
                     "apply_ms": round(ms["apply"], 4)})
    return rows


def free_gib():
    import torch
    return torch.cuda.mem_get_info()[0] / 2 ** 30


def run_workload(args, workload, with_cpu):
    """All legs of one workload; returns the JSON object of the line."""
    import statistics
    import torch
    from paper_2507_01004_amd import synth, zeco

    inp, c = synth.config_inputs(workload, device="cuda:0", g=args.g_dtype,
                                 per_head_gate=args.gate == "head")
    B, H, P, L, dk, dv = c["B"], c["H"], c["P"], c["L"], c["d_k"], c["d_v"]
    T = P * L
    if args.layout == "bhtd":   # same values, each head's tokens contiguous in memory
        inp = {n: t.transpose(1, 2).contiguous().transpose(1, 2) for n, t in inp.items()}
    q, k, v, g = inp["q"], inp["k"], inp["v"], inp["g"]
    o = torch.empty_like(v)
    S_loc = torch.empty(P, B, H, dk, dv, dtype=torch.float32, device="cuda:0")
    gdim = (dk,) if args.gate == "channel" else ()
    G_cum = torch.empty((B, T, H) + gdim, dtype=torch.float32, device="cuda:0")
    G_tot = torch.empty((P, B, H) + gdim, dtype=torch.float32, device="cuda:0")
    g_in = (dk * (4 if args.g_dtype == "f32" else 2)) if args.gate == "channel" else 4   # bytes per token-head
    g_cum = dk * 4 if args.gate == "channel" else 4
    S_init = torch.empty_like(S_loc)
    S_last = torch.empty(B, H, dk, dv, dtype=torch.float32, device="cuda:0")
    tensor_gib = sum(t.numel() * t.element_size() for t in (q, k, v, g, o, G_cum)) / 2 ** 30
    skipped = {}

    def step(ev=None):
        zeco.gla_local_fwd(q, k, v, g, P, out=(o, S_loc, G_cum, G_tot))
        if ev:
            ev[1].record()
        zeco.state_scan(S_loc, G_tot, K_blocks=args.k_blocks, out=(S_init, S_last))
        if ev:
            ev[2].record()
        zeco.apply_init_state(q, g, G_cum, S_init, o, P, first_segment_is_zero=True, dense=args.dense_correction)
        if ev:
            ev[3].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for s in range(args.steps):
        evs[s][0].record()
        step(evs[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    def timed(fn, warm=None, reps=None):
        for _ in range(args.warmup if warm is None else warm):
            fn()
        torch.cuda.synchronize()
        fe = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        n = args.steps if reps is None else reps
        fe[0].record()
        for _ in range(n):
            fn()
        fe[1].record()
        torch.cuda.synchronize()
        return fe[0].elapsed_time(fe[1]) / n

    # The same result by the fused entry point, by either of its schedules: two-phase (states, scan,
    # output pass from the scanned states) and local pass in chunk-decay form + scan + correction.
    # Reported beside the headline number, never as `value`.
    two_phase = fused_correct = chunk_decay = None
    if c["io"] == "bf16" and not (args.only_pipeline or args.only_backward):
        ws = torch.empty(max(zeco.fused_workspace_bytes(q, v, g, P), 16), dtype=torch.uint8, device="cuda:0")
        o2 = torch.empty_like(v)
        S_last2 = torch.empty_like(S_last)
        io = 2
        th = B * T * H
        fms = timed(lambda: zeco.gla_fused_fwd(q, k, v, g, P, out=(o2, S_last2), workspace=ws,
                                               schedule=zeco.SCHEDULE_TWO_PHASE))
        fb = th * (dk * io + dv * io + g_in)                        # phase 1: k, v, g
        fb += th * (2 * dk * io + dv * io + g_in + dv * io)         # phase 2
        two_phase = {"entry": "zeco_gla_fused_fwd(ZECO_SCHEDULE_TWO_PHASE)", "ms_per_step": round(fms, 4),
                     "tokens_per_s": round(B * T / (fms * 1e-3), 1), "alg_bytes": fb,
                     "GBps": round(fb / fms / 1e6, 1), "hbm_frac": round(fb / fms / 1e6 / HBM_PEAK_GBS, 4)}
        cms = timed(lambda: zeco.gla_fused_fwd(q, k, v, g, P, out=(o2, S_last2), workspace=ws,
                                               schedule=zeco.SCHEDULE_CORRECT))
        fused_correct = {"entry": "zeco_gla_fused_fwd(ZECO_SCHEDULE_CORRECT)", "ms_per_step": round(cms, 4),
                         "tokens_per_s": round(B * T / (cms * 1e-3), 1),
                         "note": "local pass (chunk-decay form) + scan + correction that stops where the decay "
                                 "has vanished; traffic depends on the gates"}
        if args.gate == "channel" and not args.only_fused:
            # the three calls of the headline with the cumulative decay kept per chunk (Alg. 1's gamma~ list)
            G_chunk = torch.empty(B, T // 64, H, dk, dtype=torch.float32, device="cuda:0")

            def step_cd():
                zeco.gla_local_fwd_chunk_decay(q, k, v, g, P, out=(o2, S_loc, G_chunk, G_tot))
                zeco.state_scan(S_loc, G_tot, K_blocks=args.k_blocks, out=(S_init, S_last2))
                zeco.apply_init_state_chunk_decay(q, g, G_chunk, S_init, o2, P, first_segment_is_zero=True)
            dms = timed(step_cd)
            lms = timed(lambda: zeco.gla_local_fwd_chunk_decay(q, k, v, g, P, out=(o2, S_loc, G_chunk, G_tot)))
            lb = th * (2 * dk * io + 2 * dv * io + g_in + dk * 4 // 64) + B * P * H * (dk * dv * 4 + dk * 4)
            chunk_decay = {"entries": "zeco_gla_local_fwd_chunk_decay, zeco_state_scan, zeco_apply_init_state_chunk_decay",
                           "ms_per_step": round(dms, 4), "tokens_per_s": round(B * T / (dms * 1e-3), 1),
                           "local_ms": round(lms, 4), "local_alg_bytes": lb,
                           "local_GBps": round(lb / lms / 1e6, 1),
                           "local_hbm_frac": round(lb / lms / 1e6 / HBM_PEAK_GBS, 4)}
            del G_chunk
            zeco.gla_local_fwd(q, k, v, g, P, out=(o, S_loc, G_cum, G_tot))   # S_loc, G_tot of the headline again
            zeco.state_scan(S_loc, G_tot, K_blocks=args.k_blocks, out=(S_init, S_last))
        del ws, o2, S_last2

    # The same pipeline with the log decay stored in bf16 (256 B per token-head less to read): a data
    # format choice of the caller, reported beside the fp32-gate headline.
    g_bf16 = None
    if c["io"] == "bf16" and args.g_dtype == "f32" and args.gate == "channel" and not args.no_variants:
        gh = g.to(torch.bfloat16)
        def step_h():
            zeco.gla_local_fwd(q, k, v, gh, P, out=(o, S_loc, G_cum, G_tot))
            zeco.state_scan(S_loc, G_tot, K_blocks=args.k_blocks, out=(S_init, S_last))
            zeco.apply_init_state(q, gh, G_cum, S_init, o, P, first_segment_is_zero=True)
        ws = torch.empty(max(zeco.fused_workspace_bytes(q, v, gh, P), 16), dtype=torch.uint8, device="cuda:0")
        o2 = torch.empty_like(v)
        res = {}
        for name, fn in (("three_call", step_h),
                         ("two_phase", lambda: zeco.gla_fused_fwd(q, k, v, gh, P, out=(o2, S_last), workspace=ws,
                                                                  schedule=zeco.SCHEDULE_TWO_PHASE)),
                         ("fused_correct", lambda: zeco.gla_fused_fwd(q, k, v, gh, P, out=(o2, S_last), workspace=ws,
                                                                      schedule=zeco.SCHEDULE_CORRECT))):
            t = timed(fn, warm=3, reps=max(1, args.steps // 2))
            res[name] = {"ms_per_step": round(t, 4), "tokens_per_s": round(B * T / (t * 1e-3), 1)}
        g_bf16 = res
        del gh, ws, o2
        step()   # the fp32-gate outputs again

    # The same three calls with the wide range of gates (zeco_gla_desc.wide_gates: decay factors of the tiles
    # counted from half the chunk's total, a second multiplication of the state per chunk).
    wide = None
    if c["io"] == "bf16" and not args.no_variants:
        with zeco.wide_gates():
            lms = timed(lambda: zeco.gla_local_fwd(q, k, v, g, P, out=(o, S_loc, G_cum, G_tot)), warm=3,
                        reps=max(1, args.steps // 2))
            t = timed(step, warm=3, reps=max(1, args.steps // 2))
        wide = {"local_fwd_ms": round(lms, 4), "ms_per_step": round(t, 4), "tokens_per_s": round(B * T / (t * 1e-3), 1)}
        step()   # the standard range's outputs again

    copy_gbs = None
    if args.calib_copy_mib:
        src = torch.empty(args.calib_copy_mib << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        zeco.hbm_copy(dst, src)
        ce = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ce[0].record()
        for _ in range(5):
            zeco.hbm_copy(dst, src)
        ce[1].record()
        torch.cuda.synchronize()
        copy_gbs = 5 * 2 * src.numel() / ce[0].elapsed_time(ce[1]) / 1e6
        del src, dst
    # What the memory system gives plain coalesced streams with the kernels' ratios of reads to writes
    # (zeco_hbm_mix: 256 MiB per stream): the scan is 1:1, the correction 4:1 (q, 2 x G_cum, o in; o out),
    # the local pass 5:3 in units of 256 B per token-head (q, k, v, 2 x g in; o, 2 x G_cum out).
    mix_gbs = None
    if args.calib_copy_mib and with_cpu:
        sl = 256 << 20
        src = torch.empty(5 * sl, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty(3 * sl, dtype=torch.uint8, device="cuda:0")
        mix_gbs = {}
        for r, w in ((1, 0), (0, 1), (1, 1), (4, 1), (5, 3)):
            zeco.hbm_mix(dst, src, sl, r, w)
            t = timed(lambda: zeco.hbm_mix(dst, src, sl, r, w), warm=1, reps=5)
            mix_gbs["%d:%d" % (r, w)] = round((r + w) * sl / t / 1e6, 1)
        # the correction rewrites one of its four input streams in place
        last = src[3 * sl:4 * sl]
        t = timed(lambda: zeco.hbm_mix(last, src, sl, 4, 1), warm=1, reps=5)
        mix_gbs["4:1 in place"] = round(5 * sl / t / 1e6, 1)
        del src, dst

    # The correction stops, per (segment, head), where the decay factor exp(G_cum) has become an exact
    # zero; the same kernel made to stream every token gives its bandwidth on the full traffic.
    dense_ms = live_frac = None
    if P > 1 and not args.dense_correction:
        # tokens per (segment, head) the default call works on: up to the first 64-token block whose
        # first token has G_cum < -105 in every channel
        live = []
        for p1 in range(1, P, 16):     # a few segments at a time: the comparison makes a temporary
            Gs = G_cum.view((B, P, L // 64, 64, H) + gdim)[:, p1:p1 + 16, :, 0]
            alive = (Gs >= -105.0).any(dim=-1) if args.gate == "channel" else (Gs >= -105.0)
            live.append((float(alive.float().sum().item()), alive.numel()))
            del Gs, alive
        live_frac = sum(x for x, _ in live) / sum(n for _, n in live)
        if not (args.only_pipeline or args.only_fused or args.only_backward):
            dense_ms = timed(lambda: zeco.apply_init_state(q, g, G_cum, S_init, o, P, first_segment_is_zero=True, dense=True),
                             warm=1, reps=max(1, args.steps // 2))

    samples = {n: [e[i].elapsed_time(e[i + 1]) for e in evs] for i, n in enumerate(["local", "scan", "apply"])}
    ms = {n: sum(x) / len(x) for n, x in samples.items()}

    # The scan's working set may sit in the 256 MB Infinity Cache when it is timed in a loop.  Cold figures: after
    # a sweep that READS 1 GiB (the caches then hold clean lines of something else: the scan's own HBM rate),
    # and after a 512 MiB FILL (dirty lines that the scan's traffic has to push out on top of its own).
    scan_cold = scan_cold_fill = None
    if not args.no_cold_scan:
        junk = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
        for mode in ("read", "fill"):
            cold = []
            for _ in range(10):
                if mode == "read":
                    junk.sum()
                else:
                    junk[:512 << 20].fill_(3)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                zeco.state_scan(S_loc, G_tot, K_blocks=args.k_blocks, out=(S_init, S_last))
                e1.record()
                torch.cuda.synchronize()
                cold.append(e0.elapsed_time(e1))
            if mode == "read":
                scan_cold = statistics.median(cold)
            else:
                scan_cold_fill = statistics.median(cold)
        del junk

    # Backward of the same workload (App. A.4), whole call: reported beside the headline number.  It needs
    # dO, four gradients and its workspace; o and G_cum are released first (nothing below reads them).
    backward = None
    if c["io"] == "bf16" and not args.no_backward:
        del o, G_cum
        torch.cuda.empty_cache()
        ws_bytes = zeco.fused_bwd_workspace_bytes(q, v, g, P)
        need = (ws_bytes + zeco.saved_states_bytes(q, v, g, P) + zeco.fused_workspace_bytes(q, v, g, P)
                + 5 * v.numel() * 2 + g.numel() * 4) / 2 ** 30
        if need + 4 > free_gib():
            skipped["backward"] = "needs %.0f GiB beside the inputs, %.0f GiB free" % (need, free_gib())
        else:
            gen = torch.Generator(device="cuda:0").manual_seed(99)
            dO = torch.empty_like(v)
            for t0 in range(0, T, 65536):
                dO[:, t0:t0 + 65536] = torch.randn((B, min(65536, T - t0), H, dv), generator=gen, device="cuda:0").to(torch.bfloat16)
            ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda:0")
            grads = (torch.empty_like(q), torch.empty_like(q), torch.empty_like(v),
                     torch.empty(g.shape, dtype=torch.float32, device="cuda:0"), torch.empty_like(S_last))
            nb = max(1, args.steps // 2)
            bms = timed(lambda: zeco.gla_fused_bwd(q, k, v, g, dO, P, out=grads, workspace=ws),
                        warm=max(1, args.warmup // 2), reps=nb)
            th = B * T * H
            # bytes of the four passes as built: forward states (k, v, g), dQ (dO, v, k, q, g in; dq and fp32 q.*dq
            # out; it also leaves the pieces' state gradients), dV (k, q, dO, g in; dv out), dK (v, dO, q, k, g, fp32
            # q.*dq in; dk and fp32 dg out)
            io = dk * 2
            pb = th * ((2 * io + g_in) + (5 * io + g_in + g_cum) + (4 * io + g_in) + (5 * io + g_in + 2 * g_cum))
            # training pair: the forward leaves the states at the backward's piece boundaries, the backward
            # starts from them instead of recomputing them
            save = torch.empty(zeco.saved_states_bytes(q, v, g, P), dtype=torch.uint8, device="cuda:0")
            wsf = torch.empty(max(zeco.fused_workspace_bytes(q, v, g, P), 16), dtype=torch.uint8, device="cuda:0")
            o4 = torch.empty_like(v)
            pair = {}
            for nm, fn in (("fwd_saving_ms", lambda: zeco.gla_fused_fwd(q, k, v, g, P, out=(o4, S_last), workspace=wsf, save=save,
                                                                        schedule=zeco.SCHEDULE_TWO_PHASE)),
                           ("bwd_from_saved_ms", lambda: zeco.gla_fused_bwd(q, k, v, g, dO, P, out=grads, workspace=ws, saved=save))):
                pair[nm] = round(timed(fn, warm=1, reps=nb), 4)
            del save, wsf, o4
            backward = {"entry": "zeco_gla_fused_bwd", "ms_per_step": round(bms, 4), **pair,
                        "tokens_per_s": round(B * T / (bms * 1e-3), 1), "pass_bytes": pb,
                        "GBps": round(pb / bms / 1e6, 1), "hbm_frac": round(pb / bms / 1e6 / HBM_PEAK_GBS, 4)}
            del ws, grads, dO

    ms_per_step = wall * 1e3 / args.steps
    ab = algorithmic_bytes(c, g_in, g_cum)
    af = algorithmic_flops(c)
    kernels = {}
    for n in ("local", "scan", "apply"):
        if ms[n] > 0:
            kernels[n] = {"ms": round(ms[n], 4), "ms_median": round(statistics.median(samples[n]), 4),
                          "ms_min": round(min(samples[n]), 4), "alg_bytes": ab[n],
                          "GBps": round(ab[n] / ms[n] / 1e6, 1),
                          "hbm_frac": round(ab[n] / ms[n] / 1e6 / HBM_PEAK_GBS, 4)}
            if n in af:
                kernels[n]["TFLOPs"] = round(af[n] / ms[n] / 1e9, 1)
                kernels[n]["mfma_frac"] = round(af[n] / ms[n] / 1e9 / MFMA_BF16_PEAK_TF, 4)
    kernels["local"]["tokens_per_s"] = round(B * T / (ms["local"] * 1e-3), 1)
    dense_step = None
    if live_frac is not None and "apply" in kernels:
        ka = kernels["apply"]
        ka["live_fraction"] = round(live_frac, 4)
        ka["alg_bytes"] = int(ab["apply"] * live_frac)
        ka["GBps"] = round(ka["alg_bytes"] / ms["apply"] / 1e6, 1)
        ka["hbm_frac"] = round(ka["GBps"] / HBM_PEAK_GBS, 4)
        ka.pop("TFLOPs", None)
        ka.pop("mfma_frac", None)
        ka["note"] = ("stops where exp(G_cum) is an exact zero in every channel (bitwise the same o); alg_bytes "
                      "counts the 64-token blocks it works on; dense_* = the same kernel streaming every token")
        if dense_ms:
            ka["dense_ms"] = round(dense_ms, 4)
            ka["dense_alg_bytes"] = ab["apply"]
            ka["dense_GBps"] = round(ab["apply"] / dense_ms / 1e6, 1)
            ka["dense_hbm_frac"] = round(ab["apply"] / dense_ms / 1e6 / HBM_PEAK_GBS, 4)
            # the step with the correction streaming every token (gates near 1 leave no other choice)
            dms = ms["local"] + ms["scan"] + dense_ms
            dense_step = {"ms_per_step": round(dms, 4), "tokens_per_s": round(B * T / (dms * 1e-3), 1),
                          "note": "local + scan as timed + the dense correction: what the step costs when no decay vanishes"}
    if scan_cold:
        kernels["scan"]["cold_cache_ms"] = round(scan_cold, 4)
        kernels["scan"]["cold_cache_GBps"] = round(ab["scan"] / scan_cold / 1e6, 1)
        kernels["scan"]["cold_after_fill_ms"] = round(scan_cold_fill, 4)
        kernels["scan"]["cold_after_fill_GBps"] = round(ab["scan"] / scan_cold_fill / 1e6, 1)
        kernels["scan"]["note"] = ("GBps is effective (working set may sit in the Infinity Cache); cold_cache_* after a "
                                   "1 GiB read sweep, cold_after_fill_* after a 512 MiB fill (dirty lines to evict)")
    ach = ab["local"] / ms["local"] / 1e6
    out = {
        "metric": "tokens/s for GLA segment fwd + state scan (1 MI355X)",
        "value": B * T / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": c["io"], "data": "synthetic",
        "config": {"workload": "%s: B=%d H=%d P=%d segments x L=%d tokens, d_k=d_v=%d, C=%d, %s q/k/v/o, "
                               "%s log-decay per %s; local fwd + segment-state scan + init-state correction"
                               % (workload, B, H, P, L, dk, c["C"], c["io"], args.g_dtype,
                                  "channel" if args.gate == "channel" else "head"),
                   "K_blocks": args.k_blocks, "layout": args.layout, "tensor_GiB": round(tensor_gib, 1)},
        "roofline": {"kernel": "gla_chunk_bf16_kernel (zeco_gla_local_fwd)", "bound": "hbm",
                     "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(ach / HBM_PEAK_GBS, 4),
                     "traffic": MEASURED_TRAFFIC.get((workload, args.g_dtype)) if args.gate == "channel" else None},
        "kernels": kernels,
        "dense_correction_step": dense_step,
        "two_phase": two_phase,
        "fused_correct": fused_correct,
        "chunk_decay": chunk_decay,
        "backward": backward,
        "g_bf16": g_bf16,
        "wide_gates": wide,
        "hbm_copy_GBps": None if copy_gbs is None else round(copy_gbs, 1),
        "hbm_mix_GBps": mix_gbs,
    }
    if skipped:
        out["skipped"] = skipped
    if workload == "c3" and not (args.only_pipeline or args.only_fused or args.only_backward):
        if c["io"] == "bf16" and args.gate == "channel" and P >= 2:
            out["unequal_segments"] = unequal_segments_case(args, inp, P, T)
    if with_cpu:
        out["cpu_baseline"] = cpu_baseline(inp, c, min(T, 131072))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c5", choices=["c2", "c3", "c4", "c5"])
    ap.add_argument("--g-dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--gate", default="channel", choices=["channel", "head"],
                    help="one log decay per (token, head, channel) as in GLA (default), or per (token, head)")
    ap.add_argument("--k-blocks", type=int, default=16)
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-backward", action="store_true", help="skip the backward timing")
    ap.add_argument("--no-cold-scan", action="store_true", help="skip the cold-cache timing of the scan")
    ap.add_argument("--no-variants", action="store_true", help="skip the bf16-gate timing")
    ap.add_argument("--no-others", action="store_true", help="skip the c3 / c2 / scan legs appended to the default workload")
    ap.add_argument("--only-pipeline", action="store_true",
                    help="time the three calls (and the calibration copy) only: no fused, backward, variant or "
                         "cold-scan legs (for profiler runs, whose per-kernel statistics then cover one launch "
                         "shape each)")
    ap.add_argument("--only-backward", action="store_true",
                    help="besides the three calls, time only the backward (and the training pair)")
    ap.add_argument("--only-fused", action="store_true",
                    help="besides the three calls, time only the fused forward (both schedules)")
    ap.add_argument("--dense-correction", action="store_true",
                    help="pass ZECO_APPLY_DENSE to the correction of the timed pipeline")
    ap.add_argument("--layout", default="bthd", choices=["bthd", "bhtd"],
                    help="memory order of q/k/v/g/o: token-major (default) or head-major")
    ap.add_argument("--calib-copy-mib", type=int, default=1024,
                    help="size of the plain copy timed beside the kernels (0 = skip)")
    args = ap.parse_args()
    if args.only_pipeline or args.only_fused:
        args.no_backward = True
    if args.only_pipeline or args.only_fused or args.only_backward:
        args.no_cold_scan = args.no_variants = args.no_others = True
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (P sequence segments resident on one MI355X); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch

    torch.cuda.set_device(0)
    out = run_workload(args, args.workload, with_cpu=not args.no_cpu)
    torch.cuda.empty_cache()
    if not args.no_others:
        others = {}
        if args.workload != "c3":
            r = run_workload(args, "c3", with_cpu=False)
            torch.cuda.empty_cache()
            others["c3"] = {n: r[n] for n in ("value", "ms_per_step", "config", "roofline", "kernels", "dense_correction_step",
                                              "two_phase", "fused_correct", "chunk_decay", "backward", "g_bf16", "wide_gates",
                                              "unequal_segments") if n in r}
        if args.workload != "c2":
            others["c2"] = single_segment_case(args)
        out["other_workloads"] = others
        out["scan_variants"] = scan_variants_case(args)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
