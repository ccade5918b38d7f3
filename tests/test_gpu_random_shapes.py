"""Seeded random draw of valid problem shapes - batch, heads, segments, segment length (ragged or not, one
chunk to thousands of tokens), d_k, d_v, gate layout - so that the launch heuristics (sibling workgroups,
sub-segments, pieces, tree scan, short first chunk) meet combinations no hand-picked case lists.  For each
shape every forward route, the three calls over a random unequal cut of the same tokens, and the backward,
against the fp64 oracle's unsegmented recurrence with an incoming state and an outgoing state gradient."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2507_01004_amd import synth, zeco
from tests.gpu_util import TOL, host, rel_err_bh

pytestmark = pytest.mark.gpu
N_CASES, SEED, MAX_TOKEN_HEADS = 40, 2, 60000      # the oracle takes well under a second per case


def draw_cases():
    rng = np.random.default_rng(SEED)
    cases = []
    for ci in range(N_CASES):
        dk, dv = int(rng.choice([64, 128])), int(rng.choice([64, 128]))
        gate = str(rng.choice(["f32", "bf16", "head"]))
        B, H = int(rng.choice([1, 1, 2, 3])), int(rng.choice([1, 2, 3, 5, 8]))
        P = int(rng.choice([1, 2, 3, 4, 7, 16]))
        kind = int(rng.integers(0, 4))
        if kind == 0:
            L = int(rng.integers(64, 200))
        elif kind == 1:
            L = int(rng.choice([64, 128, 256, 512, 1024]))
        elif kind == 2:
            L = int(rng.integers(200, 1400))
        elif B * H * P <= 4:
            L = int(rng.choice([2048, 2056, 4096, 4100, 3000, 8192]))     # long, few streams: the cut paths
        else:
            L = int(rng.integers(64, 700))
        while B * P * L * H > MAX_TOKEN_HEADS and P > 1:
            P //= 2
        while B * P * L * H > MAX_TOKEN_HEADS and H > 1:
            H //= 2
        while B * P * L * H > MAX_TOKEN_HEADS and B > 1:
            B -= 1
        T = P * L
        # a random cut of the T tokens into 1..6 unequal segments of at least 64 tokens (None if the draw fails)
        start = None
        if T >= 128:
            nseg = int(rng.integers(1, min(6, T // 64) + 1))
            cuts = []
            if nseg > 1:
                cuts = sorted(int(c) * 64 + int(j) for c, j in zip(
                    rng.choice(np.arange(1, T // 64), size=nseg - 1, replace=False), rng.integers(-20, 20, size=nseg - 1)))
            cand = [0] + cuts + [T]
            if min(np.diff(cand)) >= 64:
                start = cand
        cases.append((ci, B, H, P, L, dk, dv, gate, start))
    return cases


CASES = draw_cases()


@pytest.mark.parametrize("case", CASES, ids=["%d_B%d_H%d_P%d_L%d_%dx%d_%s" % c[:8] for c in CASES])
def test_random_shape_all_routes(case):
    with zeco.wide_gates(case[0] % 3 == 2):     # every third shape with the other range of gates
        all_routes(case)


def all_routes(case):
    ci, B, H, P, L, dk, dv, gate, start = case
    print("case", case, flush=True)
    tol = TOL["bf16"]
    per_head = gate == "head"
    inp = synth.make_inputs(B, P * L, H, dk, dv, seed=1000 * SEED + ci, io="bf16", g="f32" if per_head else gate,
                            device="cuda", per_head_gate=per_head, gate_div=64.0)
    gen = torch.Generator(device="cuda").manual_seed(5000 + 1000 * SEED + ci)
    dO = torch.randn(inp["v"].shape, generator=gen, device="cuda").to(torch.bfloat16)
    S0 = torch.randn(B, H, dk, dv, device="cuda", generator=gen) * 0.3
    dS_T = torch.randn(B, H, dk, dv, device="cuda", generator=gen) * 0.3
    q, k, v, g = (inp[n] for n in "qkvg")
    hq, hk, hv, hg = host(q), host(k), host(v), host(g)
    if per_head:
        hg = np.repeat(hg[..., None], dk, axis=-1)
    o_f, S_f = oracle.gla_recurrent(hq, hk, hv, hg, 0.5, host(S0))
    ref = oracle.gla_recurrent_bwd(hq, hk, hv, hg, host(dO), 0.5, host(S0), host(dS_T))

    def check_forward(o, S_last, what):
        torch.cuda.synchronize()
        assert rel_err_bh(host(o), o_f, (0, 2)) <= tol, what
        assert rel_err_bh(host(S_last), S_f, (0, 1)) <= tol, what

    o, S_last, _ = zeco.segmented_fwd(q, k, v, g, P, scale=0.5, S0=S0)
    check_forward(o, S_last, "three calls")
    for sched in (zeco.SCHEDULE_TWO_PHASE, zeco.SCHEDULE_CORRECT, zeco.SCHEDULE_AUTO):
        o, S_last = zeco.gla_fused_fwd(q, k, v, g, P, scale=0.5, S0=S0, schedule=sched)
        check_forward(o, S_last, "fused, schedule %d" % sched)
    if not per_head and L % 64 == 0:
        o, S_loc, G_chunk, G_tot = zeco.gla_local_fwd_chunk_decay(q, k, v, g, P, scale=0.5)
        S_init, S_last = zeco.state_scan(S_loc, G_tot, S0=S0)
        zeco.apply_init_state_chunk_decay(q, g, G_chunk, S_init, o, P, scale=0.5, first_segment_is_zero=False)
        check_forward(o, S_last, "chunk decay")
    if start is not None:
        seg = torch.tensor(start, dtype=torch.int64, device="cuda")
        bound = int(max(np.diff(start)))
        o, S_loc, G_cum, G_tot = zeco.gla_local_fwd_varlen(q, k, v, g, seg, bound, scale=0.5)
        S_init, S_last = zeco.state_scan(S_loc, G_tot, S0=S0)
        zeco.apply_init_state_varlen(q, g, G_cum, S_init, o, seg, bound, scale=0.5, first_segment_is_zero=False)
        check_forward(o, S_last, "unequal segments %s" % (start,))
        S_loc, G_tot = zeco.gla_local_state_varlen(k, v, g, seg, bound)
        S_init, S_last = zeco.state_scan(S_loc, G_tot, S0=S0)
        o = zeco.gla_fwd_from_state_varlen(q, k, v, g, S_init, seg, bound, scale=0.5)
        check_forward(o, S_last, "unequal segments, two phases %s" % (start,))

    ref_dg = ref[3].sum(axis=-1) if per_head else ref[3]
    got = zeco.gla_fused_bwd(q, k, v, g, dO, P, scale=0.5, S0=S0, dS_T=dS_T)
    torch.cuda.synchronize()
    for nm, x, r in zip(("dq", "dk", "dv"), got[:3], ref[:3]):
        assert rel_err_bh(host(x), r, (0, 2)) <= tol, nm
    assert rel_err_bh(host(got[3]), ref_dg, (0, 2)) <= tol, "dg"
    assert rel_err_bh(host(got[4]), ref[4], (0, 1)) <= tol, "dS0"

    if start is not None:   # the backward's building blocks over the unequal cut
        S_loc, G_tot = zeco.gla_local_state_varlen(k, v, g, seg, bound)
        S_init, S_last = zeco.state_scan(S_loc, G_tot, S0=S0)
        dS_loc = zeco.gla_bwd_dstate_varlen(q, g, dO, seg, bound, scale=0.5)
        dS_in, dS0 = zeco.state_scan(dS_loc, G_tot, S0=dS_T, direction=1)
        got = zeco.gla_bwd_from_state_varlen(q, k, v, g, dO, S_init, S_last, dS_in, seg, bound, scale=0.5)
        torch.cuda.synchronize()
        for nm, x, r in zip(("dq", "dk", "dv"), got[:3], ref[:3]):
            assert rel_err_bh(host(x), r, (0, 2)) <= tol, nm + ", unequal segments"
        assert rel_err_bh(host(dS0), ref[4], (0, 1)) <= tol, "dS0, unequal segments"
        assert rel_err_bh(host(got[3]), ref_dg, (0, 2)) <= tol, "dg, unequal segments"


F32_CASES = [c for c in CASES if c[7] != "head"][::3]


@pytest.mark.parametrize("case", F32_CASES, ids=["%d_B%d_H%d_P%d_L%d_%dx%d_%s" % c[:8] for c in F32_CASES])
def test_random_shape_fp32_routes(case):
    """The same shapes on fp32 tensors, chunk length drawn from the three the fp32 kernels take: three calls,
    two-phase forward, the backward in one call and, over the unequal cut, forward and backward in one call each."""
    ci, B, H, P, L, dk, dv, gate, start = case
    C = (16, 32, 64)[ci % 3]
    print("fp32 case", case, "C", C, flush=True)
    tol = TOL["f32"]
    inp = synth.make_inputs(B, P * L, H, dk, dv, seed=3000 * SEED + ci, io="f32", g="f32", device="cuda", gate_div=64.0)
    gen = torch.Generator(device="cuda").manual_seed(7000 + 1000 * SEED + ci)
    dO = torch.randn(inp["v"].shape, generator=gen, device="cuda")
    S0 = torch.randn(B, H, dk, dv, device="cuda", generator=gen) * 0.3
    dS_T = torch.randn(B, H, dk, dv, device="cuda", generator=gen) * 0.3
    q, k, v, g = (inp[n] for n in "qkvg")
    hq, hk, hv, hg = host(q), host(k), host(v), host(g)
    o_f, S_f = oracle.gla_recurrent(hq, hk, hv, hg, 0.5, host(S0))
    ref = oracle.gla_recurrent_bwd(hq, hk, hv, hg, host(dO), 0.5, host(S0), host(dS_T))

    def check_forward(o, S_last, what):
        torch.cuda.synchronize()
        assert rel_err_bh(host(o), o_f, (0, 2)) <= tol, what
        assert rel_err_bh(host(S_last), S_f, (0, 1)) <= tol, what

    def check_backward(got, what):
        torch.cuda.synchronize()
        for nm, x, r in zip(("dq", "dk", "dv", "dg"), got[:4], ref[:4]):
            assert rel_err_bh(host(x), r, (0, 2)) <= tol, nm + what
        assert rel_err_bh(host(got[4]), ref[4], (0, 1)) <= tol, "dS0" + what

    o, S_last, _ = zeco.segmented_fwd(q, k, v, g, P, scale=0.5, S0=S0, C=C)
    check_forward(o, S_last, "three calls")
    o, S_last = zeco.gla_fused_fwd(q, k, v, g, P, scale=0.5, S0=S0, C=C)
    check_forward(o, S_last, "fused")
    check_backward(zeco.gla_fused_bwd(q, k, v, g, dO, P, scale=0.5, S0=S0, dS_T=dS_T, C=C), "")
    if start is not None:
        seg = torch.tensor(start, dtype=torch.int64, device="cuda")
        bound = int(max(np.diff(start)))
        o, S_last = zeco.gla_fused_fwd_varlen(q, k, v, g, seg, bound, scale=0.5, S0=S0, C=C)
        check_forward(o, S_last, "unequal segments %s" % (start,))
        check_backward(zeco.gla_fused_bwd_varlen(q, k, v, g, dO, seg, bound, scale=0.5, C=C, S0=S0, dS_T=dS_T),
                       ", unequal segments")
