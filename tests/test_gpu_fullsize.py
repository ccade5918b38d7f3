"""Parity at the benchmark's full sizes and launch configuration, on sampled (segment, head)
slices the oracle can compute one by one.  For a segment p >= 1 the oracle is warm-started
W tokens before the segment: older history is attenuated by exp(sum of g over the window), and
the test asserts from the actual gates that this factor is below 1e-30."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2507_01004_amd import synth, zeco
from tests.gpu_util import TOL, host, log_err, rel_err_bh

pytestmark = pytest.mark.gpu
W = {"c2": 8192, "c3": 8192, "c4": 8192, "c5": 16384}   # warm-up tokens (slow heads of c5 decay 4x slower)


def slice_oracle(inp, L, p, h, W):
    """Oracle output for segment p, head h (batch 0) of the unsegmented run, and the state
    entering the segment."""
    t0 = max(0, p * L - W) if p > 0 else 0
    sl = slice(t0, (p + 1) * L)
    q, k, v, g = (host(inp[n][:1, sl, h:h + 1]) for n in ("q", "k", "v", "g"))
    if p > 0:
        warm = g[0, :p * L - t0, 0].sum(axis=0)
        assert t0 == 0 or warm.max() < np.log(1e-30), "warm-up window too short for these gates"
    o, _ = oracle.gla_recurrent(q, k, v, g)
    n_warm = p * L - t0
    S_in = None
    if n_warm:
        _, S_in = oracle.gla_recurrent(q[:, :n_warm], k[:, :n_warm], v[:, :n_warm], g[:, :n_warm])
    return o[:, n_warm:], S_in


@pytest.mark.parametrize("name,samples", [
    ("c2", [(0, 0), (0, 9), (0, 15)]),
    ("c3", [(0, 3), (1, 0), (4, 7), (7, 15)]),
    ("c4", [(0, 0), (1, 5), (37, 11), (63, 15)]),
    ("c5", [(0, 1), (1, 6), (128, 2), (255, 7)]),
])
def test_fullsize_sampled_slices(name, samples):
    inp, c = synth.config_inputs(name, device="cuda")
    P, L, H = c["P"], c["L"], c["H"]
    print("full-size", name, c, flush=True)
    o, S_last, parts = zeco.segmented_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P)
    o_fused, S_last_fused = zeco.gla_fused_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P,
                                               schedule=zeco.SCHEDULE_TWO_PHASE)
    o_corr, S_last_corr = zeco.gla_fused_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P,
                                             schedule=zeco.SCHEDULE_CORRECT)
    # the three calls with the cumulative decay kept per chunk
    o_cd, S_loc_cd, G_chunk, G_tot_cd = zeco.gla_local_fwd_chunk_decay(inp["q"], inp["k"], inp["v"], inp["g"], P)
    S_init_cd, S_last_cd = zeco.state_scan(S_loc_cd, G_tot_cd)
    zeco.apply_init_state_chunk_decay(inp["q"], inp["g"], G_chunk, S_init_cd, o_cd, P)
    del S_loc_cd, G_chunk, S_init_cd
    torch.cuda.synchronize()
    assert rel_err_bh(host(S_last_cd), host(S_last), (0, 1)) <= TOL[c["io"]]
    # all schedules end in the same state (up to bf16-operand rounding of the routes)
    assert rel_err_bh(host(S_last_fused), host(S_last), (0, 1)) <= TOL[c["io"]]
    assert rel_err_bh(host(S_last_corr), host(S_last), (0, 1)) <= TOL[c["io"]]
    for (p, h) in samples:
        print("  sample segment %d head %d" % (p, h), flush=True)
        o_ref, S_in = slice_oracle(inp, L, p, h, W[name])
        got = host(o[:1, p * L:(p + 1) * L, h:h + 1])
        assert rel_err_bh(got, o_ref, (0, 2)) <= TOL[c["io"]]
        assert rel_err_bh(host(o_fused[:1, p * L:(p + 1) * L, h:h + 1]), o_ref, (0, 2)) <= TOL[c["io"]]
        assert rel_err_bh(host(o_corr[:1, p * L:(p + 1) * L, h:h + 1]), o_ref, (0, 2)) <= TOL[c["io"]]
        assert rel_err_bh(host(o_cd[:1, p * L:(p + 1) * L, h:h + 1]), o_ref, (0, 2)) <= TOL[c["io"]]
        assert rel_err_bh(host(o_corr[:1, p * L:p * L + 256, h:h + 1]), o_ref[:, :256], (0, 2)) <= TOL[c["io"]]
        # the head of the segment is where the incoming state matters most
        assert rel_err_bh(got[:, :256], o_ref[:, :256], (0, 2)) <= TOL[c["io"]]
        if S_in is not None:
            assert rel_err_bh(host(parts["S_init"][p, :1, h:h + 1]), S_in, (0, 1)) <= TOL[c["io"]]
        Gc = np.cumsum(host(inp["g"][:1, p * L:(p + 1) * L, h:h + 1]), axis=1)
        assert log_err(host(parts["G_cum"][:1, p * L:(p + 1) * L, h:h + 1]), Gc) <= 1e-5
        assert log_err(host(parts["G_tot"][p, :1, h:h + 1]), Gc[:, -1]) <= 1e-5


def slice_oracle_bwd(inp, dO, L, p, h, P, W):
    """Oracle gradients for segment p, head h (batch 0) of the unsegmented run: the oracle runs on a
    window reaching W tokens before and after the segment; what lies outside is attenuated by the
    gates of the window, which is asserted."""
    T = P * L
    t0 = max(0, p * L - W)
    t1 = min(T, (p + 1) * L + W)
    sl = slice(t0, t1)
    q, k, v, g = (host(inp[n][:1, sl, h:h + 1]) for n in ("q", "k", "v", "g"))
    d = host(dO[:1, sl, h:h + 1])
    a, b = p * L - t0, (p + 1) * L - t0
    assert t0 == 0 or g[0, :a, 0].sum(axis=0).max() < np.log(1e-30)
    assert t1 == T or g[0, b:, 0].sum(axis=0).max() < np.log(1e-30)
    grads = oracle.gla_recurrent_bwd(q, k, v, g, d)
    return [x[:, a:b] for x in grads[:4]]


@pytest.mark.parametrize("name,samples", [
    ("c2", [(0, 0), (0, 9)]),
    ("c3", [(0, 3), (4, 7), (7, 15)]),
    ("c4", [(0, 0), (37, 11), (63, 15)]),
])
def test_fullsize_backward_sampled_slices(name, samples):
    inp, c = synth.config_inputs(name, device="cuda")
    P, L, H = c["P"], c["L"], c["H"]
    print("full-size backward", name, c, flush=True)
    gen = torch.Generator(device="cuda").manual_seed(4242)
    dO = torch.randn(inp["v"].shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    dq, dk, dv, dg, dS0 = zeco.gla_fused_bwd(inp["q"], inp["k"], inp["v"], inp["g"], dO, P)
    torch.cuda.synchronize()
    for (p, h) in samples:
        print("  sample segment %d head %d" % (p, h), flush=True)
        ref = slice_oracle_bwd(inp, dO, L, p, h, P, W[name])
        for nm, x, r in zip(("dq", "dk", "dv", "dg"), (dq, dk, dv, dg), ref):
            got = host(x[:1, p * L:(p + 1) * L, h:h + 1])
            print("    %s rel err %.4f" % (nm, rel_err_bh(got, r, (0, 2))), flush=True)
            assert rel_err_bh(got, r, (0, 2)) <= TOL[c["io"]], nm
            # both ends of the segment are where the states handed over by the scans matter most
            assert rel_err_bh(got[:, :256], r[:, :256], (0, 2)) <= TOL[c["io"]], nm
            assert rel_err_bh(got[:, -256:], r[:, -256:], (0, 2)) <= TOL[c["io"]], nm


def test_fullsize_backward_c5_sampled_slices():
    """Config 5 (8.4 M tokens, half the heads decaying four times slower): the fused backward on one fast and
    two slow heads; the slow heads are where states and state gradients carry furthest across the pieces."""
    inp, c = synth.config_inputs("c5", device="cuda")
    P, L, H = c["P"], c["L"], c["H"]
    print("full-size backward c5", c, flush=True)
    gen = torch.Generator(device="cuda").manual_seed(4245)
    dO = torch.empty_like(inp["v"])
    for t0 in range(0, P * L, 1 << 16):      # slab by slab: the fp32 draw of the whole tensor would be 32 GiB
        dO[:, t0:t0 + (1 << 16)] = torch.randn((1, 1 << 16, H, c["d_v"]), generator=gen, device="cuda").to(torch.bfloat16)
    dq, dk, dv, dg, dS0 = zeco.gla_fused_bwd(inp["q"], inp["k"], inp["v"], inp["g"], dO, P)
    torch.cuda.synchronize()
    for (p, h) in [(128, 2), (0, 6), (255, 7)]:
        print("  sample segment %d head %d" % (p, h), flush=True)
        ref = slice_oracle_bwd(inp, dO, L, p, h, P, W["c5"])
        for nm, x, r in zip(("dq", "dk", "dv", "dg"), (dq, dk, dv, dg), ref):
            got = host(x[:1, p * L:(p + 1) * L, h:h + 1])
            print("    %s rel err %.4f" % (nm, rel_err_bh(got, r, (0, 2))), flush=True)
            assert rel_err_bh(got, r, (0, 2)) <= TOL[c["io"]], nm
            assert rel_err_bh(got[:, :256], r[:, :256], (0, 2)) <= TOL[c["io"]], nm
            assert rel_err_bh(got[:, -256:], r[:, -256:], (0, 2)) <= TOL[c["io"]], nm


def test_fullsize_backward_building_blocks_sampled_slices():
    """Config 3 through the calls a sequence-parallel rank makes around the two scans, with the segments as
    given (16384 tokens each, not cut into pieces): forward states, scan, state gradients, reverse scan, gradient
    passes.  dG is a running sum over a whole segment there, re-anchored every 512 tokens.  Then the same over
    an unequal cut of the same tokens (three ragged lengths)."""
    inp, c = synth.config_inputs("c3", device="cuda")
    P, L, H = c["P"], c["L"], c["H"]
    tol = TOL[c["io"]]
    print("full-size backward building blocks", c, flush=True)
    q, k, v, g = (inp[n] for n in ("q", "k", "v", "g"))
    gen = torch.Generator(device="cuda").manual_seed(4246)
    dO = torch.randn(v.shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    S_loc, G_tot = zeco.gla_local_state(k, v, g, P)
    S_init, S_last = zeco.state_scan(S_loc, G_tot)
    dS_loc = zeco.gla_bwd_dstate(q, g, dO, P)
    dS_in, dS0 = zeco.state_scan(dS_loc, G_tot, direction=1)
    grads = zeco.gla_bwd_from_state(q, k, v, g, dO, S_init, S_last, dS_in, P)
    torch.cuda.synchronize()
    for (p, h) in [(0, 3), (4, 7), (7, 15)]:
        print("  sample segment %d head %d" % (p, h), flush=True)
        ref = slice_oracle_bwd(inp, dO, L, p, h, P, W["c3"])
        for nm, x, r in zip(("dq", "dk", "dv", "dg"), grads, ref):
            got = host(x[:1, p * L:(p + 1) * L, h:h + 1])
            print("    %s rel err %.4f" % (nm, rel_err_bh(got, r, (0, 2))), flush=True)
            assert rel_err_bh(got, r, (0, 2)) <= tol, nm
            assert rel_err_bh(got[:, :256], r[:, :256], (0, 2)) <= tol, nm
            assert rel_err_bh(got[:, -256:], r[:, -256:], (0, 2)) <= tol, nm

    lengths = [8190, 24576, 16384, 12291, 20480, 16387, 4100, 28664]
    start = [0] + [int(x) for x in np.cumsum(lengths)]
    seg = torch.tensor(start, dtype=torch.int64, device="cuda")
    bound = max(lengths)
    print("  unequal segments", lengths, flush=True)
    S_loc, G_tot = zeco.gla_local_state_varlen(k, v, g, seg, bound)
    S_init, S_last = zeco.state_scan(S_loc, G_tot)
    dS_loc = zeco.gla_bwd_dstate_varlen(q, g, dO, seg, bound)
    dS_in, dS0 = zeco.state_scan(dS_loc, G_tot, direction=1)
    grads = zeco.gla_bwd_from_state_varlen(q, k, v, g, dO, S_init, S_last, dS_in, seg, bound)
    torch.cuda.synchronize()
    T = P * L
    for (p, h) in [(0, 5), (3, 12), (7, 15)]:
        print("  sample segment %d head %d" % (p, h), flush=True)
        a, e = start[p], start[p + 1]
        t0, t1 = max(0, a - W["c3"]), min(T, e + W["c3"])
        hq, hk, hv, hg = (host(inp[n][:1, t0:t1, h:h + 1]) for n in ("q", "k", "v", "g"))
        assert t0 == 0 or hg[0, :a - t0, 0].sum(axis=0).max() < np.log(1e-30)
        assert t1 == T or hg[0, e - t0:, 0].sum(axis=0).max() < np.log(1e-30)
        ref = oracle.gla_recurrent_bwd(hq, hk, hv, hg, host(dO[:1, t0:t1, h:h + 1]))
        for nm, x, r in zip(("dq", "dk", "dv", "dg"), grads, ref[:4]):
            got, r = host(x[:1, a:e, h:h + 1]), r[:, a - t0:e - t0]
            print("    %s rel err %.4f" % (nm, rel_err_bh(got, r, (0, 2))), flush=True)
            assert rel_err_bh(got, r, (0, 2)) <= tol, nm


def test_fullsize_ragged_segment_length_sampled_slices():
    """c3's tensors cut to 8 segments of 16380 tokens (255 chunks and one of 60 tokens per segment; the
    fused backward cuts each into 35 pieces of 468): every forward route and the backward on sampled slices."""
    inp, c = synth.config_inputs("c3", device="cuda")
    P, H, L = c["P"], c["H"], 16380
    gen = torch.Generator(device="cuda").manual_seed(4243)
    dO = torch.randn(inp["v"].shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)[:, :P * L]
    inp = {n: t[:, :P * L] for n, t in inp.items()}      # views: the strides of the full tensors
    q, k, v, g = (inp[n] for n in ("q", "k", "v", "g"))
    tol = TOL[c["io"]]
    print("full-size ragged", P, L, flush=True)
    o, S_last, parts = zeco.segmented_fwd(q, k, v, g, P)
    o_tp, S_tp = zeco.gla_fused_fwd(q, k, v, g, P, schedule=zeco.SCHEDULE_TWO_PHASE)
    o_co, S_co = zeco.gla_fused_fwd(q, k, v, g, P, schedule=zeco.SCHEDULE_CORRECT)
    grads = zeco.gla_fused_bwd(q, k, v, g, dO, P)
    torch.cuda.synchronize()
    assert rel_err_bh(host(S_tp), host(S_last), (0, 1)) <= tol
    assert rel_err_bh(host(S_co), host(S_last), (0, 1)) <= tol
    for (p, h) in [(0, 2), (3, 9), (7, 15)]:
        print("  sample segment %d head %d" % (p, h), flush=True)
        seg = slice(p * L, (p + 1) * L)
        o_ref, S_in = slice_oracle(inp, L, p, h, W["c3"])
        for got in (o, o_tp, o_co):
            x = host(got[:1, seg, h:h + 1])
            assert rel_err_bh(x, o_ref, (0, 2)) <= tol
            assert rel_err_bh(x[:, :256], o_ref[:, :256], (0, 2)) <= tol
        if S_in is not None:
            assert rel_err_bh(host(parts["S_init"][p, :1, h:h + 1]), S_in, (0, 1)) <= tol
        Gc = np.cumsum(host(g[:1, seg, h:h + 1]), axis=1)
        assert log_err(host(parts["G_cum"][:1, seg, h:h + 1]), Gc) <= 1e-5
        ref = slice_oracle_bwd(inp, dO, L, p, h, P, W["c3"])
        for nm, x, r in zip(("dq", "dk", "dv", "dg"), grads, ref):
            got = host(x[:1, seg, h:h + 1])
            assert rel_err_bh(got, r, (0, 2)) <= tol, nm
            assert rel_err_bh(got[:, :256], r[:, :256], (0, 2)) <= tol, nm
            assert rel_err_bh(got[:, -256:], r[:, -256:], (0, 2)) <= tol, nm


def range_oracle(inp, a, e, h, W):
    """Oracle output for the tokens [a, e) of head h (batch 0) of the unsegmented run, warm-started W tokens
    before a, and the state entering token a."""
    t0 = max(0, a - W)
    q, k, v, g = (host(inp[n][:1, t0:e, h:h + 1]) for n in ("q", "k", "v", "g"))
    n_warm = a - t0
    if t0 > 0:
        assert g[0, :n_warm, 0].sum(axis=0).max() < np.log(1e-30), "warm-up window too short for these gates"
    o, _ = oracle.gla_recurrent(q, k, v, g)
    S_in = None
    if n_warm:
        _, S_in = oracle.gla_recurrent(q[:, :n_warm], k[:, :n_warm], v[:, :n_warm], g[:, :n_warm])
    return o[:, n_warm:], S_in


def test_fullsize_unequal_segments_sampled_slices():
    """c3's tensors cut into 8 segments of 4100 to 28664 tokens (three of them ragged): the three calls over
    unequal segments on sampled (segment, head) slices."""
    inp, c = synth.config_inputs("c3", device="cuda")
    lengths = [8190, 24576, 16384, 12291, 20480, 16387, 4100, 28664]
    T = c["P"] * c["L"]
    assert sum(lengths) == T
    start = [0] + [int(x) for x in np.cumsum(lengths)]
    seg = torch.tensor(start, dtype=torch.int64, device="cuda")
    q, k, v, g = (inp[n] for n in ("q", "k", "v", "g"))
    tol = TOL[c["io"]]
    print("full-size unequal segments", lengths, flush=True)
    o, S_loc, G_cum, G_tot = zeco.gla_local_fwd_varlen(q, k, v, g, seg, max(lengths))
    S_init, S_last = zeco.state_scan(S_loc, G_tot)
    zeco.apply_init_state_varlen(q, g, G_cum, S_init, o, seg, max(lengths))
    _, S_last_eq, _ = zeco.segmented_fwd(q, k, v, g, c["P"])
    torch.cuda.synchronize()
    assert rel_err_bh(host(S_last), host(S_last_eq), (0, 1)) <= tol     # the end state does not depend on the cut
    for (p, h) in [(0, 5), (1, 0), (3, 12), (6, 9), (7, 15)]:
        print("  sample segment %d head %d" % (p, h), flush=True)
        a, e = start[p], start[p + 1]
        o_ref, S_in = range_oracle(inp, a, e, h, W["c3"])
        got = host(o[:1, a:e, h:h + 1])
        assert rel_err_bh(got, o_ref, (0, 2)) <= tol
        assert rel_err_bh(got[:, :256], o_ref[:, :256], (0, 2)) <= tol
        if S_in is not None:
            assert rel_err_bh(host(S_init[p, :1, h:h + 1]), S_in, (0, 1)) <= tol
        Gc = np.cumsum(host(g[:1, a:e, h:h + 1]), axis=1)
        assert log_err(host(G_cum[:1, a:e, h:h + 1]), Gc) <= 1e-5
        assert log_err(host(G_tot[p, :1, h:h + 1]), Gc[:, -1]) <= 1e-5


@pytest.mark.parametrize("name", ["c2", "c3"])
def test_fullsize_whole_forward_against_unsegmented_oracle(name):
    """Every token and head of configs 2 and 3 against Eq. (1) run over the whole sequence (the oracle
    needs a few seconds for 131072 tokens x 16 heads): the three calls, the fused call, and the three calls with
    the wide range of gates."""
    inp, c = synth.config_inputs(name, device="cuda")
    P = c["P"]
    print("whole forward", name, c, flush=True)
    o, S_last, _ = zeco.segmented_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P)
    o_fused, S_last_fused = zeco.gla_fused_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P)
    with zeco.wide_gates():      # the other reference point of the tiles' decay factors, in the same launch shapes
        o_wide, S_last_wide, _ = zeco.segmented_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P)
    torch.cuda.synchronize()
    o_ref, S_ref = oracle.gla_recurrent(*(host(inp[n]) for n in ("q", "k", "v", "g")))
    print("  oracle done", flush=True)
    for got, got_S in ((o, S_last), (o_fused, S_last_fused), (o_wide, S_last_wide)):
        assert rel_err_bh(host(got), o_ref, (0, 2)) <= TOL[c["io"]]
        assert rel_err_bh(host(got_S), S_ref, (0, 1)) <= TOL[c["io"]]
        # Frobenius norm of the error beside the max norm
        diff = host(got) - o_ref
        assert np.linalg.norm(diff) <= TOL[c["io"]] * np.linalg.norm(o_ref)


def test_fullsize_whole_backward_c2_against_oracle():
    """Config 2 (one segment of 16384 tokens, 16 heads): all four gradients at every token."""
    inp, c = synth.config_inputs("c2", device="cuda")
    print("whole backward c2", c, flush=True)
    gen = torch.Generator(device="cuda").manual_seed(4243)
    dO = torch.randn(inp["v"].shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    got = zeco.gla_fused_bwd(inp["q"], inp["k"], inp["v"], inp["g"], dO, c["P"])
    torch.cuda.synchronize()
    ref = oracle.gla_recurrent_bwd(*(host(inp[n]) for n in ("q", "k", "v", "g")), host(dO))
    print("  oracle done", flush=True)
    for nm, x, r in zip(("dq", "dk", "dv", "dg"), got[:4], ref[:4]):
        e = rel_err_bh(host(x), r, (0, 2))
        print("    %s rel err %.4f" % (nm, e), flush=True)
        assert e <= TOL[c["io"]], nm
    assert rel_err_bh(host(got[4]), ref[4], (0, 1)) <= TOL[c["io"]]
