"""Segments of unequal length (zeco_gla_local_fwd_varlen, zeco_apply_init_state_varlen, and the two phases
zeco_gla_local_state_varlen, zeco_gla_fwd_from_state_varlen, and the backward's building blocks): the local pass of
every segment against the oracle's local pass of that token range on its own, and the three calls (the scan is
the ordinary one) against the unsegmented fp64 recurrence over the whole sequence.  Lengths mix multiples of
the chunk size with ragged ones, one chunk with many, and differ by up to 30x inside one call; tokens before
the first segment and after the last must come back untouched."""
import zlib

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2507_01004_amd import synth, zeco
from tests.gpu_util import TOL, host, log_err, rel_err_bh

pytestmark = pytest.mark.gpu

# (name, B, H, lengths, d_k, d_v, g dtype, per-head gate); io is fp32 where the name says so, else bf16
CASES = [
    ("f32_mixed", 1, 2, (100, 64, 191, 320), 64, 64, "f32", False),
    ("f32_d128", 2, 1, (65, 1100, 129), 128, 128, "f32", False),                 # correction: 2 workgroups for the longest
    ("mixed_d128", 1, 4, (64, 200, 65, 1000, 128), 128, 128, "f32", False),       # sibling workgroups split d_v
    ("mixed_whole", 2, 16, (127, 64, 300, 191, 77), 128, 128, "f32", False),     # one workgroup per stream
    ("long_and_short", 1, 2, (2100, 70, 1320), 128, 128, "f32", False),          # correction: 3 workgroups for the longest
    ("gbf16_d64", 1, 3, (100, 640, 90, 257), 64, 64, "bf16", False),
    ("dk64_dv128", 1, 2, (129, 64, 512), 64, 128, "f32", False),
    ("head_gate", 1, 4, (200, 64, 1000, 333), 128, 128, "f32", True),
    ("equal", 1, 2, (256, 256, 256), 128, 128, "f32", False),                    # must agree with the ordinary call
]


def offsets(lengths):
    return [0] + [int(x) for x in np.cumsum(lengths)]


def io_of(name):
    return "f32" if name.startswith("f32") else "bf16"


def make(case, T, **kw):
    name, B, H, lengths, dk, dv, gd, ph = case
    return synth.make_inputs(B, T, H, dk, dv, seed=zlib.crc32(name.encode()) % 10000 + 21, io=io_of(name), g=gd,
                             device="cuda", per_head_gate=ph, **kw)


def widen(g, dk):
    """Host copy of the gate as the oracle takes it: [B,T,H,d_k]."""
    g = host(g)
    return g if g.ndim == 4 else np.repeat(g[..., None], dk, axis=-1)


def first_channel(G, per_head):
    return G[..., 0] if per_head else G


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_varlen_local_pass_and_three_calls(case):
    name, B, H, lengths, dk, dv, gd, ph = case
    print("case", case, flush=True)
    tol = TOL[io_of(name)]
    P, T, Lmax = len(lengths), sum(lengths), max(lengths)
    start = offsets(lengths)
    seg = torch.tensor(start, dtype=torch.int64, device="cuda")
    inp = make(case, T)
    o, S_loc, G_cum, G_tot = zeco.gla_local_fwd_varlen(inp["q"], inp["k"], inp["v"], inp["g"], seg, Lmax, scale=0.5)
    torch.cuda.synchronize()
    q, k, v, g = host(inp["q"]), host(inp["k"]), host(inp["v"]), widen(inp["g"], dk)
    for p in range(P):
        a, e = start[p], start[p + 1]
        o_r, S_r, Gc_r, Gt_r = oracle.gla_local(q[:, a:e], k[:, a:e], v[:, a:e], g[:, a:e], 1, 0.5)
        assert rel_err_bh(host(o)[:, a:e], o_r, (0, 2)) <= tol, p
        assert rel_err_bh(host(S_loc)[p], S_r[0], (0, 1)) <= tol, p
        assert log_err(host(G_cum)[:, a:e], first_channel(Gc_r, ph)) <= 1e-5, p
        assert log_err(host(G_tot)[p], first_channel(Gt_r[0], ph)) <= 1e-5, p
    if name == "equal":   # the same kernels on the same data: identical to the call with one length
        o2, S2, Gc2, Gt2 = zeco.gla_local_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P, scale=0.5)
        assert torch.equal(o, o2) and torch.equal(S_loc, S2) and torch.equal(G_cum, Gc2) and torch.equal(G_tot, Gt2)

    # the three calls against the unsegmented recurrence, slow decay so that the correction reaches every token
    inp = make(case, T, gate_div=64.0)
    gen = torch.Generator(device="cuda").manual_seed(zlib.crc32(name.encode()) % 10000 + 22)
    S0 = torch.randn(B, H, dk, dv, device="cuda", generator=gen) * 0.5
    o, S_loc, G_cum, G_tot = zeco.gla_local_fwd_varlen(inp["q"], inp["k"], inp["v"], inp["g"], seg, Lmax, scale=0.5)
    o_local = host(o).copy()
    S_init, S_last = zeco.state_scan(S_loc, G_tot, S0=S0)
    for dense in (False, True):
        o_c = o.clone()
        zeco.apply_init_state_varlen(inp["q"], inp["g"], G_cum, S_init, o_c, seg, Lmax, scale=0.5,
                                     first_segment_is_zero=False, dense=dense)
        torch.cuda.synchronize()
        o_f, S_f = oracle.gla_recurrent(host(inp["q"]), host(inp["k"]), host(inp["v"]), widen(inp["g"], dk), 0.5,
                                        host(S0))
        assert rel_err_bh(host(o_c), o_f, (0, 2)) <= tol, dense
    assert rel_err_bh(host(S_last), S_f, (0, 1)) <= tol
    assert rel_err_bh(o_local, o_f, (0, 2)) > 5 * tol     # the correction matters here
    if io_of(name) == "bf16":   # Alg. 1's own schedule over the same table: states, scan, output from the states
        S_loc2, G_tot2 = zeco.gla_local_state_varlen(inp["k"], inp["v"], inp["g"], seg, Lmax)
        S_init2, S_last2 = zeco.state_scan(S_loc2, G_tot2, S0=S0)
        o2 = zeco.gla_fwd_from_state_varlen(inp["q"], inp["k"], inp["v"], inp["g"], S_init2, seg, Lmax, scale=0.5)
        torch.cuda.synchronize()
        assert log_err(host(G_tot2), host(G_tot)) <= 1e-5     # (the two modes sum the gates in different orders)
        assert rel_err_bh(host(S_loc2), host(S_loc), (1, 2)) <= tol
        assert rel_err_bh(host(o2), o_f, (0, 2)) <= tol
        assert rel_err_bh(host(S_last2), S_f, (0, 1)) <= tol
        # the same three phases as one call: the same kernels on the same data
        o3, S_last3 = zeco.gla_fused_fwd_varlen(inp["q"], inp["k"], inp["v"], inp["g"], seg, Lmax, scale=0.5, S0=S0)
        torch.cuda.synchronize()
        assert torch.equal(o3, o2) and torch.equal(S_last3, S_last2)


@pytest.mark.parametrize("case", [c for c in CASES if not c[0].startswith("f32")], ids=lambda c: c[0])
def test_varlen_backward_building_blocks(case):
    """Forward states, their scan, the state gradients, the reverse scan and the gradient passes, all over the
    same table, against the oracle's backward of the unsegmented recurrence with S0 and dS_T."""
    name, B, H, lengths, dk, dv, gd, ph = case
    print("case", case, flush=True)
    tol = TOL["bf16"]
    P, T, Lmax = len(lengths), sum(lengths), max(lengths)
    seg = torch.tensor(offsets(lengths), dtype=torch.int64, device="cuda")
    inp = make(case, T, gate_div=64.0)
    q, k, v, g = (inp[n] for n in "qkvg")
    gen = torch.Generator(device="cuda").manual_seed(zlib.crc32(name.encode()) % 10000 + 23)
    dO = torch.randn(v.shape, generator=gen, device="cuda").to(torch.bfloat16)
    S0 = torch.randn(B, H, dk, dv, device="cuda", generator=gen) * 0.3
    dS_T = torch.randn(B, H, dk, dv, device="cuda", generator=gen) * 0.3
    S_loc, G_tot = zeco.gla_local_state_varlen(k, v, g, seg, Lmax)
    S_init, S_last = zeco.state_scan(S_loc, G_tot, S0=S0)
    dS_loc = zeco.gla_bwd_dstate_varlen(q, g, dO, seg, Lmax, scale=0.5)
    dS_in, dS0 = zeco.state_scan(dS_loc, G_tot, S0=dS_T, direction=1)
    got = zeco.gla_bwd_from_state_varlen(q, k, v, g, dO, S_init, S_last, dS_in, seg, Lmax, scale=0.5)
    torch.cuda.synchronize()
    ref = oracle.gla_recurrent_bwd(host(q), host(k), host(v), widen(g, dk), host(dO), 0.5, host(S0), host(dS_T))
    for nm, x, r in zip(("dq", "dk", "dv"), got[:3], ref[:3]):
        assert rel_err_bh(host(x), r, (0, 2)) <= tol, nm
    # (dg: the running sum over a segment is re-anchored every 512 tokens, so long segments hold the bound too)
    assert rel_err_bh(host(got[3]), ref[3].sum(axis=-1) if ph else ref[3], (0, 2)) <= tol, "dg"
    assert rel_err_bh(host(dS0), ref[4], (0, 1)) <= tol, "dS0"
    # the whole backward as one call (its dQ pass also emits the state gradients, so dS_loc is rounded differently)
    one = zeco.gla_fused_bwd_varlen(q, k, v, g, dO, seg, Lmax, scale=0.5, S0=S0, dS_T=dS_T)
    torch.cuda.synchronize()
    for nm, x, r in zip(("dq", "dk", "dv"), one[:3], ref[:3]):
        assert rel_err_bh(host(x), r, (0, 2)) <= tol, nm + ", one call"
    assert rel_err_bh(host(one[3]), ref[3].sum(axis=-1) if ph else ref[3], (0, 2)) <= tol, "dg, one call"
    assert rel_err_bh(host(one[4]), ref[4], (0, 1)) <= tol, "dS0, one call"


def test_varlen_tokens_outside_the_segments_stay_untouched_and_bound_may_be_loose():
    """Tokens before the first segment and after the last one belong to no segment: their rows of o and G_cum
    keep the pattern they held.  The bound on the lengths is far above the longest segment."""
    B, H, dk, dv = 1, 4, 128, 128
    lengths, lead, tail = (150, 64, 400), 37, 7
    print("outside tokens", lengths, lead, tail, flush=True)
    seg = torch.tensor([lead + s for s in offsets(lengths)], dtype=torch.int64, device="cuda")
    T = lead + sum(lengths) + tail
    inp = synth.make_inputs(B, T, H, dk, dv, seed=78, io="bf16", g="f32", device="cuda", gate_div=64.0)
    mark = 123.0
    o = torch.full((B, T, H, dv), mark, dtype=torch.bfloat16, device="cuda")
    G_cum = torch.full((B, T, H, dk), mark, dtype=torch.float32, device="cuda")
    P = len(lengths)
    S_loc = torch.empty(P, B, H, dk, dv, device="cuda")
    G_tot = torch.empty(P, B, H, dk, device="cuda")
    zeco.gla_local_fwd_varlen(inp["q"], inp["k"], inp["v"], inp["g"], seg, 4096, scale=1.0,
                              out=(o, S_loc, G_cum, G_tot))
    S_init, S_last = zeco.state_scan(S_loc, G_tot)
    zeco.apply_init_state_varlen(inp["q"], inp["g"], G_cum, S_init, o, seg, 4096, scale=1.0)
    torch.cuda.synchronize()
    a, e = lead, lead + sum(lengths)
    assert torch.all(o[:, :a] == mark) and torch.all(o[:, e:] == mark)
    assert torch.all(G_cum[:, :a] == mark) and torch.all(G_cum[:, e:] == mark)
    sl = {n: host(inp[n])[:, a:e] for n in "qkvg"}
    o_f, S_f = oracle.gla_recurrent(sl["q"], sl["k"], sl["v"], sl["g"], 1.0, None)
    assert rel_err_bh(host(o)[:, a:e], o_f, (0, 2)) <= TOL["bf16"]
    assert rel_err_bh(host(S_last), S_f, (0, 1)) <= TOL["bf16"]


def test_varlen_segment_outside_the_rules_is_skipped():
    """A segment shorter than a chunk, or longer than the bound, is left alone by both kernels - its rows of
    o and its S_loc keep their contents - while the other segments are computed as usual."""
    B, H, dk, dv = 1, 2, 128, 128
    lengths = (128, 40, 200, 300)                        # 40 < 64; 300 > the bound of 256
    print("skipped segments", lengths, flush=True)
    start = offsets(lengths)
    T = start[-1]
    seg = torch.tensor(start, dtype=torch.int64, device="cuda")
    inp = synth.make_inputs(B, T, H, dk, dv, seed=79, io="bf16", g="f32", device="cuda")
    mark = 99.0
    o = torch.full((B, T, H, dv), mark, dtype=torch.bfloat16, device="cuda")
    G_cum = torch.full((B, T, H, dk), mark, dtype=torch.float32, device="cuda")
    S_loc = torch.full((4, B, H, dk, dv), mark, device="cuda")
    G_tot = torch.full((4, B, H, dk), mark, device="cuda")
    # T >= P * 64 holds (668 >= 256), so the host accepts the call
    zeco.gla_local_fwd_varlen(inp["q"], inp["k"], inp["v"], inp["g"], seg, 256, scale=1.0,
                              out=(o, S_loc, G_cum, G_tot))
    S_init = torch.zeros_like(S_loc)
    zeco.apply_init_state_varlen(inp["q"], inp["g"], G_cum, S_init, o, seg, 256, first_segment_is_zero=False)
    torch.cuda.synchronize()
    for p, taken in enumerate((True, False, True, False)):
        a, e = start[p], start[p + 1]
        if taken:
            sl = {n: host(inp[n])[:, a:e] for n in "qkvg"}
            o_r, S_r, _, _ = oracle.gla_local(sl["q"], sl["k"], sl["v"], sl["g"], 1, 1.0)
            assert rel_err_bh(host(o)[:, a:e], o_r, (0, 2)) <= TOL["bf16"], p
            assert rel_err_bh(host(S_loc)[p], S_r[0], (0, 1)) <= TOL["bf16"], p
        else:
            assert torch.all(o[:, a:e] == mark) and torch.all(S_loc[p] == mark) and torch.all(G_tot[p] == mark), p

    # offsets far outside the tensor: both segments that touch them are skipped, the others computed
    start = [0, 128, 2 ** 62, 368, 668]
    seg = torch.tensor(start, dtype=torch.int64, device="cuda")
    o.fill_(mark); S_loc.fill_(mark); G_tot.fill_(mark); G_cum.fill_(mark)
    zeco.gla_local_fwd_varlen(inp["q"], inp["k"], inp["v"], inp["g"], seg, 512, scale=1.0,
                              out=(o, S_loc, G_cum, G_tot))
    zeco.apply_init_state_varlen(inp["q"], inp["g"], G_cum, S_init, o, seg, 512, first_segment_is_zero=False)
    torch.cuda.synchronize()
    assert torch.all(o[:, 128:368] == mark) and torch.all(S_loc[1:3] == mark) and torch.all(G_tot[1:3] == mark)
    for p, (a, e) in ((0, (0, 128)), (3, (368, 668))):
        sl = {n: host(inp[n])[:, a:e] for n in "qkvg"}
        o_r, S_r, _, _ = oracle.gla_local(sl["q"], sl["k"], sl["v"], sl["g"], 1, 1.0)
        assert rel_err_bh(host(o)[:, a:e], o_r, (0, 2)) <= TOL["bf16"], p
        assert rel_err_bh(host(S_loc)[p], S_r[0], (0, 1)) <= TOL["bf16"], p
