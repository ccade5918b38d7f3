"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle, element by element,
on seeded synthetic inputs small enough for the oracle yet spanning several chunks, tiles,
segments and both workgroup decompositions of the bf16 chunk kernel."""
import zlib

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2507_01004_amd import synth, zeco
from tests.gpu_util import TOL, dev, host, log_err, oracle_full, oracle_local, rel_err_bh, randn_seeded

pytestmark = pytest.mark.gpu

# (name, B, H, P, L, d_k, d_v, io, g dtype)
CASES = [
    ("c1_f32", 1, 1, 4, 64, 64, 64, "f32", "f32"),                 # BASELINE config 1
    ("f32_d128", 2, 3, 2, 192, 128, 128, "f32", "f32"),
    ("f32_dk64_dv128", 1, 2, 3, 128, 64, 128, "f32", "f32"),
    ("f32_dk128_dv64", 1, 2, 2, 128, 128, 64, "f32", "f32"),
    ("bf16_sliced", 1, 4, 2, 320, 128, 128, "bf16", "f32"),        # 8 streams -> two sibling workgroups split d_v
    ("bf16_whole", 2, 16, 8, 128, 128, 128, "bf16", "f32"),        # 256 streams -> one workgroup per stream
    ("bf16_subseg", 1, 2, 2, 1024, 128, 128, "bf16", "f32"),       # 4 streams -> 4 sub-segments per segment
    ("bf16_subseg_d64", 1, 1, 1, 2048, 64, 64, "bf16", "bf16"),    # 1 stream  -> 8 sub-segments
    ("bf16_gbf16", 1, 3, 2, 256, 128, 128, "bf16", "bf16"),
    ("bf16_onechunk", 1, 2, 4, 64, 128, 128, "bf16", "f32"),       # N = 1: pipeline prologue only
    ("bf16_whole_onechunk", 1, 16, 16, 64, 128, 128, "bf16", "f32"),
    ("bf16_d64", 1, 2, 4, 192, 64, 64, "bf16", "f32"),
    ("bf16_dk64_dv128", 1, 2, 2, 128, 64, 128, "bf16", "f32"),
    ("bf16_dk128_dv64", 1, 2, 2, 128, 128, 64, "bf16", "bf16"),
]


def make(case, **kw):
    name, B, H, P, L, dk, dv, io, gd = case
    return synth.make_inputs(B, P * L, H, dk, dv, seed=zlib.crc32(name.encode()) % 10000 + 7, io=io, g=gd,
                             device="cuda", **kw)


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_local_fwd_matches_oracle(case):
    name, B, H, P, L, dk, dv, io, gd = case
    print("case", case, flush=True)
    inp = make(case)
    o, S_loc, G_cum, G_tot = zeco.gla_local_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P, scale=0.5)
    torch.cuda.synchronize()
    o_r, S_r, Gc_r, Gt_r = oracle_local(inp, P, scale=0.5)
    tol = TOL[io]
    assert rel_err_bh(host(o), o_r, (0, 2)) <= tol
    assert rel_err_bh(host(S_loc), S_r, (0, 1, 2)) <= tol
    assert log_err(host(G_cum), Gc_r) <= 1e-5
    assert log_err(host(G_tot), Gt_r) <= 1e-5


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_pipeline_matches_unsegmented_oracle(case):
    """Local pass + scan + correction against Eq. (1) run over the whole sequence."""
    name, B, H, P, L, dk, dv, io, gd = case
    print("case", case, flush=True)
    inp = make(case, gate_div=64.0)      # slow decay: the incoming state matters at every token
    o, S_last, parts = zeco.segmented_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P)
    torch.cuda.synchronize()
    o_r, Sf_r = oracle_full(inp)
    tol = TOL[io]
    assert rel_err_bh(host(o), o_r, (0, 2)) <= tol
    assert rel_err_bh(host(S_last), Sf_r, (0, 1)) <= tol
    # the correction must matter in this test, otherwise it proves nothing about it
    o_loc, _, _, _ = oracle_local(inp, P)
    assert rel_err_bh(o_loc, o_r, (0, 2)) > 10 * tol or P == 1


@pytest.mark.parametrize("case", [CASES[0], CASES[4], CASES[5]], ids=lambda c: c[0])
def test_pipeline_with_incoming_state_and_zero_gate(case):
    """g == 0 (plain causal linear attention) and a non-zero S0: nothing decays, so the state
    and the correction reach every token with full weight."""
    name, B, H, P, L, dk, dv, io, gd = case
    print("case", case, flush=True)
    inp = make(case, zero_gate=True)
    S0 = randn_seeded((B, H, dk, dv), 7100) * 0.3
    o, S_last, _ = zeco.segmented_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P, S0=S0)
    torch.cuda.synchronize()
    o_r, Sf_r = oracle_full(inp, S0=host(S0))
    assert rel_err_bh(host(o), o_r, (0, 2)) <= TOL[io]
    assert rel_err_bh(host(S_last), Sf_r, (0, 1)) <= TOL[io]


def random_states(P, BH, dk, dv, seed):
    r = np.random.default_rng(seed)
    S_loc = r.standard_normal((P, BH, dk, dv)).astype(np.float32)
    G_tot = (-r.random((P, BH, dk)) * 3).astype(np.float32)
    S0 = r.standard_normal((BH, dk, dv)).astype(np.float32)
    return S_loc, G_tot, S0


@pytest.mark.parametrize("shape", [(4, 1, 64, 64), (8, 16, 128, 128), (1, 3, 128, 64), (37, 2, 64, 128)])
def test_state_scan_matches_oracle_and_is_block_independent(shape):
    P, BH, dk, dv = shape
    print("scan", shape, flush=True)
    S_loc, G_tot, S0 = random_states(P, BH, dk, dv, seed=P)
    for s0 in (None, S0):
        ref_init, ref_last = oracle.state_scan(S_loc, G_tot, s0)
        base = None
        for K in (1, 2, 8, dk // 4, dk):
            S_init, S_last = zeco.state_scan(dev(S_loc), dev(G_tot), None if s0 is None else dev(s0),
                                             K_blocks=K)
            torch.cuda.synchronize()
            assert rel_err_bh(host(S_init), ref_init, (1,)) <= 1e-5
            assert rel_err_bh(host(S_last), ref_last, (0,)) <= 1e-5
            if base is None:
                base = (S_init.clone(), S_last.clone())
            else:   # bitwise independent of the row-block count
                assert torch.equal(S_init, base[0]) and torch.equal(S_last, base[1])


@pytest.mark.parametrize("shape", [(64, 16, 128, 128), (256, 8, 128, 128), (33, 4, 128, 128), (100, 2, 64, 64)])
def test_state_scan_at_full_size_with_decays_of_order_one(shape):
    """The benchmark configurations' scan shapes (64 segments x 16 heads, 256 x 8) and two narrow ones, which
    take the other thread widths of the kernel, with log decays in (-3, 0): at the workloads' own gates
    exp(G_tot) is an exact zero, so only a case like this one checks the chained decay term at scale.  Both
    directions, against the oracle's serial chain."""
    P, BH, dk, dv = shape
    print("scan, full size", shape, flush=True)
    S_loc, G_tot, S0 = random_states(P, BH, dk, dv, seed=300 + P)
    ref_init, ref_last = oracle.state_scan(S_loc, G_tot, S0)
    S_init, S_last = zeco.state_scan(dev(S_loc), dev(G_tot), dev(S0))
    torch.cuda.synchronize()
    assert rel_err_bh(host(S_init), ref_init, (1,)) <= 1e-5
    assert rel_err_bh(host(S_last), ref_last, (0,)) <= 1e-5
    rev_init, rev_last = oracle.state_scan(np.flip(S_loc, 0), np.flip(G_tot, 0), None)
    S_init, S_last = zeco.state_scan(dev(S_loc), dev(G_tot), None, direction=1)
    torch.cuda.synchronize()
    assert rel_err_bh(host(S_init), np.flip(rev_init, 0), (1,)) <= 1e-5
    assert rel_err_bh(host(S_last), rev_last, (0,)) <= 1e-5


@pytest.mark.parametrize("shape", [(36, 2, 128, 128), (256, 1, 128, 64), (12, 3, 64, 128), (37, 2, 64, 64), (4, 1, 64, 64),
                                   (1, 2, 128, 128)])
def test_state_scan_tree_matches_oracle(shape):
    """The scan as a tree of depth two, both directions, with and without an incoming state, against the
    oracle's serial chain (the reverse chain = the oracle on the flipped segments); P = 37 (prime), 4 and 1
    have no divisor that shortens the chain and take the serial path."""
    P, BH, dk, dv = shape
    print("tree scan", shape, flush=True)
    S_loc, G_tot, S0 = random_states(P, BH, dk, dv, seed=100 + P)
    for s0 in (None, S0):
        ref_init, ref_last = oracle.state_scan(S_loc, G_tot, s0)
        S_init, S_last = zeco.state_scan_tree(dev(S_loc), dev(G_tot), None if s0 is None else dev(s0))
        again = zeco.state_scan_tree(dev(S_loc), dev(G_tot), None if s0 is None else dev(s0))
        torch.cuda.synchronize()
        assert rel_err_bh(host(S_init), ref_init, (1,)) <= 1e-5
        assert rel_err_bh(host(S_last), ref_last, (0,)) <= 1e-5
        assert torch.equal(S_init, again[0]) and torch.equal(S_last, again[1])      # deterministic
        rev_init, rev_last = oracle.state_scan(np.flip(S_loc, 0), np.flip(G_tot, 0), s0)
        S_init, S_last = zeco.state_scan_tree(dev(S_loc), dev(G_tot), None if s0 is None else dev(s0), direction=1)
        torch.cuda.synchronize()
        assert rel_err_bh(host(S_init), np.flip(rev_init, 0), (1,)) <= 1e-5
        assert rel_err_bh(host(S_last), rev_last, (0,)) <= 1e-5
    # one log decay per head: the oracle fed the broadcast value
    Gh = G_tot[..., 0].copy()
    ref_init, ref_last = oracle.state_scan(S_loc, np.repeat(Gh[..., None], dk, axis=-1), S0)
    S_init, S_last = zeco.state_scan_tree(dev(S_loc), dev(Gh), dev(S0))
    torch.cuda.synchronize()
    assert rel_err_bh(host(S_init), ref_init, (1,)) <= 1e-5
    assert rel_err_bh(host(S_last), ref_last, (0,)) <= 1e-5


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("dims", [(64, 64), (128, 128), (64, 128), (128, 64)])
def test_apply_init_state_matches_oracle(io, dims):
    dk, dv = dims
    B, H, P, L = 2, 2, 3, 128
    print("apply", io, dims, flush=True)
    r = np.random.default_rng(dk + dv)
    dt = synth.torch_dtype(io)
    q = torch.from_numpy(r.standard_normal((B, P * L, H, dk))).to(dt).cuda()
    o0 = torch.from_numpy(r.standard_normal((B, P * L, H, dv))).to(dt).cuda()
    G = -np.cumsum(r.random((B, P * L, H, dk)) * 0.05, axis=1).astype(np.float32)
    S = r.standard_normal((P, B, H, dk, dv)).astype(np.float32)
    for first_zero in (True, False):
        Sx = S.copy()
        if first_zero:
            Sx[0] = 0
        o = o0.clone()
        zeco.apply_init_state(q, torch.empty(0), dev(G), dev(Sx), o, P, scale=0.7,
                              first_segment_is_zero=first_zero)
        torch.cuda.synchronize()
        ref = oracle.apply_init_state(host(q), G.astype(np.float64), Sx.astype(np.float64), host(o0), 0.7)
        assert rel_err_bh(host(o), ref, (0, 2)) <= TOL[io]
    # zero incoming states leave o bitwise unchanged
    o = o0.clone()
    zeco.apply_init_state(q, torch.empty(0), dev(G), dev(np.zeros_like(S)), o, P, first_segment_is_zero=False)
    torch.cuda.synchronize()
    assert torch.equal(o, o0)


@pytest.mark.parametrize("io,per_head", [("f32", False), ("bf16", False), ("bf16", True)])   # per-head gates: bf16 only
def test_apply_init_state_stops_where_the_decay_has_vanished(io, per_head):
    """Once exp(G_cum) is an exact zero in every channel the correction adds nothing; the call that
    stops there and the call that streams every token (ZECO_APPLY_DENSE) must give the same o, and
    both must match the oracle.  Crossing points: inside a 64-token block, on a block boundary, on a
    workgroup boundary (1024 tokens), never (one slow channel), and before the first token."""
    dk, dv, B, H, L = 128, 64, 1, 5, 2048
    P = 2
    print("apply vanish", io, per_head, flush=True)
    r = np.random.default_rng(17)
    dt = synth.torch_dtype(io)
    q = torch.from_numpy(r.standard_normal((B, P * L, H, dk))).to(dt).cuda()
    o0 = torch.from_numpy(r.standard_normal((B, P * L, H, dv))).to(dt).cuda()
    S = r.standard_normal((P, B, H, dk, dv)).astype(np.float32)
    # per head: number of tokens after which every channel is below the threshold
    cross = [700, 1024, 1536, None, 0]
    g = np.zeros((B, P * L, H, dk), dtype=np.float32)
    for h, c in enumerate(cross):
        if c is None:
            g[:, :, h] = -0.2
            g[:, :, h, 5] = -0.01          # one channel that never vanishes within the segment
        elif c == 0:
            g[:, :, h] = -200.0
        else:
            g[:, :, h] = -106.0 / c * (1.0 + 0.3 * r.random(dk))
    if per_head:
        g = np.ascontiguousarray(g[..., 0])
    G = np.cumsum(g.reshape((B, P, L) + g.shape[2:]), axis=2).reshape(g.shape).astype(np.float32)
    G_full = G if not per_head else np.repeat(G[..., None], dk, axis=-1)
    outs = []
    for dense in (False, True):
        o = o0.clone()
        zeco.apply_init_state(q, torch.empty(0), dev(G), dev(S), o, P, scale=1.3,
                              first_segment_is_zero=False, dense=dense)
        torch.cuda.synchronize()
        outs.append(o)
    assert torch.equal(outs[0].float() + 0.0, outs[1].float() + 0.0)   # "+ 0.0": -0 and +0 compare equal anyway
    ref = oracle.apply_init_state(host(q), G_full.astype(np.float64), S.astype(np.float64), host(o0), 1.3)
    assert rel_err_bh(host(outs[0]), ref, (0, 2)) <= TOL[io]
    # where the decay has vanished o is untouched, bit for bit
    for h, c in enumerate(cross):
        if c is not None:
            c64 = -(-c // 64) * 64
            for p in range(P):
                assert torch.equal(outs[0][:, p * L + c64:(p + 1) * L, h], o0[:, p * L + c64:(p + 1) * L, h])


def test_correction_with_a_ragged_number_of_streams():
    """133 (segment, batch, head) streams: one full group of 128 and a partial one whose last block of 8
    is incomplete, for the workgroup-to-stream mapping of both correction kernels."""
    dk, dv, B, H, P, L = 64, 64, 1, 19, 8, 128
    r = np.random.default_rng(5)
    q = torch.from_numpy(r.standard_normal((B, P * L, H, dk))).to(torch.bfloat16).cuda()
    o0 = torch.from_numpy(r.standard_normal((B, P * L, H, dv))).to(torch.bfloat16).cuda()
    g = (-r.random((B, P * L, H, dk)) * 0.05).astype(np.float32)
    S = r.standard_normal((P, B, H, dk, dv)).astype(np.float32)
    S[0] = 0
    G = np.cumsum(g.reshape(B, P, L, H, dk), axis=2)
    Gk = np.zeros((B, P, L // 64, H, dk))
    Gk[:, :, 1:] = G.reshape(B, P, L // 64, 64, H, dk)[:, :, :-1, 63]
    ref = oracle.apply_init_state(host(q), G.reshape(B, P * L, H, dk), S.astype(np.float64), host(o0), 1.0)
    o = o0.clone()
    zeco.apply_init_state(q, torch.empty(0), dev(G.reshape(B, P * L, H, dk)), dev(S), o, P, first_segment_is_zero=True)
    o2 = o0.clone()
    zeco.apply_init_state_chunk_decay(q, dev(g), dev(Gk.reshape(B, P * L // 64, H, dk)), dev(S), o2, P,
                                      first_segment_is_zero=True)
    torch.cuda.synchronize()
    assert rel_err_bh(host(o), ref, (0, 2)) <= TOL["bf16"]
    assert rel_err_bh(host(o2), ref, (0, 2)) <= TOL["bf16"]
    assert torch.equal(o[:, :L], o0[:, :L]) and torch.equal(o2[:, :L], o0[:, :L])   # segment 0 untouched


def test_strided_views_and_determinism():
    """q, k, g, v taken as views of one fused projection buffer; two runs are bitwise equal."""
    B, T, H, d, P = 1, 256, 4, 128, 2
    gen = torch.Generator(device="cuda").manual_seed(5)
    fused = torch.randn(B, T, H, 4 * d, generator=gen, device="cuda").to(torch.bfloat16)
    q, k, v = fused[..., :d], fused[..., d:2 * d], fused[..., 2 * d:3 * d]
    g = (torch.nn.functional.logsigmoid(fused[..., 3 * d:].float()) / 16).to(torch.bfloat16)
    gbuf = torch.empty_like(fused)
    gbuf[..., :d] = g
    gv = gbuf[..., :d]
    outs = []
    for _ in range(2):
        o, S_last, parts = zeco.segmented_fwd(q, k, v, gv, P)
        torch.cuda.synchronize()
        outs.append((o.clone(), S_last.clone(), parts["G_cum"].clone()))
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    o_r, Sf_r = oracle.gla_recurrent(host(q), host(k), host(v), host(gv))
    assert rel_err_bh(host(outs[0][0]), o_r, (0, 2)) <= TOL["bf16"]
    assert rel_err_bh(host(outs[0][1]), Sf_r, (0, 1)) <= TOL["bf16"]


def test_errors_surface_as_exceptions():
    q = torch.zeros(1, 96, 1, 64, device="cuda")
    with pytest.raises(zeco.ZecoError):
        zeco.gla_local_fwd(q, q, q, q, 2)            # L = 48 is shorter than a chunk


def test_fp32_path_holds_its_tolerance_on_long_segments():
    """The accuracy path over 4 segments of 4096 tokens (64 chunks each, a ragged variant beside it): the
    relative error against the fp64 oracle stays below 1e-4 where rounding has thousands of steps to add up."""
    B, H, P, dk, dv = 1, 2, 4, 128, 128
    for L in (4096, 4000):
        print("fp32 long", L, flush=True)
        inp = synth.make_inputs(B, P * L, H, dk, dv, seed=4096 + L, io="f32", g="f32", device="cuda", gate_div=64.0)
        S0 = randn_seeded((B, H, dk, dv), 7101) * 0.3
        o, S_last, parts = zeco.segmented_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P, scale=0.5, S0=S0)
        torch.cuda.synchronize()
        o_r, Sf_r = oracle_full(inp, scale=0.5, S0=host(S0))
        assert rel_err_bh(host(o), o_r, (0, 2)) <= TOL["f32"]
        assert rel_err_bh(host(S_last), Sf_r, (0, 1)) <= TOL["f32"]
        Gc = np.cumsum(host(inp["g"]).reshape(B, P, L, H, dk), axis=2).reshape(B, P * L, H, dk)
        assert log_err(host(parts["G_cum"]), Gc) <= 1e-5


@pytest.mark.parametrize("per_head", [False, True])
def test_strong_gates_up_to_the_documented_range(per_head):
    """Log decays between -1.2 and -0.4 per token: up to 77 per chunk and channel, just inside the documented
    range (below 80) of the direct form K / Lambda, whose largest factor is then e^77.  Forward by every route
    and backward against the oracle; the correction dies out within the first chunk of a segment."""
    B, H, P, L, dk, dv = 1, 3, 2, 256, 128, 128
    print("strong gates", per_head, flush=True)
    inp = synth.make_inputs(B, P * L, H, dk, dv, seed=91, io="bf16", g="f32", device="cuda", per_head_gate=per_head)
    gen = torch.Generator(device="cuda").manual_seed(92)
    inp["g"] = -(0.4 + 0.8 * torch.rand(inp["g"].shape, generator=gen, device="cuda"))
    inp["g"][:, 64:128] = -1.2                          # one chunk at the strongest decay in every channel
    dO = torch.randn(inp["v"].shape, generator=gen, device="cuda").to(torch.bfloat16)
    q, k, v, g = (inp[n] for n in ("q", "k", "v", "g"))
    h = {n: host(t) for n, t in inp.items()}
    if per_head:
        h["g"] = np.repeat(h["g"][..., None], dk, axis=-1)
    o_r, S_r = oracle.gla_recurrent(h["q"], h["k"], h["v"], h["g"], 0.5)
    ref = oracle.gla_recurrent_bwd(h["q"], h["k"], h["v"], h["g"], host(dO), 0.5, None, None)
    o, S_last, _ = zeco.segmented_fwd(q, k, v, g, P, scale=0.5)
    outs = [o] + [zeco.gla_fused_fwd(q, k, v, g, P, scale=0.5, schedule=sc)[0]
                  for sc in (zeco.SCHEDULE_TWO_PHASE, zeco.SCHEDULE_CORRECT)]
    grads = zeco.gla_fused_bwd(q, k, v, g, dO, P, scale=0.5)
    torch.cuda.synchronize()
    for x in outs:
        assert torch.isfinite(x.float()).all()
        assert rel_err_bh(host(x), o_r, (0, 2)) <= TOL["bf16"]
    assert rel_err_bh(host(S_last), S_r, (0, 1)) <= TOL["bf16"]
    for name_, x, r in zip(("dq", "dk", "dv"), grads[:3], ref[:3]):
        assert rel_err_bh(host(x), r, (0, 2)) <= TOL["bf16"], name_
    # dG is a sum of nearly cancelling terms (exactly zero at a segment's first token): with decays this strong
    # the sum itself is small while the bf16 rounding noise of its terms is not, and the per-head layout adds up
    # 128 channels of it - the bound here is 5e-2 instead of the 2e-2 that holds on the workloads' gates
    dg_r = ref[3].sum(axis=-1) if per_head else ref[3]
    assert rel_err_bh(host(grads[3]), dg_r, (0, 2)) <= (5e-2 if per_head else TOL["bf16"])


@pytest.mark.parametrize("per_head", [False, True])
def test_wide_range_of_gates(per_head):
    """The wide range of gates (zeco_gla_desc.wide_gates): log decays of -1.2 to -2.4 per token, 77 to 154 per
    chunk and channel, and one chunk with all of its 150 in its first 30 tokens.  The decay factors of the operand
    tiles are then counted from half the chunk's total, so half a chunk's decay is what has to fit their range
    (below 80) wherever in the chunk it falls; counted from the chunk's start these gates overflow.  Forward by
    every route and backward against the oracle."""
    B, H, P, L, dk, dv = 1, 3, 2, 320, 128, 128
    print("gates beyond a whole-chunk reference", per_head, flush=True)
    inp = synth.make_inputs(B, P * L, H, dk, dv, seed=93, io="bf16", g="f32", device="cuda", per_head_gate=per_head)
    gen = torch.Generator(device="cuda").manual_seed(94)
    inp["g"] = -(1.2 + 1.2 * torch.rand(inp["g"].shape, generator=gen, device="cuda"))
    inp["g"][:, 64:128] = -2.4                          # one chunk at the strongest decay in every channel
    inp["g"][:, 192:222] = -5.0                         # one with all of its decay early ...
    inp["g"][:, 222:256] = -1e-3                        # ... and next to none late
    dO = torch.randn(inp["v"].shape, generator=gen, device="cuda").to(torch.bfloat16)
    q, k, v, g = (inp[n] for n in ("q", "k", "v", "g"))
    h = {n: host(t) for n, t in inp.items()}
    if per_head:
        h["g"] = np.repeat(h["g"][..., None], dk, axis=-1)
    o_r, S_r = oracle.gla_recurrent(h["q"], h["k"], h["v"], h["g"], 0.5)
    ref = oracle.gla_recurrent_bwd(h["q"], h["k"], h["v"], h["g"], host(dO), 0.5, None, None)
    with zeco.wide_gates():
        o, S_last, _ = zeco.segmented_fwd(q, k, v, g, P, scale=0.5)
        outs = [o] + [zeco.gla_fused_fwd(q, k, v, g, P, scale=0.5, schedule=sc)[0]
                      for sc in (zeco.SCHEDULE_TWO_PHASE, zeco.SCHEDULE_CORRECT)]
        grads = zeco.gla_fused_bwd(q, k, v, g, dO, P, scale=0.5)
    torch.cuda.synchronize()
    for x in outs:
        assert torch.isfinite(x.float()).all()
        assert rel_err_bh(host(x), o_r, (0, 2)) <= TOL["bf16"]
    assert rel_err_bh(host(S_last), S_r, (0, 1)) <= TOL["bf16"]
    for name_, x, r in zip(("dq", "dk", "dv"), grads[:3], ref[:3]):
        assert torch.isfinite(x.float()).all(), name_
        assert rel_err_bh(host(x), r, (0, 2)) <= TOL["bf16"], name_
    dg_r = ref[3].sum(axis=-1) if per_head else ref[3]
    assert torch.isfinite(grads[3]).all()
    print("  dg rel err %.4f" % rel_err_bh(host(grads[3]), dg_r, (0, 2)), flush=True)
    # dG under gates this strong: the state lives a token or two, so the sum of nearly cancelling terms is small
    # against its terms' bf16 rounding noise (the effect of the test above, here in both gate layouts)
    assert rel_err_bh(host(grads[3]), dg_r, (0, 2)) <= 6e-2


@pytest.mark.parametrize("per_head,L", [(False, 448), (True, 448), (False, 200)])
def test_wide_range_on_ordinary_gates(per_head, L):
    """wide_gates only moves the reference point of the tiles' decay factors: on the workloads' gates it gives the
    results of the standard range up to rounding.  Forward by every route and backward against the oracle, whole
    and ragged chunks."""
    B, H, P, dk, dv = 2, 3, 3, 128, 128
    print("wide range, ordinary gates", per_head, L, flush=True)
    inp = synth.make_inputs(B, P * L, H, dk, dv, seed=95 + L, io="bf16", g="f32", device="cuda", per_head_gate=per_head)
    dO = randn_seeded(inp["v"].shape, 96).to(torch.bfloat16)
    q, k, v, g = (inp[n] for n in ("q", "k", "v", "g"))
    h = {n: host(t) for n, t in inp.items()}
    if per_head:
        h["g"] = np.repeat(h["g"][..., None], dk, axis=-1)
    o_r, S_r = oracle.gla_recurrent(h["q"], h["k"], h["v"], h["g"], 0.5)
    ref = oracle.gla_recurrent_bwd(h["q"], h["k"], h["v"], h["g"], host(dO), 0.5, None, None)
    with zeco.wide_gates():
        o, S_last, _ = zeco.segmented_fwd(q, k, v, g, P, scale=0.5)
        outs = [o] + [zeco.gla_fused_fwd(q, k, v, g, P, scale=0.5, schedule=sc)[0]
                      for sc in (zeco.SCHEDULE_TWO_PHASE, zeco.SCHEDULE_CORRECT)]
        grads = zeco.gla_fused_bwd(q, k, v, g, dO, P, scale=0.5)
    torch.cuda.synchronize()
    for x in outs:
        assert rel_err_bh(host(x), o_r, (0, 2)) <= TOL["bf16"]
    assert rel_err_bh(host(S_last), S_r, (0, 1)) <= TOL["bf16"]
    dg_r = ref[3].sum(axis=-1) if per_head else ref[3]
    for name_, x, r in zip(("dq", "dk", "dv", "dg"), grads, (ref[0], ref[1], ref[2], dg_r)):
        assert rel_err_bh(host(x), r, (0, 2)) <= TOL["bf16"], name_


def test_empty_batch_is_a_no_op():
    """B = 0 through the binding: the calls succeed, return empty tensors and launch nothing."""
    q = torch.empty(0, 256, 2, 128, dtype=torch.bfloat16, device="cuda")
    g = torch.empty(0, 256, 2, 128, device="cuda")
    o, S_last, parts = zeco.segmented_fwd(q, q, q, g, 2)
    assert o.shape == q.shape and S_last.shape == (0, 2, 128, 128) and parts["S_loc"].shape == (2, 0, 2, 128, 128)
    o2, S2 = zeco.gla_fused_fwd(q, q, q, g, 2)
    grads = zeco.gla_fused_bwd(q, q, q, g, q, 2)
    torch.cuda.synchronize()
    assert o2.numel() == 0 and all(t.numel() == 0 for t in grads)


BF16_CASES = [c for c in CASES if c[7] == "bf16"]


@pytest.mark.parametrize("case", BF16_CASES, ids=[c[0] for c in BF16_CASES])
def test_two_phase_forward_matches_oracle(case):
    """Alg. 1's own schedule: states only, scan, output pass from the scanned states; and the fused
    entry point, with and without a state entering the first segment."""
    name, B, H, P, L, dk, dv, io, gd = case
    print("case", case, flush=True)
    inp = make(case, gate_div=64.0)
    q, k, v, g = inp["q"], inp["k"], inp["v"], inp["g"]
    tol = TOL[io]
    # phase 1 against the oracle's local pass
    S_loc, G_tot = zeco.gla_local_state(k, v, g, P)
    torch.cuda.synchronize()
    _, S_r, _, Gt_r = oracle_local(inp, P)
    assert rel_err_bh(host(S_loc), S_r, (0, 1, 2)) <= tol
    assert log_err(host(G_tot), Gt_r) <= 1e-5
    # phase 2 from the oracle's own scanned states (fp32 copies), against the unsegmented run
    S0 = randn_seeded((B, H, dk, dv), 7102) * 0.3
    for s0 in (None, S0):
        o_r, Sf_r = oracle_full(inp, scale=0.5, S0=None if s0 is None else host(s0))
        Si_r, _ = oracle.state_scan(S_r.reshape(P, B * H, dk, dv), Gt_r.reshape(P, B * H, dk),
                                    None if s0 is None else host(s0).reshape(B * H, dk, dv))
        o2 = zeco.gla_fwd_from_state(q, k, v, g, dev(Si_r.reshape(P, B, H, dk, dv)), P, scale=0.5)
        torch.cuda.synchronize()
        assert rel_err_bh(host(o2), o_r, (0, 2)) <= tol
        # everything in one call, by either schedule
        for sched in (zeco.SCHEDULE_TWO_PHASE, zeco.SCHEDULE_CORRECT, zeco.SCHEDULE_AUTO):
            o3, S_last = zeco.gla_fused_fwd(q, k, v, g, P, scale=0.5, S0=s0, schedule=sched)
            torch.cuda.synchronize()
            assert rel_err_bh(host(o3), o_r, (0, 2)) <= tol
            assert rel_err_bh(host(S_last), Sf_r, (0, 1)) <= tol


@pytest.mark.parametrize("case", BF16_CASES, ids=[c[0] for c in BF16_CASES])
def test_chunk_decay_form_matches_oracle(case):
    """The local pass that keeps the cumulative decay per chunk (Alg. 1's gamma~_[n] list) and the
    correction that rebuilds the in-chunk factor from g: each against the oracle, then chained."""
    name, B, H, P, L, dk, dv, io, gd = case
    print("case", case, flush=True)
    inp = make(case, gate_div=64.0)
    q, k, v, g = inp["q"], inp["k"], inp["v"], inp["g"]
    tol = TOL[io]
    o, S_loc, G_chunk, G_tot = zeco.gla_local_fwd_chunk_decay(q, k, v, g, P, scale=0.5)
    torch.cuda.synchronize()
    o_r, S_r, Gc_r, Gt_r = oracle_local(inp, P, scale=0.5)
    assert rel_err_bh(host(o), o_r, (0, 2)) <= tol
    assert rel_err_bh(host(S_loc), S_r, (0, 1, 2)) <= tol
    assert log_err(host(G_tot), Gt_r) <= 1e-5
    # G_chunk[n] = cumulative log decay at the last token before chunk n, zero at a segment's first chunk
    N = L // 64
    Gk_r = np.zeros((B, P, N, H, dk))
    Gk_r[:, :, 1:] = Gc_r.reshape(B, P, N, 64, H, dk)[:, :, :-1, 63]
    assert log_err(host(G_chunk), Gk_r.reshape(B, P * N, H, dk)) <= 1e-5
    # correction from the oracle's scanned states and the oracle's chunk decays, on the oracle's local output
    S0 = randn_seeded((B, H, dk, dv), 7103) * 0.3
    o_full, _ = oracle_full(inp, scale=0.5, S0=host(S0))
    Si_r, _ = oracle.state_scan(S_r.reshape(P, B * H, dk, dv), Gt_r.reshape(P, B * H, dk), host(S0).reshape(B * H, dk, dv))
    o2 = torch.from_numpy(o_r).to(q.dtype).cuda()
    zeco.apply_init_state_chunk_decay(q, g, dev(Gk_r.reshape(B, P * N, H, dk)), dev(Si_r.reshape(P, B, H, dk, dv)),
                                      o2, P, scale=0.5, first_segment_is_zero=False)
    torch.cuda.synchronize()
    assert rel_err_bh(host(o2), o_full, (0, 2)) <= tol
    # chained on the GPU
    S_init, S_last = zeco.state_scan(S_loc, G_tot, S0=S0)
    zeco.apply_init_state_chunk_decay(q, g, G_chunk, S_init, o, P, scale=0.5, first_segment_is_zero=False)
    torch.cuda.synchronize()
    assert rel_err_bh(host(o), o_full, (0, 2)) <= tol


@pytest.mark.parametrize("gd", ["f32", "bf16"])
def test_chunk_decay_correction_stops_where_the_decay_has_vanished(gd):
    """As test_apply_init_state_stops_where_the_decay_has_vanished, for the correction that works from g
    and the per-chunk decay: crossing inside a chunk, on a chunk boundary, on a workgroup boundary,
    never, and before the first token."""
    dk, dv, B, H, L, P = 128, 128, 1, 5, 2048, 2
    print("chunk-decay vanish", gd, flush=True)
    r = np.random.default_rng(23)
    q = torch.from_numpy(r.standard_normal((B, P * L, H, dk))).to(torch.bfloat16).cuda()
    o0 = torch.from_numpy(r.standard_normal((B, P * L, H, dv))).to(torch.bfloat16).cuda()
    S = r.standard_normal((P, B, H, dk, dv)).astype(np.float32)
    cross = [700, 1024, 1536, None, 0]
    g = np.zeros((B, P * L, H, dk), dtype=np.float32)
    for h, c in enumerate(cross):
        if c is None:
            g[:, :, h] = -0.2
            g[:, :, h, 5] = -0.01
        elif c == 0:
            g[:, :, h] = -200.0
        else:
            g[:, :, h] = -106.0 / c * (1.0 + 0.3 * r.random(dk))
    gt = torch.from_numpy(g).to(synth.torch_dtype(gd)).cuda()
    gh = host(gt)                                              # the gates as the kernel sees them
    G = np.cumsum(gh.reshape(B, P, L, H, dk), axis=2)
    Gk = np.zeros((B, P, L // 64, H, dk))
    Gk[:, :, 1:] = G.reshape(B, P, L // 64, 64, H, dk)[:, :, :-1, 63]
    Gk_dev = dev(Gk.reshape(B, P * L // 64, H, dk))
    outs = []
    for dense in (False, True):
        o = o0.clone()
        zeco.apply_init_state_chunk_decay(q, gt, Gk_dev, dev(S), o, P, scale=1.3, first_segment_is_zero=False,
                                          dense=dense)
        torch.cuda.synchronize()
        outs.append(o)
    assert torch.equal(outs[0].float() + 0.0, outs[1].float() + 0.0)
    ref = oracle.apply_init_state(host(q), G.reshape(B, P * L, H, dk), S.astype(np.float64), host(o0), 1.3)
    assert rel_err_bh(host(outs[0]), ref, (0, 2)) <= TOL["bf16"]
    for h, c in enumerate(cross):
        if c is not None:   # untouched from the first chunk whose incoming decay has vanished
            Gk_h = host(Gk_dev).reshape(B, P, L // 64, H, dk)[0, 0, :, h]
            n_stop = int(np.argmax((Gk_h < -105.0).all(axis=-1)))
            for p in range(P):
                assert torch.equal(outs[0][:, p * L + 64 * n_stop:(p + 1) * L, h], o0[:, p * L + 64 * n_stop:(p + 1) * L, h])


def test_fused_forward_fp32_has_the_two_phases_only():
    """fp32 inputs take Alg. 1's schedule (tests/test_gpu_f32_chunks.py); the chunk-decay correction schedule and
    the states saved for a backward exist for bf16 only."""
    q = torch.zeros(1, 64, 1, 64, device="cuda")
    o, _ = zeco.gla_fused_fwd(q, q, q, q, 1)
    assert torch.equal(o, q)
    with pytest.raises(zeco.ZecoError) as e:
        zeco.gla_fused_fwd(q, q, q, q, 1, schedule=zeco.SCHEDULE_CORRECT)
    assert e.value.status == zeco.ZECO_ERR_UNSUPPORTED
    with pytest.raises(zeco.ZecoError) as e:
        zeco.gla_fused_fwd(q, q, q, q, 1, save=torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))
    assert e.value.status == zeco.ZECO_ERR_UNSUPPORTED
