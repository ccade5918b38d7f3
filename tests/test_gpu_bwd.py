"""GPU parity of the backward pass (App. A.4): the HIP path through the C ABI against the fp64 oracle's
token-by-token reverse recurrence, on seeded synthetic inputs spanning several chunks, segments, the
d_v split and the cut into shorter pieces."""
import zlib

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2507_01004_amd import synth, zeco
from tests.gpu_util import TOL, dev, host, rel_err_bh

pytestmark = pytest.mark.gpu

# (name, B, H, P, L, d_k, d_v, g dtype)
CASES = [
    ("bwd_split", 1, 4, 2, 320, 128, 128, "f32"),          # 8 streams: d_v split in the dV pass, 5 chunks
    ("bwd_whole", 2, 16, 8, 128, 128, 128, "f32"),         # 256 streams
    ("bwd_pieces", 1, 2, 2, 1024, 128, 128, "f32"),        # fused call cuts each segment in 4
    ("bwd_pieces_d64", 1, 1, 1, 2048, 64, 64, "bf16"),
    ("bwd_gbf16", 1, 3, 2, 256, 128, 128, "bf16"),
    ("bwd_pieces_odd", 1, 1, 1, 1920, 128, 128, "f32"),    # 30 chunks: forward 2 pieces, backward 6 of 5 chunks
    ("bwd_pieces_prime", 1, 2, 1, 1664, 64, 128, "f32"),   # 26 chunks: 2 pieces of 13, which no factor divides
    ("bwd_onechunk", 1, 2, 4, 64, 128, 128, "f32"),
    ("bwd_dk64_dv128", 1, 2, 2, 192, 64, 128, "f32"),
    ("bwd_dk128_dv64", 1, 2, 2, 192, 128, 64, "bf16"),
]
GRADS = ("dq", "dk", "dv", "dg")
AXES = (0, 2)


def make(case, **kw):
    name, B, H, P, L, dk, dv, gd = case
    inp = synth.make_inputs(B, P * L, H, dk, dv, seed=zlib.crc32(name.encode()) % 10000 + 11, io="bf16", g=gd,
                            device="cuda", **kw)
    gen = torch.Generator(device="cuda").manual_seed(zlib.crc32(name.encode()) % 10000 + 12)
    inp["dO"] = torch.randn(inp["v"].shape, generator=gen, device="cuda").to(torch.bfloat16)
    return inp


def oracle_bwd(inp, scale, S0=None, dS_T=None):
    return oracle.gla_recurrent_bwd(host(inp["q"]), host(inp["k"]), host(inp["v"]), host(inp["g"]),
                                    host(inp["dO"]), scale, S0, dS_T)


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_bwd_dstate_matches_oracle(case):
    """Each segment's outgoing state gradient = d loss / d S0 of that segment run on its own."""
    name, B, H, P, L, dk, dv, gd = case
    print("case", case, flush=True)
    inp = make(case, gate_div=64.0)
    dS_loc = zeco.gla_bwd_dstate(inp["q"], inp["g"], inp["dO"], P, scale=0.5)
    torch.cuda.synchronize()
    for p in range(P):
        sl = {n: t[:, p * L:(p + 1) * L] for n, t in inp.items()}
        ref = oracle_bwd(sl, 0.5)[4]
        assert rel_err_bh(host(dS_loc[p]), ref, (0, 1)) <= TOL["bf16"], p


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_fused_bwd_matches_unsegmented_oracle(case):
    name, B, H, P, L, dk, dv, gd = case
    print("case", case, flush=True)
    inp = make(case, gate_div=64.0)      # slow decay: states and state gradients reach every token
    gen = torch.Generator(device="cuda").manual_seed(zlib.crc32(name.encode()) % 10000 + 13)
    S0 = torch.randn(B, H, dk, dv, device="cuda", generator=gen) * 0.3
    dS_T = torch.randn(B, H, dk, dv, device="cuda", generator=gen) * 0.3
    for s0, dst in ((None, None), (S0, dS_T)):
        got = zeco.gla_fused_bwd(inp["q"], inp["k"], inp["v"], inp["g"], inp["dO"], P, scale=0.5, S0=s0, dS_T=dst)
        torch.cuda.synchronize()
        ref = oracle_bwd(inp, 0.5, None if s0 is None else host(s0), None if dst is None else host(dst))
        for name_, x, r in zip(GRADS, got[:4], ref[:4]):
            assert rel_err_bh(host(x), r, AXES) <= TOL["bf16"], name_
        assert rel_err_bh(host(got[4]), ref[4], (0, 1)) <= TOL["bf16"]


# segments far beyond 512 tokens, where the dK pass re-anchors the running sum of dG at the forward-state
# checkpoints the dQ pass left: whole chunks, a ragged length (the two passes must cut it at the same tokens),
# a chunk count that is no multiple of 8, both state shapes and gate formats
LONG_CASES = [
    ("blocks_long", 1, 2, 2, 4096, 128, 128, "f32"),
    ("blocks_long_ragged", 1, 2, 2, 4133, 128, 128, "f32"),
    ("blocks_long_odd", 2, 1, 1, 3008, 64, 128, "bf16"),       # 47 chunks: 5 checkpoints, 7 chunks after the last
    ("blocks_long_ragged_d64", 1, 3, 1, 1601, 64, 64, "f32"),  # 26 chunks, the last one holds a single token
    ("blocks_513", 1, 2, 3, 513, 128, 64, "f32"),              # one checkpoint, nine chunks, the short one last
]


@pytest.mark.parametrize("case", [CASES[0], CASES[4]] + LONG_CASES, ids=lambda c: c[0])
def test_bwd_building_blocks_chain(case):
    """The calls a sequence-parallel run makes around the two All-Scans: forward states, their scan,
    state gradients, the reverse scan, then the gradient passes, with P segments as given."""
    name, B, H, P, L, dk, dv, gd = case
    print("case", case, flush=True)
    inp = make(case, gate_div=64.0)
    q, k, v, g, dO = (inp[n] for n in ("q", "k", "v", "g", "dO"))
    S_loc, G_tot = zeco.gla_local_state(k, v, g, P)
    S_init, S_last = zeco.state_scan(S_loc, G_tot)
    dS_loc = zeco.gla_bwd_dstate(q, g, dO, P, scale=0.7)
    dS_in, dS0 = zeco.state_scan(dS_loc, G_tot, direction=1)
    got = zeco.gla_bwd_from_state(q, k, v, g, dO, S_init, S_last, dS_in, P, scale=0.7)
    torch.cuda.synchronize()
    ref = oracle_bwd(inp, 0.7)
    for name_, x, r in zip(GRADS, got, ref[:4]):
        assert rel_err_bh(host(x), r, AXES) <= TOL["bf16"], name_
    assert rel_err_bh(host(dS0), ref[4], (0, 1)) <= TOL["bf16"]
    # the reverse scan against the oracle's scan run on the flipped chain
    Si_r, Sl_r = oracle.state_scan(np.flip(host(dS_loc), 0).reshape(P, B * H, dk, dv),
                                   np.flip(host(G_tot), 0).reshape(P, B * H, dk))
    assert rel_err_bh(host(dS_in), np.flip(Si_r, 0).reshape(P, B, H, dk, dv), (1, 2)) <= 1e-5
    assert rel_err_bh(host(dS0), Sl_r.reshape(B, H, dk, dv), (0, 1)) <= 1e-5


def test_bwd_zero_gate_and_strided_views():
    """g == 0 (nothing decays, every state term at full weight), on head-sliced views of wider tensors."""
    B, H, P, L, dk, dv = 1, 3, 2, 128, 128, 128
    wide = synth.make_inputs(B, P * L, H + 2, dk, dv, seed=77, io="bf16", g="f32", device="cuda", zero_gate=True)
    inp = {n: t[:, :, 1:1 + H] for n, t in wide.items()}
    gen = torch.Generator(device="cuda").manual_seed(78)
    inp["dO"] = torch.randn(wide["v"].shape, generator=gen, device="cuda").to(torch.bfloat16)[:, :, 1:1 + H]
    got = zeco.gla_fused_bwd(inp["q"], inp["k"], inp["v"], inp["g"], inp["dO"], P, scale=1.0)
    again = zeco.gla_fused_bwd(inp["q"], inp["k"], inp["v"], inp["g"], inp["dO"], P, scale=1.0)
    torch.cuda.synchronize()
    ref = oracle_bwd(inp, 1.0)
    for name_, x, y, r in zip(GRADS, got[:4], again[:4], ref[:4]):
        assert rel_err_bh(host(x), r, AXES) <= TOL["bf16"], name_
        assert torch.equal(x, y), name_            # no atomics: bitwise reproducible


def test_bwd_rejects_a_small_workspace():
    q = torch.zeros(1, 64, 1, 64, device="cuda")
    qb = q.to(torch.bfloat16)
    with pytest.raises(zeco.ZecoError) as e:
        zeco.gla_fused_bwd(qb, qb, qb, q, qb, 1, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == zeco.ZECO_ERR_WORKSPACE


@pytest.mark.parametrize("case", [CASES[0], CASES[2], CASES[3], CASES[5], CASES[6],
                                  ("bwd_saved_ragged", 1, 2, 2, 1000, 128, 128, "f32"),
                                  ("bwd_saved_long", 1, 1, 1, 16384, 128, 128, "f32")], ids=lambda c: c[0])
def test_backward_from_states_saved_by_the_forward(case):
    """The forward, by either schedule, leaves the states entering the backward's pieces; the backward started
    from them (no recomputation of the forward states) gives the same gradients within tolerance."""
    name, B, H, P, L, dk, dv, gd = case
    print("case", case, flush=True)
    inp = make(case, gate_div=64.0)
    q, k, v, g, dO = (inp[n] for n in ("q", "k", "v", "g", "dO"))
    gen = torch.Generator(device="cuda").manual_seed(zlib.crc32(name.encode()) % 10000 + 14)
    S0 = torch.randn(B, H, dk, dv, device="cuda", generator=gen) * 0.3
    ref = oracle_bwd(inp, 0.5, host(S0), None)
    for sched in (zeco.SCHEDULE_TWO_PHASE, zeco.SCHEDULE_CORRECT):
        save = torch.empty(zeco.saved_states_bytes(q, v, g, P), dtype=torch.uint8, device="cuda")
        o, S_last = zeco.gla_fused_fwd(q, k, v, g, P, scale=0.5, S0=S0, save=save, schedule=sched)
        o_plain, S_last_plain = zeco.gla_fused_fwd(q, k, v, g, P, scale=0.5, S0=S0, schedule=sched)
        assert torch.equal(o, o_plain) and torch.equal(S_last, S_last_plain)     # saving changes nothing
        got = zeco.gla_fused_bwd(q, k, v, g, dO, P, scale=0.5, saved=save)       # S0 comes with the saved states
        torch.cuda.synchronize()
        for name_, x, r in zip(GRADS, got[:4], ref[:4]):
            assert rel_err_bh(host(x), r, AXES) <= TOL["bf16"], name_
        assert rel_err_bh(host(got[4]), ref[4], (0, 1)) <= TOL["bf16"]


@pytest.mark.parametrize("H", [1, 2])
def test_few_heads_long_sequence_scans_the_pieces_as_a_tree(H):
    """One or two heads and 32768 tokens per segment: the fused calls cut the sequence into 128 pieces and more
    and scan them with the two-level scan (a serial chain that short on width is latency-bound).  Forward by
    both schedules and backward against the oracle, with a state entering and a state gradient leaving."""
    B, P, L, dk, dv = 1, 2, 32768, 64, 64
    print("few heads", H, flush=True)
    inp = synth.make_inputs(B, P * L, H, dk, dv, seed=500 + H, io="bf16", g="f32", device="cuda", gate_div=64.0)
    gen = torch.Generator(device="cuda").manual_seed(501)
    dO = torch.randn(inp["v"].shape, generator=gen, device="cuda").to(torch.bfloat16)
    q, k, v, g = (inp[n] for n in ("q", "k", "v", "g"))
    S0 = torch.randn(B, H, dk, dv, device="cuda", generator=gen) * 0.3
    dS_T = torch.randn(B, H, dk, dv, device="cuda", generator=gen) * 0.3
    o_r, S_r = oracle.gla_recurrent(host(q), host(k), host(v), host(g), 0.5, host(S0))
    ref = oracle.gla_recurrent_bwd(host(q), host(k), host(v), host(g), host(dO), 0.5, host(S0), host(dS_T))
    for sched in (zeco.SCHEDULE_TWO_PHASE, zeco.SCHEDULE_CORRECT):
        o, S_last = zeco.gla_fused_fwd(q, k, v, g, P, scale=0.5, S0=S0, schedule=sched)
        torch.cuda.synchronize()
        assert rel_err_bh(host(o), o_r, (0, 2)) <= TOL["bf16"]
        assert rel_err_bh(host(S_last), S_r, (0, 1)) <= TOL["bf16"]
    got = zeco.gla_fused_bwd(q, k, v, g, dO, P, scale=0.5, S0=S0, dS_T=dS_T)
    torch.cuda.synchronize()
    for name_, x, r in zip(GRADS, got[:4], ref[:4]):
        assert rel_err_bh(host(x), r, AXES) <= TOL["bf16"], name_
    assert rel_err_bh(host(got[4]), ref[4], (0, 1)) <= TOL["bf16"]
