"""GPU parity with one log decay per (token, head) shared by all channels (the scalar-decay members of
the family, Sec. 2.1): g, G_cum, dg are [B,T,H].  The oracle is the per-channel one, fed the gate
broadcast over the channels; the gradient of a shared gate is the sum of the per-channel gradients."""
import zlib

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2507_01004_amd import synth, zeco
from tests.gpu_util import TOL, host, log_err, rel_err_bh, randn_seeded

pytestmark = pytest.mark.gpu

# (name, B, H, P, L, d_k, d_v)
CASES = [
    ("hg_split", 1, 4, 2, 320, 128, 128),        # 8 streams: sibling workgroups split d_v
    ("hg_whole", 2, 16, 8, 128, 128, 128),       # 256 streams
    ("hg_pieces", 1, 2, 2, 2048, 128, 128),      # few streams: sub-segmented local pass, fused calls cut the segments
    ("hg_pieces_ragged", 1, 1, 1, 4100, 64, 64), # the same with a length that is no multiple of 64 (4 x 1025)
    ("hg_halves", 1, 8, 10, 8192, 128, 128),     # 80 streams of 8192 tokens: the local pass runs every segment as two halves
    ("hg_onechunk", 1, 2, 4, 64, 128, 128),
    ("hg_d64", 1, 2, 3, 192, 64, 64),
    ("hg_dk128_dv64", 1, 2, 2, 192, 128, 64),    # state of the Mamba-2 shape: wide key, narrow value
    ("hg_dk64_dv128", 1, 2, 2, 128, 64, 128),
]
TOLB = TOL["bf16"]


def make(case, **kw):
    name, B, H, P, L, dk, dv = case
    seed = zlib.crc32(name.encode()) % 10000 + 21
    inp = synth.make_inputs(B, P * L, H, dk, dv, seed=seed, io="bf16", g="f32", device="cuda",
                            per_head_gate=True, **kw)
    gen = torch.Generator(device="cuda").manual_seed(seed + 1)
    inp["dO"] = torch.randn(inp["v"].shape, generator=gen, device="cuda").to(torch.bfloat16)
    return inp


def wide(inp, dk):
    """Host copies with the gate broadcast to [B,T,H,d_k]."""
    h = {n: host(t) for n, t in inp.items()}
    h["g"] = np.repeat(h["g"][..., None], dk, axis=-1)
    return h


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_head_gate_three_call_forward(case):
    name, B, H, P, L, dk, dv = case
    print("case", case, flush=True)
    inp = make(case, gate_div=64.0)
    h = wide(inp, dk)
    o, S_loc, G_cum, G_tot = zeco.gla_local_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P, scale=0.5)
    torch.cuda.synchronize()
    assert G_cum.shape == (B, P * L, H) and G_tot.shape == (P, B, H)
    o_r, S_r, Gc_r, Gt_r = oracle.gla_local(h["q"], h["k"], h["v"], h["g"], P, 0.5)
    assert rel_err_bh(host(o), o_r, (0, 2)) <= TOLB
    assert rel_err_bh(host(S_loc), S_r, (0, 1, 2)) <= TOLB
    assert log_err(host(G_cum), Gc_r[..., 0]) <= 1e-5
    assert log_err(host(G_tot), Gt_r[..., 0]) <= 1e-5
    S0 = randn_seeded((B, H, dk, dv), 7000) * 0.3
    o, S_last, parts = zeco.segmented_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P, scale=0.5, S0=S0)
    torch.cuda.synchronize()
    o_f, S_f = oracle.gla_recurrent(h["q"], h["k"], h["v"], h["g"], 0.5, host(S0))
    assert rel_err_bh(host(o), o_f, (0, 2)) <= TOLB
    assert rel_err_bh(host(S_last), S_f, (0, 1)) <= TOLB


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_head_gate_two_phase_forward_and_backward(case):
    name, B, H, P, L, dk, dv = case
    print("case", case, flush=True)
    inp = make(case, gate_div=64.0)
    h = wide(inp, dk)
    S0 = randn_seeded((B, H, dk, dv), 7001) * 0.3
    dS_T = randn_seeded((B, H, dk, dv), 7002) * 0.3
    for s0, dst in ((None, None), (S0, dS_T)):
        for sched in (zeco.SCHEDULE_CORRECT, zeco.SCHEDULE_TWO_PHASE):
            o, S_last = zeco.gla_fused_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P, scale=0.5, S0=s0, schedule=sched)
            torch.cuda.synchronize()
            o_f, S_f = oracle.gla_recurrent(h["q"], h["k"], h["v"], h["g"], 0.5, None if s0 is None else host(s0))
            assert rel_err_bh(host(o), o_f, (0, 2)) <= TOLB
            assert rel_err_bh(host(S_last), S_f, (0, 1)) <= TOLB
        got = zeco.gla_fused_bwd(inp["q"], inp["k"], inp["v"], inp["g"], inp["dO"], P, scale=0.5, S0=s0, dS_T=dst)
        torch.cuda.synchronize()
        s0h = None if s0 is None else host(s0)
        o_f, S_f = oracle.gla_recurrent(h["q"], h["k"], h["v"], h["g"], 0.5, s0h)
        assert rel_err_bh(host(o), o_f, (0, 2)) <= TOLB
        assert rel_err_bh(host(S_last), S_f, (0, 1)) <= TOLB
        ref = oracle.gla_recurrent_bwd(h["q"], h["k"], h["v"], h["g"], h["dO"], 0.5, s0h,
                                       None if dst is None else host(dst))
        assert got[3].shape == (B, P * L, H)
        for nm, x, r in zip(("dq", "dk", "dv"), got[:3], ref[:3]):
            assert rel_err_bh(host(x), r, (0, 2)) <= TOLB, nm
        assert rel_err_bh(host(got[3]), ref[3].sum(axis=-1), (0, 2)) <= TOLB, "dg"
        assert rel_err_bh(host(got[4]), ref[4], (0, 1)) <= TOLB
