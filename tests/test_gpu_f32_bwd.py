"""GPU parity of the fp32 backward pass (App. A.4 on fp32 tensors, fp32 MFMA): the one-call backward and the calls
a sequence-parallel run makes around the two All-Scans, against the fp64 oracle's token-by-token reverse
recurrence at the fp32 tolerance; every chunk length the fp32 kernels take, whole and ragged segment lengths,
lengths beyond a checkpoint of the forward state, both state shapes, unequal segments."""
import zlib

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2507_01004_amd import synth, zeco
from tests.gpu_util import TOL, host, rel_err_bh

pytestmark = pytest.mark.gpu

# (name, B, H, P, L, d_k, d_v, C)
CASES = [
    ("f32bwd_c64", 1, 2, 2, 320, 128, 128, 64),
    ("f32bwd_c32", 2, 2, 3, 192, 128, 128, 32),
    ("f32bwd_c16", 1, 3, 2, 208, 128, 128, 16),
    ("f32bwd_ragged_c64", 1, 2, 2, 203, 128, 128, 64),
    ("f32bwd_ragged_c16", 1, 2, 2, 203, 64, 128, 16),
    ("f32bwd_d64", 1, 2, 2, 256, 64, 64, 32),
    ("f32bwd_dk128_dv64", 1, 2, 1, 257, 128, 64, 64),
    ("f32bwd_anchor", 1, 2, 2, 1100, 128, 128, 64),        # two checkpoints of the forward state per segment
    ("f32bwd_anchor_c16", 1, 1, 1, 1601, 64, 64, 16),      # three, 32 chunks apart; the last chunk holds one token
    ("f32bwd_pieces_c16", 2, 16, 4, 1024, 128, 128, 16),   # 128 streams cut into 4 pieces each (four workgroups share a compute unit at C = 16)
]
GRADS = ("dq", "dk", "dv", "dg")
AXES = (0, 2)


def make(case, **kw):
    name, B, H, P, L, dk, dv, C = case
    seed = zlib.crc32(name.encode()) % 10000
    inp = synth.make_inputs(B, P * L, H, dk, dv, seed=seed + 21, io="f32", g="f32", device="cuda", **kw)
    gen = torch.Generator(device="cuda").manual_seed(seed + 22)
    inp["dO"] = torch.randn(inp["v"].shape, generator=gen, device="cuda")
    return inp, gen


def oracle_bwd(inp, scale, S0=None, dS_T=None):
    return oracle.gla_recurrent_bwd(host(inp["q"]), host(inp["k"]), host(inp["v"]), host(inp["g"]),
                                    host(inp["dO"]), scale, S0, dS_T)


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_fused_bwd_fp32_matches_unsegmented_oracle(case):
    name, B, H, P, L, dk, dv, C = case
    print("case", case, flush=True)
    inp, gen = make(case, gate_div=64.0)      # slow decay: states and state gradients reach every token
    S0 = torch.randn(B, H, dk, dv, device="cuda", generator=gen) * 0.3
    dS_T = torch.randn(B, H, dk, dv, device="cuda", generator=gen) * 0.3
    for s0, dst in ((None, None), (S0, dS_T)):
        got = zeco.gla_fused_bwd(inp["q"], inp["k"], inp["v"], inp["g"], inp["dO"], P, scale=0.5, S0=s0, dS_T=dst, C=C)
        o, S_last = zeco.gla_fused_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P, scale=0.5, S0=s0, C=C)   # the same cut
        torch.cuda.synchronize()
        assert got[0].dtype == torch.float32
        o_r, S_r = oracle.gla_recurrent(host(inp["q"]), host(inp["k"]), host(inp["v"]), host(inp["g"]), 0.5,
                                        None if s0 is None else host(s0))
        assert rel_err_bh(host(o), o_r, AXES) <= TOL["f32"] and rel_err_bh(host(S_last), S_r, (0, 1)) <= TOL["f32"]
        ref = oracle_bwd(inp, 0.5, None if s0 is None else host(s0), None if dst is None else host(dst))
        for name_, x, r in zip(GRADS, got[:4], ref[:4]):
            assert rel_err_bh(host(x), r, AXES) <= TOL["f32"], name_
        assert rel_err_bh(host(got[4]), ref[4], (0, 1)) <= TOL["f32"]


@pytest.mark.parametrize("case", [CASES[0], CASES[2], CASES[3], CASES[7]], ids=lambda c: c[0])
def test_bwd_building_blocks_fp32(case):
    """Forward states, their scan, state gradients (checked per segment against the oracle run on that segment
    alone), the reverse scan, then the gradient passes, with P segments as given."""
    name, B, H, P, L, dk, dv, C = case
    print("case", case, flush=True)
    inp, _ = make(case, gate_div=64.0)
    q, k, v, g, dO = (inp[n] for n in ("q", "k", "v", "g", "dO"))
    S_loc, G_tot = zeco.gla_local_state(k, v, g, P, C=C)
    S_init, S_last = zeco.state_scan(S_loc, G_tot)
    dS_loc = zeco.gla_bwd_dstate(q, g, dO, P, scale=0.7, C=C)
    dS_in, dS0 = zeco.state_scan(dS_loc, G_tot, direction=1)
    got = zeco.gla_bwd_from_state(q, k, v, g, dO, S_init, S_last, dS_in, P, scale=0.7, C=C)
    torch.cuda.synchronize()
    for p in range(P):
        sl = {n: t[:, p * L:(p + 1) * L] for n, t in inp.items()}
        assert rel_err_bh(host(dS_loc[p]), oracle_bwd(sl, 0.7)[4], (0, 1)) <= TOL["f32"], p
    ref = oracle_bwd(inp, 0.7)
    for name_, x, r in zip(GRADS, got, ref[:4]):
        assert rel_err_bh(host(x), r, AXES) <= TOL["f32"], name_
    assert rel_err_bh(host(dS0), ref[4], (0, 1)) <= TOL["f32"]


def test_fused_bwd_fp32_strong_gates_and_strided_views():
    """Log decays of -1.5 to -2.4 per token at C = 64 (96 to 154 per chunk: the factors counted from half the
    chunk's total), on head-sliced views of wider tensors; twice, bitwise the same."""
    B, H, P, L, dk, dv = 1, 2, 2, 192, 128, 128
    wide = synth.make_inputs(B, P * L, H + 2, dk, dv, seed=31, io="f32", g="f32", device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(32)
    wide["g"] = -(1.5 + 0.9 * torch.rand(wide["g"].shape, generator=gen, device="cuda"))
    wide["dO"] = torch.randn(wide["v"].shape, generator=gen, device="cuda")
    inp = {n: t[:, :, 1:1 + H] for n, t in wide.items()}
    got = zeco.gla_fused_bwd(inp["q"], inp["k"], inp["v"], inp["g"], inp["dO"], P, scale=1.0)
    again = zeco.gla_fused_bwd(inp["q"], inp["k"], inp["v"], inp["g"], inp["dO"], P, scale=1.0)
    torch.cuda.synchronize()
    ref = oracle_bwd(inp, 1.0)
    for name_, x, y, r in zip(GRADS, got[:4], again[:4], ref[:4]):
        assert torch.isfinite(x).all(), name_
        assert rel_err_bh(host(x), r, AXES) <= TOL["f32"], name_
        assert torch.equal(x, y), name_            # no atomics: bitwise reproducible


def test_fused_bwd_fp32_unequal_segments():
    """The whole backward over a table of unequal segment lengths (one of them beyond a checkpoint), chunk length 32."""
    B, H, dk, dv, C = 2, 2, 128, 128, 32
    lens = [70, 600, 129, 257]
    T = sum(lens)
    inp = synth.make_inputs(B, T, H, dk, dv, seed=41, io="f32", g="f32", device="cuda", gate_div=64.0)
    gen = torch.Generator(device="cuda").manual_seed(42)
    inp["dO"] = torch.randn(inp["v"].shape, generator=gen, device="cuda")
    seg = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int64, device="cuda")
    got = zeco.gla_fused_bwd_varlen(inp["q"], inp["k"], inp["v"], inp["g"], inp["dO"], seg, max(lens), scale=0.5, C=C)
    torch.cuda.synchronize()
    ref = oracle_bwd(inp, 0.5)
    for name_, x, r in zip(GRADS, got[:4], ref[:4]):
        assert rel_err_bh(host(x), r, AXES) <= TOL["f32"], name_
    assert rel_err_bh(host(got[4]), ref[4], (0, 1)) <= TOL["f32"]
