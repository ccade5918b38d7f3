"""Segment lengths that are no multiple of the chunk size: the forward entry points make the first chunk of
every segment the short one.  Each of them against the fp64 oracle (which knows no chunks), on lengths with
1, 36, 40 and 63 tokens in the short chunk, one and several chunks, both workgroup decompositions of the
bf16 chunk kernel, all gate layouts, and a correction whose last workgroup has fewer blocks than the
others."""
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
    ("f32_100", 1, 2, 3, 100, 64, 64, "f32", "f32"),
    ("f32_65_d128", 2, 1, 2, 65, 128, 128, "f32", "f32"),            # one token in the short chunk
    ("f32_191", 1, 2, 2, 191, 64, 128, "f32", "f32"),                # 63 tokens
    ("bf16_sliced_100", 1, 4, 2, 100, 128, 128, "bf16", "f32"),      # sibling workgroups split d_v
    ("bf16_sliced_65", 1, 2, 3, 65, 128, 128, "bf16", "f32"),
    ("bf16_whole_127", 2, 16, 5, 127, 128, 128, "bf16", "f32"),      # one workgroup per stream
    ("bf16_1000", 1, 3, 2, 1000, 128, 128, "bf16", "f32"),           # 16 chunks, the first of 40 tokens
    ("bf16_2100", 1, 2, 2, 2100, 128, 128, "bf16", "f32"),           # correction: 3 workgroups per segment, the last of one block
    ("bf16_subseg_2056", 1, 2, 2, 2056, 128, 128, "bf16", "f32"),    # 4 streams: 8 sub-segments of 257 tokens per segment
    ("bf16_subseg_4100", 1, 1, 1, 4100, 64, 64, "bf16", "bf16"),      # 1 stream: 4 sub-segments of 1025 tokens
    ("bf16_gbf16_300", 1, 3, 2, 300, 128, 128, "bf16", "bf16"),
    ("bf16_d64_200", 1, 2, 4, 200, 64, 64, "bf16", "f32"),
    ("bf16_dk64_dv128_100", 1, 2, 2, 100, 64, 128, "bf16", "f32"),
    ("bf16_dk128_dv64_129", 1, 2, 2, 129, 128, 64, "bf16", "bf16"),
]
BF16_CASES = [c for c in CASES if c[7] == "bf16"]


def make(case, **kw):
    name, B, H, P, L, dk, dv, io, gd = case
    return synth.make_inputs(B, P * L, H, dk, dv, seed=zlib.crc32(name.encode()) % 10000 + 11, io=io, g=gd,
                             device="cuda", **kw)


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_ragged_local_fwd_and_pipeline(case):
    name, B, H, P, L, dk, dv, io, gd = case
    print("case", case, flush=True)
    tol = TOL[io]
    inp = make(case)
    o, S_loc, G_cum, G_tot = zeco.gla_local_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P, scale=0.5)
    torch.cuda.synchronize()
    o_r, S_r, Gc_r, Gt_r = oracle_local(inp, P, scale=0.5)
    assert rel_err_bh(host(o), o_r, (0, 2)) <= tol
    assert rel_err_bh(host(S_loc), S_r, (0, 1, 2)) <= tol
    assert log_err(host(G_cum), Gc_r) <= 1e-5
    assert log_err(host(G_tot), Gt_r) <= 1e-5
    # the three calls against the unsegmented recurrence, slow decay so that the correction reaches every token
    inp = make(case, gate_div=64.0)
    gen = torch.Generator(device="cuda").manual_seed(zlib.crc32(name.encode()) % 10000 + 12)
    S0 = torch.randn(B, H, dk, dv, device="cuda", generator=gen) * 0.5
    o, S_last, _ = zeco.segmented_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P, scale=0.5, S0=S0)
    torch.cuda.synchronize()
    o_f, S_f = oracle_full(inp, scale=0.5, S0=host(S0))
    assert rel_err_bh(host(o), o_f, (0, 2)) <= tol
    assert rel_err_bh(host(S_last), S_f, (0, 1)) <= tol
    o_loc, _, _, _ = oracle_local(inp, P, scale=0.5)
    assert rel_err_bh(o_loc, o_f, (0, 2)) > 5 * tol     # the correction matters here


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_ragged_correction_alone_dense_and_default(io):
    """zeco_apply_init_state on its own: every token corrected exactly once (the window of the short first
    block overlaps the second block), dense and default calls equal, rows past the vanishing point untouched."""
    B, H, P, L, dk, dv = 1, 3, 2, 1320, 128, 128      # 21 blocks, the first of 40 tokens; workgroups of 16, 5 blocks
    print("ragged correction", io, flush=True)
    r = np.random.default_rng(5)
    td = synth.torch_dtype(io)
    q = torch.from_numpy(r.standard_normal((B, P * L, H, dk))).to(td).cuda()
    o0 = torch.from_numpy(r.standard_normal((B, P * L, H, dv))).to(td).cuda()
    S = r.standard_normal((P, B, H, dk, dv)).astype(np.float32)
    g = np.zeros((B, P * L, H, dk), dtype=np.float32)
    g[:, :, 0] = -0.002 * (1.0 + r.random(dk))            # never vanishes
    g[:, :, 1] = -106.0 / 500 * (1.0 + 0.3 * r.random(dk))   # vanishes near token 500
    g[:, :, 2] = -106.0 / 30 * (1.0 + 0.3 * r.random(dk))    # vanishes inside the short block
    G = np.cumsum(g.reshape(B, P, L, H, dk).astype(np.float64), axis=2).reshape(B, P * L, H, dk)
    outs = []
    for dense in (False, True):
        o = o0.clone()
        zeco.apply_init_state(q, torch.zeros(1), dev(G), dev(S), o, P, scale=1.3, first_segment_is_zero=False, dense=dense)
        torch.cuda.synchronize()
        outs.append(o)
    assert torch.equal(outs[0].float() + 0.0, outs[1].float() + 0.0)
    ref = oracle.apply_init_state(host(q), host(dev(G)), S.astype(np.float64), host(o0), 1.3)
    assert rel_err_bh(host(outs[0]), ref, (0, 2)) <= TOL[io]


@pytest.mark.parametrize("case", BF16_CASES, ids=[c[0] for c in BF16_CASES])
def test_ragged_two_phase_chunk_decay_and_fused_forward(case):
    name, B, H, P, L, dk, dv, io, gd = case
    print("case", case, flush=True)
    tol = TOL[io]
    inp = make(case, gate_div=64.0)
    q, k, v, g = inp["q"], inp["k"], inp["v"], inp["g"]
    S0 = randn_seeded((B, H, dk, dv), 7200) * 0.3
    o_l, S_r, Gc_r, Gt_r = oracle_local(inp, P, scale=0.5)
    # states only, output pass from the oracle's scanned states
    S_loc, G_tot = zeco.gla_local_state(k, v, g, P)
    torch.cuda.synchronize()
    assert rel_err_bh(host(S_loc), S_r, (0, 1, 2)) <= tol
    assert log_err(host(G_tot), Gt_r) <= 1e-5
    for s0 in (None, S0):
        o_f, S_f = oracle_full(inp, scale=0.5, S0=None if s0 is None else host(s0))
        Si_r, _ = oracle.state_scan(S_r.reshape(P, B * H, dk, dv), Gt_r.reshape(P, B * H, dk),
                                    None if s0 is None else host(s0).reshape(B * H, dk, dv))
        o2 = zeco.gla_fwd_from_state(q, k, v, g, dev(Si_r.reshape(P, B, H, dk, dv)), P, scale=0.5)
        torch.cuda.synchronize()
        assert rel_err_bh(host(o2), o_f, (0, 2)) <= tol
        for sched in (zeco.SCHEDULE_TWO_PHASE, zeco.SCHEDULE_CORRECT, zeco.SCHEDULE_AUTO):
            o3, S_last = zeco.gla_fused_fwd(q, k, v, g, P, scale=0.5, S0=s0, schedule=sched)
            torch.cuda.synchronize()
            assert rel_err_bh(host(o3), o_f, (0, 2)) <= tol
            assert rel_err_bh(host(S_last), S_f, (0, 1)) <= tol
    # chunk-decay form: G_chunk[n] = cumulative log decay at the last token before chunk n; chunk 0 holds the
    # first L - 64 (N - 1) tokens
    o, S_loc, G_chunk, G_tot = zeco.gla_local_fwd_chunk_decay(q, k, v, g, P, scale=0.5)
    torch.cuda.synchronize()
    assert rel_err_bh(host(o), o_l, (0, 2)) <= tol
    assert rel_err_bh(host(S_loc), S_r, (0, 1, 2)) <= tol
    N = -(-L // 64)
    r0 = L - 64 * (N - 1)
    Gseg = Gc_r.reshape(B, P, L, H, dk)
    Gk_r = np.zeros((B, P, N, H, dk))
    for n in range(1, N):
        Gk_r[:, :, n] = Gseg[:, :, r0 + 64 * (n - 1) - 1]
    assert G_chunk.shape == (B, P * N, H, dk)
    assert log_err(host(G_chunk), Gk_r.reshape(B, P * N, H, dk)) <= 1e-5
    o_f, _ = oracle_full(inp, scale=0.5, S0=host(S0))
    S_init, S_last = zeco.state_scan(S_loc, G_tot, S0=S0)
    zeco.apply_init_state_chunk_decay(q, g, G_chunk, S_init, o, P, scale=0.5, first_segment_is_zero=False)
    torch.cuda.synchronize()
    assert rel_err_bh(host(o), o_f, (0, 2)) <= tol


def test_ragged_per_head_gates():
    B, H, P, L, dk, dv = 1, 3, 3, 230, 128, 128
    print("ragged per-head gates", flush=True)
    inp = synth.make_inputs(B, P * L, H, dk, dv, seed=77, io="bf16", g="f32", device="cuda", gate_div=64.0,
                            per_head_gate=True)
    h = {n: host(t) for n, t in inp.items()}
    h["g"] = np.repeat(h["g"][..., None], dk, axis=-1)
    S0 = randn_seeded((B, H, dk, dv), 7201) * 0.3
    o_f, S_f = oracle.gla_recurrent(h["q"], h["k"], h["v"], h["g"], 0.5, host(S0))
    o, S_last, _ = zeco.segmented_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P, scale=0.5, S0=S0)
    torch.cuda.synchronize()
    assert rel_err_bh(host(o), o_f, (0, 2)) <= TOL["bf16"]
    assert rel_err_bh(host(S_last), S_f, (0, 1)) <= TOL["bf16"]
    for sched in (zeco.SCHEDULE_TWO_PHASE, zeco.SCHEDULE_CORRECT):
        o3, S_last = zeco.gla_fused_fwd(inp["q"], inp["k"], inp["v"], inp["g"], P, scale=0.5, S0=S0, schedule=sched)
        torch.cuda.synchronize()
        assert rel_err_bh(host(o3), o_f, (0, 2)) <= TOL["bf16"]
        assert rel_err_bh(host(S_last), S_f, (0, 1)) <= TOL["bf16"]


BWD_CASES = [
    # (name, B, H, P, L, d_k, d_v, g dtype)
    ("rb_100", 1, 4, 2, 100, 128, 128, "f32"),            # d_v split in the dV pass; chunks of 36 + 64
    ("rb_65", 1, 2, 3, 65, 128, 128, "f32"),              # one token in the short chunk
    ("rb_whole_127", 2, 16, 5, 127, 128, 128, "f32"),     # 160 streams
    ("rb_1000", 1, 2, 2, 1000, 128, 128, "bf16"),         # fused call: 2 pieces of 500 tokens per segment
    ("rb_1046", 1, 1, 2, 1046, 64, 64, "f32"),            # 1046 = 2 x 523: no divisor gives pieces of 64..512 tokens, left whole
    ("rb_dk64_dv128_200", 1, 2, 2, 200, 64, 128, "f32"),
    ("rb_dk128_dv64_129", 1, 2, 2, 129, 128, 64, "bf16"),
]
GRADS = ("dq", "dk", "dv", "dg")


def make_bwd(case, **kw):
    name, B, H, P, L, dk, dv, gd = case
    inp = synth.make_inputs(B, P * L, H, dk, dv, seed=zlib.crc32(name.encode()) % 10000 + 11, io="bf16", g=gd,
                            device="cuda", **kw)
    gen = torch.Generator(device="cuda").manual_seed(zlib.crc32(name.encode()) % 10000 + 12)
    inp["dO"] = torch.randn(inp["v"].shape, generator=gen, device="cuda").to(torch.bfloat16)
    return inp


def oracle_bwd(inp, scale, S0=None, dS_T=None):
    return oracle.gla_recurrent_bwd(host(inp["q"]), host(inp["k"]), host(inp["v"]), host(inp["g"]),
                                    host(inp["dO"]), scale, S0, dS_T)


@pytest.mark.parametrize("case", BWD_CASES, ids=[c[0] for c in BWD_CASES])
def test_ragged_backward(case):
    """The fused backward, and the chain of building blocks around the two scans, against the oracle's
    token-by-token reverse recurrence over the whole sequence."""
    name, B, H, P, L, dk, dv, gd = case
    print("case", case, flush=True)
    tol = TOL["bf16"]
    inp = make_bwd(case, gate_div=64.0)
    q, k, v, g, dO = (inp[n] for n in ("q", "k", "v", "g", "dO"))
    S0 = randn_seeded((B, H, dk, dv), 7202) * 0.3
    dS_T = randn_seeded((B, H, dk, dv), 7203) * 0.3
    for s0, dst in ((None, None), (S0, dS_T)):
        got = zeco.gla_fused_bwd(q, k, v, g, dO, P, scale=0.5, S0=s0, dS_T=dst)
        torch.cuda.synchronize()
        ref = oracle_bwd(inp, 0.5, None if s0 is None else host(s0), None if dst is None else host(dst))
        for name_, x, r in zip(GRADS, got[:4], ref[:4]):
            assert rel_err_bh(host(x), r, (0, 2)) <= tol, name_
        assert rel_err_bh(host(got[4]), ref[4], (0, 1)) <= tol
    S_loc, G_tot = zeco.gla_local_state(k, v, g, P)
    S_init, S_last = zeco.state_scan(S_loc, G_tot)
    dS_loc = zeco.gla_bwd_dstate(q, g, dO, P, scale=0.7)
    torch.cuda.synchronize()
    for p in range(P):      # each segment's outgoing state gradient on its own
        sl = {n: t[:, p * L:(p + 1) * L] for n, t in inp.items()}
        assert rel_err_bh(host(dS_loc[p]), oracle_bwd(sl, 0.7)[4], (0, 1)) <= tol, p
    dS_in, dS0 = zeco.state_scan(dS_loc, G_tot, direction=1)
    got = zeco.gla_bwd_from_state(q, k, v, g, dO, S_init, S_last, dS_in, P, scale=0.7)
    torch.cuda.synchronize()
    ref = oracle_bwd(inp, 0.7)
    for name_, x, r in zip(GRADS, got, ref[:4]):
        assert rel_err_bh(host(x), r, (0, 2)) <= tol, name_
    assert rel_err_bh(host(dS0), ref[4], (0, 1)) <= tol


def test_ragged_backward_per_head_gates():
    B, H, P, L, dk, dv = 1, 3, 2, 230, 128, 128
    print("ragged backward, per-head gates", flush=True)
    inp = synth.make_inputs(B, P * L, H, dk, dv, seed=79, io="bf16", g="f32", device="cuda", gate_div=64.0,
                            per_head_gate=True)
    gen = torch.Generator(device="cuda").manual_seed(80)
    dO = torch.randn(inp["v"].shape, generator=gen, device="cuda").to(torch.bfloat16)
    h = {n: host(t) for n, t in inp.items()}
    h["g"] = np.repeat(h["g"][..., None], dk, axis=-1)
    ref = oracle.gla_recurrent_bwd(h["q"], h["k"], h["v"], h["g"], host(dO), 0.5, None, None)
    got = zeco.gla_fused_bwd(inp["q"], inp["k"], inp["v"], inp["g"], dO, P, scale=0.5)
    torch.cuda.synchronize()
    for name_, x, r in zip(GRADS[:3], got[:3], ref[:3]):
        assert rel_err_bh(host(x), r, (0, 2)) <= TOL["bf16"], name_
    assert rel_err_bh(host(got[3]), ref[3].sum(axis=-1), (0, 2)) <= TOL["bf16"]


def test_ragged_lengths_a_segment_must_hold_a_chunk():
    inp = synth.make_inputs(1, 200, 2, 128, 128, seed=3, io="bf16", g="f32", device="cuda")
    q, k, v, g = inp["q"], inp["k"], inp["v"], inp["g"]
    assert zeco.saved_states_bytes(q, v, g, 2) > 0       # states are saved per piece, whatever its length
    with pytest.raises(zeco.ZecoError):      # shorter than a chunk
        zeco.gla_local_fwd(q[:, :80], k[:, :80], v[:, :80], g[:, :80], 2)
