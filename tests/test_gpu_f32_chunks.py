"""The fp32 path with chunk lengths 16, 32 and 64, and its two-phase forward (Alg. 1's schedule): Sec. 2.1 leaves
the chunk length free and the result does not depend on it, so every case is held against the chunk-free fp64
recurrence at the fp32 tolerance.  A shorter chunk spans less decay in K / Lambda and therefore takes stronger
gates: the last test runs decays that a 64-token chunk could not represent."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2507_01004_amd import synth, zeco
from tests.gpu_util import TOL, host, log_err, oracle_full, oracle_local, randn_seeded, rel_err_bh

pytestmark = pytest.mark.gpu
tol = TOL["f32"]

# (B, H, P, L, d_k, d_v): whole chunks, lengths that are multiples of 16 but not of 64, and ragged ones
SHAPES = [(1, 1, 4, 64, 64, 64), (2, 2, 2, 208, 128, 128), (1, 2, 3, 135, 64, 128), (1, 3, 2, 321, 128, 64)]


@pytest.mark.parametrize("C", [16, 32, 64])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_f32_every_forward_route_at_every_chunk_length(shape, C):
    B, H, P, L, dk, dv = shape
    print("f32 chunks", shape, C, flush=True)
    inp = synth.make_inputs(B, P * L, H, dk, dv, seed=600 + C + L, io="f32", g="f32", device="cuda", gate_div=32.0)
    q, k, v, g = (inp[n] for n in "qkvg")
    S0 = randn_seeded((B, H, dk, dv), 8000 + C) * 0.3
    # the local pass on its own
    o, S_loc, G_cum, G_tot = zeco.gla_local_fwd(q, k, v, g, P, scale=0.5, C=C)
    torch.cuda.synchronize()
    o_r, S_r, Gc_r, Gt_r = oracle_local(inp, P, scale=0.5)
    assert rel_err_bh(host(o), o_r, (0, 2)) <= tol
    assert rel_err_bh(host(S_loc), S_r, (0, 1, 2)) <= tol
    assert log_err(host(G_cum), Gc_r) <= 1e-5 and log_err(host(G_tot), Gt_r) <= 1e-5
    # three calls, two phases, one call: against the unsegmented recurrence with an incoming state
    o_f, S_f = oracle_full(inp, scale=0.5, S0=host(S0))
    o3, S3, _ = zeco.segmented_fwd(q, k, v, g, P, scale=0.5, S0=S0, C=C)
    S_loc2, G_tot2 = zeco.gla_local_state(k, v, g, P, C=C)
    S_init2, S2 = zeco.state_scan(S_loc2, G_tot2, S0=S0)
    o2 = zeco.gla_fwd_from_state(q, k, v, g, S_init2, P, scale=0.5, C=C)
    o1, S1 = zeco.gla_fused_fwd(q, k, v, g, P, scale=0.5, S0=S0, C=C)
    torch.cuda.synchronize()
    assert rel_err_bh(host(S_loc2), S_r, (0, 1, 2)) <= tol and log_err(host(G_tot2), Gt_r) <= 1e-5
    for o_x, S_x in ((o3, S3), (o2, S2), (o1, S1)):
        assert rel_err_bh(host(o_x), o_f, (0, 2)) <= tol
        assert rel_err_bh(host(S_x), S_f, (0, 1)) <= tol
    assert rel_err_bh(o_r, o_f, (0, 2)) > 10 * tol      # the incoming states matter here


@pytest.mark.parametrize("C", [16, 32, 64])
def test_f32_unequal_segments_at_every_chunk_length(C):
    B, H, dk, dv = 1, 2, 64, 128
    lengths = (100, 64, 333, 208)
    start = [0] + [int(x) for x in np.cumsum(lengths)]
    seg = torch.tensor(start, dtype=torch.int64, device="cuda")
    T, bound = sum(lengths), max(lengths)
    print("f32 chunks, unequal segments", C, flush=True)
    inp = synth.make_inputs(B, T, H, dk, dv, seed=650 + C, io="f32", g="f32", device="cuda", gate_div=32.0)
    q, k, v, g = (inp[n] for n in "qkvg")
    S0 = randn_seeded((B, H, dk, dv), 8100 + C) * 0.3
    o_f, S_f = oracle_full(inp, scale=0.5, S0=host(S0))
    o, S_loc, G_cum, G_tot = zeco.gla_local_fwd_varlen(q, k, v, g, seg, bound, scale=0.5, C=C)
    S_init, S_last = zeco.state_scan(S_loc, G_tot, S0=S0)
    zeco.apply_init_state_varlen(q, g, G_cum, S_init, o, seg, bound, scale=0.5, C=C, first_segment_is_zero=False)
    o1, S1 = zeco.gla_fused_fwd_varlen(q, k, v, g, seg, bound, scale=0.5, C=C, S0=S0)
    torch.cuda.synchronize()
    for o_x, S_x in ((o, S_last), (o1, S1)):
        assert rel_err_bh(host(o_x), o_f, (0, 2)) <= tol
        assert rel_err_bh(host(S_x), S_f, (0, 1)) <= tol
    for p in range(len(lengths)):
        Gc = np.cumsum(host(g[:, start[p]:start[p + 1]]), axis=1)
        assert log_err(host(G_cum[:, start[p]:start[p + 1]]), Gc) <= 1e-5


def test_f32_short_chunks_take_gates_a_long_chunk_cannot():
    """Log decays of -2.5 to -4.5 per token: up to 72 over a chunk of 16 tokens (inside the range of K / Lambda),
    288 over 64 tokens (far outside: exp overflows).  C = 16 matches the oracle; C = 64 is documented to fail."""
    B, H, P, L, dk, dv = 1, 2, 2, 128, 64, 64
    inp = synth.make_inputs(B, P * L, H, dk, dv, seed=660, io="f32", g="f32", device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(661)
    inp["g"] = -(2.5 + 2.0 * torch.rand(inp["g"].shape, generator=gen, device="cuda"))
    q, k, v, g = (inp[n] for n in "qkvg")
    o_f, S_f = oracle_full(inp, scale=1.0)
    o, S_last, _ = zeco.segmented_fwd(q, k, v, g, P, C=16)
    o1, S1 = zeco.gla_fused_fwd(q, k, v, g, P, C=16)
    torch.cuda.synchronize()
    for o_x, S_x in ((o, S_last), (o1, S1)):
        assert torch.isfinite(o_x).all()
        assert rel_err_bh(host(o_x), o_f, (0, 2)) <= tol
        assert rel_err_bh(host(S_x), S_f, (0, 1)) <= tol
    o64, _, _ = zeco.segmented_fwd(q, k, v, g, P, C=64)
    torch.cuda.synchronize()
    assert not torch.isfinite(o64).all()       # the documented outcome beyond the range: inf / NaN, status OK


def test_chunk_lengths_the_kernels_do_not_have_are_refused():
    qb = torch.zeros(1, 128, 1, 64, dtype=torch.bfloat16, device="cuda")
    gf = torch.zeros(1, 128, 1, 64, device="cuda")
    with pytest.raises(zeco.ZecoError) as e:
        zeco.gla_local_fwd(qb, qb, qb, gf, 1, C=32)          # bf16: 64 only
    assert e.value.status == zeco.ZECO_ERR_UNSUPPORTED
    with pytest.raises(zeco.ZecoError) as e:
        zeco.gla_local_fwd(gf, gf, gf, gf, 1, C=48)
    assert e.value.status == zeco.ZECO_ERR_UNSUPPORTED
