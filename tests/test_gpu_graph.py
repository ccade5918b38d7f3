"""The library allocates nothing and never synchronises, so its calls can be recorded into a HIP graph:
capture the three-call pipeline, the tree scan, the fused forward (both schedules), the fused backward and the
three calls over segments of unequal length once, replay them on new input values - and, for the last, on a
new table of segment offsets, which is device data like any other input - and compare every replay bitwise
with the eager calls."""
import pytest
import torch

from paper_2507_01004_amd import synth, zeco
from tests.gpu_util import randn_seeded

pytestmark = pytest.mark.gpu


def test_pipeline_forward_backward_replay_from_a_graph():
    B, H, P, L, dk, dv = 1, 4, 16, 128, 128, 128     # 16 segments: the tree scan really splits (8 groups of 2)
    inp = synth.make_inputs(B, P * L, H, dk, dv, seed=31, io="bf16", g="f32", device="cuda")
    q, k, v, g = (inp[n] for n in ("q", "k", "v", "g"))
    dO = randn_seeded(v.shape, 7301, v.dtype)
    T = P * L
    # every output and workspace is allocated before the capture
    o3 = torch.empty_like(v)
    S_loc = torch.empty(P, B, H, dk, dv, device="cuda")
    G_cum = torch.empty(B, T, H, dk, device="cuda")
    G_tot = torch.empty(P, B, H, dk, device="cuda")
    S_init, S_last3 = torch.empty_like(S_loc), torch.empty(B, H, dk, dv, device="cuda")
    S_init_t, S_last_t = torch.empty_like(S_loc), torch.empty(B, H, dk, dv, device="cuda")
    ws_t = torch.empty(max(16, int(zeco.lib().zeco_state_scan_tree_workspace(P, B * H, dk, dv, 0))), dtype=torch.uint8,
                       device="cuda")
    o2, S_last2 = torch.empty_like(v), torch.empty(B, H, dk, dv, device="cuda")
    o4, S_last4 = torch.empty_like(v), torch.empty(B, H, dk, dv, device="cuda")
    ws_f = torch.empty(zeco.fused_workspace_bytes(q, v, g, P), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(zeco.fused_bwd_workspace_bytes(q, v, g, P), dtype=torch.uint8, device="cuda")
    grads = (torch.empty_like(q), torch.empty_like(q), torch.empty_like(v), torch.empty(B, T, H, dk, device="cuda"),
             torch.empty(B, H, dk, dv, device="cuda"))
    ws_l = torch.empty(max(zeco.local_fwd_workspace_bytes(q, v, g, P), 16), dtype=torch.uint8, device="cuda")
    seg = torch.arange(P + 1, dtype=torch.int64, device="cuda") * L      # P+1 token offsets, rewritten per replay
    o5, S_loc5, G_cum5, G_tot5 = torch.empty_like(v), torch.empty_like(S_loc), torch.empty_like(G_cum), torch.empty_like(G_tot)
    S_init5, S_last5 = torch.empty_like(S_loc), torch.empty(B, H, dk, dv, device="cuda")

    def run():
        zeco.gla_local_fwd(q, k, v, g, P, out=(o3, S_loc, G_cum, G_tot), workspace=ws_l)
        zeco.state_scan(S_loc, G_tot, out=(S_init, S_last3))
        zeco.state_scan_tree(S_loc, G_tot, out=(S_init_t, S_last_t), workspace=ws_t)
        zeco.apply_init_state(q, g, G_cum, S_init, o3, P)
        zeco.gla_fused_fwd(q, k, v, g, P, out=(o2, S_last2), workspace=ws_f, schedule=zeco.SCHEDULE_TWO_PHASE)
        zeco.gla_fused_fwd(q, k, v, g, P, out=(o4, S_last4), workspace=ws_f, schedule=zeco.SCHEDULE_CORRECT)
        zeco.gla_fused_bwd(q, k, v, g, dO, P, out=grads, workspace=ws_b)
        zeco.gla_local_fwd_varlen(q, k, v, g, seg, 512, out=(o5, S_loc5, G_cum5, G_tot5))
        zeco.state_scan(S_loc5, G_tot5, out=(S_init5, S_last5))
        zeco.apply_init_state_varlen(q, g, G_cum5, S_init5, o5, seg, 512)

    outs = (o3, S_last3, S_init_t, S_last_t, o2, S_last2, o4, S_last4, o5, S_last5) + grads
    lengths = ([128] * 16, [64, 192] * 8, [100, 156] * 8)                # each sums to T
    run()                      # warm-up outside the capture (loads the code objects)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for rep in range(3):
        gen = torch.Generator(device="cuda").manual_seed(100 + rep)
        q.copy_(torch.randn(q.shape, generator=gen, device="cuda"))
        v.copy_(torch.randn(v.shape, generator=gen, device="cuda"))
        dO.copy_(torch.randn(v.shape, generator=gen, device="cuda"))
        seg.copy_(torch.tensor([0] + list(torch.tensor(lengths[rep]).cumsum(0)), dtype=torch.int64))
        run()
        torch.cuda.synchronize()
        eager = [t.clone() for t in outs]
        for t in outs:
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(outs, eager)):
            assert torch.equal(a, b), (rep, i)
        if rep == 0:   # equal lengths: the same result as the ordinary three calls
            assert torch.equal(o5, o3) and torch.equal(S_last5, S_last3)


def test_fp32_forward_backward_replay_from_a_graph():
    """The fp32 kernels recorded the same way: the one-call forward and backward at a chunk length of 32, replayed
    on new values, bitwise equal to the eager calls."""
    B, H, P, L, dk, dv, C = 1, 2, 4, 200, 128, 64, 32
    inp = synth.make_inputs(B, P * L, H, dk, dv, seed=33, io="f32", g="f32", device="cuda")
    q, k, v, g = (inp[n] for n in ("q", "k", "v", "g"))
    dO = randn_seeded(v.shape, 7302, v.dtype)
    o, S_last = torch.empty_like(v), torch.empty(B, H, dk, dv, device="cuda")
    ws_f = torch.empty(zeco.fused_workspace_bytes(q, v, g, P, C=C), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(zeco.fused_bwd_workspace_bytes(q, v, g, P, C=C), dtype=torch.uint8, device="cuda")
    grads = (torch.empty_like(q), torch.empty_like(q), torch.empty_like(v), torch.empty(B, P * L, H, dk, device="cuda"),
             torch.empty(B, H, dk, dv, device="cuda"))

    def run():
        zeco.gla_fused_fwd(q, k, v, g, P, out=(o, S_last), workspace=ws_f, C=C)
        zeco.gla_fused_bwd(q, k, v, g, dO, P, out=grads, workspace=ws_b, C=C)

    outs = (o, S_last) + grads
    run()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for rep in range(3):
        gen = torch.Generator(device="cuda").manual_seed(200 + rep)
        q.copy_(torch.randn(q.shape, generator=gen, device="cuda"))
        dO.copy_(torch.randn(v.shape, generator=gen, device="cuda"))
        run()
        torch.cuda.synchronize()
        eager = [t.clone() for t in outs]
        for t in outs:
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(outs, eager)):
            assert torch.equal(a, b), (rep, i)
