"""zeco_state_scan_tree_static, the entry point that allocates nothing, against zeco_state_scan_tree on a
caller workspace: same kernels in the same order, so the results must be bitwise equal.  Two calls in a row
on the same GPU, the second with a smaller problem (the fixed scratch still holds the first call's group
states), then the first problem again."""
import pytest
import torch

from paper_2507_01004_amd import zeco

pytestmark = pytest.mark.gpu


def _problem(P, BH, dk, dv, per_head, seed):
    gen = torch.Generator(device="cuda:0").manual_seed(seed)
    S_loc = torch.randn(P, BH, dk, dv, device="cuda:0", generator=gen)
    G_tot = -0.3 * torch.rand((P, BH) + (() if per_head else (dk,)), device="cuda:0", generator=gen)
    S0 = torch.randn(BH, dk, dv, device="cuda:0", generator=gen)
    return S_loc, G_tot, S0


def _both(P, BH, dk, dv, per_head, direction, seed, with_s0=True):
    S_loc, G_tot, S0 = _problem(P, BH, dk, dv, per_head, seed)
    s0 = S0 if with_s0 else None
    ref = zeco.state_scan_tree(S_loc, G_tot, s0, direction=direction)
    out = (torch.full_like(S_loc, float("nan")), torch.full_like(S0, float("nan")))
    print("static scan P=%d BH=%d d=%dx%d per_head=%d dir=%d" % (P, BH, dk, dv, per_head, direction), flush=True)
    got = zeco.state_scan_tree_static(S_loc, G_tot, s0, out, direction=direction)
    torch.cuda.synchronize()
    assert torch.equal(got[0], ref[0]) and torch.equal(got[1], ref[1])
    return got


def test_static_scratch_scan_matches_workspace_scan_on_consecutive_calls():
    lim = int(zeco.lib().zeco_state_scan_tree_static_limit())
    big = (256, 2, 128, 128)
    assert 0 < int(zeco.lib().zeco_state_scan_tree_workspace(*big, 0)) <= lim
    _both(*big, per_head=False, direction=0, seed=1)
    _both(36, 1, 64, 128, per_head=False, direction=0, seed=2)          # smaller, right after the large one
    _both(*big, per_head=False, direction=1, seed=3, with_s0=False)     # and the large one again, reversed
    _both(48, 3, 128, 64, per_head=True, direction=1, seed=4)
    _both(37, 2, 128, 128, per_head=False, direction=0, seed=5)         # a prime count: the plain chain, no scratch


def test_static_scratch_scan_refuses_what_does_not_fit():
    P, BH = 1024, 8
    assert int(zeco.lib().zeco_state_scan_tree_workspace(P, BH, 128, 128, 0)) > int(zeco.lib().zeco_state_scan_tree_static_limit())
    S_loc = torch.empty(1, device="cuda:0")   # never read: the size check comes first
    st = zeco.lib().zeco_state_scan_tree_static(P, BH, 128, 128, S_loc.data_ptr(), S_loc.data_ptr(), None,
                                                S_loc.data_ptr(), None, 0, 0, None)
    assert st == zeco.ZECO_ERR_SCRATCH_LIMIT
