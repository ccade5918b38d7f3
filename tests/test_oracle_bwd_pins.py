"""Pins of the fp64 backward oracle (CPU only).

The oracle walks the token recurrence in reverse.  The pins reach the same gradients another way:
reverse-mode differentiation (torch.autograd, float64) of the unrolled quadratic form, central
finite differences of the forward oracle, the closed matmul form at g == 0, the reverse cumulative
sum of App. A.4 for the gate gradient, and the chaining of segments through dS (the backward
All-Scan of App. A.4)."""
import numpy as np
import pytest
import torch

from oracle import oracle
from tests.pins import tiny_inputs

TOL = 1e-9


def relerr(a, b):
    return np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300)


def torch_quadratic(q, k, v, g, scale, S0):
    """Eq. (1) unrolled with dense tensors: o = scale * (tril(A) V + (q .* e^G) S0),
    A_ts = sum_i q_ti k_si exp(G_ti - G_si); S_T = sum_s (e^(G_T - G_s) .* k_s)^T v_s + e^G_T .* S0."""
    B, T, H, dk = q.shape
    G = torch.cumsum(g, dim=1)
    diff = G[:, :, None] - G[:, None, :]                       # [B, t, s, H, dk]
    mask = torch.tril(torch.ones(T, T, dtype=torch.bool))[None, :, :, None, None]
    w = torch.where(mask, torch.exp(torch.where(mask, diff, torch.zeros_like(diff))), torch.zeros_like(diff))
    A = torch.einsum("bthi,bshi,btshi->btsh", q, k, w)
    o = torch.einsum("btsh,bshj->bthj", A, v)
    kd = k * torch.exp(G[:, -1:, :, :] - G)
    S_T = torch.einsum("bshi,bshj->bhij", kd, v)
    if S0 is not None:
        o = o + torch.einsum("bthi,bhij->bthj", q * torch.exp(G), S0)
        S_T = S_T + torch.exp(G[:, -1])[..., None] * S0
    return scale * o, S_T


def autograd_reference(q, k, v, g, dO, scale, S0, dS_T):
    ts = [torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v, g)]
    s0 = None if S0 is None else torch.tensor(S0, dtype=torch.float64, requires_grad=True)
    o, S_T = torch_quadratic(*ts, scale, s0)
    loss = (o * torch.tensor(dO)).sum()
    if dS_T is not None:
        loss = loss + (S_T * torch.tensor(dS_T)).sum()
    loss.backward()
    out = [t.grad.numpy() for t in ts]
    out.append(None if s0 is None else s0.grad.numpy())
    return out


@pytest.mark.parametrize("shape", [(1, 9, 1, 3, 2), (2, 37, 2, 5, 7), (1, 160, 2, 4, 6)])
@pytest.mark.parametrize("with_state", [False, True])
def test_bwd_vs_autograd_of_quadratic_form(shape, with_state):
    """Every gradient against reverse-mode differentiation of an independently written forward;
    d_k != d_v catches transposed operands, T > 128 crosses the oracle's recompute block."""
    B, T, H, dk, dv = shape
    q, k, v, g = tiny_inputs(B, T, H, dk, dv, seed=T + 1)
    r = np.random.default_rng(T)
    dO = r.standard_normal((B, T, H, dv))
    S0 = r.standard_normal((B, H, dk, dv)) if with_state else None
    dS_T = r.standard_normal((B, H, dk, dv)) if with_state else None
    got = oracle.gla_recurrent_bwd(q, k, v, g, dO, scale=0.6, S0=S0, dS_T=dS_T)
    ref = autograd_reference(q, k, v, g, dO, 0.6, S0, dS_T)
    for name, a, b in zip(("dq", "dk", "dv", "dg"), got[:4], ref[:4]):
        assert relerr(a, b) < TOL, name
    if with_state:
        assert relerr(got[4], ref[4]) < TOL


def test_bwd_vs_finite_differences_of_forward_oracle():
    """Central differences of loss = <o, dO> + <S_T, dS_T> through the forward oracle."""
    B, T, H, dk, dv = 1, 21, 2, 4, 3
    q, k, v, g = tiny_inputs(B, T, H, dk, dv, seed=5)
    r = np.random.default_rng(6)
    dO = r.standard_normal((B, T, H, dv))
    S0 = r.standard_normal((B, H, dk, dv))
    dS_T = r.standard_normal((B, H, dk, dv))
    grads = oracle.gla_recurrent_bwd(q, k, v, g, dO, scale=1.3, S0=S0, dS_T=dS_T)

    def loss(q_, k_, v_, g_, s0_):
        o, Sf = oracle.gla_recurrent(q_, k_, v_, g_, scale=1.3, S0=s0_)
        return np.sum(o * dO) + np.sum(Sf * dS_T)

    args = [q, k, v, g, S0]
    eps = 1e-6
    for which in range(5):
        for _ in range(6):
            idx = tuple(r.integers(0, n) for n in args[which].shape)
            plus = [a.copy() for a in args]
            minus = [a.copy() for a in args]
            plus[which][idx] += eps
            minus[which][idx] -= eps
            fd = (loss(*plus) - loss(*minus)) / (2 * eps)
            assert abs(fd - grads[which][idx]) <= 1e-6 * max(1.0, abs(fd)), (which, idx)


def test_bwd_zero_gate_is_linear_attention_backward():
    """g == 0: o = scale tril(Q K^T) V, so dQ = scale tril(dO V^T) K, dK = scale tril(dO V^T)^T Q,
    dV = scale tril(Q K^T)^T dO."""
    B, T, H, dk, dv = 1, 48, 1, 6, 5
    q, k, v, _ = tiny_inputs(B, T, H, dk, dv, seed=2)
    dO = np.random.default_rng(3).standard_normal((B, T, H, dv))
    dq, dkk, dvv, dg, dS0 = oracle.gla_recurrent_bwd(q, k, v, np.zeros_like(q), dO, scale=0.5)
    Q, K, V, D = q[0, :, 0], k[0, :, 0], v[0, :, 0], dO[0, :, 0]
    dA = np.tril(D @ V.T)
    assert relerr(dq[0, :, 0], 0.5 * dA @ K) < TOL
    assert relerr(dkk[0, :, 0], 0.5 * dA.T @ Q) < TOL
    assert relerr(dvv[0, :, 0], 0.5 * np.tril(Q @ K.T).T @ D) < TOL
    # d loss / d S0 = scale * sum_t q_t^T dO_t when nothing decays
    assert relerr(dS0[0, 0], 0.5 * Q.T @ D) < TOL


def test_gate_gradient_is_reverse_cumsum():
    """Last line of App. A.4: dG = revcum(Q .* dQ - K .* dK) when no gradient enters the final state;
    with dS_T the sum gains the constant row sums of dS_T .* S_T."""
    B, T, H, dk, dv = 2, 50, 2, 5, 4
    q, k, v, g = tiny_inputs(B, T, H, dk, dv, seed=8)
    r = np.random.default_rng(9)
    dO = r.standard_normal((B, T, H, dv))
    dq, dkk, _, dg, _ = oracle.gla_recurrent_bwd(q, k, v, g, dO, scale=0.9)
    dA = q * dq - k * dkk
    assert relerr(dg, np.flip(np.cumsum(np.flip(dA, 1), 1), 1)) < TOL
    dS_T = r.standard_normal((B, H, dk, dv))
    S0 = r.standard_normal((B, H, dk, dv))
    dq, dkk, _, dg, _ = oracle.gla_recurrent_bwd(q, k, v, g, dO, scale=0.9, S0=S0, dS_T=dS_T)
    _, S_T = oracle.gla_recurrent(q, k, v, g, scale=0.9, S0=S0)
    dA = q * dq - k * dkk
    tail = np.sum(dS_T * S_T, axis=-1)[:, None]                # [B, 1, H, dk]
    assert relerr(dg, np.flip(np.cumsum(np.flip(dA, 1), 1), 1) + tail) < TOL


@pytest.mark.parametrize("P", [2, 4, 8])
def test_bwd_segments_chain_through_dS(P):
    """Backward All-Scan of App. A.4: running the backward segment by segment, each segment started
    from the forward state entering it and handing d loss / d S0 to the segment before it, gives
    the gradients of the unsegmented run."""
    B, T, H, dk, dv = 1, 64, 2, 4, 5
    L = T // P
    q, k, v, g = tiny_inputs(B, T, H, dk, dv, seed=P)
    dO = np.random.default_rng(P + 1).standard_normal((B, T, H, dv))
    full = oracle.gla_recurrent_bwd(q, k, v, g, dO, scale=0.8)
    S_in = [np.zeros((B, H, dk, dv))]
    for p in range(P):
        sl = slice(p * L, (p + 1) * L)
        _, Sf = oracle.gla_recurrent(q[:, sl], k[:, sl], v[:, sl], g[:, sl], scale=0.8, S0=S_in[-1])
        S_in.append(Sf)
    dS = None
    parts = [None] * P
    for p in reversed(range(P)):
        sl = slice(p * L, (p + 1) * L)
        parts[p] = oracle.gla_recurrent_bwd(q[:, sl], k[:, sl], v[:, sl], g[:, sl], dO[:, sl], scale=0.8,
                                            S0=S_in[p], dS_T=dS)
        dS = parts[p][4]
    for i, name in enumerate(("dq", "dk", "dv", "dg")):
        assert relerr(np.concatenate([x[i] for x in parts], axis=1), full[i]) < TOL, name
    assert relerr(dS, full[4]) < TOL


def test_bwd_is_linear_in_dO_and_scale():
    B, T, H, dk, dv = 1, 30, 1, 3, 4
    q, k, v, g = tiny_inputs(B, T, H, dk, dv, seed=4)
    r = np.random.default_rng(5)
    d1, d2 = r.standard_normal((2, B, T, H, dv))
    a = oracle.gla_recurrent_bwd(q, k, v, g, d1, scale=0.5)
    b = oracle.gla_recurrent_bwd(q, k, v, g, d2, scale=0.5)
    c = oracle.gla_recurrent_bwd(q, k, v, g, 2 * d1 - 3 * d2, scale=1.5)
    for x, y, z in zip(a, b, c):
        assert relerr(z, 3 * (2 * x - 3 * y)) < TOL
