"""Pins of the fp64 oracle against what the paper and the mathematics fix (CPU only).

Every pin is a derivation other than the oracle's own token loop, chosen so that a dropped
term, a wrong sign or index, or a transposed operand fails at least one of them."""
import numpy as np
import pytest

from oracle import oracle
from tests.pins import quadratic_form, tiny_inputs

TOL = 1e-10


def relerr(a, b):
    return np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300)


# ---- Eq. (1) ------------------------------------------------------------------------------
@pytest.mark.parametrize("shape", [(1, 7, 1, 3, 2), (2, 33, 2, 5, 8), (1, 64, 3, 8, 4)])
def test_recurrent_vs_quadratic_unrolling(shape):
    """Eq. (1) unrolled by hand: decay enters as exp(G_t - G_s), diagonal weight exactly 1,
    state rows (d_k index) carry the decay; d_k != d_v catches transposed operands."""
    B, T, H, dk, dv = shape
    q, k, v, g = tiny_inputs(B, T, H, dk, dv, seed=T)
    S0 = np.random.default_rng(1).standard_normal((B, H, dk, dv))
    for s0 in (None, S0):
        o, Sf = oracle.gla_recurrent(q, k, v, g, scale=0.7, S0=s0)
        o_ref, Sf_ref = quadratic_form(q, k, v, g, scale=0.7, S0=s0)
        assert relerr(o, o_ref) < TOL
        assert relerr(Sf, Sf_ref) < TOL


@pytest.mark.parametrize("alpha", [0.5, 0.9, 1.0])
def test_geometric_closed_form(alpha):
    """d_k = d_v = 1, q = k = v = 1, constant alpha: S_t = sum_{r<=t} alpha^(t-r)
    => o_t = (1 - alpha^(t+1)) / (1 - alpha) for 0-based t, and o_t = t + 1 when alpha = 1."""
    T = 40
    one = np.ones((1, T, 1, 1))
    g = np.full((1, T, 1, 1), np.log(alpha))
    o, Sf = oracle.gla_recurrent(one, one, one, g)
    t = np.arange(T)
    ref = t + 1.0 if alpha == 1.0 else (1 - alpha ** (t + 1)) / (1 - alpha)
    assert relerr(o[0, :, 0, 0], ref) < TOL
    assert abs(Sf[0, 0, 0, 0] - ref[-1]) < TOL * ref[-1]


def test_zero_gate_is_causal_linear_attention():
    """alpha == 1 reduces GLA to plain causal linear attention (Sec. 1, Sec. 2.1):
    o = tril(Q K^T) V, computed with library matmuls."""
    B, T, H, dk, dv = 2, 50, 2, 6, 5
    q, k, v, _ = tiny_inputs(B, T, H, dk, dv, seed=3)
    g = np.zeros_like(q)
    o, Sf = oracle.gla_recurrent(q, k, v, g)
    for b in range(B):
        for h in range(H):
            A = np.tril(q[b, :, h] @ k[b, :, h].T)
            assert relerr(o[b, :, h], A @ v[b, :, h]) < TOL
            assert relerr(Sf[b, h], k[b, :, h].T @ v[b, :, h]) < TOL


def test_single_chunk_masked_matmul_form():
    """One chunk from the zero state (Sec. 2.1 chunk output with S_[i-1] = 0, Alg. 1 scores):
    O = [((Q .* Lambda)(K / Lambda)^T) .* M] V, Lambda = inclusive cumulative product of alpha,
    M lower triangular including the diagonal; final state = (K .* Gamma)^T V."""
    T, dk, dv = 64, 8, 12
    q, k, v, g = tiny_inputs(1, T, 1, dk, dv, seed=11, gate_div=16.0)
    o, Sf = oracle.gla_recurrent(q, k, v, g)
    Q, K, V = q[0, :, 0], k[0, :, 0], v[0, :, 0]
    Lam = np.exp(np.cumsum(g[0, :, 0], axis=0))
    P = np.tril((Q * Lam) @ (K / Lam).T)
    assert relerr(o[0, :, 0], P @ V) < 1e-9
    Gam = Lam[-1] / Lam
    assert relerr(Sf[0, 0], (K * Gam).T @ V) < 1e-9


def test_chunkwise_recurrence_matches():
    """Chunk state recurrence (Eq. (3)) and chunk output equation of Sec. 2.1 evaluated with
    numpy matmuls for C = 16 over 5 chunks (intra scores read with K / Lambda, as Alg. 1)."""
    T, C, dk, dv = 80, 16, 6, 7
    q, k, v, g = tiny_inputs(1, T, 1, dk, dv, seed=5, gate_div=8.0)
    o, Sf = oracle.gla_recurrent(q, k, v, g)
    S = np.zeros((dk, dv))
    M = np.tril(np.ones((C, C)))
    out = np.zeros((T, dv))
    for n in range(T // C):
        sl = slice(n * C, (n + 1) * C)
        Q, K, V = q[0, sl, 0], k[0, sl, 0], v[0, sl, 0]
        Lam = np.exp(np.cumsum(g[0, sl, 0], axis=0))
        gam = Lam[-1]
        Gam = gam / Lam
        out[sl] = (Q * Lam) @ S + (((Q * Lam) @ (K / Lam).T) * M) @ V
        S = gam[:, None] * S + (K * Gam).T @ V
    assert relerr(o[0, :, 0], out) < 1e-9
    assert relerr(Sf[0, 0], S) < 1e-9


def test_linearity_in_v_and_state():
    B, T, H, dk, dv = 1, 20, 2, 4, 3
    q, k, v, g = tiny_inputs(B, T, H, dk, dv, seed=8)
    r = np.random.default_rng(9)
    v2 = r.standard_normal(v.shape)
    S0 = r.standard_normal((B, H, dk, dv))
    oa, _ = oracle.gla_recurrent(q, k, v, g, S0=S0)
    ob, _ = oracle.gla_recurrent(q, k, v2, g, S0=None)
    oc, _ = oracle.gla_recurrent(q, k, 2 * v - 3 * v2, g, S0=2 * S0)
    assert relerr(oc, 2 * oa - 3 * ob) < TOL


# ---- local pass ----------------------------------------------------------------------------
def test_local_pass_is_per_segment_zero_state_run():
    B, P, L, H, dk, dv = 2, 3, 10, 2, 4, 5
    q, k, v, g = tiny_inputs(B, P * L, H, dk, dv, seed=21)
    o, S_loc, G_cum, G_tot = oracle.gla_local(q, k, v, g, P, scale=1.3)
    for p in range(P):
        sl = slice(p * L, (p + 1) * L)
        o_ref, Sf_ref = quadratic_form(q[:, sl], k[:, sl], v[:, sl], g[:, sl], scale=1.3)
        assert relerr(o[:, sl], o_ref) < TOL
        assert relerr(S_loc[p], Sf_ref) < TOL
        assert relerr(G_cum[:, sl], np.cumsum(g[:, sl], axis=1)) < TOL
        assert relerr(G_tot[p], np.sum(g[:, sl], axis=1)) < TOL


# ---- segmentation invariance (Eq. (global-correction), App. A.1) ----------------------------
@pytest.mark.parametrize("P", [1, 2, 4, 8])
def test_segmented_equals_unsegmented(P):
    B, T, H, dk, dv = 1, 96, 2, 5, 6
    q, k, v, g = tiny_inputs(B, T, H, dk, dv, seed=31)
    S0 = np.random.default_rng(2).standard_normal((B, H, dk, dv))
    for s0 in (None, S0):
        o_ref, Sf_ref = oracle.gla_recurrent(q, k, v, g, scale=0.9, S0=s0)
        o, S_last = oracle.segmented_forward(q, k, v, g, P, scale=0.9, S0=s0)
        assert relerr(o, o_ref) < 1e-9
        assert relerr(S_last, Sf_ref) < 1e-9


def test_segments_of_unequal_length_equal_unsegmented():
    """The same invariance for an uneven cut: the local pass of every token range on its own, the state
    recurrence over the ranges, the correction of every range by the state entering it."""
    B, T, H, dk, dv = 2, 90, 2, 4, 3
    q, k, v, g = tiny_inputs(B, T, H, dk, dv, seed=33)
    S0 = np.random.default_rng(3).standard_normal((B, H, dk, dv))
    start = [0, 7, 8, 40, 41, 77, 90]
    P = len(start) - 1
    parts = [oracle.gla_local(q[:, a:e], k[:, a:e], v[:, a:e], g[:, a:e], 1, scale=0.9)
             for a, e in zip(start[:-1], start[1:])]
    S_loc = np.stack([x[1][0] for x in parts]).reshape(P, B * H, dk, dv)
    G_tot = np.stack([x[3][0] for x in parts]).reshape(P, B * H, dk)
    S_init, S_last = oracle.state_scan(S_loc, G_tot, S0.reshape(B * H, dk, dv))
    o = np.concatenate([oracle.apply_init_state(q[:, a:e], x[2], S_init[p:p + 1].reshape(1, B, H, dk, dv), x[0], 0.9)
                        for p, (a, e, x) in enumerate(zip(start[:-1], start[1:], parts))], axis=1)
    o_ref, Sf_ref = oracle.gla_recurrent(q, k, v, g, scale=0.9, S0=S0)
    assert relerr(o, o_ref) < 1e-9
    assert relerr(S_last.reshape(B, H, dk, dv), Sf_ref) < 1e-9


def test_scan_states_are_global_states_at_segment_boundaries():
    """S_init[p] must be the unsegmented run's state right before segment p."""
    B, P, L, H, dk, dv = 1, 4, 12, 1, 3, 4
    q, k, v, g = tiny_inputs(B, P * L, H, dk, dv, seed=41)
    _, S_loc, _, G_tot = oracle.gla_local(q, k, v, g, P)
    S_init, _ = oracle.state_scan(S_loc.reshape(P, B * H, dk, dv), G_tot.reshape(P, B * H, dk))
    for p in range(P):
        if p == 0:
            ref = np.zeros((B, H, dk, dv))
        else:
            _, ref = quadratic_form(q[:, :p * L], k[:, :p * L], v[:, :p * L], g[:, :p * L])
        assert np.max(np.abs(S_init[p].reshape(B, H, dk, dv) - ref)) < 1e-10


# ---- segment scan (Sec. 3.2) -----------------------------------------------------------------
def test_scan_unit_decay_is_exclusive_cumsum():
    r = np.random.default_rng(51)
    P, BH, dk, dv = 6, 3, 4, 5
    S_loc = r.standard_normal((P, BH, dk, dv))
    S0 = r.standard_normal((BH, dk, dv))
    S_init, S_last = oracle.state_scan(S_loc, np.zeros((P, BH, dk)), S0)
    inc = S0[None] + np.cumsum(S_loc, axis=0)
    assert relerr(S_init[0], S0) < TOL
    assert relerr(S_init[1:], inc[:-1]) < TOL
    assert relerr(S_last, inc[-1]) < TOL


def test_scan_single_source_is_product_of_decays():
    """Only segment 0 contributes: S_init[p] = exp(sum_{0<r<p} G_tot[r]) .* S_loc[0] (rows)."""
    r = np.random.default_rng(52)
    P, BH, dk, dv = 5, 2, 3, 4
    S_loc = np.zeros((P, BH, dk, dv))
    S_loc[0] = r.standard_normal((BH, dk, dv))
    G_tot = -r.random((P, BH, dk))
    S_init, S_last = oracle.state_scan(S_loc, G_tot)
    assert np.all(S_init[0] == 0)
    for p in range(1, P + 1):
        ref = np.exp(np.sum(G_tot[1:p], axis=0))[..., None] * S_loc[0]
        got = S_last if p == P else S_init[p]
        assert relerr(got, ref) < TOL


def test_scan_associativity_pair_merge():
    """Merging neighbouring segments (G1+G2, exp(G2) .* S1 + S2) and scanning the merged list
    must reproduce the even-index results."""
    r = np.random.default_rng(53)
    P, BH, dk, dv = 8, 2, 3, 3
    S_loc = r.standard_normal((P, BH, dk, dv))
    G_tot = -r.random((P, BH, dk))
    S_init, S_last = oracle.state_scan(S_loc, G_tot)
    Gm = G_tot[0::2] + G_tot[1::2]
    Sm = np.exp(G_tot[1::2])[..., None] * S_loc[0::2] + S_loc[1::2]
    S_init_m, S_last_m = oracle.state_scan(Sm, Gm)
    assert relerr(S_init_m, S_init[0::2]) < TOL
    assert relerr(S_last_m, S_last) < TOL


def test_scan_single_segment():
    r = np.random.default_rng(54)
    S_loc = r.standard_normal((1, 2, 3, 4))
    G = -r.random((1, 2, 3))
    S0 = r.standard_normal((2, 3, 4))
    S_init, S_last = oracle.state_scan(S_loc, G, S0)
    assert np.array_equal(S_init[0], S0)
    assert relerr(S_last, np.exp(G[0])[..., None] * S0 + S_loc[0]) < TOL


# ---- correction ------------------------------------------------------------------------------
def test_correction_zero_state_is_identity_and_zero_gate_is_gemm():
    r = np.random.default_rng(61)
    B, P, L, H, dk, dv = 1, 2, 6, 2, 3, 4
    q = r.standard_normal((B, P * L, H, dk))
    o = r.standard_normal((B, P * L, H, dv))
    G = -r.random((B, P * L, H, dk))
    Z = np.zeros((P, B, H, dk, dv))
    assert np.array_equal(oracle.apply_init_state(q, G, Z, o), o)
    S = r.standard_normal((P, B, H, dk, dv))
    got = oracle.apply_init_state(q, np.zeros_like(G), S, o, scale=0.5)
    ref = o.copy()
    for p in range(P):
        sl = slice(p * L, (p + 1) * L)
        ref[:, sl] += 0.5 * np.einsum("bthi,bhij->bthj", q[:, sl], S[p])
    assert relerr(got, ref) < TOL


def test_correction_first_token_uses_its_own_decay():
    """o_0 += (q_0 .* alpha_0) S_init : the incoming state is decayed by the token's own gate."""
    r = np.random.default_rng(62)
    dk, dv = 3, 2
    q = r.standard_normal((1, 1, 1, dk))
    g = -r.random((1, 1, 1, dk))
    S = r.standard_normal((1, 1, 1, dk, dv))
    got = oracle.apply_init_state(q, g, S, np.zeros((1, 1, 1, dv)))
    ref = (q[0, 0, 0] * np.exp(g[0, 0, 0])) @ S[0, 0, 0]
    assert relerr(got[0, 0, 0], ref) < TOL
    o2, _ = oracle.gla_recurrent(q, np.zeros_like(q), np.zeros((1, 1, 1, dv)), g, S0=S[0])
    assert relerr(o2[0, 0, 0], ref) < TOL
