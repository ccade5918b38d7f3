"""Independent numpy restatements used to pin the oracle (never imported by the oracle or the
HIP path).  Each is a different derivation from the token recurrence the oracle implements."""
import numpy as np


def tiny_inputs(B, T, H, dk, dv, seed, gate_div=4.0):
    r = np.random.default_rng(seed)
    q = r.standard_normal((B, T, H, dk))
    k = r.standard_normal((B, T, H, dk))
    k /= np.linalg.norm(k, axis=-1, keepdims=True)
    v = r.standard_normal((B, T, H, dv))
    x = r.standard_normal((B, T, H, dk))
    g = -np.log1p(np.exp(-x)) / gate_div      # logsigmoid(x)/gate_div
    return q, k, v, g


def quadratic_form(q, k, v, g, scale=1.0, S0=None):
    """Unrolled Eq. (1):  o_t = scale * sum_{s<=t} (sum_i q_ti k_si exp(G_ti - G_si)) v_s
                               + scale * (q_t .* exp(G_t)) S0,   G = inclusive cumsum of g.
    O(T^2 d) with explicit loops over (t, s).  Also returns the final state
    S_T = sum_s (exp(G_T - G_s) .* k_s)^T v_s + exp(G_T) .* S0."""
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    o = np.zeros((B, T, H, dv))
    Sf = np.zeros((B, H, dk, dv))
    for b in range(B):
        for h in range(H):
            G = np.cumsum(g[b, :, h, :], axis=0)
            for t in range(T):
                acc = np.zeros(dv)
                for s in range(t + 1):
                    w = np.sum(q[b, t, h] * k[b, s, h] * np.exp(G[t] - G[s]))
                    acc += w * v[b, s, h]
                if S0 is not None:
                    acc += (q[b, t, h] * np.exp(G[t])) @ S0[b, h]
                o[b, t, h] = scale * acc
            for s in range(T):
                Sf[b, h] += np.outer(np.exp(G[T - 1] - G[s]) * k[b, s, h], v[b, s, h])
            if S0 is not None:
                Sf[b, h] += np.exp(G[T - 1])[:, None] * S0[b, h]
    return o, Sf
