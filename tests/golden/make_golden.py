"""Writes tests/golden/tiny_gla.json: the oracle's results on a tiny seeded input, as text.

The paper prints no worked numeric example, so nothing here is a value from the paper: the stored
numbers are what the fp64 oracle (oracle/, and nothing else) computes for inputs drawn by numpy's
PCG64 generator with the seed below.  The file pins the oracle against silent changes of its own
arithmetic; the independent pins of the oracle live in tests/test_oracle_pins.py and
tests/test_oracle_bwd_pins.py.  Run from the repository root:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import oracle  # noqa: E402

SEED, B, T, H, DK, DV, P, SCALE = 20250701, 1, 12, 2, 3, 2, 3, 0.75


def inputs():
    r = np.random.default_rng(SEED)
    q = r.standard_normal((B, T, H, DK))
    k = r.standard_normal((B, T, H, DK))
    k /= np.linalg.norm(k, axis=-1, keepdims=True)
    v = r.standard_normal((B, T, H, DV))
    g = -np.log1p(np.exp(-r.standard_normal((B, T, H, DK)))) / 4.0     # logsigmoid(x) / 4
    dO = r.standard_normal((B, T, H, DV))
    S0 = r.standard_normal((B, H, DK, DV))
    return q, k, v, g, dO, S0


def main():
    q, k, v, g, dO, S0 = inputs()
    o, S_T = oracle.gla_recurrent(q, k, v, g, SCALE, S0)
    o_loc, S_loc, G_cum, G_tot = oracle.gla_local(q, k, v, g, P, SCALE)
    S_init, S_last = oracle.state_scan(S_loc.reshape(P, B * H, DK, DV), G_tot.reshape(P, B * H, DK),
                                       S0.reshape(B * H, DK, DV))
    dq, dk, dv, dg, dS0 = oracle.gla_recurrent_bwd(q, k, v, g, dO, SCALE, S0)
    out = dict(seed=SEED, shape=dict(B=B, T=T, H=H, d_k=DK, d_v=DV, P=P), scale=SCALE,
               o=o.tolist(), S_T=S_T.tolist(), o_local=o_loc.tolist(), S_loc=S_loc.tolist(),
               G_tot=G_tot.tolist(), S_init=S_init.tolist(), S_last=S_last.tolist(),
               dq=dq.tolist(), dk=dk.tolist(), dv=dv.tolist(), dg=dg.tolist(), dS0=dS0.tolist())
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_gla.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=0)
    print("wrote", path)


if __name__ == "__main__":
    main()
