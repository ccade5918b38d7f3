"""The stored results of tests/golden/tiny_gla.json (written by tests/golden/make_golden.py, which calls
only the oracle) must be reproduced by the oracle as it stands: a change of the oracle's arithmetic
shows up here and has to be justified against the paper before the file is regenerated."""
import json
import os

import numpy as np

from oracle import oracle
from tests.golden.make_golden import B, DK, DV, H, P, SCALE, inputs

PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tiny_gla.json")


def test_oracle_reproduces_stored_values():
    gold = json.load(open(PATH))
    q, k, v, g, dO, S0 = inputs()
    o, S_T = oracle.gla_recurrent(q, k, v, g, SCALE, S0)
    o_loc, S_loc, G_cum, G_tot = oracle.gla_local(q, k, v, g, P, SCALE)
    S_init, S_last = oracle.state_scan(S_loc.reshape(P, B * H, DK, DV), G_tot.reshape(P, B * H, DK),
                                       S0.reshape(B * H, DK, DV))
    dq, dk, dv, dg, dS0 = oracle.gla_recurrent_bwd(q, k, v, g, dO, SCALE, S0)
    got = dict(o=o, S_T=S_T, o_local=o_loc, S_loc=S_loc, G_tot=G_tot, S_init=S_init, S_last=S_last,
               dq=dq, dk=dk, dv=dv, dg=dg, dS0=dS0)
    for name, x in got.items():
        ref = np.asarray(gold[name])
        assert ref.shape == x.shape, name
        assert np.max(np.abs(x - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref))), name
