"""ctypes front end of the fp64 CPU oracle (gla_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module; the
product path (the HIP library and its binding) never does.  Everything here is numpy float64.

Array layouts follow gla_oracle.c: q, k, g, G_cum [B,T,H,d_k]; v, o [B,T,H,d_v];
S_loc, S_init [P,B,H,d_k,d_v]; G_tot [P,B,H,d_k]; g is the log decay (alpha = exp(g)).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gla_oracle.c")
_LIB = os.path.join(_HERE, "libgla_oracle.so")
_lib = None


def build(force=False):
    """Compile gla_oracle.c with gcc (OpenMP) into libgla_oracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _bind(lib):
    """Declare the argument types of every oracle_* function of a loaded library."""
    dp = ctypes.POINTER(ctypes.c_double)
    ci, cd = ctypes.c_int, ctypes.c_double
    lib.oracle_gla_recurrent.argtypes = [ci] * 5 + [dp] * 4 + [cd] + [dp] * 3
    lib.oracle_gla_recurrent.restype = None
    lib.oracle_gla_local.argtypes = [ci] * 6 + [dp] * 4 + [cd] + [dp] * 4
    lib.oracle_gla_local.restype = None
    lib.oracle_state_scan.argtypes = [ci] * 4 + [dp] * 5
    lib.oracle_state_scan.restype = None
    lib.oracle_apply_init_state.argtypes = [ci] * 6 + [dp] * 3 + [cd] + [dp]
    lib.oracle_apply_init_state.restype = None
    lib.oracle_gla_recurrent_bwd.argtypes = [ci] * 5 + [dp] * 4 + [cd] + [dp] * 8
    lib.oracle_gla_recurrent_bwd.restype = None
    lib.oracle_num_threads.argtypes = []
    lib.oracle_num_threads.restype = ci
    return lib


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = _bind(ctypes.CDLL(_LIB))
    return _lib


def _c(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def num_threads():
    return int(_load().oracle_num_threads())


def gla_recurrent(q, k, v, g, scale=1.0, S0=None):
    """Eq. (1) token by token over the whole sequence.  Returns (o [B,T,H,d_v], S_final [B,H,d_k,d_v])."""
    q, k, v, g = _c(q), _c(k), _c(v), _c(g)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    assert k.shape == q.shape == g.shape and v.shape == (B, T, H, dv)
    if S0 is not None:
        S0 = _c(S0)
        assert S0.shape == (B, H, dk, dv)
    o = np.empty((B, T, H, dv))
    Sf = np.empty((B, H, dk, dv))
    _load().oracle_gla_recurrent(B, T, H, dk, dv, _p(q), _p(k), _p(v), _p(g), float(scale),
                                 _p(S0), _p(o), _p(Sf))
    return o, Sf


def gla_recurrent_bwd(q, k, v, g, dO, scale=1.0, S0=None, dS_T=None):
    """Gradients of sum(o * dO) + sum(S_T * dS_T) for the unsegmented recurrence (App. A.4 computes
    the same quantities chunkwise).  Returns (dq, dk, dv, dg, dS0 [B,H,d_k,d_v])."""
    q, k, v, g, dO = _c(q), _c(k), _c(v), _c(g), _c(dO)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    assert k.shape == q.shape and g.shape == q.shape and v.shape == (B, T, H, dv) and dO.shape == v.shape
    if S0 is not None:
        S0 = _c(S0)
        assert S0.shape == (B, H, dk, dv)
    if dS_T is not None:
        dS_T = _c(dS_T)
        assert dS_T.shape == (B, H, dk, dv)
    dq, dkk, dg = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    dvv = np.empty_like(v)
    dS0 = np.empty((B, H, dk, dv))
    _load().oracle_gla_recurrent_bwd(B, T, H, dk, dv, _p(q), _p(k), _p(v), _p(g), float(scale), _p(S0),
                                     _p(dO), _p(dS_T), _p(dq), _p(dkk), _p(dvv), _p(dg), _p(dS0))
    return dq, dkk, dvv, dg, dS0


def gla_local(q, k, v, g, P, scale=1.0):
    """Local pass (Sec. 3.1): each of the P segments from the zero state.
    Returns (o_local, S_loc [P,B,H,d_k,d_v], G_cum [B,T,H,d_k], G_tot [P,B,H,d_k])."""
    q, k, v, g = _c(q), _c(k), _c(v), _c(g)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    assert T % P == 0
    L = T // P
    o = np.empty((B, T, H, dv))
    S_loc = np.empty((P, B, H, dk, dv))
    G_cum = np.empty((B, T, H, dk))
    G_tot = np.empty((P, B, H, dk))
    _load().oracle_gla_local(B, P, H, L, dk, dv, _p(q), _p(k), _p(v), _p(g), float(scale),
                             _p(o), _p(S_loc), _p(G_cum), _p(G_tot))
    return o, S_loc, G_cum, G_tot


def state_scan(S_loc, G_tot, S0=None):
    """Segment-state recurrence (Sec. 3.2).  S_loc [P,BH,d_k,d_v], G_tot [P,BH,d_k].
    Returns (S_init [P,BH,d_k,d_v], S_last [BH,d_k,d_v])."""
    S_loc, G_tot = _c(S_loc), _c(G_tot)
    P, BH, dk, dv = S_loc.shape
    assert G_tot.shape == (P, BH, dk)
    if S0 is not None:
        S0 = _c(S0)
        assert S0.shape == (BH, dk, dv)
    S_init = np.empty((P, BH, dk, dv))
    S_last = np.empty((BH, dk, dv))
    _load().oracle_state_scan(P, BH, dk, dv, _p(S_loc), _p(G_tot), _p(S0), _p(S_init), _p(S_last))
    return S_init, S_last


def apply_init_state(q, G_cum, S_init, o, scale=1.0):
    """o_t += (scale q_t .* exp(G_cum_t)) S_init[p]; returns a new array.  S_init [P,B,H,d_k,d_v]."""
    q, G_cum, S_init = _c(q), _c(G_cum), _c(S_init)
    o = np.array(o, dtype=np.float64, order="C", copy=True)
    B, T, H, dk = q.shape
    P = S_init.shape[0]
    dv = o.shape[-1]
    assert T % P == 0 and S_init.shape == (P, B, H, dk, dv)
    _load().oracle_apply_init_state(B, P, H, T // P, dk, dv, _p(q), _p(G_cum), _p(S_init),
                                    float(scale), _p(o))
    return o


def segmented_forward(q, k, v, g, P, scale=1.0, S0=None):
    """The three steps chained (local pass, segment scan, correction).  Returns (o, S_last)."""
    o_loc, S_loc, G_cum, G_tot = gla_local(q, k, v, g, P, scale)
    Pn, B, H, dk, dv = S_loc.shape
    S_init, S_last = state_scan(S_loc.reshape(Pn, B * H, dk, dv), G_tot.reshape(Pn, B * H, dk),
                                None if S0 is None else np.asarray(S0).reshape(B * H, dk, dv))
    o = apply_init_state(q, G_cum, S_init.reshape(Pn, B, H, dk, dv), o_loc, scale)
    return o, S_last.reshape(B, H, dk, dv)
