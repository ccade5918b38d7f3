"""Helpers of the GPU parity tests: error metrics and oracle calls on host copies of the inputs."""
import numpy as np
import torch

from oracle import oracle
from paper_2507_01004_amd import synth

# Tolerances: relative error per (batch, head) = max|x - ref| / max|ref|; 1e-4 for fp32 inputs,
# 2e-2 for bf16 inputs with fp32 accumulation.  Cumulative log decays are compared as logs:
# |dG| <= 1e-5 * max(1, |G|) (fp32 inputs; bf16 gates are exact inputs too, same bound).
TOL = {"f32": 1e-4, "bf16": 2e-2}


def rel_err_bh(x, ref, bh_axes):
    """max over (b, h) of max|x - ref| / max|ref|; `bh_axes` are the axes that index (b, h)."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    other = tuple(a for a in range(ref.ndim) if a not in bh_axes)
    num = np.max(np.abs(x - ref), axis=other)
    den = np.maximum(np.max(np.abs(ref), axis=other), 1e-30)
    return float(np.max(num / den))


def log_err(G, G_ref):
    G = np.asarray(G, dtype=np.float64)
    return float(np.max(np.abs(G - G_ref) / np.maximum(1.0, np.abs(G_ref))))


def host(t):
    return synth.to_f64(t)


def oracle_local(inp, P, scale=1.0):
    return oracle.gla_local(host(inp["q"]), host(inp["k"]), host(inp["v"]), host(inp["g"]), P, scale)


def oracle_full(inp, scale=1.0, S0=None):
    return oracle.gla_recurrent(host(inp["q"]), host(inp["k"]), host(inp["v"]), host(inp["g"]), scale, S0)


def dev(a, dtype=torch.float32):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dtype).cuda()


def randn_seeded(shape, seed, dtype=torch.float32):
    """Standard normal values on the GPU from a generator of their own (a failure must be reproducible)."""
    gen = torch.Generator(device="cuda").manual_seed(int(seed))
    return torch.randn(tuple(shape), device="cuda", generator=gen).to(dtype)
