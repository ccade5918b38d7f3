"""Seeded synthetic GLA workloads (inputs only: none of the method's arithmetic lives here).

Serves both the HIP path and the CPU oracle, which otherwise share nothing.  The recipe follows
the operator benchmark of the paper (App. A.3: random tensors, H heads of d_k = d_v = d/H):
q, k, v ~ N(0,1) with k L2-normalised per token, log decay g = logsigmoid(x) / 16 with
x ~ N(mu, 1) drawn per (token, head, d_k channel); mu = 0, or `slow_shift` for heads >=
`slow_head_from` (slowly decaying heads).  Tensors are laid out [B, T, H, d].
"""
import torch

# (B, H, P, L, d_k, d_v, C, io dtype, seed, first slow head or None)
CONFIGS = {
    "c1": dict(B=1, H=1, P=4, L=64, d_k=64, d_v=64, C=64, io="f32", seed=1001, slow_from=None),
    "c2": dict(B=1, H=16, P=1, L=16384, d_k=128, d_v=128, C=64, io="bf16", seed=1002, slow_from=None),
    "c3": dict(B=1, H=16, P=8, L=16384, d_k=128, d_v=128, C=64, io="bf16", seed=1003, slow_from=None),
    "c4": dict(B=1, H=16, P=64, L=16384, d_k=128, d_v=128, C=64, io="bf16", seed=1004, slow_from=None),
    "c5": dict(B=1, H=8, P=256, L=32768, d_k=128, d_v=128, C=64, io="bf16", seed=1005, slow_from=4),
}

_DT = {"f32": torch.float32, "bf16": torch.bfloat16}


def torch_dtype(name):
    return _DT[name]


def make_inputs(B, T, H, d_k, d_v, *, seed, io="bf16", g="f32", device="cpu", slow_from=None,
                slow_shift=2.0, gate_div=16.0, zero_gate=False, slab_tokens=8192, per_head_gate=False):
    """Returns dict(q, k, v, g) of torch tensors on `device`, generated slab by slab over T so that
    the fp32 temporaries stay small next to the result.  per_head_gate: g is [B,T,H] (one log decay per
    token and head, the first channel's draw) instead of [B,T,H,d_k]."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(int(seed))
    io_dt, g_dt = _DT[io], _DT[g]
    q = torch.empty(B, T, H, d_k, dtype=io_dt, device=dev)
    k = torch.empty(B, T, H, d_k, dtype=io_dt, device=dev)
    v = torch.empty(B, T, H, d_v, dtype=io_dt, device=dev)
    gt = torch.empty((B, T, H) if per_head_gate else (B, T, H, d_k), dtype=g_dt, device=dev)
    for t0 in range(0, T, slab_tokens):
        t1 = min(T, t0 + slab_tokens)
        n = t1 - t0
        q[:, t0:t1] = torch.randn(B, n, H, d_k, generator=gen, device=dev).to(io_dt)
        kk = torch.randn(B, n, H, d_k, generator=gen, device=dev)
        k[:, t0:t1] = (kk / kk.norm(dim=-1, keepdim=True)).to(io_dt)
        v[:, t0:t1] = torch.randn(B, n, H, d_v, generator=gen, device=dev).to(io_dt)
        x = torch.randn(B, n, H, d_k, generator=gen, device=dev)
        if slow_from is not None:
            x[:, :, slow_from:] += slow_shift
        if per_head_gate:
            x = x[..., 0]
        if zero_gate:
            gt[:, t0:t1] = 0
        else:
            gt[:, t0:t1] = (torch.nn.functional.logsigmoid(x) / gate_div).to(g_dt)
    return dict(q=q, k=k, v=v, g=gt)


def config_inputs(name, *, device="cpu", g="f32", **over):
    c = dict(CONFIGS[name])
    c.update(over)
    per_head = bool(c.pop("per_head_gate", False))
    return make_inputs(c["B"], c["P"] * c["L"], c["H"], c["d_k"], c["d_v"], seed=c["seed"],
                       io=c["io"], g=g, device=device, slow_from=c["slow_from"], per_head_gate=per_head), c


def to_f64(t):
    """Host float64 copy of a tensor's (already rounded) values."""
    return t.detach().to("cpu").to(torch.float64).numpy()
