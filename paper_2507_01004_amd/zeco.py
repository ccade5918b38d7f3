"""Thin ctypes binding of libzeco.so (C ABI in include/zeco.h): argument marshalling only.

Every step of the path runs in the HIP kernels; PyTorch supplies device memory and the stream.
There is no CPU fallback: a missing library raises.  Tensor layouts: q, k, g [B,T,H,d_k];
v, o [B,T,H,d_v] (any strides with a contiguous last dimension); S_loc, S_init [P,B,H,d_k,d_v]
fp32; G_cum [B,T,H,d_k] fp32; G_tot [P,B,H,d_k] fp32.
"""
import contextlib
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "csrc", "libzeco.so")

ZECO_OK, ZECO_ERR_INVALID_ARG, ZECO_ERR_UNSUPPORTED, ZECO_ERR_WORKSPACE, ZECO_ERR_HIP, ZECO_ERR_SCRATCH_LIMIT = range(6)
ZECO_F32, ZECO_BF16 = 0, 1
APPLY_FIRST_SEGMENT_ZERO, APPLY_DENSE = 1, 2
SCHEDULE_AUTO, SCHEDULE_TWO_PHASE, SCHEDULE_CORRECT = 0, 1, 2
EXPORTS = ("zeco_gla_local_fwd_workspace", "zeco_gla_local_fwd", "zeco_state_scan",
           "zeco_state_scan_tree_workspace", "zeco_state_scan_tree",
           "zeco_state_scan_tree_static_limit", "zeco_state_scan_tree_static",
           "zeco_apply_init_state", "zeco_gla_local_fwd_varlen", "zeco_apply_init_state_varlen",
           "zeco_gla_local_state_varlen", "zeco_gla_fwd_from_state_varlen",
           "zeco_gla_bwd_dstate_varlen", "zeco_gla_bwd_from_state_varlen",
           "zeco_gla_fused_fwd_varlen_workspace", "zeco_gla_fused_fwd_varlen",
           "zeco_gla_fused_bwd_varlen_workspace", "zeco_gla_fused_bwd_varlen",
           "zeco_gla_local_fwd_chunk_decay", "zeco_apply_init_state_chunk_decay",
           "zeco_gla_local_state", "zeco_gla_fwd_from_state",
           "zeco_gla_fused_fwd_workspace", "zeco_gla_saved_states_bytes", "zeco_gla_fused_fwd", "zeco_gla_bwd_dstate",
           "zeco_gla_bwd_from_state_workspace", "zeco_gla_bwd_from_state", "zeco_gla_fused_bwd_workspace", "zeco_gla_fused_bwd",
           "zeco_hbm_copy", "zeco_hbm_mix", "zeco_status_string", "zeco_version")


class GlaDesc(ctypes.Structure):
    """Mirror of zeco_gla_desc."""
    _fields_ = [("B", ctypes.c_int32), ("P", ctypes.c_int32), ("H", ctypes.c_int32),
                ("L", ctypes.c_int32), ("d_k", ctypes.c_int32), ("d_v", ctypes.c_int32),
                ("C", ctypes.c_int32), ("io_dtype", ctypes.c_int32), ("g_dtype", ctypes.c_int32),
                ("scale", ctypes.c_float),
                ("stride_b", ctypes.c_int64), ("stride_t", ctypes.c_int64), ("stride_h", ctypes.c_int64),
                ("vstride_b", ctypes.c_int64), ("vstride_t", ctypes.c_int64), ("vstride_h", ctypes.c_int64),
                ("g_per_head", ctypes.c_int32),
                ("wide_gates", ctypes.c_int32)]


class ZecoError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__("%s: %s (status %d)" % (where, status_string(status), status))


_lib = None


def lib():
    """The loaded library.  Raises if it has not been built (python -m paper_2507_01004_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libzeco.so is not built: run __graft_entry__.build() "
                               "(expected at %s); there is no fallback path" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, fp = ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p
        dp = ctypes.POINTER(GlaDesc)
        L.zeco_gla_local_fwd_workspace.argtypes = [dp]
        L.zeco_gla_local_fwd_workspace.restype = ctypes.c_size_t
        L.zeco_gla_local_fwd.argtypes = [dp, vp, vp, vp, vp, vp, fp, fp, fp, vp, ctypes.c_size_t, vp]
        L.zeco_gla_local_fwd.restype = i32
        L.zeco_state_scan.argtypes = [i32, i32, i32, i32, i32, fp, fp, fp, fp, fp, i32, i32, vp]
        L.zeco_state_scan.restype = i32
        L.zeco_state_scan_tree_workspace.argtypes = [i32, i32, i32, i32, i32]
        L.zeco_state_scan_tree_workspace.restype = ctypes.c_size_t
        L.zeco_state_scan_tree.argtypes = [i32, i32, i32, i32, fp, fp, fp, fp, fp, i32, i32, vp, ctypes.c_size_t, vp]
        L.zeco_state_scan_tree.restype = i32
        L.zeco_state_scan_tree_static_limit.argtypes = []
        L.zeco_state_scan_tree_static_limit.restype = ctypes.c_size_t
        L.zeco_state_scan_tree_static.argtypes = [i32, i32, i32, i32, fp, fp, fp, fp, fp, i32, i32, vp]
        L.zeco_state_scan_tree_static.restype = i32
        L.zeco_apply_init_state.argtypes = [dp, vp, fp, fp, vp, i32, vp]
        L.zeco_apply_init_state.restype = i32
        L.zeco_gla_local_fwd_varlen.argtypes = [dp, vp, ctypes.c_int64, vp, vp, vp, vp, vp, fp, fp, fp, vp]
        L.zeco_gla_local_fwd_varlen.restype = i32
        L.zeco_apply_init_state_varlen.argtypes = [dp, vp, ctypes.c_int64, vp, fp, fp, vp, i32, vp]
        L.zeco_apply_init_state_varlen.restype = i32
        L.zeco_gla_local_state_varlen.argtypes = [dp, vp, ctypes.c_int64, vp, vp, vp, fp, fp, vp]
        L.zeco_gla_local_state_varlen.restype = i32
        L.zeco_gla_fwd_from_state_varlen.argtypes = [dp, vp, ctypes.c_int64, vp, vp, vp, vp, fp, vp, vp]
        L.zeco_gla_fwd_from_state_varlen.restype = i32
        L.zeco_gla_bwd_dstate_varlen.argtypes = [dp, vp, ctypes.c_int64, vp, vp, vp, fp, vp]
        L.zeco_gla_bwd_dstate_varlen.restype = i32
        L.zeco_gla_bwd_from_state_varlen.argtypes = [dp, vp, ctypes.c_int64] + [vp] * 5 + [fp] * 3 + [vp] * 3 + [fp, vp, ctypes.c_size_t, vp]
        L.zeco_gla_bwd_from_state_varlen.restype = i32
        for nm in ("zeco_gla_fused_fwd_varlen_workspace", "zeco_gla_fused_bwd_varlen_workspace"):
            getattr(L, nm).argtypes = [dp]
            getattr(L, nm).restype = ctypes.c_size_t
        L.zeco_gla_fused_fwd_varlen.argtypes = [dp, vp, ctypes.c_int64] + [vp] * 4 + [fp, vp, fp, vp, ctypes.c_size_t, vp]
        L.zeco_gla_fused_fwd_varlen.restype = i32
        L.zeco_gla_fused_bwd_varlen.argtypes = [dp, vp, ctypes.c_int64] + [vp] * 5 + [fp, fp] + [vp] * 3 + [fp, fp, vp, ctypes.c_size_t, vp]
        L.zeco_gla_fused_bwd_varlen.restype = i32
        L.zeco_gla_local_fwd_chunk_decay.argtypes = [dp, vp, vp, vp, vp, vp, fp, fp, fp, vp]
        L.zeco_gla_local_fwd_chunk_decay.restype = i32
        L.zeco_apply_init_state_chunk_decay.argtypes = [dp, vp, vp, fp, fp, vp, i32, vp]
        L.zeco_apply_init_state_chunk_decay.restype = i32
        L.zeco_gla_local_state.argtypes = [dp, vp, vp, vp, fp, fp, vp]
        L.zeco_gla_local_state.restype = i32
        L.zeco_gla_fwd_from_state.argtypes = [dp, vp, vp, vp, vp, fp, vp, vp]
        L.zeco_gla_fwd_from_state.restype = i32
        L.zeco_gla_fused_fwd_workspace.argtypes = [dp]
        L.zeco_gla_fused_fwd_workspace.restype = ctypes.c_size_t
        L.zeco_gla_saved_states_bytes.argtypes = [dp]
        L.zeco_gla_saved_states_bytes.restype = ctypes.c_size_t
        L.zeco_gla_fused_fwd.argtypes = [dp, vp, vp, vp, vp, fp, vp, fp, fp, i32, vp, ctypes.c_size_t, vp]
        L.zeco_gla_fused_fwd.restype = i32
        L.zeco_gla_bwd_dstate.argtypes = [dp, vp, vp, vp, fp, vp]
        L.zeco_gla_bwd_dstate.restype = i32
        L.zeco_gla_bwd_from_state.argtypes = [dp] + [vp] * 5 + [fp] * 3 + [vp] * 3 + [fp, vp, ctypes.c_size_t, vp]
        L.zeco_gla_bwd_from_state_workspace.argtypes = [dp]
        L.zeco_gla_bwd_from_state_workspace.restype = ctypes.c_size_t
        L.zeco_gla_bwd_from_state.restype = i32
        L.zeco_gla_fused_bwd_workspace.argtypes = [dp]
        L.zeco_gla_fused_bwd_workspace.restype = ctypes.c_size_t
        L.zeco_gla_fused_bwd.argtypes = [dp] + [vp] * 5 + [fp] * 3 + [vp] * 3 + [fp, fp, vp, ctypes.c_size_t, vp]
        L.zeco_gla_fused_bwd.restype = i32
        L.zeco_hbm_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.zeco_hbm_copy.restype = i32
        L.zeco_hbm_mix.argtypes = [vp, vp, ctypes.c_size_t, i32, i32, vp]
        L.zeco_hbm_mix.restype = i32
        L.zeco_status_string.argtypes = [i32]
        L.zeco_status_string.restype = ctypes.c_char_p
        L.zeco_version.argtypes = []
        L.zeco_version.restype = i32
        _lib = L
    return _lib


def status_string(status):
    return lib().zeco_status_string(int(status)).decode()


def version():
    return int(lib().zeco_version())


def _dtype_code(t):
    if t.dtype == torch.float32:
        return ZECO_F32
    if t.dtype == torch.bfloat16:
        return ZECO_BF16
    raise TypeError("unsupported dtype %s" % t.dtype)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


_WIDE_GATES = False


@contextlib.contextmanager
def wide_gates(on=True):
    """Within the block every descriptor asks for the wide range of gates (zeco_gla_desc.wide_gates: the sum of
    |g| over a chunk may reach 160 instead of 80 with bf16 q/k/v, at about 3 % more time in the chunk kernels)."""
    global _WIDE_GATES
    before, _WIDE_GATES = _WIDE_GATES, bool(on)
    try:
        yield
    finally:
        _WIDE_GATES = before


def _desc(q, v, g_code, per_head, P, C, scale):
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    if T % P != 0:
        raise ValueError("T=%d is not a multiple of P=%d" % (T, P))
    if q.stride(-1) != 1 or v.stride(-1) != 1:
        raise ValueError("innermost dimension must be contiguous")
    return GlaDesc(B, P, H, T // P, dk, dv, C, _dtype_code(q), g_code, float(scale),
                   q.stride(0), q.stride(1), q.stride(2), v.stride(0), v.stride(1), v.stride(2),
                   int(per_head), int(_WIDE_GATES))


def make_desc(q, v, g, P, C=64, scale=1.0):
    """Descriptor of a call that reads the gate g: [B,T,H,d_k] laid out like q, or, with one log decay
    per (token, head), a contiguous [B,T,H] tensor."""
    B, T, H, dk = q.shape
    per_head = g.dim() == 3
    if per_head:
        if tuple(g.shape) != (B, T, H) or not g.is_contiguous():
            raise ValueError("a per-head gate must be a contiguous [B,T,H] tensor")
    elif g.shape != q.shape or g.stride() != q.stride():
        raise ValueError("a per-channel gate must have the shape and strides of q")
    return _desc(q, v, _dtype_code(g), per_head, P, C, scale)


def _gate_dims(g, dk):
    """Trailing dimensions of the gate-shaped outputs (G_cum, G_tot, dg)."""
    return () if g.dim() == 3 else (dk,)


def _check_same_layout(ref, *others):
    for t in others:
        if t.shape != ref.shape or t.stride() != ref.stride() or t.device != ref.device:
            raise ValueError("tensors sharing a descriptor must share shape, strides and device")


def local_fwd_workspace_bytes(q, v, g, P, C=64):
    return int(lib().zeco_gla_local_fwd_workspace(ctypes.byref(make_desc(q, v, g, P, C, 1.0))))


def gla_local_fwd(q, k, v, g, P, scale=1.0, C=64, out=None, workspace=None):
    """zeco_gla_local_fwd.  Returns (o, S_loc, G_cum, G_tot); `out` and `workspace` may be supplied
    preallocated (then the call allocates nothing)."""
    if not q.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    _check_same_layout(q, k)
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise TypeError("q, k, v must share a dtype")
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    desc = make_desc(q, v, g, P, C, scale)
    if out is None:
        o = torch.empty_strided(v.shape, v.stride(), dtype=v.dtype, device=v.device)
        S_loc = torch.empty(P, B, H, dk, dv, dtype=torch.float32, device=q.device)
        G_cum = torch.empty((B, T, H) + _gate_dims(g, dk), dtype=torch.float32, device=q.device)
        G_tot = torch.empty((P, B, H) + _gate_dims(g, dk), dtype=torch.float32, device=q.device)
    else:
        o, S_loc, G_cum, G_tot = out
        _check_same_layout(v, o)
    L = lib()
    ws_bytes = L.zeco_gla_local_fwd_workspace(ctypes.byref(desc))
    ws = workspace
    if ws is None and ws_bytes:
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device=q.device)
    ws_bytes = ws.numel() if ws is not None else 0
    st = L.zeco_gla_local_fwd(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(g), _ptr(o),
                              _ptr(S_loc), _ptr(G_cum), _ptr(G_tot), _ptr(ws), ws_bytes, _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_gla_local_fwd")
    return o, S_loc, G_cum, G_tot


def state_scan(S_loc, G_tot, S0=None, K_blocks=16, out=None, direction=0):
    """zeco_state_scan on [P,B,H,d_k,d_v] (or [P,BH,d_k,d_v]) states.  Returns (S_init, S_last)."""
    if not S_loc.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    P, dk, dv = S_loc.shape[0], S_loc.shape[-2], S_loc.shape[-1]
    BH = S_loc.numel() // (P * dk * dv)
    if not (S_loc.is_contiguous() and G_tot.is_contiguous()):
        raise ValueError("S_loc and G_tot must be contiguous")
    if out is None:
        S_init = torch.empty_like(S_loc)
        S_last = torch.empty(S_loc.shape[1:], dtype=torch.float32, device=S_loc.device)
    else:
        S_init, S_last = out
    if G_tot.numel() not in (P * BH, P * BH * dk):
        raise ValueError("G_tot must be [P,BH,d_k] or, for per-head gates, [P,BH]")
    per_head = int(G_tot.numel() == P * BH and dk != 1)
    st = lib().zeco_state_scan(P, BH, dk, dv, int(K_blocks), _ptr(S_loc), _ptr(G_tot), _ptr(S0),
                               _ptr(S_init), _ptr(S_last), int(direction), per_head, _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_state_scan")
    return S_init, S_last


def state_scan_tree(S_loc, G_tot, S0=None, out=None, direction=0, workspace=None):
    """zeco_state_scan_tree: the scan as a tree of depth two (groups of segments scanned in parallel).
    Same arguments and result as state_scan, up to rounding.  Returns (S_init, S_last)."""
    if not S_loc.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    P, dk, dv = S_loc.shape[0], S_loc.shape[-2], S_loc.shape[-1]
    BH = S_loc.numel() // (P * dk * dv)
    if not (S_loc.is_contiguous() and G_tot.is_contiguous()):
        raise ValueError("S_loc and G_tot must be contiguous")
    if out is None:
        S_init = torch.empty_like(S_loc)
        S_last = torch.empty(S_loc.shape[1:], dtype=torch.float32, device=S_loc.device)
    else:
        S_init, S_last = out
    if G_tot.numel() not in (P * BH, P * BH * dk):
        raise ValueError("G_tot must be [P,BH,d_k] or, for per-head gates, [P,BH]")
    per_head = int(G_tot.numel() == P * BH and dk != 1)
    need = int(lib().zeco_state_scan_tree_workspace(P, BH, dk, dv, per_head))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=S_loc.device)
    st = lib().zeco_state_scan_tree(P, BH, dk, dv, _ptr(S_loc), _ptr(G_tot), _ptr(S0), _ptr(S_init), _ptr(S_last),
                                    int(direction), per_head, _ptr(workspace), workspace.numel(), _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_state_scan_tree")
    return S_init, S_last


def state_scan_tree_static(S_loc, G_tot, S0, out, direction=0):
    """zeco_state_scan_tree_static: zeco_state_scan_tree on the library's own fixed scratch.  The call
    allocates nothing, and neither does this wrapper: the outputs (S_init, S_last) are the caller's."""
    if not S_loc.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    P, dk, dv = S_loc.shape[0], S_loc.shape[-2], S_loc.shape[-1]
    BH = S_loc.numel() // (P * dk * dv)
    if not (S_loc.is_contiguous() and G_tot.is_contiguous()):
        raise ValueError("S_loc and G_tot must be contiguous")
    S_init, S_last = out
    if G_tot.numel() not in (P * BH, P * BH * dk):
        raise ValueError("G_tot must be [P,BH,d_k] or, for per-head gates, [P,BH]")
    per_head = int(G_tot.numel() == P * BH and dk != 1)
    st = lib().zeco_state_scan_tree_static(P, BH, dk, dv, _ptr(S_loc), _ptr(G_tot), _ptr(S0), _ptr(S_init),
                                           _ptr(S_last), int(direction), per_head, _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_state_scan_tree_static")
    return S_init, S_last


def apply_init_state(q, g_like, G_cum, S_init, o, P, scale=1.0, C=64, first_segment_is_zero=True,
                     dense=False):
    """zeco_apply_init_state: o += (scale q .* exp(G_cum)) S_init[p], in place.  `g_like` only
    supplies the gate dtype recorded in the descriptor; G_cum [B,T,H] selects per-head gates.
    dense: also stream the tokens whose decay factor has vanished (ZECO_APPLY_DENSE)."""
    if not q.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    desc = _desc(q, o, _dtype_code(g_like), G_cum.dim() == 3, P, C, scale)
    st = lib().zeco_apply_init_state(ctypes.byref(desc), _ptr(q), _ptr(G_cum), _ptr(S_init), _ptr(o),
                                     _apply_flags(first_segment_is_zero, dense), _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_apply_init_state")
    return o


def _varlen_desc(q, v, g_code, per_head, seg_start, max_len, scale, C=64):
    """Descriptor of a call over segments of unequal length: L is the bound on the lengths."""
    if seg_start.dtype != torch.int64 or not seg_start.is_cuda or seg_start.dim() != 1 or not seg_start.is_contiguous():
        raise ValueError("seg_start must be a contiguous int64 device vector of P+1 token offsets")
    if q.stride(-1) != 1 or v.stride(-1) != 1:
        raise ValueError("innermost dimension must be contiguous")
    B, T, H, dk = q.shape
    return GlaDesc(B, seg_start.numel() - 1, H, int(max_len), dk, v.shape[-1], int(C), _dtype_code(q), g_code,
                   float(scale), q.stride(0), q.stride(1), q.stride(2), v.stride(0), v.stride(1), v.stride(2),
                   int(per_head), int(_WIDE_GATES))


def gla_local_fwd_varlen(q, k, v, g, seg_start, max_len, scale=1.0, C=64, out=None):
    """zeco_gla_local_fwd_varlen: the local pass over segments [seg_start[p], seg_start[p+1]) of the token
    axis, none longer than max_len.  seg_start: int64 device vector.  Returns (o, S_loc, G_cum, G_tot)."""
    if not q.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    _check_same_layout(q, k)
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise TypeError("q, k, v must share a dtype")
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    per_head = g.dim() == 3
    if per_head:
        if tuple(g.shape) != (B, T, H) or not g.is_contiguous():
            raise ValueError("a per-head gate must be a contiguous [B,T,H] tensor")
    elif g.shape != q.shape or g.stride() != q.stride():
        raise ValueError("a per-channel gate must have the shape and strides of q")
    desc = _varlen_desc(q, v, _dtype_code(g), per_head, seg_start, max_len, scale, C)
    P = desc.P
    if out is None:
        o = torch.empty_strided(v.shape, v.stride(), dtype=v.dtype, device=v.device)
        S_loc = torch.empty(P, B, H, dk, dv, dtype=torch.float32, device=q.device)
        G_cum = torch.empty((B, T, H) + _gate_dims(g, dk), dtype=torch.float32, device=q.device)
        G_tot = torch.empty((P, B, H) + _gate_dims(g, dk), dtype=torch.float32, device=q.device)
    else:
        o, S_loc, G_cum, G_tot = out
        _check_same_layout(v, o)
    st = lib().zeco_gla_local_fwd_varlen(ctypes.byref(desc), _ptr(seg_start), T, _ptr(q), _ptr(k), _ptr(v), _ptr(g),
                                         _ptr(o), _ptr(S_loc), _ptr(G_cum), _ptr(G_tot), _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_gla_local_fwd_varlen")
    return o, S_loc, G_cum, G_tot


def apply_init_state_varlen(q, g_like, G_cum, S_init, o, seg_start, max_len, scale=1.0, C=64, first_segment_is_zero=True,
                            dense=False):
    """zeco_apply_init_state_varlen: the correction over the segments of gla_local_fwd_varlen, in place."""
    if not q.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    desc = _varlen_desc(q, o, _dtype_code(g_like), G_cum.dim() == 3, seg_start, max_len, scale, C)
    st = lib().zeco_apply_init_state_varlen(ctypes.byref(desc), _ptr(seg_start), q.shape[1], _ptr(q), _ptr(G_cum),
                                            _ptr(S_init), _ptr(o), _apply_flags(first_segment_is_zero, dense),
                                            _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_apply_init_state_varlen")
    return o


def _gate_per_head(q, g):
    per_head = g.dim() == 3
    if per_head:
        if tuple(g.shape) != tuple(q.shape[:3]) or not g.is_contiguous():
            raise ValueError("a per-head gate must be a contiguous [B,T,H] tensor")
    elif g.shape != q.shape or g.stride() != q.stride():
        raise ValueError("a per-channel gate must have the shape and strides of q")
    return per_head


def gla_local_state_varlen(k, v, g, seg_start, max_len, C=64, out=None):
    """zeco_gla_local_state_varlen: end state and total log decay of every segment of the table from the
    zero state.  Returns (S_loc, G_tot)."""
    if not k.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    B, T, H, dk = k.shape
    dv = v.shape[-1]
    desc = _varlen_desc(k, v, _dtype_code(g), _gate_per_head(k, g), seg_start, max_len, 1.0, C)
    if out is None:
        S_loc = torch.empty(desc.P, B, H, dk, dv, dtype=torch.float32, device=k.device)
        G_tot = torch.empty((desc.P, B, H) + _gate_dims(g, dk), dtype=torch.float32, device=k.device)
    else:
        S_loc, G_tot = out
    st = lib().zeco_gla_local_state_varlen(ctypes.byref(desc), _ptr(seg_start), T, _ptr(k), _ptr(v), _ptr(g),
                                           _ptr(S_loc), _ptr(G_tot), _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_gla_local_state_varlen")
    return S_loc, G_tot


def gla_fwd_from_state_varlen(q, k, v, g, S_init, seg_start, max_len, scale=1.0, C=64, out=None):
    """zeco_gla_fwd_from_state_varlen: the forward of every segment of the table from S_init[p].  Returns o."""
    if not q.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    _check_same_layout(q, k)
    desc = _varlen_desc(q, v, _dtype_code(g), _gate_per_head(q, g), seg_start, max_len, scale, C)
    o = torch.empty_strided(v.shape, v.stride(), dtype=v.dtype, device=v.device) if out is None else out
    st = lib().zeco_gla_fwd_from_state_varlen(ctypes.byref(desc), _ptr(seg_start), q.shape[1], _ptr(q), _ptr(k),
                                              _ptr(v), _ptr(g), _ptr(S_init), _ptr(o), _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_gla_fwd_from_state_varlen")
    return o


def gla_bwd_dstate_varlen(q, g, dO, seg_start, max_len, scale=1.0, C=64, out=None):
    """zeco_gla_bwd_dstate_varlen: the state gradient leaving every segment of the table towards the earlier
    ones, from dS = 0.  Returns dS_loc [P,B,H,d_k,d_v]."""
    if not q.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    B, T, H, dk = q.shape
    dv = dO.shape[-1]
    desc = _varlen_desc(q, dO, _dtype_code(g), _gate_per_head(q, g), seg_start, max_len, scale, C)
    dS_loc = torch.empty(desc.P, B, H, dk, dv, dtype=torch.float32, device=q.device) if out is None else out
    st = lib().zeco_gla_bwd_dstate_varlen(ctypes.byref(desc), _ptr(seg_start), T, _ptr(q), _ptr(g), _ptr(dO),
                                          _ptr(dS_loc), _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_gla_bwd_dstate_varlen")
    return dS_loc


def _bwd_from_state_workspace(desc, workspace, device):
    need = int(lib().zeco_gla_bwd_from_state_workspace(ctypes.byref(desc)))
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
    return workspace, (workspace.numel() if workspace is not None else 0)


def gla_bwd_from_state_varlen(q, k, v, g, dO, S_init, S_last, dS_in, seg_start, max_len, scale=1.0, C=64, out=None,
                              workspace=None):
    """zeco_gla_bwd_from_state_varlen: dq, dk, dv, dg of every segment of the table from the scanned forward
    states and state gradients.  Returns (dq, dk, dv, dg)."""
    if not q.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    _check_same_layout(q, k)
    _check_same_layout(v, dO)
    desc = _varlen_desc(q, v, _dtype_code(g), _gate_per_head(q, g), seg_start, max_len, scale, C)
    dq, dk, dv, dg = _grad_outputs(q, v, g) if out is None else out
    workspace, ws_bytes = _bwd_from_state_workspace(desc, workspace, q.device)
    st = lib().zeco_gla_bwd_from_state_varlen(ctypes.byref(desc), _ptr(seg_start), q.shape[1], _ptr(q), _ptr(k),
                                              _ptr(v), _ptr(g), _ptr(dO), _ptr(S_init), _ptr(S_last), _ptr(dS_in),
                                              _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dg), _ptr(workspace), ws_bytes,
                                              _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_gla_bwd_from_state_varlen")
    return dq, dk, dv, dg


def gla_fused_fwd_varlen(q, k, v, g, seg_start, max_len, scale=1.0, C=64, S0=None, out=None, workspace=None):
    """zeco_gla_fused_fwd_varlen: the whole forward over a table of unequal segments.  Returns (o, S_last)."""
    if not q.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    _check_same_layout(q, k)
    B, T, H, dk = q.shape
    desc = _varlen_desc(q, v, _dtype_code(g), _gate_per_head(q, g), seg_start, max_len, scale, C)
    if out is None:
        out = (torch.empty_strided(v.shape, v.stride(), dtype=v.dtype, device=v.device),
               torch.empty(B, H, dk, v.shape[-1], dtype=torch.float32, device=q.device))
    o, S_last = out
    need = int(lib().zeco_gla_fused_fwd_varlen_workspace(ctypes.byref(desc)))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    st = lib().zeco_gla_fused_fwd_varlen(ctypes.byref(desc), _ptr(seg_start), T, _ptr(q), _ptr(k), _ptr(v), _ptr(g),
                                         _ptr(S0), _ptr(o), _ptr(S_last), _ptr(workspace), workspace.numel(), _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_gla_fused_fwd_varlen")
    return o, S_last


def gla_fused_bwd_varlen(q, k, v, g, dO, seg_start, max_len, scale=1.0, C=64, S0=None, dS_T=None, out=None, workspace=None):
    """zeco_gla_fused_bwd_varlen: the whole backward over a table of unequal segments.
    Returns (dq, dk, dv, dg, dS0)."""
    if not q.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    _check_same_layout(q, k)
    _check_same_layout(v, dO)
    B, T, H, dk = q.shape
    desc = _varlen_desc(q, v, _dtype_code(g), _gate_per_head(q, g), seg_start, max_len, scale, C)
    if out is None:
        out = _grad_outputs(q, v, g) + (torch.empty(B, H, dk, v.shape[-1], dtype=torch.float32, device=q.device),)
    dq, dk_, dv, dg, dS0 = out
    need = int(lib().zeco_gla_fused_bwd_varlen_workspace(ctypes.byref(desc)))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    st = lib().zeco_gla_fused_bwd_varlen(ctypes.byref(desc), _ptr(seg_start), T, _ptr(q), _ptr(k), _ptr(v), _ptr(g),
                                         _ptr(dO), _ptr(S0), _ptr(dS_T), _ptr(dq), _ptr(dk_), _ptr(dv), _ptr(dg),
                                         _ptr(dS0), _ptr(workspace), workspace.numel(), _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_gla_fused_bwd_varlen")
    return dq, dk_, dv, dg, dS0


def _apply_flags(first_segment_is_zero, dense):
    return (APPLY_FIRST_SEGMENT_ZERO if first_segment_is_zero else 0) | (APPLY_DENSE if dense else 0)


def gla_local_fwd_chunk_decay(q, k, v, g, P, scale=1.0, C=64, out=None):
    """zeco_gla_local_fwd_chunk_decay: the local pass with the cumulative log decay kept per chunk.
    Returns (o, S_loc, G_chunk [B, P*ceil(L/C), H, d_k], G_tot)."""
    if not q.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    _check_same_layout(q, k)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    desc = make_desc(q, v, g, P, C, scale)
    if out is None:
        o = torch.empty_strided(v.shape, v.stride(), dtype=v.dtype, device=v.device)
        S_loc = torch.empty(P, B, H, dk, dv, dtype=torch.float32, device=q.device)
        G_chunk = torch.empty(B, P * -(-(T // P) // C), H, dk, dtype=torch.float32, device=q.device)
        G_tot = torch.empty(P, B, H, dk, dtype=torch.float32, device=q.device)
    else:
        o, S_loc, G_chunk, G_tot = out
        _check_same_layout(v, o)
    st = lib().zeco_gla_local_fwd_chunk_decay(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(g), _ptr(o),
                                              _ptr(S_loc), _ptr(G_chunk), _ptr(G_tot), _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_gla_local_fwd_chunk_decay")
    return o, S_loc, G_chunk, G_tot


def apply_init_state_chunk_decay(q, g, G_chunk, S_init, o, P, scale=1.0, C=64, first_segment_is_zero=True,
                                 dense=False):
    """zeco_apply_init_state_chunk_decay: the correction from g and the per-chunk cumulative log decay."""
    if not q.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    desc = make_desc(q, o, g, P, C, scale)
    st = lib().zeco_apply_init_state_chunk_decay(ctypes.byref(desc), _ptr(q), _ptr(g), _ptr(G_chunk),
                                                 _ptr(S_init), _ptr(o),
                                                 _apply_flags(first_segment_is_zero, dense), _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_apply_init_state_chunk_decay")
    return o


def gla_local_state(k, v, g, P, C=64, out=None):
    """zeco_gla_local_state (phase 1 of the two-phase forward).  Returns (S_loc, G_tot)."""
    if not k.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    B, T, H, dk = k.shape
    dv = v.shape[-1]
    desc = make_desc(k, v, g, P, C, 1.0)
    if out is None:
        S_loc = torch.empty(P, B, H, dk, dv, dtype=torch.float32, device=k.device)
        G_tot = torch.empty((P, B, H) + _gate_dims(g, dk), dtype=torch.float32, device=k.device)
    else:
        S_loc, G_tot = out
    st = lib().zeco_gla_local_state(ctypes.byref(desc), _ptr(k), _ptr(v), _ptr(g), _ptr(S_loc),
                                    _ptr(G_tot), _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_gla_local_state")
    return S_loc, G_tot


def gla_fwd_from_state(q, k, v, g, S_init, P, scale=1.0, C=64, out=None):
    """zeco_gla_fwd_from_state (phase 2): forward of each segment p started from S_init[p].  Returns o."""
    if not q.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    _check_same_layout(q, k)
    desc = make_desc(q, v, g, P, C, scale)
    o = torch.empty_strided(v.shape, v.stride(), dtype=v.dtype, device=v.device) if out is None else out
    st = lib().zeco_gla_fwd_from_state(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(g),
                                       _ptr(S_init), _ptr(o), _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_gla_fwd_from_state")
    return o


def fused_workspace_bytes(q, v, g, P, C=64):
    return int(lib().zeco_gla_fused_fwd_workspace(ctypes.byref(make_desc(q, v, g, P, C, 1.0))))


def saved_states_bytes(q, v, g, P, C=64):
    return int(lib().zeco_gla_saved_states_bytes(ctypes.byref(make_desc(q, v, g, P, C, 1.0))))


def gla_fused_fwd(q, k, v, g, P, scale=1.0, S0=None, C=64, out=None, workspace=None, want_last=True,
                  save=None, schedule=SCHEDULE_AUTO):
    """zeco_gla_fused_fwd: the whole forward in one call.  Returns (o, S_last).  `save`: a uint8
    tensor of saved_states_bytes() that receives the forward states for gla_fused_bwd(saved=...).
    schedule: SCHEDULE_AUTO, SCHEDULE_TWO_PHASE or SCHEDULE_CORRECT."""
    if not q.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    _check_same_layout(q, k)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    desc = make_desc(q, v, g, P, C, scale)
    L = lib()
    need = L.zeco_gla_fused_fwd_workspace(ctypes.byref(desc))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    if out is None:
        o = torch.empty_strided(v.shape, v.stride(), dtype=v.dtype, device=v.device)
        S_last = torch.empty(B, H, dk, dv, dtype=torch.float32, device=q.device) if want_last else None
    else:
        o, S_last = out
    if save is not None and save.numel() < L.zeco_gla_saved_states_bytes(ctypes.byref(desc)):
        raise ValueError("`save` is smaller than saved_states_bytes()")
    st = L.zeco_gla_fused_fwd(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(g), _ptr(S0), _ptr(o),
                              _ptr(S_last), _ptr(save), int(schedule), _ptr(workspace), workspace.numel(),
                              _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_gla_fused_fwd")
    return o, S_last


def gla_bwd_dstate(q, g, dO, P, scale=1.0, C=64, out=None):
    """zeco_gla_bwd_dstate: per segment, the state gradient it sends to the segment before it.
    Returns dS_loc [P,B,H,d_k,d_v]."""
    if not q.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    B, T, H, dk = q.shape
    dv = dO.shape[-1]
    desc = make_desc(q, dO, g, P, C, scale)
    dS_loc = torch.empty(P, B, H, dk, dv, dtype=torch.float32, device=q.device) if out is None else out
    st = lib().zeco_gla_bwd_dstate(ctypes.byref(desc), _ptr(q), _ptr(g), _ptr(dO), _ptr(dS_loc), _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_gla_bwd_dstate")
    return dS_loc


def _grad_outputs(q, v, g):
    dq = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    dk = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    dv = torch.empty_strided(v.shape, v.stride(), dtype=v.dtype, device=v.device)
    dg = torch.empty(g.shape, dtype=torch.float32, device=q.device)
    return dq, dk, dv, dg


def gla_bwd_from_state(q, k, v, g, dO, S_init, S_last, dS_in, P, scale=1.0, C=64, out=None, workspace=None):
    """zeco_gla_bwd_from_state: dq, dk, dv, dg of every segment from the scanned forward states and
    state gradients.  Returns (dq, dk, dv, dg)."""
    if not q.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    _check_same_layout(q, k)
    _check_same_layout(v, dO)
    desc = make_desc(q, v, g, P, C, scale)
    dq, dk, dv, dg = _grad_outputs(q, v, g) if out is None else out
    workspace, ws_bytes = _bwd_from_state_workspace(desc, workspace, q.device)
    st = lib().zeco_gla_bwd_from_state(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(g), _ptr(dO),
                                       _ptr(S_init), _ptr(S_last), _ptr(dS_in), _ptr(dq), _ptr(dk),
                                       _ptr(dv), _ptr(dg), _ptr(workspace), ws_bytes, _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_gla_bwd_from_state")
    return dq, dk, dv, dg


def fused_bwd_workspace_bytes(q, v, g, P, C=64):
    return int(lib().zeco_gla_fused_bwd_workspace(ctypes.byref(make_desc(q, v, g, P, C, 1.0))))


def gla_fused_bwd(q, k, v, g, dO, P, scale=1.0, S0=None, dS_T=None, C=64, out=None, workspace=None,
                  want_dS0=True, saved=None):
    """zeco_gla_fused_bwd: the whole backward in one call.  Returns (dq, dk, dv, dg, dS0)."""
    if not q.is_cuda:
        raise RuntimeError("zeco kernels run on the GPU only")
    _check_same_layout(q, k)
    _check_same_layout(v, dO)
    B, T, H, dk_ = q.shape
    dv_ = v.shape[-1]
    desc = make_desc(q, v, g, P, C, scale)
    L = lib()
    need = L.zeco_gla_fused_bwd_workspace(ctypes.byref(desc))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    if out is None:
        dq, dk, dv, dg = _grad_outputs(q, v, g)
        dS0 = torch.empty(B, H, dk_, dv_, dtype=torch.float32, device=q.device) if want_dS0 else None
    else:
        dq, dk, dv, dg, dS0 = out
    st = L.zeco_gla_fused_bwd(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(g), _ptr(dO), _ptr(S0),
                              _ptr(dS_T), _ptr(saved), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dg), _ptr(dS0),
                              _ptr(workspace), workspace.numel(), _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_gla_fused_bwd")
    return dq, dk, dv, dg, dS0


def hbm_copy(dst, src):
    """zeco_hbm_copy: plain device copy used for bandwidth / counter calibration."""
    if not (dst.is_cuda and src.is_cuda and dst.is_contiguous() and src.is_contiguous()):
        raise RuntimeError("hbm_copy needs contiguous GPU tensors")
    nbytes = src.numel() * src.element_size()
    if nbytes != dst.numel() * dst.element_size():
        raise ValueError("size mismatch")
    st = lib().zeco_hbm_copy(_ptr(dst), _ptr(src), nbytes, _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_hbm_copy")
    return dst


def hbm_mix(dst, src, slice_bytes, reads, writes):
    """zeco_hbm_mix: `reads` x `writes` streams of slice_bytes each (bandwidth calibration for a traffic mix)."""
    if src.numel() * src.element_size() < reads * slice_bytes or dst.numel() * dst.element_size() < max(16, writes * slice_bytes):
        raise ValueError("buffers too small for the mix")
    st = lib().zeco_hbm_mix(_ptr(dst), _ptr(src), int(slice_bytes), int(reads), int(writes), _stream())
    if st != ZECO_OK:
        raise ZecoError(st, "zeco_hbm_mix")


def segmented_fwd(q, k, v, g, P, scale=1.0, S0=None, K_blocks=16, C=64):
    """Local pass, segment-state scan and correction chained.  Returns (o, S_last, parts) with
    parts = dict(S_loc, G_cum, G_tot, S_init)."""
    o, S_loc, G_cum, G_tot = gla_local_fwd(q, k, v, g, P, scale, C=C)
    S_init, S_last = state_scan(S_loc, G_tot, S0=S0, K_blocks=K_blocks)
    apply_init_state(q, g, G_cum, S_init, o, P, scale, C=C, first_segment_is_zero=S0 is None)
    return o, S_last, dict(S_loc=S_loc, G_cum=G_cum, G_tot=G_tot, S_init=S_init)
