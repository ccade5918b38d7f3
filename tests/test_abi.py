"""C-ABI checks that need no GPU: the library loads, exports every symbol the header declares,
and rejects bad arguments with a status code before touching the HIP runtime."""
import ctypes
import os
import re

import pytest

from paper_2507_01004_amd import zeco

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(zeco.LIB_PATH):
        from paper_2507_01004_amd.build import build_lib
        build_lib()
    return zeco.lib()


def header_functions():
    text = open(os.path.join(ROOT, "include", "zeco.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(zeco_[a-z_]+)\s*\(", text)))


def test_exports_match_header(L):
    names = header_functions()
    assert set(names) == set(zeco.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_version_and_strings(L):
    assert zeco.version() >= 100
    assert zeco.status_string(zeco.ZECO_OK) == "ok"
    for s in range(1, 6):
        assert zeco.status_string(s) not in ("ok", "unknown status")
    assert zeco.status_string(99) == "unknown status"


def good_desc(**kw):
    d = dict(B=1, P=2, H=2, L=128, d_k=128, d_v=128, C=64, io_dtype=zeco.ZECO_BF16,
             g_dtype=zeco.ZECO_F32, scale=1.0, stride_b=2 * 256 * 128 * 2, stride_t=256, stride_h=128,
             vstride_b=2 * 256 * 128 * 2, vstride_t=256, vstride_h=128, g_per_head=0, wide_gates=0)
    d.update(kw)
    return zeco.GlaDesc(*[d[f[0]] for f in zeco.GlaDesc._fields_])


FAKE = ctypes.c_void_p(0x1000)   # aligned, never dereferenced: validation fails first


def call_local(L, desc, q=FAKE, o=FAKE, ws_bytes=0):
    return L.zeco_gla_local_fwd(ctypes.byref(desc), q, FAKE, FAKE, FAKE, o, FAKE, FAKE, FAKE, None,
                                ws_bytes, None)


@pytest.mark.parametrize("kw,expect", [
    (dict(B=-1), zeco.ZECO_ERR_INVALID_ARG),
    (dict(wide_gates=2), zeco.ZECO_ERR_INVALID_ARG),
    (dict(P=0), zeco.ZECO_ERR_INVALID_ARG),
    (dict(L=(1 << 30) + 64, P=1, stride_b=1 << 44), zeco.ZECO_ERR_INVALID_ARG),   # beyond the length limit
    (dict(L=40), zeco.ZECO_ERR_UNSUPPORTED),           # shorter than a chunk
    (dict(stride_t=100), zeco.ZECO_ERR_INVALID_ARG),   # stride not a multiple of 8
    (dict(stride_t=(1 << 24) + 8, stride_b=1 << 40), zeco.ZECO_ERR_UNSUPPORTED),   # token stride beyond 2^24 elements
    (dict(stride_h=64), zeco.ZECO_ERR_INVALID_ARG),    # heads overlap
    (dict(io_dtype=7), zeco.ZECO_ERR_INVALID_ARG),
    (dict(scale=float("nan")), zeco.ZECO_ERR_INVALID_ARG),
    (dict(C=32, L=128), zeco.ZECO_ERR_UNSUPPORTED),
    (dict(d_k=96, stride_h=96), zeco.ZECO_ERR_UNSUPPORTED),
    (dict(io_dtype=zeco.ZECO_F32, g_dtype=zeco.ZECO_BF16), zeco.ZECO_ERR_UNSUPPORTED),
    (dict(g_per_head=2), zeco.ZECO_ERR_INVALID_ARG),
    (dict(g_per_head=1, g_dtype=zeco.ZECO_BF16), zeco.ZECO_ERR_UNSUPPORTED),   # per-head gates are fp32
    (dict(g_per_head=1, io_dtype=zeco.ZECO_F32), zeco.ZECO_ERR_UNSUPPORTED),
])
def test_local_fwd_rejects_bad_descriptors(L, kw, expect):
    assert call_local(L, good_desc(**kw)) == expect
    assert L.zeco_apply_init_state(ctypes.byref(good_desc(**kw)), FAKE, FAKE, FAKE, FAKE, 1, None) == expect


def test_segment_lengths_that_are_no_multiple_of_the_chunk(L):
    """The entry points take them (validation gets past the descriptor: the next check, a null pointer,
    answers), saved states included."""
    d, ref = good_desc(L=100), ctypes.byref
    assert call_local(L, d, q=None) == zeco.ZECO_ERR_INVALID_ARG
    assert L.zeco_apply_init_state(ref(d), None, FAKE, FAKE, FAKE, 1, None) == zeco.ZECO_ERR_INVALID_ARG
    assert L.zeco_gla_local_fwd_chunk_decay(ref(d), None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None) == zeco.ZECO_ERR_INVALID_ARG
    assert L.zeco_gla_fused_fwd_workspace(ref(d)) > 0
    assert L.zeco_gla_fused_bwd_workspace(ref(d)) > 0 and L.zeco_gla_saved_states_bytes(ref(d)) > 0
    assert L.zeco_gla_bwd_dstate(ref(d), None, FAKE, FAKE, FAKE, None) == zeco.ZECO_ERR_INVALID_ARG
    fwd = [None] + [FAKE] * 3 + [None, FAKE, None]
    assert L.zeco_gla_fused_fwd(ref(d), *fwd, FAKE, 0, FAKE, 1 << 30, None) == zeco.ZECO_ERR_INVALID_ARG   # with S_save
    fused = [FAKE] * 5 + [None, None, FAKE] + [FAKE] * 4 + [None, FAKE]
    fused[0] = None
    assert L.zeco_gla_fused_bwd(ref(d), *fused, 1 << 30, None) == zeco.ZECO_ERR_INVALID_ARG


def test_an_empty_batch_is_a_valid_no_op(L):
    """B = 0: every entry point returns ZECO_OK before it looks at a pointer (all null here, no GPU needed)."""
    d, ref, N = good_desc(B=0), ctypes.byref, None
    assert L.zeco_gla_local_fwd(ref(d), N, N, N, N, N, N, N, N, N, 0, N) == zeco.ZECO_OK
    assert L.zeco_apply_init_state(ref(d), N, N, N, N, 0, N) == zeco.ZECO_OK
    assert L.zeco_state_scan(4, 0, 128, 128, 16, N, N, N, N, N, 0, 0, N) == zeco.ZECO_OK
    assert L.zeco_gla_local_fwd_chunk_decay(ref(d), N, N, N, N, N, N, N, N, N) == zeco.ZECO_OK
    assert L.zeco_apply_init_state_chunk_decay(ref(d), N, N, N, N, N, 0, N) == zeco.ZECO_OK
    assert L.zeco_gla_local_state(ref(d), N, N, N, N, N, N) == zeco.ZECO_OK
    assert L.zeco_gla_fwd_from_state(ref(d), N, N, N, N, N, N, N) == zeco.ZECO_OK
    assert L.zeco_gla_fused_fwd(ref(d), N, N, N, N, N, N, N, N, 0, N, 0, N) == zeco.ZECO_OK
    assert L.zeco_gla_bwd_dstate(ref(d), N, N, N, N, N) == zeco.ZECO_OK
    assert L.zeco_gla_bwd_from_state(ref(d), *([N] * 12), N, 0, N) == zeco.ZECO_OK
    assert L.zeco_gla_fused_bwd(ref(d), *([N] * 14), 0, N) == zeco.ZECO_OK
    assert L.zeco_gla_fused_fwd_workspace(ref(d)) == 0 and L.zeco_gla_local_fwd_workspace(ref(d)) == 0


def test_state_scan_tree_validates_and_sizes_its_workspace(L):
    ws = L.zeco_state_scan_tree_workspace
    assert ws(36, 2, 128, 128, 0) == (2 * 9 * 2 * 128 * 128 + 9 * 2 * 128) * 4      # groups of 4: 2*4 + 9 = 17 < 36
    assert ws(36, 2, 128, 128, 1) == (2 * 9 * 2 * 128 * 128 + 9 * 2) * 4
    assert ws(37, 2, 128, 128, 0) == 0 and ws(4, 2, 128, 128, 0) == 0 and ws(0, 2, 128, 128, 0) == 0
    tree = lambda P=36, ws_bytes=1 << 30, S_loc=FAKE, w=FAKE, direction=0: L.zeco_state_scan_tree(
        P, 2, 128, 128, S_loc, FAKE, None, FAKE, None, direction, 0, w, ws_bytes, None)
    assert tree(ws_bytes=16) == zeco.ZECO_ERR_WORKSPACE
    assert tree(S_loc=None) == zeco.ZECO_ERR_INVALID_ARG
    assert tree(w=None) == zeco.ZECO_ERR_INVALID_ARG
    assert tree(direction=2) == zeco.ZECO_ERR_INVALID_ARG
    assert tree(P=0) == zeco.ZECO_ERR_INVALID_ARG
    assert tree(P=37, S_loc=None, w=None, ws_bytes=0) == zeco.ZECO_ERR_INVALID_ARG     # the serial path's own check


def test_apply_init_state_rejects_unknown_flags(L):
    assert L.zeco_apply_init_state(ctypes.byref(good_desc()), FAKE, FAKE, FAKE, FAKE, 4, None) == zeco.ZECO_ERR_INVALID_ARG
    assert L.zeco_apply_init_state(ctypes.byref(good_desc()), None, FAKE, FAKE, FAKE, 3, None) == zeco.ZECO_ERR_INVALID_ARG


def test_unequal_segment_lengths_validate_before_any_launch(L):
    """The six entry points over a table of segment offsets: descriptor, T and the table's pointer."""
    ref = ctypes.byref
    loc = lambda d=None, seg=FAKE, T=4096, q=FAKE: L.zeco_gla_local_fwd_varlen(
        ref(d or good_desc(L=1000)), seg, T, q, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None)
    app = lambda d=None, seg=FAKE, T=4096, q=FAKE, flags=0: L.zeco_apply_init_state_varlen(
        ref(d or good_desc(L=1000)), seg, T, q, FAKE, FAKE, FAKE, flags, None)
    sta = lambda d=None, seg=FAKE, T=4096, q=FAKE: L.zeco_gla_local_state_varlen(
        ref(d or good_desc(L=1000)), seg, T, q, FAKE, FAKE, FAKE, FAKE, None)
    out = lambda d=None, seg=FAKE, T=4096, q=FAKE: L.zeco_gla_fwd_from_state_varlen(
        ref(d or good_desc(L=1000)), seg, T, q, FAKE, FAKE, FAKE, FAKE, FAKE, None)
    dst = lambda d=None, seg=FAKE, T=4096, q=FAKE: L.zeco_gla_bwd_dstate_varlen(
        ref(d or good_desc(L=1000)), seg, T, q, FAKE, FAKE, FAKE, None)
    bwd = lambda d=None, seg=FAKE, T=4096, q=FAKE: L.zeco_gla_bwd_from_state_varlen(
        ref(d or good_desc(L=1000)), seg, T, q, *([FAKE] * 11), FAKE, 1 << 30, None)
    ffw = lambda d=None, seg=FAKE, T=4096, q=FAKE, ws=1 << 30: L.zeco_gla_fused_fwd_varlen(
        ref(d or good_desc(L=1000)), seg, T, q, FAKE, FAKE, FAKE, None, FAKE, None, FAKE, ws, None)
    fbw = lambda d=None, seg=FAKE, T=4096, q=FAKE, ws=1 << 30: L.zeco_gla_fused_bwd_varlen(
        ref(d or good_desc(L=1000)), seg, T, q, *([FAKE] * 4), None, None, *([FAKE] * 4), None, FAKE, ws, None)
    need_f = L.zeco_gla_fused_fwd_varlen_workspace(ref(good_desc(L=1000)))
    need_b = L.zeco_gla_fused_bwd_varlen_workspace(ref(good_desc(L=1000)))
    assert 0 < need_f < need_b
    assert L.zeco_gla_fused_bwd_varlen_workspace(ref(good_desc(L=1000, io_dtype=zeco.ZECO_F32))) == need_b   # fp32 too
    assert ffw(ws=need_f - 1) == zeco.ZECO_ERR_WORKSPACE and fbw(ws=need_b - 1) == zeco.ZECO_ERR_WORKSPACE
    for call in (loc, app, sta, out, dst, bwd, ffw, fbw):
        assert call(seg=None) == zeco.ZECO_ERR_INVALID_ARG
        assert call(seg=ctypes.c_void_p(0x1004)) == zeco.ZECO_ERR_INVALID_ARG        # not 8-byte aligned
        assert call(T=127) == zeco.ZECO_ERR_INVALID_ARG                             # under P * C tokens
        assert call(T=(1 << 40) + 1) == zeco.ZECO_ERR_INVALID_ARG
        assert call(q=None) == zeco.ZECO_ERR_INVALID_ARG
        assert call(q=ctypes.c_void_p(0x1008)) == zeco.ZECO_ERR_INVALID_ARG
        assert call(d=good_desc(L=48)) == zeco.ZECO_ERR_UNSUPPORTED                  # bound under one chunk
        assert call(d=good_desc(io_dtype=zeco.ZECO_F32, g_dtype=zeco.ZECO_BF16)) == zeco.ZECO_ERR_UNSUPPORTED
        assert call(d=good_desc(B=0), seg=None, q=None) == zeco.ZECO_OK              # empty batch
    assert app(flags=4) == zeco.ZECO_ERR_INVALID_ARG


def test_local_fwd_rejects_bad_pointers(L):
    assert call_local(L, good_desc(), q=None) == zeco.ZECO_ERR_INVALID_ARG
    assert call_local(L, good_desc(), o=ctypes.c_void_p(0x1004)) == zeco.ZECO_ERR_INVALID_ARG
    assert L.zeco_gla_local_fwd(None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, 0,
                                None) == zeco.ZECO_ERR_INVALID_ARG
    assert L.zeco_gla_local_fwd_workspace(None) == 0


def test_state_scan_rejects_bad_arguments(L):
    def scan(P=4, BH=2, dk=128, dv=128, K=8, S_loc=FAKE, G=FAKE, S0=None, S_init=FAKE, S_last=None, d=0):
        return L.zeco_state_scan(P, BH, dk, dv, K, S_loc, G, S0, S_init, S_last, d, 0, None)
    assert scan(P=0) == zeco.ZECO_ERR_INVALID_ARG
    assert scan(K=3) == zeco.ZECO_ERR_INVALID_ARG          # does not divide d_k
    assert scan(S_loc=None) == zeco.ZECO_ERR_INVALID_ARG
    assert scan(S_init=ctypes.c_void_p(0x1008)) == zeco.ZECO_ERR_INVALID_ARG
    assert scan(d=2) == zeco.ZECO_ERR_INVALID_ARG
    assert scan(dv=126) == zeco.ZECO_ERR_UNSUPPORTED


def test_binding_refuses_cpu_tensors():
    import torch
    q = torch.zeros(1, 64, 1, 64)
    with pytest.raises(RuntimeError):
        zeco.gla_local_fwd(q, q, q, q, 1)
    with pytest.raises(RuntimeError):
        zeco.state_scan(torch.zeros(1, 1, 64, 64), torch.zeros(1, 1, 64))


def test_backward_entry_points_reject_bad_arguments(L):
    d = good_desc()
    f32 = good_desc(io_dtype=zeco.ZECO_F32)
    ref = ctypes.byref
    assert L.zeco_gla_bwd_dstate(ref(d), None, FAKE, FAKE, FAKE, None) == zeco.ZECO_ERR_INVALID_ARG
    assert L.zeco_gla_bwd_dstate(ref(f32), None, FAKE, FAKE, FAKE, None) == zeco.ZECO_ERR_INVALID_ARG   # fp32 is taken
    assert L.zeco_gla_bwd_dstate(ref(good_desc(L=40)), FAKE, FAKE, FAKE, FAKE, None) == zeco.ZECO_ERR_UNSUPPORTED   # shorter than a chunk
    args = [FAKE] * 12
    args[7] = None                                         # dS_in missing
    assert L.zeco_gla_bwd_from_state(ref(d), *args, None, 0, None) == zeco.ZECO_ERR_INVALID_ARG
    assert L.zeco_gla_bwd_from_state(ref(f32), *args, None, 0, None) == zeco.ZECO_ERR_INVALID_ARG
    # checkpoints of the forward state that re-anchor dG: one per 512 tokens inside a segment, none up to 512
    wsz = L.zeco_gla_bwd_from_state_workspace
    assert wsz(ref(d)) == 0 and wsz(ref(good_desc(L=512))) == 0 and wsz(ref(f32)) == 0
    assert wsz(ref(good_desc(L=513, io_dtype=zeco.ZECO_F32, C=16))) == 1 * 2 * 2 * 1 * 128 * 128 * 4   # whatever C
    long = good_desc(L=16384)
    assert wsz(ref(long)) == 1 * 2 * 2 * 31 * 128 * 128 * 4
    assert wsz(ref(good_desc(L=513))) == 1 * 2 * 2 * 1 * 128 * 128 * 4
    args = [FAKE] * 12
    assert L.zeco_gla_bwd_from_state(ref(long), *args, FAKE, wsz(ref(long)) - 1, None) == zeco.ZECO_ERR_WORKSPACE
    assert L.zeco_gla_bwd_from_state(ref(long), *args, None, wsz(ref(long)), None) == zeco.ZECO_ERR_INVALID_ARG
    need = L.zeco_gla_fused_bwd_workspace(ref(d))
    assert need > 0 and L.zeco_gla_fused_bwd_workspace(ref(f32)) == need
    fused = [FAKE] * 5 + [None, None, None] + [FAKE] * 4 + [None, FAKE]
    assert L.zeco_gla_fused_bwd(ref(d), *fused, need - 1, None) == zeco.ZECO_ERR_WORKSPACE
    assert L.zeco_gla_fused_bwd(ref(f32), *fused, need - 1, None) == zeco.ZECO_ERR_WORKSPACE
    saved = list(fused)
    saved[7] = FAKE                                        # the fp32 forward saves no states to start from
    assert L.zeco_gla_fused_bwd(ref(f32), *saved, need, None) == zeco.ZECO_ERR_UNSUPPORTED
    fused[0] = ctypes.c_void_p(0x1004)
    assert L.zeco_gla_fused_bwd(ref(d), *fused, need, None) == zeco.ZECO_ERR_INVALID_ARG


def test_chunk_decay_and_fused_forward_reject_bad_arguments(L):
    d = good_desc()
    f32 = good_desc(io_dtype=zeco.ZECO_F32)
    head = good_desc(g_per_head=1)
    ref = ctypes.byref
    loc = [FAKE] * 9
    assert L.zeco_gla_local_fwd_chunk_decay(ref(f32), *loc, None) == zeco.ZECO_ERR_UNSUPPORTED
    assert L.zeco_gla_local_fwd_chunk_decay(ref(head), *loc, None) == zeco.ZECO_ERR_UNSUPPORTED
    loc[6] = None                                          # G_chunk missing
    assert L.zeco_gla_local_fwd_chunk_decay(ref(d), *loc, None) == zeco.ZECO_ERR_INVALID_ARG
    app = [FAKE] * 5
    assert L.zeco_apply_init_state_chunk_decay(ref(d), *app, 8, None) == zeco.ZECO_ERR_INVALID_ARG
    assert L.zeco_apply_init_state_chunk_decay(ref(head), *app, 0, None) == zeco.ZECO_ERR_UNSUPPORTED
    app[1] = ctypes.c_void_p(0x1008)                       # g misaligned
    assert L.zeco_apply_init_state_chunk_decay(ref(d), *app, 0, None) == zeco.ZECO_ERR_INVALID_ARG
    need = L.zeco_gla_fused_fwd_workspace(ref(d))
    assert need > 0
    # q, k, v, g, S0, o, S_last, S_save, schedule, workspace, bytes, stream
    fused = [FAKE, FAKE, FAKE, FAKE, None, FAKE, None, None]
    assert L.zeco_gla_fused_fwd(ref(d), *fused, 7, FAKE, need, None) == zeco.ZECO_ERR_INVALID_ARG
    assert L.zeco_gla_fused_fwd(ref(d), *fused, zeco.SCHEDULE_CORRECT, FAKE, need - 1, None) == zeco.ZECO_ERR_WORKSPACE
    f32 = good_desc(io_dtype=zeco.ZECO_F32)                # fp32: two phases only, no saved states
    assert L.zeco_gla_fused_fwd(ref(f32), *fused, zeco.SCHEDULE_CORRECT, FAKE, 1 << 30, None) == zeco.ZECO_ERR_UNSUPPORTED
    fused[7] = FAKE
    assert L.zeco_gla_fused_fwd(ref(f32), *fused, zeco.SCHEDULE_TWO_PHASE, FAKE, 1 << 30, None) == zeco.ZECO_ERR_UNSUPPORTED


def test_a_missing_library_raises_instead_of_falling_back(monkeypatch):
    """The binding has no other path: without libzeco.so every call fails with a message that says how to build it."""
    monkeypatch.setattr(zeco, "_lib", None)
    monkeypatch.setattr(zeco, "LIB_PATH", os.path.join(os.path.dirname(zeco.LIB_PATH), "no_such_libzeco.so"))
    with pytest.raises(RuntimeError, match="not built"):
        zeco.lib()
    with pytest.raises(RuntimeError, match="not built"):
        zeco.version()


def test_static_scratch_scan_checks_its_limit_before_any_hip_call(L):
    """zeco_state_scan_tree_static: the limit is the stated 33 MiB; a problem whose group states do not fit
    is refused with its own status, with no pointer read and no HIP call made."""
    limit = L.zeco_state_scan_tree_static_limit()
    assert limit == 33 << 20
    call = lambda P, BH, S_loc=FAKE: L.zeco_state_scan_tree_static(P, BH, 128, 128, S_loc, FAKE, None, FAKE, None, 0, 0, None)
    assert L.zeco_state_scan_tree_workspace(1024, 4, 128, 128, 0) <= limit      # the largest case it is meant for
    assert L.zeco_state_scan_tree_workspace(1024, 8, 128, 128, 0) > limit
    assert call(1024, 8) == zeco.ZECO_ERR_SCRATCH_LIMIT
    assert call(1024, 8, S_loc=None) == zeco.ZECO_ERR_SCRATCH_LIMIT             # the size check comes first
    assert call(36, 2, S_loc=None) == zeco.ZECO_ERR_INVALID_ARG
    assert call(0, 2) == zeco.ZECO_ERR_INVALID_ARG
    assert call(37, 0) == zeco.ZECO_OK                                          # empty batch


def test_hbm_mix_takes_only_the_mixes_it_was_built_for(L):
    assert L.zeco_hbm_mix(FAKE, FAKE, 1 << 20, 7, 1, None) == zeco.ZECO_ERR_UNSUPPORTED
    assert L.zeco_hbm_mix(FAKE, FAKE, 1 << 20, 0, 0, None) == zeco.ZECO_ERR_UNSUPPORTED
    assert L.zeco_hbm_mix(None, FAKE, 1 << 20, 4, 1, None) == zeco.ZECO_ERR_INVALID_ARG
    assert L.zeco_hbm_mix(FAKE, FAKE, 24, 4, 1, None) == zeco.ZECO_ERR_INVALID_ARG


def test_chunk_length_per_precision(L):
    """C = 64 for bf16 q/k/v; the fp32 kernel also has 16 and 32.  Segments shorter than 64 tokens are refused
    whatever the chunk length (the correction works on windows of 64 tokens)."""
    ref = ctypes.byref
    f32 = lambda **kw: good_desc(io_dtype=zeco.ZECO_F32, **kw)
    ws = L.zeco_gla_fused_fwd_workspace
    assert ws(ref(f32())) > 0 and ws(ref(f32(C=16))) > 0 and ws(ref(f32(C=32))) > 0
    assert ws(ref(f32(C=48))) == 0 and ws(ref(f32(C=128))) == 0 and ws(ref(good_desc(C=32))) == 0
    assert call_local(L, good_desc(C=32)) == zeco.ZECO_ERR_UNSUPPORTED
    assert call_local(L, f32(C=8)) == zeco.ZECO_ERR_UNSUPPORTED
    assert call_local(L, f32(C=16, L=48)) == zeco.ZECO_ERR_UNSUPPORTED
    assert call_local(L, f32(C=16, L=80), q=None) == zeco.ZECO_ERR_INVALID_ARG      # the descriptor itself is fine
