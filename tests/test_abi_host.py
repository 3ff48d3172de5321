"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
function include/energon.h declares, and rejects bad arguments before touching a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2209_02341_amd import binding as E

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # non-NULL, 256-byte aligned; never dereferenced because validation fails first


def declared_functions():
    text = open(os.path.join(ROOT, "include", "energon.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(energon_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"energon_pack", "energon_unpack", "energon_layer_forward"} <= set(names)
    lib = E.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_strerror():
    assert E.strerror(0) == "ok"
    for code in range(-7, 0):
        assert E.strerror(code) not in ("ok", "unknown status")
    assert E.strerror(-99) == "unknown status"


def cfg(**kw):
    base = dict(hidden=1024, n_heads=16, head_dim=64, ffn=4096, ln_eps=1e-5, dtype=E.BF16)
    base.update(kw)
    return E.LayerConfig(**base)


def test_workspace_sizes():
    c = cfg()
    assert E.energon_workspace_bytes(c, 0) > 0
    T = 577
    need = sum(T * n * 2 for n in (1024, 3072, 1024, 1024, 1024, 4096))
    got = E.energon_workspace_bytes(c, T)
    assert need <= got <= need + 6 * 256
    off = E.energon_workspace_layout(c, T)
    assert off[0] == 0 and all(o % 256 == 0 for o in off) and off == sorted(off)
    assert off[E.WS_QKV] >= T * 1024 * 2
    assert E.energon_workspace_bytes(cfg(head_dim=96, n_heads=8), 10) == 0
    assert E.energon_workspace_bytes(cfg(hidden=1000), 10) == 0
    assert E.energon_workspace_bytes(c, -1) == 0
    assert E.energon_workspace_bytes(cfg(dtype=E.F32, hidden=260, n_heads=1, ffn=8), 3) > 0


def pack_status(lengths, B=2, S=4, H=64, dt=E.BF16, x=FAKE, xp=FAKE, cap=8, cu=FAKE, idx=FAKE):
    lens = np.asarray(lengths, dtype=np.int32)
    tot = C.c_int64(-5)
    st = E.lib().energon_pack(x, lens.ctypes.data, B, S, H, dt, xp, cap, cu, idx, C.byref(tot), None)
    assert tot.value == -5      # never written on failure
    return st


def test_pack_rejects_bad_arguments_before_any_launch():
    assert pack_status([1, 2], x=None) == -1
    assert pack_status([1, 2], cu=None) == -1
    assert pack_status([1, 2], dt=7) == -6
    assert pack_status([1, 2], H=60) == -2
    assert pack_status([1, 2], B=0) == -2
    assert pack_status([1, 5]) == -3
    assert pack_status([-1, 2]) == -3
    assert pack_status([4, 4], cap=7) == -4
    assert pack_status([1, 2], x=FAKE + 8) == -5
    assert pack_status([1, 2], B=2, S=1 << 30) == -2


def test_unpack_rejects_bad_arguments():
    f = E.lib().energon_unpack
    assert f(None, FAKE, 3, 2, 4, 64, E.BF16, FAKE, None) == -1
    assert f(FAKE, FAKE, 9, 2, 4, 64, E.BF16, FAKE, None) == -2
    assert f(FAKE, FAKE, 3, 2, 4, 63, E.F32, FAKE, None) == -2
    assert f(FAKE, FAKE, 3, 2, 4, 64, 5, FAKE, None) == -6
    assert f(FAKE, FAKE + 4, 3, 2, 4, 64, E.BF16, FAKE + 2, None) == -5


def layer_status(c=None, w=None, lengths=(3, 2), T=5, max_len=4, x=FAKE, y=FAKE, cu=FAKE, ws=FAKE, ws_bytes=1 << 30):
    c = c or cfg()
    if w is None:
        w = E.LayerWeights(*([FAKE] * 12))
    lens = np.asarray(lengths, dtype=np.int32)
    return E.lib().energon_layer_forward(C.byref(c), C.byref(w), x, y, T, cu, lens.ctypes.data, len(lens), max_len,
                                         ws, ws_bytes, None)


def test_layer_forward_rejects_bad_arguments():
    assert layer_status(x=None) == -1
    w = E.LayerWeights(*([FAKE] * 12)); w.w_fc1 = None
    assert layer_status(w=w) == -1
    assert layer_status(c=cfg(head_dim=80, n_heads=16)) == -6
    assert layer_status(c=cfg(dtype=3)) == -6
    assert layer_status(c=cfg(ffn=4100)) == -2
    assert layer_status(c=cfg(hidden=0)) == -2
    assert layer_status(T=6) == -3                 # lengths do not sum to T
    assert layer_status(lengths=(5, 0)) == -3      # longer than max_len
    assert layer_status(ws_bytes=1024) == -4
    # limits of the kernels behind the call: a LayerNorm row must fit one workgroup's registers,
    # a contraction addresses a tile's rows with 32-bit byte offsets
    assert layer_status(c=cfg(hidden=32768 + 64, n_heads=513, head_dim=64)) == -6
    assert layer_status(c=cfg(dtype=E.F32, hidden=16384 + 64, n_heads=257, head_dim=64)) == -6
    assert layer_status(c=cfg(ffn=1 << 24)) == -6
    assert layer_status(c=cfg(n_heads=1 << 18, head_dim=64, hidden=1024)) == -6
    assert layer_status(ws=FAKE + 16) == -5
    assert layer_status(y=FAKE + 2) == -5
    st = E.lib().energon_layer_forward_profiled
    c, w = cfg(), E.LayerWeights(*([FAKE] * 12))
    lens = np.asarray([3, 2], dtype=np.int32)
    assert st(C.byref(c), C.byref(w), FAKE, FAKE, 5, FAKE, lens.ctypes.data, 2, 4, FAKE, 1 << 30, None, None) == -1


def test_stage_entry_points_reject_bad_arguments():
    l = E.lib()
    assert l.energon_layernorm(FAKE, FAKE, None, FAKE, 4, 64, 1e-5, E.BF16, None) == -1
    assert l.energon_layernorm(FAKE, FAKE, FAKE, FAKE, 4, 62, 1e-5, E.BF16, None) == -2
    assert l.energon_layernorm(FAKE, FAKE, FAKE, FAKE, 4, 1 << 20, 1e-5, E.BF16, None) == -6
    assert l.energon_linear(FAKE, FAKE, None, None, FAKE, 4, 64, 64, E.EPI_BIAS_RESIDUAL, E.BF16, None) == -1
    assert l.energon_linear(FAKE, FAKE, None, None, FAKE, 4, 64, 96, E.EPI_BIAS, E.BF16, None) == -2
    assert l.energon_linear(FAKE, FAKE, None, None, FAKE, 4, 64, 64, 9, E.BF16, None) == -6
    assert l.energon_linear(FAKE, FAKE, None, None, FAKE, 4, 64, 1 << 24, E.EPI_BIAS, E.BF16, None) == -6
    assert l.energon_linear(FAKE, FAKE, FAKE + 2, None, FAKE, 4, 64, 64, E.EPI_BIAS, E.BF16, None) == -5
    assert l.energon_attention(FAKE, FAKE, FAKE, 5, 2, 4, 2, 32, E.BF16, None) == -6
    assert l.energon_attention(FAKE, None, FAKE, 5, 2, 4, 2, 64, E.BF16, None) == -1
    assert l.energon_attention(FAKE, FAKE, FAKE, 5, 0, 4, 2, 64, E.BF16, None) == -2
    assert l.energon_attention(FAKE, FAKE, FAKE, 0, 2, 4, 2, 64, E.BF16, None) == 0   # T = 0: nothing to do


def test_padded_attention_path_entry_points_reject_bad_arguments():
    l = E.lib()
    assert l.energon_rebuild_qkv(FAKE, FAKE, 5, 2, 4, 2, 64, E.BF16, FAKE, FAKE, None, None) == -1
    assert l.energon_rebuild_qkv(FAKE, FAKE, 5, 2, 4, 2, 64, E.F32, FAKE, FAKE, FAKE, None) == -6
    assert l.energon_rebuild_qkv(FAKE, FAKE, 5, 2, 4, 2, 96, E.BF16, FAKE, FAKE, FAKE, None) == -6
    assert l.energon_rebuild_qkv(FAKE, FAKE, 9, 2, 4, 2, 64, E.BF16, FAKE, FAKE, FAKE, None) == -2   # T > B*S
    assert l.energon_rebuild_qkv(FAKE, FAKE, 5, 2, 4, 2, 64, E.BF16, FAKE + 8, FAKE, FAKE, None) == -5
    assert l.energon_attention_padded(FAKE, FAKE, FAKE, None, 2, 4, 2, 64, E.BF16, FAKE, None) == -1
    assert l.energon_attention_padded(FAKE, FAKE, FAKE, FAKE, 2, 0, 2, 64, E.BF16, FAKE, None) == -2
    assert l.energon_remove_attn_padding(FAKE, FAKE, 5, 2, 4, 2, 64, E.BF16, None, None) == -1
    assert l.energon_remove_attn_padding(FAKE, FAKE, 0, 2, 4, 2, 64, E.BF16, FAKE, None) == 0   # T = 0: nothing to do
    c = cfg()
    assert E.energon_drce_workspace_bytes(c, 2, 4) == 4 * 2 * 4 * c.n_heads * c.head_dim * 2
    assert E.energon_drce_workspace_bytes(c, 0, 4) == 0
    w = E.LayerWeights(*([FAKE] * 12))
    lens = np.asarray([3, 2], dtype=np.int32)
    f = l.energon_layer_forward_drce
    args = (C.byref(c), C.byref(w), FAKE, FAKE, 5, FAKE, lens.ctypes.data, 2, 4, FAKE, 1 << 30)
    assert f(*args, None, 1 << 30, None, None) == -1
    assert f(*args, FAKE, 16, None, None) == -4
    assert f(*args, FAKE + 16, 1 << 30, None, None) == -5


def test_ln_folded_entry_points_reject_bad_arguments():
    l = E.lib()
    f = l.energon_fold_layernorm
    assert f(FAKE, None, FAKE, FAKE, 8, 64, E.BF16, FAKE + 256, None, FAKE, None) == -1
    assert f(FAKE, None, FAKE, FAKE, 8, 64, E.F32, FAKE + 256, FAKE, FAKE, None) == -6
    assert f(FAKE, None, FAKE, FAKE, 8, 60, E.BF16, FAKE + 256, FAKE, FAKE, None) == -2
    assert f(FAKE, None, FAKE, FAKE, 8, 64, E.BF16, FAKE, FAKE, FAKE, None) == -6          # in place
    assert f(FAKE, None, FAKE, FAKE, 8, 64, E.BF16, FAKE + 256, FAKE + 4, FAKE, None) == -5
    s = l.energon_row_stats
    assert s(FAKE, 4, 64, E.BF16, 1e-5, None, None) == -1
    assert s(FAKE, 4, 64, E.F32, 1e-5, FAKE, None) == -6
    assert s(FAKE, 4, 60, E.BF16, 1e-5, FAKE, None) == -2
    assert s(FAKE, 4, 1 << 16, E.BF16, 1e-5, FAKE, None) == -6
    assert s(FAKE, 4, 64, E.BF16, -1.0, FAKE, None) == -2
    assert s(FAKE, 0, 64, E.BF16, 1e-5, FAKE, None) == 0                                   # M = 0: nothing to do
    g = l.energon_linear_ln_folded
    assert g(FAKE, FAKE, FAKE, FAKE, None, FAKE, 4, 64, 64, 0, E.BF16, None) == -1
    assert g(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 4, 64, 96, 0, E.BF16, None) == -2
    assert g(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 4, 64, 64, 0, E.F32, None) == -6
    assert g(FAKE, FAKE, FAKE + 4, FAKE, FAKE, FAKE, 4, 64, 64, 0, E.BF16, None) == -5
    assert E.energon_stats_scratch_bytes(1000, 5120) == 1000 * 40 * 8
    assert E.energon_stats_scratch_bytes(3, 200) == 256
    assert E.energon_stats_scratch_bytes(-1, 64) == 0
    r = l.energon_linear_residual_stats
    assert r(FAKE, FAKE, None, None, FAKE, 4, 64, 64, E.BF16, 1e-5, FAKE, FAKE, 1 << 20, None) == -1
    assert r(FAKE, FAKE, None, FAKE, FAKE, 4, 64, 64, E.BF16, 1e-5, FAKE, FAKE, 16, None) == -4
    assert r(FAKE, FAKE, None, FAKE, FAKE, 4, 64, 64, E.BF16, 1e-5, FAKE, FAKE + 16, 1 << 20, None) == -5
    assert r(FAKE, FAKE, None, FAKE, FAKE, 4, 1 << 16, 64, E.BF16, 1e-5, FAKE, FAKE, 1 << 30, None) == -6
    c = cfg()
    w = E.FoldedLayerWeights(*([FAKE] * 10))
    lens = np.asarray([3, 2], dtype=np.int32)
    lf = l.energon_layer_forward_ln_folded
    assert lf(C.byref(c), C.byref(w), FAKE, FAKE, 5, FAKE, lens.ctypes.data, 2, 4, FAKE, 16, None, None, None) == -4
    assert lf(C.byref(c), C.byref(w), FAKE, FAKE, 6, FAKE, lens.ctypes.data, 2, 4, FAKE, 1 << 30, None, None, None) == -3
    assert lf(C.byref(c), C.byref(w), FAKE, FAKE, 5, FAKE, lens.ctypes.data, 2, 4, FAKE, 1 << 30, FAKE + 4, None, None) == -5
    w.c_fc1 = None
    assert lf(C.byref(c), C.byref(w), FAKE, FAKE, 5, FAKE, lens.ctypes.data, 2, 4, FAKE, 1 << 30, None, None, None) == -1
    c32 = cfg()
    c32.dtype = E.F32
    w = E.FoldedLayerWeights(*([FAKE] * 10))
    assert lf(C.byref(c32), C.byref(w), FAKE, FAKE, 5, FAKE, lens.ctypes.data, 2, 4, FAKE, 1 << 30, None, None, None) == -6


def test_decode_and_model_end_entry_points_reject_bad_arguments():
    l = E.lib()
    a = l.energon_decode_attention
    assert a(FAKE, FAKE, FAKE, None, 2, 8, 2, 64, E.BF16, FAKE, None) == -1
    assert a(FAKE, FAKE, FAKE, FAKE, 2, 8, 2, 96, E.BF16, FAKE, None) == -6
    assert a(FAKE, FAKE, FAKE, FAKE, 2, 8, 2, 64, E.F32, FAKE, None) == -6
    assert a(FAKE, FAKE, FAKE, FAKE, 2, 0, 2, 64, E.BF16, FAKE, None) == -2
    assert a(FAKE, FAKE, FAKE, FAKE + 2, 2, 8, 2, 64, E.BF16, FAKE, None) == -5
    assert a(FAKE, FAKE, FAKE, FAKE, 0, 8, 2, 64, E.BF16, FAKE, None) == 0       # B = 0: nothing to do
    c = cfg()
    assert E.energon_decode_workspace_bytes(c, 4) >= E.energon_workspace_bytes(c, 4)
    assert E.energon_decode_workspace_bytes(c, 4) % 256 == 0
    w = E.LayerWeights(*([FAKE] * 12))
    lens = np.asarray([3, 8], dtype=np.int32)
    f = l.energon_decode_layer_forward
    assert f(C.byref(c), C.byref(w), FAKE, FAKE + 256, 2, None, None, FAKE, FAKE, 8, FAKE, 1 << 30, None) == -1
    assert f(C.byref(c), C.byref(w), FAKE, FAKE, 2, FAKE, None, FAKE, FAKE, 8, FAKE, 1 << 30, None) == -6   # x aliases y
    assert f(C.byref(c), C.byref(w), FAKE, FAKE + 256, 2, FAKE, lens.ctypes.data, FAKE, FAKE, 8, FAKE, 1 << 30, None) == -3
    assert f(C.byref(c), C.byref(w), FAKE, FAKE + 256, 2, FAKE, None, FAKE, FAKE, 8, FAKE, 16, None) == -4
    assert f(C.byref(c), C.byref(w), FAKE, FAKE + 256, 2, FAKE, None, FAKE, FAKE, 0, FAKE, 1 << 30, None) == -2
    e = l.energon_embed_packed
    assert e(FAKE, FAKE, 5, 2, FAKE, 100, None, 16, 64, E.BF16, FAKE, None) == -1
    assert e(FAKE, FAKE, 5, 2, FAKE, 100, FAKE, 16, 60, E.BF16, FAKE, None) == -2
    assert e(FAKE, FAKE, 5, 2, FAKE, 100, FAKE, 16, 64, E.F32, FAKE, None) == -6
    assert e(FAKE, FAKE, 0, 2, FAKE, 100, FAKE, 16, 64, E.BF16, FAKE, None) == 0
    r = l.energon_last_token_rows
    assert r(FAKE, None, 2, 64, E.BF16, FAKE, None) == -1
    assert r(FAKE, FAKE, 2, 60, E.BF16, FAKE, None) == -2
    assert r(FAKE, FAKE, 0, 64, E.BF16, FAKE, None) == 0


def test_cache_fill_and_embed_at_reject_bad_arguments():
    l = E.lib()
    f = l.energon_cache_fill
    assert f(FAKE, FAKE, 5, 2, 128, 8, E.BF16, None, FAKE, None) == -1
    assert f(FAKE, FAKE, 5, 2, 100, 8, E.BF16, FAKE, FAKE, None) == -2
    assert f(FAKE, FAKE, 5, 2, 128, 8, E.F32, FAKE, FAKE, None) == -6
    assert f(FAKE, FAKE + 2, 5, 2, 128, 8, E.BF16, FAKE, FAKE, None) == -5
    assert f(None, FAKE, 0, 2, 128, 8, E.BF16, FAKE, FAKE, None) == 0          # T = 0: nothing to do
    e = l.energon_embed_at
    assert e(FAKE, None, 4, FAKE, 100, FAKE, 16, 64, E.BF16, FAKE, None) == -1
    assert e(FAKE, FAKE, 4, FAKE, 100, FAKE, 16, 60, E.BF16, FAKE, None) == -2
    assert e(FAKE, FAKE, 4, FAKE, 100, FAKE, 16, 64, E.F32, FAKE, None) == -6
    assert e(FAKE, FAKE, 0, FAKE, 100, FAKE, 16, 64, E.BF16, FAKE, None) == 0


def test_static_scratch_generation_step_rejects_bad_arguments_before_touching_the_device():
    f = E.lib().energon_decode_layer_forward_static
    c, w = cfg(), E.LayerWeights(*([FAKE] * 12))
    lens = np.asarray([3, 2], dtype=np.int32)
    ok_args = lambda **kw: [kw.get("c", C.byref(c)), C.byref(w), kw.get("x", FAKE), kw.get("y", FAKE + 4096), kw.get("B", 2),
                            FAKE, kw.get("lens", lens.ctypes.data), FAKE, FAKE, kw.get("S_cap", 8), None]
    assert f(*ok_args(x=None)) == -1
    assert f(*ok_args(y=FAKE)) == -6                      # x and y may not alias
    assert f(*ok_args(S_cap=0)) == -2
    assert f(*ok_args(S_cap=3)) == -3                     # a cached length that does not fit the cache
    assert f(*ok_args(x=FAKE + 2)) == -5
    assert f(*ok_args(B=60000, lens=None)) == -4          # beyond the fixed scratch array
    c32 = cfg(dtype=E.F32)
    assert f(*ok_args(c=C.byref(c32))) == -6


def test_linear_with_scratch_rejects_bad_arguments():
    f = E.lib().energon_linear_with_scratch
    assert E.energon_linear_scratch_bytes(577, 1024, 1024, E.BF16) == 0        # too few tiles for the persistent kernel
    assert E.energon_linear_scratch_bytes(577, 1024, 1000, E.BF16) == 0        # invalid shape
    assert E.energon_linear_scratch_bytes(8428, 5120, 20480, E.F32) == 0
    need = E.energon_linear_scratch_bytes(3184, 6144, 12288, E.BF16)           # 312 long tiles on 256 workgroups
    assert need > 0 and need % 256 == 0
    args = lambda **kw: [kw.get("x", FAKE), FAKE, None, None, FAKE, 3184, 6144, kw.get("K", 12288), E.EPI_BIAS, E.BF16,
                         kw.get("scratch", FAKE), kw.get("nbytes", need), None]
    assert f(*args(x=None)) == -1
    assert f(*args(K=12290)) == -2
    assert f(*args(scratch=None)) == -1
    assert f(*args(scratch=FAKE + 16)) == -5
    assert f(*args(nbytes=need - 1)) == -4


def test_streamed_stack_rejects_bad_arguments_before_touching_the_device():
    f = E.lib().energon_stack_forward_streamed
    c, w = cfg(), E.LayerWeights(*([FAKE] * 12))
    lens = np.asarray([3, 2], dtype=np.int32)
    need = E.energon_layer_weights_bytes(c)
    assert need >= 2 * (1024 * 3072 + 1024 * 1024 + 2 * 1024 * 4096) and need % 256 == 0
    assert E.energon_layer_weights_bytes(cfg(head_dim=80)) == 0
    args = lambda **kw: [C.byref(c), kw.get("w", C.byref(w)), kw.get("L", 1), kw.get("x", FAKE), 5, FAKE, lens.ctypes.data, 2, 4,
                         FAKE, 1 << 30, kw.get("s0", FAKE), kw.get("s1", FAKE + 4096), kw.get("nbytes", need), None,
                         kw.get("cs", 1)]
    assert f(*args(w=None)) == -1
    assert f(*args(L=0)) == -2
    assert f(*args(cs=None)) == -6          # copy stream = compute stream
    assert f(*args(s1=FAKE)) == -5          # the two slots must be distinct
    assert f(*args(s0=FAKE + 16)) == -5
    assert f(*args(x=None)) == -1
    assert f(*args(nbytes=need - 1)) == -4
    w2 = E.LayerWeights(*([FAKE] * 12)); w2.w_fc2 = None
    assert f(*args(w=C.byref(w2))) == -1
