"""ctypes binding of libenergon.so: same names as the C ABI, argument marshalling only.

Every step of the path runs in the library's HIP kernels.  Tensors are torch tensors used
as typed device memory (data_ptr) and the stream is torch's current HIP stream; nothing is
computed here.  If the library has not been built, importing a function fails loudly:
there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libenergon.so")

F32, BF16, F16 = 0, 1, 2
EPI_BIAS, EPI_BIAS_GELU, EPI_BIAS_RESIDUAL = 0, 1, 2
WS_U, WS_QKV, WS_ATTN, WS_Y1, WS_W, WS_M, WS_COUNT = 0, 1, 2, 3, 4, 5, 6
STAGE_NAMES = ("ln1", "qkv", "attn", "out", "ln2", "fc1", "fc2")


class EnergonError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status} ({strerror(status)})")


class LayerConfig(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("ffn", C.c_int32), ("ln_eps", C.c_float), ("dtype", C.c_int32)]


_WEIGHT_FIELDS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b",
                  "w_fc1", "b_fc1", "w_fc2", "b_fc2")


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _WEIGHT_FIELDS]


_FOLDED_FIELDS = ("wf_qkv", "c_qkv", "bf_qkv", "w_o", "b_o", "wf_fc1", "c_fc1", "bf_fc1", "w_fc2", "b_fc2")


class FoldedLayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _FOLDED_FIELDS]


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it was not built (python -m paper_2209_02341_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with __graft_entry__.build(); "
                               "there is no fallback path")
        l = C.CDLL(_LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        pcfg, pw = C.POINTER(LayerConfig), C.POINTER(LayerWeights)
        l.energon_strerror.restype = C.c_char_p
        l.energon_strerror.argtypes = [C.c_int]
        l.energon_workspace_bytes.restype = sz
        l.energon_workspace_bytes.argtypes = [pcfg, i64]
        l.energon_workspace_layout.argtypes = [pcfg, i64, C.POINTER(sz)]
        l.energon_pack.argtypes = [vp, vp, i32, i32, i32, i32, vp, i64, vp, vp, C.POINTER(i64), vp]
        l.energon_unpack.argtypes = [vp, vp, i64, i32, i32, i32, i32, vp, vp]
        layer_args = [pcfg, pw, vp, vp, i64, vp, vp, i32, i32, vp, sz, vp]
        l.energon_layer_forward.argtypes = layer_args
        l.energon_layer_forward_profiled.argtypes = layer_args + [C.POINTER(C.c_float)]
        l.energon_layer_weights_bytes.restype = sz
        l.energon_layer_weights_bytes.argtypes = [pcfg]
        l.energon_stack_forward_streamed.argtypes = [pcfg, pw, i32, vp, i64, vp, vp, i32, i32, vp, sz, vp, vp, sz, vp, vp]
        l.energon_stack_forward_streamed.restype = C.c_int
        l.energon_layernorm.argtypes = [vp, vp, vp, vp, i64, i32, C.c_float, i32, vp]
        l.energon_linear.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, vp]
        l.energon_linear_scratch_bytes.restype = sz
        l.energon_linear_scratch_bytes.argtypes = [i64, i32, i32, i32]
        l.energon_linear_with_scratch.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, vp, sz, vp]
        l.energon_linear_with_scratch.restype = C.c_int
        l.energon_linear_plan_selfcheck.argtypes = [i64, i32, i32, i32, i32, C.POINTER(i32)]
        l.energon_linear_plan_selfcheck.restype = C.c_int
        l.energon_attention.argtypes = [vp, vp, vp, i64, i32, i32, i32, i32, i32, vp]
        l.energon_rebuild_qkv.argtypes = [vp, vp, i64, i32, i32, i32, i32, i32, vp, vp, vp, vp]
        l.energon_attention_padded.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, vp]
        l.energon_remove_attn_padding.argtypes = [vp, vp, i64, i32, i32, i32, i32, i32, vp, vp]
        l.energon_drce_workspace_bytes.restype = sz
        l.energon_drce_workspace_bytes.argtypes = [pcfg, i32, i32]
        l.energon_layer_forward_drce.argtypes = layer_args[:-1] + [vp, sz, vp, C.POINTER(C.c_float)]
        l.energon_fold_layernorm.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp]
        l.energon_row_stats.argtypes = [vp, i64, i32, i32, C.c_float, vp, vp]
        l.energon_linear_ln_folded.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, vp]
        l.energon_stats_scratch_bytes.restype = sz
        l.energon_stats_scratch_bytes.argtypes = [i64, i32]
        l.energon_linear_residual_stats.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, i32, C.c_float, vp, vp, sz, vp]
        l.energon_layer_forward_ln_folded.argtypes = [pcfg, C.POINTER(FoldedLayerWeights), vp, vp, i64, vp, vp, i32,
                                                      i32, vp, sz, vp, vp, vp]
        l.energon_cache_fill.argtypes = [vp, vp, i64, i32, i32, i32, i32, vp, vp, vp]
        l.energon_cache_fill.restype = C.c_int
        l.energon_decode_attention.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, vp]
        l.energon_decode_workspace_bytes.restype = sz
        l.energon_decode_workspace_bytes.argtypes = [pcfg, i32]
        l.energon_decode_layer_forward.argtypes = [pcfg, pw, vp, vp, i32, vp, vp, vp, vp, i32, vp, sz, vp]
        l.energon_decode_layer_forward_static.argtypes = [pcfg, pw, vp, vp, i32, vp, vp, vp, vp, i32, vp]
        l.energon_decode_layer_forward_static.restype = C.c_int
        l.energon_embed_packed.argtypes = [vp, vp, i64, i32, vp, i32, vp, i32, i32, i32, vp, vp]
        l.energon_embed_at.argtypes = [vp, vp, i64, vp, i32, vp, i32, i32, i32, vp, vp]
        l.energon_embed_at.restype = C.c_int
        l.energon_last_token_rows.argtypes = [vp, vp, i32, i32, i32, vp, vp]
        for name in ("energon_decode_attention", "energon_decode_layer_forward", "energon_embed_packed",
                     "energon_last_token_rows"):
            getattr(l, name).restype = C.c_int
        for name in ("energon_fold_layernorm", "energon_row_stats", "energon_linear_ln_folded",
                     "energon_linear_residual_stats", "energon_layer_forward_ln_folded"):
            getattr(l, name).restype = C.c_int
        for name in ("energon_workspace_layout", "energon_pack", "energon_unpack", "energon_layer_forward",
                     "energon_layer_forward_profiled", "energon_layernorm", "energon_linear",
                     "energon_attention", "energon_rebuild_qkv", "energon_attention_padded",
                     "energon_remove_attn_padding", "energon_layer_forward_drce"):
            getattr(l, name).restype = C.c_int
        _lib = l
    return _lib


# ------------------------------------------------------------------ marshalling helpers
def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array / raw int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float16:
        return F16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _stream(stream):
    if stream is not None:
        return stream
    import torch
    return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None


def _lengths(lengths) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(lengths), dtype=np.int32)


def _check(status: int, where: str):
    if status != 0:
        raise EnergonError(status, where)


def make_weights(tensors: dict) -> LayerWeights:
    """LayerWeights from a dict of device tensors (missing / None bias = NULL).  The caller
    keeps the tensors alive."""
    w = LayerWeights()
    for n in _WEIGHT_FIELDS:
        setattr(w, n, _ptr(tensors.get(n)))
    return w


def make_folded_weights(tensors: dict) -> FoldedLayerWeights:
    """FoldedLayerWeights from a dict of device tensors (missing / None bias = NULL).  The caller
    keeps the tensors alive."""
    w = FoldedLayerWeights()
    for n in _FOLDED_FIELDS:
        setattr(w, n, _ptr(tensors.get(n)))
    return w


# ------------------------------------------------------------------ the C ABI, same names
def strerror(status: int) -> str:
    return lib().energon_strerror(int(status)).decode()


def energon_workspace_bytes(cfg: LayerConfig, max_tokens: int) -> int:
    return int(lib().energon_workspace_bytes(C.byref(cfg), int(max_tokens)))


def energon_workspace_layout(cfg: LayerConfig, max_tokens: int) -> list:
    off = (C.c_size_t * WS_COUNT)()
    _check(lib().energon_workspace_layout(C.byref(cfg), int(max_tokens), off), "energon_workspace_layout")
    return [int(v) for v in off]


def energon_pack(x_padded, lengths, x_packed, cu_seqlens, token_idx, stream=None) -> int:
    """x_padded [B,S,H] device; lengths host int32 [B]; outputs device.  Returns T."""
    B, S, H = x_padded.shape
    lens = _lengths(lengths)
    total = C.c_int64(-1)
    _check(lib().energon_pack(_ptr(x_padded), _ptr(lens), B, S, H, _dtype_code(x_padded), _ptr(x_packed),
                              int(x_packed.shape[0]), _ptr(cu_seqlens), _ptr(token_idx), C.byref(total),
                              _stream(stream)), "energon_pack")
    return int(total.value)


def energon_unpack(y_packed, cu_seqlens, T: int, y_padded, stream=None) -> None:
    B, S, H = y_padded.shape
    _check(lib().energon_unpack(_ptr(y_packed), _ptr(cu_seqlens), int(T), B, S, H, _dtype_code(y_padded),
                                _ptr(y_padded), _stream(stream)), "energon_unpack")


def energon_layer_forward(cfg: LayerConfig, weights: LayerWeights, x_packed, y_packed, T: int, cu_seqlens,
                          lengths, max_len: int, workspace, stream=None) -> None:
    lens = _lengths(lengths)
    _check(lib().energon_layer_forward(C.byref(cfg), C.byref(weights), _ptr(x_packed), _ptr(y_packed), int(T),
                                       _ptr(cu_seqlens), _ptr(lens), len(lens), int(max_len), _ptr(workspace),
                                       int(workspace.numel() * workspace.element_size()), _stream(stream)),
           "energon_layer_forward")


def energon_layer_forward_profiled(cfg: LayerConfig, weights: LayerWeights, x_packed, y_packed, T: int,
                                   cu_seqlens, lengths, max_len: int, workspace, stream=None) -> dict:
    lens = _lengths(lengths)
    ms = (C.c_float * len(STAGE_NAMES))()
    _check(lib().energon_layer_forward_profiled(C.byref(cfg), C.byref(weights), _ptr(x_packed), _ptr(y_packed),
                                                int(T), _ptr(cu_seqlens), _ptr(lens), len(lens), int(max_len),
                                                _ptr(workspace),
                                                int(workspace.numel() * workspace.element_size()),
                                                _stream(stream), ms), "energon_layer_forward_profiled")
    return dict(zip(STAGE_NAMES, (float(v) for v in ms)))


def energon_layer_weights_bytes(cfg: LayerConfig) -> int:
    return int(lib().energon_layer_weights_bytes(C.byref(cfg)))


def energon_stack_forward_streamed(cfg: LayerConfig, host_layers: list, x_packed, T: int, cu_seqlens, lengths,
                                   max_len: int, workspace, slot0, slot1, copy_stream, stream=None) -> None:
    """host_layers: LayerWeights structs whose pointers are (pinned) HOST addresses.  copy_stream: a raw
    HIP stream handle (e.g. torch.cuda.Stream().cuda_stream)."""
    lens = _lengths(lengths)
    arr = (LayerWeights * len(host_layers))(*host_layers)
    _check(lib().energon_stack_forward_streamed(C.byref(cfg), arr, len(host_layers), _ptr(x_packed), int(T),
                                                _ptr(cu_seqlens), _ptr(lens), len(lens), int(max_len),
                                                _ptr(workspace), int(workspace.numel() * workspace.element_size()),
                                                _ptr(slot0), _ptr(slot1), int(slot0.numel() * slot0.element_size()),
                                                _stream(stream), int(copy_stream)),
           "energon_stack_forward_streamed")


def energon_layernorm(x, gamma, beta, y, eps: float, stream=None) -> None:
    T, H = x.shape
    _check(lib().energon_layernorm(_ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), T, H, float(eps), _dtype_code(x),
                                   _stream(stream)), "energon_layernorm")


def energon_linear(x, w, bias, residual, y, epilogue: int, stream=None) -> None:
    M, K = x.shape
    N = w.shape[0]
    _check(lib().energon_linear(_ptr(x), _ptr(w), _ptr(bias), _ptr(residual), _ptr(y), M, N, K, int(epilogue),
                                _dtype_code(x), _stream(stream)), "energon_linear")


def energon_linear_scratch_bytes(M: int, N: int, K: int, dtype: int) -> int:
    return int(lib().energon_linear_scratch_bytes(int(M), int(N), int(K), int(dtype)))


def energon_linear_with_scratch(x, w, bias, residual, y, epilogue: int, scratch, stream=None) -> None:
    M, K = x.shape
    N = w.shape[0]
    nbytes = 0 if scratch is None else int(scratch.numel() * scratch.element_size())
    _check(lib().energon_linear_with_scratch(_ptr(x), _ptr(w), _ptr(bias), _ptr(residual), _ptr(y), M, N, K,
                                             int(epilogue), _dtype_code(x), _ptr(scratch), nbytes, _stream(stream)),
           "energon_linear_with_scratch")


def energon_linear_plan_selfcheck(M: int, N: int, K: int, workgroups_per_xcd: int = 32, with_scratch: bool = True):
    """(status, pieces): status 0 = the decomposition covers every tile and slab once; -1 = shape not taken."""
    pieces = C.c_int32(0)
    st = lib().energon_linear_plan_selfcheck(int(M), int(N), int(K), int(workgroups_per_xcd), int(bool(with_scratch)),
                                             C.byref(pieces))
    return int(st), int(pieces.value)


def energon_attention(qkv, out, cu_seqlens, B: int, max_len: int, n_heads: int, head_dim: int,
                      stream=None) -> None:
    T = qkv.shape[0]
    _check(lib().energon_attention(_ptr(qkv), _ptr(out), _ptr(cu_seqlens), T, int(B), int(max_len), int(n_heads),
                                   int(head_dim), _dtype_code(qkv), _stream(stream)), "energon_attention")


# ---- the paper's own attention path (rebuild padding + transpose, padded core, remove padding)
def energon_rebuild_qkv(qkv_packed, cu_seqlens, B: int, S: int, n_heads: int, head_dim: int, q_pad, k_pad, v_pad,
                        stream=None) -> None:
    T = qkv_packed.shape[0]
    _check(lib().energon_rebuild_qkv(_ptr(qkv_packed), _ptr(cu_seqlens), int(T), int(B), int(S), int(n_heads),
                                     int(head_dim), _dtype_code(qkv_packed), _ptr(q_pad), _ptr(k_pad), _ptr(v_pad),
                                     _stream(stream)), "energon_rebuild_qkv")


def energon_attention_padded(q_pad, k_pad, v_pad, cu_seqlens, out_pad, stream=None) -> None:
    B, nh, S, d = q_pad.shape
    _check(lib().energon_attention_padded(_ptr(q_pad), _ptr(k_pad), _ptr(v_pad), _ptr(cu_seqlens), B, S, nh, d,
                                          _dtype_code(q_pad), _ptr(out_pad), _stream(stream)),
           "energon_attention_padded")


def energon_remove_attn_padding(out_pad, cu_seqlens, attn_packed, stream=None) -> None:
    B, nh, S, d = out_pad.shape
    T = attn_packed.shape[0]
    _check(lib().energon_remove_attn_padding(_ptr(out_pad), _ptr(cu_seqlens), int(T), B, S, nh, d,
                                             _dtype_code(out_pad), _ptr(attn_packed), _stream(stream)),
           "energon_remove_attn_padding")


def energon_drce_workspace_bytes(cfg: LayerConfig, B: int, S: int) -> int:
    return int(lib().energon_drce_workspace_bytes(C.byref(cfg), int(B), int(S)))


def energon_layer_forward_drce(cfg: LayerConfig, weights: LayerWeights, x_packed, y_packed, T: int, cu_seqlens,
                               lengths, max_len: int, workspace, pad_workspace, stream=None, timed=False):
    """Returns the per-stage milliseconds (dict) if timed, else None."""
    lens = _lengths(lengths)
    ms = (C.c_float * len(STAGE_NAMES))() if timed else None
    _check(lib().energon_layer_forward_drce(C.byref(cfg), C.byref(weights), _ptr(x_packed), _ptr(y_packed), int(T),
                                            _ptr(cu_seqlens), _ptr(lens), len(lens), int(max_len), _ptr(workspace),
                                            int(workspace.numel() * workspace.element_size()), _ptr(pad_workspace),
                                            int(pad_workspace.numel() * pad_workspace.element_size()),
                                            _stream(stream), ms), "energon_layer_forward_drce")
    return dict(zip(STAGE_NAMES, (float(v) for v in ms))) if timed else None


# ---- LayerNorm folded into the following linear
def energon_fold_layernorm(w, b, gamma, beta, w_folded, colsum, bias_folded, stream=None) -> None:
    N, K = w.shape
    _check(lib().energon_fold_layernorm(_ptr(w), _ptr(b), _ptr(gamma), _ptr(beta), N, K, _dtype_code(w),
                                        _ptr(w_folded), _ptr(colsum), _ptr(bias_folded), _stream(stream)),
           "energon_fold_layernorm")


def energon_row_stats(x, eps: float, stats, stream=None) -> None:
    M, K = x.shape
    _check(lib().energon_row_stats(_ptr(x), M, K, _dtype_code(x), float(eps), _ptr(stats), _stream(stream)),
           "energon_row_stats")


def energon_linear_ln_folded(x, w_folded, colsum, bias_folded, stats, y, gelu: bool, stream=None) -> None:
    M, K = x.shape
    N = w_folded.shape[0]
    _check(lib().energon_linear_ln_folded(_ptr(x), _ptr(w_folded), _ptr(colsum), _ptr(bias_folded), _ptr(stats),
                                          _ptr(y), M, N, K, int(bool(gelu)), _dtype_code(x), _stream(stream)),
           "energon_linear_ln_folded")


def energon_stats_scratch_bytes(M: int, N: int) -> int:
    return int(lib().energon_stats_scratch_bytes(int(M), int(N)))


def energon_linear_residual_stats(x, w, bias, residual, y, eps: float, stats_out, scratch, stream=None) -> None:
    M, K = x.shape
    N = w.shape[0]
    _check(lib().energon_linear_residual_stats(_ptr(x), _ptr(w), _ptr(bias), _ptr(residual), _ptr(y), M, N, K,
                                               _dtype_code(x), float(eps), _ptr(stats_out), _ptr(scratch),
                                               int(scratch.numel() * scratch.element_size()), _stream(stream)),
           "energon_linear_residual_stats")


def energon_layer_forward_ln_folded(cfg: LayerConfig, weights: FoldedLayerWeights, x_packed, y_packed, T: int,
                                    cu_seqlens, lengths, max_len: int, workspace, stats_in=None, stats_out=None,
                                    stream=None) -> None:
    lens = _lengths(lengths)
    _check(lib().energon_layer_forward_ln_folded(C.byref(cfg), C.byref(weights), _ptr(x_packed), _ptr(y_packed),
                                                 int(T), _ptr(cu_seqlens), _ptr(lens), len(lens), int(max_len),
                                                 _ptr(workspace),
                                                 int(workspace.numel() * workspace.element_size()),
                                                 _ptr(stats_in), _ptr(stats_out), _stream(stream)),
           "energon_layer_forward_ln_folded")


# ---- one generation step on cached keys / values; the two ends of the model
def energon_cache_fill(qkv_packed, cu_seqlens, k_cache, v_cache, stream=None) -> None:
    T = qkv_packed.shape[0]
    B, S_cap, A = k_cache.shape
    _check(lib().energon_cache_fill(_ptr(qkv_packed), _ptr(cu_seqlens), T, B, A, S_cap, _dtype_code(k_cache),
                                    _ptr(k_cache), _ptr(v_cache), _stream(stream)), "energon_cache_fill")


def energon_decode_attention(qkv, k_cache, v_cache, cache_lens_dev, n_heads: int, head_dim: int, out,
                             stream=None) -> None:
    B, S_cap = k_cache.shape[0], k_cache.shape[1]
    _check(lib().energon_decode_attention(_ptr(qkv), _ptr(k_cache), _ptr(v_cache), _ptr(cache_lens_dev), B, S_cap,
                                          int(n_heads), int(head_dim), _dtype_code(qkv), _ptr(out), _stream(stream)),
           "energon_decode_attention")


def energon_decode_workspace_bytes(cfg: LayerConfig, B: int) -> int:
    return int(lib().energon_decode_workspace_bytes(C.byref(cfg), int(B)))


def energon_decode_layer_forward(cfg: LayerConfig, weights: LayerWeights, x, y, cache_lens_dev, cache_lens_host,
                                 k_cache, v_cache, workspace, stream=None) -> None:
    B, S_cap = k_cache.shape[0], k_cache.shape[1]
    lens = None if cache_lens_host is None else _lengths(cache_lens_host)
    _check(lib().energon_decode_layer_forward(C.byref(cfg), C.byref(weights), _ptr(x), _ptr(y), B,
                                              _ptr(cache_lens_dev), _ptr(lens), _ptr(k_cache), _ptr(v_cache), S_cap,
                                              _ptr(workspace), int(workspace.numel() * workspace.element_size()),
                                              _stream(stream)), "energon_decode_layer_forward")


STATIC_SCRATCH_BYTES = 64 << 20   # ENERGON_STATIC_SCRATCH_BYTES


def energon_decode_layer_forward_static(cfg: LayerConfig, weights: LayerWeights, x, y, cache_lens_dev,
                                        cache_lens_host, k_cache, v_cache, stream=None) -> None:
    """energon_decode_layer_forward without a workspace argument (the library's fixed scratch array)."""
    B, S_cap = k_cache.shape[0], k_cache.shape[1]
    lens = None if cache_lens_host is None else _lengths(cache_lens_host)
    _check(lib().energon_decode_layer_forward_static(C.byref(cfg), C.byref(weights), _ptr(x), _ptr(y), B,
                                                     _ptr(cache_lens_dev), _ptr(lens), _ptr(k_cache),
                                                     _ptr(v_cache), S_cap, _stream(stream)),
           "energon_decode_layer_forward_static")


def energon_embed_packed(ids_dev, cu_seqlens, wte, wpe, x_packed, stream=None) -> None:
    T, H = x_packed.shape
    B = cu_seqlens.shape[0] - 1
    _check(lib().energon_embed_packed(_ptr(ids_dev), _ptr(cu_seqlens), T, B, _ptr(wte), wte.shape[0], _ptr(wpe),
                                      wpe.shape[0], H, _dtype_code(wte), _ptr(x_packed), _stream(stream)),
           "energon_embed_packed")


def energon_embed_at(ids_dev, positions_dev, wte, wpe, x, stream=None) -> None:
    n, H = x.shape
    _check(lib().energon_embed_at(_ptr(ids_dev), _ptr(positions_dev), n, _ptr(wte), wte.shape[0], _ptr(wpe),
                                  wpe.shape[0], H, _dtype_code(wte), _ptr(x), _stream(stream)), "energon_embed_at")


def energon_last_token_rows(x_packed, cu_seqlens, out, stream=None) -> None:
    B, H = out.shape
    _check(lib().energon_last_token_rows(_ptr(x_packed), _ptr(cu_seqlens), B, H, _dtype_code(out), _ptr(out),
                                         _stream(stream)), "energon_last_token_rows")
