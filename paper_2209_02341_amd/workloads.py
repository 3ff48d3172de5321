"""Seeded synthetic workloads for the packed (padding-free) transformer-layer forward.

This module only *draws data*: sequence lengths, padded activations and layer
weights with the shapes, value distributions and length mixes of the GPT-style
layers the paper evaluates (Sec. 5.1: GPT-3 layer geometry, heads of width 128;
Sec. 5.5: batches whose valid length is a fraction of the padded length).  It
holds none of the method's arithmetic (no LayerNorm, GEMM, attention, scan); both
the CPU oracle's tests and the GPU harness consume its output as plain arrays.

Every tensor has its own random streams keyed by (seed, tensor name, layer, row chunk),
so any tensor can be regenerated alone, in any order, on any number of threads.
Values are drawn in fp32 and, for bf16 workloads, rounded to bf16 (round to
nearest even) once here; the oracle and the GPU path both start from those
rounded values.
"""
from __future__ import annotations

import os
import zlib
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

F32 = "f32"
BF16 = "bf16"
F16 = "f16"     # the paper's precision (Sec. 5.1)


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str          # F32 or BF16: storage type of activations and weights
    layers: int         # L
    hidden: int         # H : model width
    n_heads: int        # nh: heads held by this GPU
    head_dim: int       # d
    ffn: int            # F : FFN width held by this GPU
    batch: int          # B
    max_len: int        # S : padded length
    length_dist: str    # "uniform" | "lognormal" | "full"
    len_lo: int
    len_hi: int
    len_median: float = 0.0
    len_sigma: float = 0.6
    row_split_bias: bool = True   # False: out-proj / FC2 carry no bias (row-split shard)
    ln_eps: float = 1e-5

    @property
    def attn_width(self) -> int:      # A = nh * d
        return self.n_heads * self.head_dim


# The five workloads of the build target, plus the zero-padding control of the last.
WORKLOADS = {
    w.name: w
    for w in [
        Workload("tiny_f32", F32, 1, 256, 4, 64, 1024, 4, 32, "uniform", 1, 32),
        Workload("small_bf16", BF16, 1, 1024, 16, 64, 4096, 8, 128, "uniform", 16, 128),
        Workload("small_f16", F16, 1, 1024, 16, 64, 4096, 8, 128, "uniform", 16, 128),
        Workload("gpt13b_f16", F16, 4, 5120, 40, 128, 20480, 32, 512, "uniform", 32, 512),
        Workload("gpt13b_bf16", BF16, 4, 5120, 40, 128, 20480, 32, 512, "uniform", 32, 512),
        Workload("gpt175b_tp8_shard_bf16", BF16, 1, 12288, 12, 128, 6144, 16, 1024,
                 "lognormal", 8, 1024, len_median=200.0, row_split_bias=False),
        Workload("heavy_pad_bf16", BF16, 1, 8192, 64, 128, 32768, 64, 2048,
                 "lognormal", 1, 2048, len_median=256.0),
        Workload("heavy_pad_control_bf16", BF16, 1, 8192, 64, 128, 32768, 64, 2048,
                 "full", 2048, 2048),
    ]
}


def _stream(seed: int, name: str, layer: int = 0, chunk: int = 0) -> np.random.Generator:
    key = zlib.crc32(name.encode("ascii"))
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, key, layer, chunk])))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (nearest even); returns the 16-bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_dtype(a: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 array whose values are exactly representable in `dtype`."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == F32:
        return a
    if dtype == F16:
        return a.astype(np.float16).astype(np.float32)   # round to nearest even
    return bf16_bits_to_f32(f32_to_bf16_bits(a))


def sample_lengths(w: Workload, seed: int = 0) -> np.ndarray:
    rng = _stream(seed, "lengths")
    if w.length_dist == "uniform":
        lens = rng.integers(w.len_lo, w.len_hi + 1, size=w.batch)
    elif w.length_dist == "lognormal":
        raw = np.exp(rng.normal(np.log(w.len_median), w.len_sigma, size=w.batch))
        lens = np.clip(np.rint(raw), w.len_lo, w.len_hi)
    elif w.length_dist == "full":
        lens = np.full(w.batch, w.max_len)
    else:
        raise ValueError(w.length_dist)
    return lens.astype(np.int32)


_CHUNK_ROWS = 1024
_POOL = ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1))


def _normal(seed: int, name: str, layer: int, shape, std: float, dtype: str) -> np.ndarray:
    """N(0, std) values rounded to `dtype`.  Rows are drawn in fixed chunks of 1024, each
    chunk from its own stream (seed, name, layer, chunk), so chunks can be filled in
    parallel and the result does not depend on the number of threads."""
    out = np.empty(shape, dtype=np.float32)
    flat = out.reshape(shape[0], -1) if len(shape) > 1 else out.reshape(1, -1)

    def fill(c):
        r0 = c * _CHUNK_ROWS
        dst = flat[r0:r0 + _CHUNK_ROWS]
        blk = _stream(seed, name, layer, c).standard_normal(dst.shape, dtype=np.float32)
        if std != 1.0:
            blk *= np.float32(std)
        dst[...] = round_to_dtype(blk, dtype)

    n_chunks = (flat.shape[0] + _CHUNK_ROWS - 1) // _CHUNK_ROWS
    if n_chunks <= 1:
        fill(0)
    else:
        list(_POOL.map(fill, range(n_chunks)))
    return out


def sample_x(w: Workload, seed: int = 0, seqs=None) -> np.ndarray:
    """Padded activations [B, S, H] ~ N(0,1); pad positions hold N(0,1) values too,
    so a path that wrongly reads them is caught.  `seqs` lists the sequences wanted;
    each sequence has its own stream so a subset costs only its share."""
    idx = list(range(w.batch)) if seqs is None else [int(b) for b in seqs]
    out = np.empty((len(idx), w.max_len, w.hidden), dtype=np.float32)
    def one(ob):
        out[ob[0]] = _normal(seed, "x", ob[1], (w.max_len, w.hidden), 1.0, w.dtype)

    if w.max_len <= _CHUNK_ROWS:      # one chunk per sequence: spread the sequences over threads
        list(_POOL.map(one, enumerate(idx)))
    else:                             # several chunks per sequence: _normal spreads those
        for ob in enumerate(idx):
            one(ob)
    return out


WEIGHT_STD = 0.02


def sample_layer(w: Workload, layer: int, seed: int = 0) -> dict:
    """One layer's parameters, stored [out, in] (both GEMM operands contiguous along
    the reduction).  w_qkv rows are Q | K | V, each head-major.  LayerNorm gain 1,
    shift 0; weights and biases ~ N(0, 0.02).  A row-split shard (Sec. 4.1.3) has
    no out-proj / FC2 bias: that bias is added after the cross-GPU sum."""
    H, A, F = w.hidden, w.attn_width, w.ffn
    g = lambda name, shape: _normal(seed, name, layer, shape, WEIGHT_STD, w.dtype)
    p = {
        "ln1_g": np.ones(H, np.float32), "ln1_b": np.zeros(H, np.float32),
        "w_qkv": g("w_qkv", (3 * A, H)), "b_qkv": g("b_qkv", (3 * A,)),
        "w_o": g("w_o", (H, A)), "b_o": g("b_o", (H,)) if w.row_split_bias else None,
        "ln2_g": np.ones(H, np.float32), "ln2_b": np.zeros(H, np.float32),
        "w_fc1": g("w_fc1", (F, H)), "b_fc1": g("b_fc1", (F,)),
        "w_fc2": g("w_fc2", (H, F)), "b_fc2": g("b_fc2", (H,)) if w.row_split_bias else None,
    }
    return p


def random_small_layer(rng: np.random.Generator, H: int, nh: int, d: int, F: int,
                       dtype: str = F32, ln_random: bool = True, bias: bool = True,
                       std: float = 0.2) -> dict:
    """Small layer with non-trivial LayerNorm gain/shift, for tests."""
    A = nh * d
    n = lambda *s: round_to_dtype(rng.standard_normal(s, dtype=np.float32) * np.float32(std), dtype)
    return {
        "ln1_g": round_to_dtype(1 + 0.3 * rng.standard_normal(H), dtype) if ln_random else np.ones(H, np.float32),
        "ln1_b": n(H) if ln_random else np.zeros(H, np.float32),
        "w_qkv": n(3 * A, H), "b_qkv": n(3 * A),
        "w_o": n(H, A), "b_o": n(H) if bias else None,
        "ln2_g": round_to_dtype(1 + 0.3 * rng.standard_normal(H), dtype) if ln_random else np.ones(H, np.float32),
        "ln2_b": n(H) if ln_random else np.zeros(H, np.float32),
        "w_fc1": n(F, H), "b_fc1": n(F),
        "w_fc2": n(H, F), "b_fc2": n(H) if bias else None,
    }
