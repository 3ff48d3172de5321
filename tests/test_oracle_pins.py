"""Pins for the CPU oracle: each test checks it against something other than itself
(hand-computed values, closed forms, brute force, textbook library routines)."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import energon_oracle as orc
from paper_2209_02341_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small_case(seed, B=3, S=9, H=8, nh=2, d=4, F=16, lengths=None, bias=True):
    rng = np.random.default_rng(seed)
    p = wl.random_small_layer(rng, H, nh, d, F, bias=bias)
    x = rng.standard_normal((B, S, H))
    if lengths is None:
        lengths = rng.integers(1, S + 1, size=B)
    return x, np.asarray(lengths, dtype=np.int32), p


# ------------------------------------------------------------------ pack indices
@pytest.mark.parametrize("lengths,S", [([3, 0, 5, 5, 1], 5), ([1], 1), ([0, 0], 4), ([7, 2, 7], 7)])
def test_pack_indices_closed_form(lengths, S):
    cu, idx = orc.pack_indices(lengths, S)
    assert cu.dtype == np.int32 and idx.dtype == np.int32
    assert cu[0] == 0 and cu[-1] == sum(lengths) == idx.size
    for b, n in enumerate(lengths):
        assert cu[b + 1] - cu[b] == n
        for s in range(n):
            assert idx[cu[b] + s] == b * S + s
    assert np.all(np.diff(idx) > 0)
    grid = np.arange(S)[None, :] < np.asarray(lengths)[:, None]
    assert np.array_equal(idx, np.flatnonzero(grid.reshape(-1)))


def test_pack_indices_rejects_bad_length():
    with pytest.raises(ValueError):
        orc.pack_indices([3, 6], 5)
    with pytest.raises(ValueError):
        orc.pack_indices([-1], 5)


def test_pack_unpack_roundtrip():
    rng = np.random.default_rng(1)
    lengths = [2, 0, 4, 1]
    x = rng.standard_normal((4, 4, 3))
    xp = orc.pack(x, lengths)
    assert xp.shape == (7, 3)
    assert np.array_equal(xp[2], x[2, 0]) and np.array_equal(xp[6], x[3, 0])
    back = orc.unpack(xp, lengths, 4)
    for b, n in enumerate(lengths):
        assert np.array_equal(back[b, :n], x[b, :n])
        assert np.all(back[b, n:] == 0)


# ------------------------------------------------------------------ hand-computed case
def read_golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            vals[k] = np.array([float(t) for t in v])
    return vals


def test_one_token_one_head_hand_computed():
    g = read_golden("one_token_one_head.txt")
    assert abs(0.5 * (1 + math.erf(2 / math.sqrt(2))) - 0.9772498680518208) < 1e-15
    p = {
        "ln1_g": [1, 1], "ln1_b": [0, 0],
        "w_qkv": [[0.3, -1.1], [2.0, 0.7], [-0.4, 0.9], [1.5, 1.5], [1, 0], [0, 2]],
        "b_qkv": [0.1, -0.2, 0.3, 0.4, 0.5, -0.5],
        "w_o": [[2, 0], [1, 1]], "b_o": [0, 1],
        "ln2_g": [2, 1], "ln2_b": [0, 1],
        "w_fc1": [[1, 0], [0, 1]], "b_fc1": [0, 0],
        "w_fc2": [[1, 1], [1, -1]], "b_fc2": [0.5, 0],
    }
    x = np.array([[[1.0, 3.0]]])
    st = {}
    y = orc.stack_forward(x, [1], [p], n_heads=1, head_dim=2, eps=0.0, stages=st)
    for k in ("attn", "y1", "w", "m"):
        np.testing.assert_allclose(st[k][0, 0], g[k], rtol=0, atol=1e-14)
    np.testing.assert_allclose(y[0, 0], g["y"], rtol=0, atol=1e-14)


# ------------------------------------------------------------------ closed forms
def single_token_formula(x0, p, A, eps):
    """Block output for a token that sees only itself: attention output = its own v.
    Written with scalar loops, independent of the oracle's routines."""
    H = len(x0)

    def ln(v, g, b):
        mu = sum(v) / H
        var = sum((t - mu) ** 2 for t in v) / H
        return [(t - mu) / math.sqrt(var + eps) * g[i] + b[i] for i, t in enumerate(v)]

    def lin(v, w, b):
        out = []
        for r in range(len(w)):
            acc = 0.0 if b is None else float(b[r])
            for c in range(len(v)):
                acc += float(w[r][c]) * v[c]
            out.append(acc)
        return out

    u = ln(list(x0), p["ln1_g"], p["ln1_b"])
    v = lin(u, p["w_qkv"][2 * A:3 * A], None if p["b_qkv"] is None else p["b_qkv"][2 * A:3 * A])
    y1 = [a + b for a, b in zip(x0, lin(v, p["w_o"], p["b_o"]))]
    w = ln(y1, p["ln2_g"], p["ln2_b"])
    z = lin(w, p["w_fc1"], p["b_fc1"])
    m = [0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in z]
    return np.array([a + b for a, b in zip(y1, lin(m, p["w_fc2"], p["b_fc2"]))])


@pytest.mark.parametrize("bias", [True, False])
def test_position_zero_closed_form(bias):
    x, lengths, p = small_case(3, bias=bias)
    y = orc.stack_forward(x, lengths, [p], 2, 4)
    for b in range(x.shape[0]):
        ref = single_token_formula(x[b, 0], p, 8, 1e-5)
        np.testing.assert_allclose(y[b, 0], ref, rtol=1e-12, atol=1e-12)


def test_zero_output_weights_give_identity():
    x, lengths, p = small_case(4)
    for k in ("w_o", "b_o", "w_fc2", "b_fc2"):
        p[k] = np.zeros_like(p[k])
    y = orc.stack_forward(x, lengths, [p, p], 2, 4)
    for b, n in enumerate(lengths):
        assert np.array_equal(y[b, :n], x[b, :n])
        assert np.all(y[b, n:] == 0)


def test_uniform_attention_is_running_mean_of_values():
    """Q = K = 0 makes every allowed score equal, so o_i is the mean of v_j over the
    allowed keys: checks the causal extent, the length clip and the normalisation."""
    rng = np.random.default_rng(5)
    S, nh, d = 7, 2, 3
    v = rng.standard_normal((S, nh * d))
    z = np.zeros_like(v)
    for length in (0, 1, 4, 7):
        out = orc.masked_causal_attention(z, z, v, length, nh, d)
        for i in range(S):
            n = min(i + 1, length)
            ref = v[:n].mean(axis=0) if n > 0 else np.zeros(nh * d)
            np.testing.assert_allclose(out[i], ref, rtol=1e-13, atol=1e-13)


def test_attention_two_keys_by_hand():
    """d = 1, one head: o_1 = (e^{q1 k0} v0 + e^{q1 k1} v1) / (e^{q1 k0} + e^{q1 k1})."""
    q = np.array([[0.7], [-1.3]]); k = np.array([[0.2], [1.1]]); v = np.array([[3.0], [-2.0]])
    out = orc.masked_causal_attention(q, k, v, 2, 1, 1)
    e0, e1 = math.exp(-1.3 * 0.2), math.exp(-1.3 * 1.1)
    assert abs(out[0, 0] - 3.0) < 1e-15
    assert abs(out[1, 0] - (e0 * 3.0 + e1 * -2.0) / (e0 + e1)) < 1e-15
    # softmax scale 1/sqrt(d): with d = 4 and all weight in one coordinate
    q4 = np.zeros((2, 4)); k4 = np.zeros((2, 4)); v4 = np.zeros((2, 4))
    q4[:, 0] = q[:, 0]; k4[:, 0] = k[:, 0]; v4[:, 0] = v[:, 0]
    out4 = orc.masked_causal_attention(q4, k4, v4, 2, 1, 4)
    e0, e1 = math.exp(-1.3 * 0.2 / 2), math.exp(-1.3 * 1.1 / 2)
    assert abs(out4[1, 0] - (e0 * 3.0 + e1 * -2.0) / (e0 + e1)) < 1e-15


# ------------------------------------------------------------------ structure
def test_batched_equals_unbatched_brute_force():
    x, lengths, p = small_case(6, B=4, S=11)
    y = orc.stack_forward(x, lengths, [p, p], 2, 4)
    for b, n in enumerate(lengths):
        alone = orc.stack_forward(x[b:b + 1, :n], [n], [p, p], 2, 4)
        np.testing.assert_allclose(y[b, :n], alone[0], rtol=1e-11, atol=1e-12)


def test_padding_invariance():
    x, lengths, p = small_case(7, B=3, S=6, lengths=[2, 6, 4])
    base = orc.stack_forward(x, lengths, [p], 2, 4)
    rng = np.random.default_rng(70)
    for S2, fill in ((6, 0.0), (13, None), (12, 1e4), (9, -3.0)):
        x2 = rng.standard_normal((3, S2, 8)) if fill is None else np.full((3, S2, 8), fill)
        for b, n in enumerate(lengths):
            x2[b, :n] = x[b, :n]
        y2 = orc.stack_forward(x2, lengths, [p], 2, 4)
        for b, n in enumerate(lengths):
            np.testing.assert_allclose(y2[b, :n], base[b, :n], rtol=1e-11, atol=1e-11)
            assert np.all(y2[b, n:] == 0)


def test_batch_permutation_equivariance():
    x, lengths, p = small_case(8, B=4)
    perm = np.array([2, 0, 3, 1])
    y = orc.stack_forward(x, lengths, [p], 2, 4)
    yp = orc.stack_forward(x[perm], lengths[perm], [p], 2, 4)
    np.testing.assert_allclose(yp, y[perm], rtol=1e-12, atol=1e-12)


def test_zero_length_sequence_rows_are_zero_and_harmless():
    x, lengths, p = small_case(9, B=3, S=5, lengths=[3, 0, 5])
    y = orc.stack_forward(x, lengths, [p], 2, 4)
    assert np.all(y[1] == 0) and np.all(np.isfinite(y))


# ------------------------------------------------------------------ invariants
def test_gelu_and_layernorm_invariants():
    z = np.linspace(-6, 6, 49)
    np.testing.assert_allclose(orc.gelu(-z), orc.gelu(z) - z, atol=1e-14)
    assert orc.gelu(np.array([0.0]))[0] == 0.0
    assert abs(orc.gelu(np.array([30.0]))[0] - 30.0) < 1e-12
    for t in (-1.5, 0.3, 2.0):
        assert abs(orc.gelu(np.array([t]))[0] - 0.5 * t * (1 + math.erf(t / math.sqrt(2)))) < 1e-15
    rng = np.random.default_rng(10)
    x = rng.standard_normal((5, 16)) * 3 + 1
    eps = 1e-5
    u = orc.layer_norm(x, np.ones(16), np.zeros(16), eps)
    var = x.var(axis=1)
    np.testing.assert_allclose(u.mean(axis=1), 0, atol=1e-14)
    np.testing.assert_allclose(u.var(axis=1), var / (var + eps), rtol=1e-12)


# ------------------------------------------------------------------ library second opinion
def test_against_torch_fp64_routines():
    """Each stage reduces to a textbook routine: layer_norm, linear, exact gelu and
    causal scaled-dot-product attention on the unpadded sequence."""
    x, lengths, p = small_case(11, B=3, S=10, H=12, nh=3, d=4, F=20)
    nh, d, A = 3, 4, 12
    st = {}
    y = orc.stack_forward(x, lengths, [p], nh, d, stages=st)
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    F = torch.nn.functional
    for b, n in enumerate(lengths):
        xb = t(x[b, :n])
        u = F.layer_norm(xb, (12,), t(p["ln1_g"]), t(p["ln1_b"]), 1e-5)
        qkv = F.linear(u, t(p["w_qkv"]), t(p["b_qkv"]))
        q, k, v = [qkv[:, i * A:(i + 1) * A].reshape(n, nh, d).transpose(0, 1) for i in range(3)]
        a = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(0, 1).reshape(n, A)
        y1 = xb + F.linear(a, t(p["w_o"]), t(p["b_o"]))
        w = F.layer_norm(y1, (12,), t(p["ln2_g"]), t(p["ln2_b"]), 1e-5)
        m = F.gelu(F.linear(w, t(p["w_fc1"]), t(p["b_fc1"])), approximate="none")
        yy = y1 + F.linear(m, t(p["w_fc2"]), t(p["b_fc2"]))
        np.testing.assert_allclose(st["attn"][b, :n], a.numpy(), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(st["m"][b, :n], m.numpy(), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(y[b, :n], yy.numpy(), rtol=1e-10, atol=1e-12)
