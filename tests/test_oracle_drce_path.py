"""Pins of the oracle's padded attention path (Sec. 4.3: rebuild padding + head transpose,
padded attention core, inverse transpose + remove padding).  CPU only."""
import numpy as np
import pytest

from oracle import energon_oracle as orc


def _case(seed, B, S, nh, d, lengths=None):
    rng = np.random.default_rng(seed)
    lengths = np.asarray(lengths if lengths is not None else rng.integers(0, S + 1, size=B))
    T = int(lengths.sum())
    qkv = rng.standard_normal((T, 3 * nh * d))
    return qkv, lengths


def test_rebuild_closed_form_indices_and_zero_pads():
    B, S, nh, d = 4, 7, 3, 4
    qkv, lengths = _case(0, B, S, nh, d, [7, 0, 3, 5])
    q, k, v = orc.rebuild_qkv_heads(qkv, lengths, S, nh, d)
    cu = np.concatenate([[0], np.cumsum(lengths)])
    A = nh * d
    for b in range(B):
        for h in range(nh):
            for s in range(S):
                if s < lengths[b]:
                    t = cu[b] + s
                    assert np.array_equal(q[b, h, s], qkv[t, h * d:(h + 1) * d])
                    assert np.array_equal(k[b, h, s], qkv[t, A + h * d:A + (h + 1) * d])
                    assert np.array_equal(v[b, h, s], qkv[t, 2 * A + h * d:2 * A + (h + 1) * d])
                else:
                    assert not q[b, h, s].any() and not k[b, h, s].any() and not v[b, h, s].any()


def test_remove_inverts_rebuild():
    B, S, nh, d = 5, 9, 2, 8
    qkv, lengths = _case(1, B, S, nh, d)
    q, k, v = orc.rebuild_qkv_heads(qkv, lengths, S, nh, d)
    A = nh * d
    assert np.array_equal(orc.remove_padding_heads(q, lengths), qkv[:, :A])
    assert np.array_equal(orc.remove_padding_heads(k, lengths), qkv[:, A:2 * A])
    assert np.array_equal(orc.remove_padding_heads(v, lengths), qkv[:, 2 * A:])


def test_rebuild_equals_library_reshape_when_nothing_is_padded():
    B, S, nh, d = 3, 5, 4, 2
    qkv, lengths = _case(2, B, S, nh, d, [5, 5, 5])
    q, _, _ = orc.rebuild_qkv_heads(qkv, lengths, S, nh, d)
    ref = qkv[:, :nh * d].reshape(B, S, nh, d).transpose(0, 2, 1, 3)
    assert np.array_equal(q, ref)


@pytest.mark.parametrize("seed", [3, 4])
def test_padded_path_equals_variable_length_attention_on_valid_tokens(seed):
    B, S, nh, d = 4, 11, 2, 4
    qkv, lengths = _case(seed, B, S, nh, d, [11, 1, 0, 6])
    A = nh * d
    q, k, v = orc.rebuild_qkv_heads(qkv, lengths, S, nh, d)
    got = orc.remove_padding_heads(orc.padded_attention_heads(q, k, v, lengths), lengths)
    # each sequence alone, no padding at all
    rows, t = [], 0
    for L in lengths:
        seq = qkv[t:t + L]
        rows.append(orc.masked_causal_attention(seq[:, :A], seq[:, A:2 * A], seq[:, 2 * A:], int(L), nh, d))
        t += L
    np.testing.assert_allclose(got, np.concatenate(rows, axis=0), rtol=0, atol=1e-12)


def test_pad_queries_attend_all_valid_keys_and_empty_sequences_give_zero():
    # Q = 0 at pads after the rebuild: uniform weights over the len valid keys
    B, S, nh, d = 2, 6, 1, 3
    qkv, lengths = _case(5, B, S, nh, d, [2, 0])
    q, k, v = orc.rebuild_qkv_heads(qkv, lengths, S, nh, d)
    o = orc.padded_attention_heads(q, k, v, lengths)
    for s in range(2, S):
        np.testing.assert_allclose(o[0, 0, s], v[0, 0, :2].mean(axis=0), atol=1e-12)
    assert not o[1].any()
