"""Plant one plausible mistake at a time in the oracle (on the CPU, by monkeypatching)
and require that at least one pin notices.  Guards the pins, not the oracle."""
import numpy as np
import pytest
from scipy.special import erf

from oracle import energon_oracle as orc
import test_oracle_pins as pins

PIN_FUNCS = [
    pins.test_one_token_one_head_hand_computed,
    lambda: pins.test_position_zero_closed_form(True),
    lambda: pins.test_position_zero_closed_form(False),
    pins.test_zero_output_weights_give_identity,
    pins.test_uniform_attention_is_running_mean_of_values,
    pins.test_attention_two_keys_by_hand,
    pins.test_batched_equals_unbatched_brute_force,
    pins.test_padding_invariance,
    pins.test_gelu_and_layernorm_invariants,
    pins.test_against_torch_fp64_routines,
    pins.test_pack_unpack_roundtrip,
    lambda: pins.test_pack_indices_closed_form([3, 0, 5, 5, 1], 5),
]


def some_pin_fails():
    for f in PIN_FUNCS:
        try:
            f()
        except (AssertionError, ValueError, IndexError):
            return True
    return False


def test_pins_pass_unmodified():
    assert not some_pin_fails()


def _ln_unbiased(x, g, b, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).sum(axis=-1, keepdims=True) / (x.shape[-1] - 1)
    return (x - mu) / np.sqrt(var + eps) * g + b


def _ln_no_shift(x, g, b, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g


def _gelu_tanh(z):
    return 0.5 * z * (1 + np.tanh(np.sqrt(2 / np.pi) * (z + 0.044715 * z ** 3)))


def _linear_no_bias(x, w, b):
    return x @ w.T


def _linear_transposed(x, w, b):
    y = x @ (w if w.shape[0] == w.shape[1] else w.T)
    return y if b is None else y + b


def _attn(variant):
    def f(q, k, v, length, nh, d):
        S = q.shape[0]
        out = np.zeros_like(q)
        scale = 1.0 if variant == "noscale" else 1.0 / np.sqrt(d)
        j = np.arange(S)
        for i in range(S):
            if variant == "noncausal":
                J = j[j < length]
            elif variant == "strict":
                J = j[(j < i) & (j < length)]
            elif variant == "nolen":
                J = j[j <= i]
            else:
                J = j[(j <= i) & (j < length)]
            if J.size == 0:
                continue
            for h in range(nh):
                c0, c1 = h * d, (h + 1) * d
                if variant == "headmix":
                    c0k = ((h + 1) % nh) * d
                    s = (k[J, c0k:c0k + d] @ q[i, c0:c1]) * scale
                else:
                    s = (k[J, c0:c1] @ q[i, c0:c1]) * scale
                p = np.exp(s - s.max())
                p = p / p.sum()
                out[i, c0:c1] = p @ v[J, c0:c1]
        return out
    return f


def _pack_indices_off(lengths, S):
    cu, idx = _orig_pack_indices(lengths, S)
    return cu, idx + (np.arange(idx.size) > 2)


_orig_pack_indices = orc.pack_indices

MUTATIONS = [
    ("layer_norm", _ln_unbiased), ("layer_norm", _ln_no_shift), ("gelu", _gelu_tanh),
    ("linear", _linear_no_bias), ("linear", _linear_transposed),
    ("masked_causal_attention", _attn("noscale")), ("masked_causal_attention", _attn("noncausal")),
    ("masked_causal_attention", _attn("strict")), ("masked_causal_attention", _attn("nolen")),
    ("masked_causal_attention", _attn("headmix")), ("pack_indices", _pack_indices_off),
]


@pytest.mark.parametrize("name,bad", MUTATIONS, ids=[f"{n}-{i}" for i, (n, _) in enumerate(MUTATIONS)])
def test_planted_mistake_is_caught(monkeypatch, name, bad):
    monkeypatch.setattr(orc, name, bad)
    assert some_pin_fails(), f"no pin noticed a broken {name}"
