"""Pins for the oracle's generation step (one new token per sequence on cached keys / values)
and for the two ends of the model (embedding on the packed layout, last-token rows)."""
import numpy as np

from oracle import energon_oracle as O
from paper_2209_02341_amd import workloads as wl


def small_layer(seed, H=32, nh=2, d=8, F=48):
    rng = np.random.default_rng(seed)
    return wl.random_small_layer(rng, H, nh, d, F), H, nh, d


def test_decode_step_is_the_last_row_of_the_whole_sequence_forward():
    """Feed a sequence token by token through decode_layer, appending K/V; at every position the
    output must equal that row of the (separately pinned) whole-sequence forward."""
    p, H, nh, d = small_layer(3)
    rng = np.random.default_rng(4)
    lens = [7, 1, 4]
    S = max(lens)
    x = rng.normal(0, 1, (len(lens), S, H))
    st = {}
    full = O.layer_forward_padded(x, np.array(lens), p, nh, d, 1e-5, stages=st)
    A = nh * d
    caches = [(np.zeros((0, A)), np.zeros((0, A))) for _ in lens]
    for pos in range(S):
        live = [b for b in range(len(lens)) if pos < lens[b]]
        y, kn, vn = O.decode_layer(x[live, pos], [caches[b] for b in live], p, nh, d, 1e-5)
        for i, b in enumerate(live):
            assert np.abs(y[i] - full[b, pos]).max() < 1e-12
            # the appended rows are the K and V columns of the whole-sequence QKV
            assert np.abs(kn[i] - st["qkv"][b, pos, A:2 * A]).max() < 1e-12
            assert np.abs(vn[i] - st["qkv"][b, pos, 2 * A:]).max() < 1e-12
            caches[b] = (np.vstack([caches[b][0], kn[i]]), np.vstack([caches[b][1], vn[i]]))


def test_decode_attention_empty_cache_returns_own_value():
    rng = np.random.default_rng(0)
    q, k, v = rng.normal(size=(3, 16))
    out = O.decode_attention(q, k, v, np.zeros((0, 16)), np.zeros((0, 16)), 2, 8)
    assert np.array_equal(out, v)


def test_decode_attention_hand_computed_two_keys():
    # one head of width 1: scores q*k = (0, ln 3) -> weights (1/4, 3/4) -> 0.25*8 + 0.75*4 = 5
    out = O.decode_attention(np.array([1.0]), np.array([np.log(3.0)]), np.array([4.0]),
                             np.array([[0.0]]), np.array([[8.0]]), 1, 1)
    assert abs(out[0] - 5.0) < 1e-14


def test_decode_attention_heads_do_not_mix_and_cache_order_matters_only_with_values():
    rng = np.random.default_rng(1)
    nh, d, p = 3, 4, 6
    A = nh * d
    q, k, v = rng.normal(size=(3, A))
    kc, vc = rng.normal(size=(2, p, A))
    base = O.decode_attention(q, k, v, kc, vc, nh, d)
    kc2 = kc.copy(); kc2[:, d:2 * d] += 1.0            # disturb head 1's keys only
    other = O.decode_attention(q, k, v, kc2, vc, nh, d)
    assert np.array_equal(base[:d], other[:d]) and np.array_equal(base[2 * d:], other[2 * d:])
    assert not np.allclose(base[d:2 * d], other[d:2 * d])
    perm = rng.permutation(p)                          # keys and values permuted together: same result
    same = O.decode_attention(q, k, v, kc[perm], vc[perm], nh, d)
    assert np.abs(same - base).max() < 1e-14


def test_embed_packed_and_last_rows_closed_forms():
    lens = np.array([3, 0, 2])
    ids = np.array([5, 1, 5, 2, 0])
    V, S, H = 6, 4, 3
    wte = np.arange(V * H, dtype=np.float64).reshape(V, H)          # wte[v, j] = 3 v + j
    wpe = 100.0 * np.arange(S)[:, None] + np.zeros((S, H))          # wpe[i, j] = 100 i
    x = O.embed_packed(ids, lens, wte, wpe)
    want_pos = np.array([0, 1, 2, 0, 1])
    for t in range(5):
        for j in range(H):
            assert x[t, j] == 3 * ids[t] + j + 100 * want_pos[t]
    last = O.last_token_rows(x, lens)
    assert np.array_equal(last[0], x[2]) and np.array_equal(last[2], x[4]) and np.all(last[1] == 0)


def test_cache_from_packed_closed_form():
    lens = np.array([2, 0, 3])
    A, S_cap = 2, 4
    T = int(lens.sum())
    # packed row t holds (t, t) | (10 + t, 10 + t) | (20 + t, 20 + t)
    qkv = np.stack([np.repeat([t, 10 + t, 20 + t], A) for t in range(T)]).astype(np.float64)
    k, v = O.cache_from_packed(qkv, lens, S_cap, A, fill=-1.0)
    want_rows = {(0, 0): 0, (0, 1): 1, (2, 0): 2, (2, 1): 3, (2, 2): 4}
    for b in range(3):
        for i in range(S_cap):
            if (b, i) in want_rows:
                t = want_rows[(b, i)]
                assert np.all(k[b, i] == 10 + t) and np.all(v[b, i] == 20 + t)
            else:
                assert np.all(k[b, i] == -1.0) and np.all(v[b, i] == -1.0)
