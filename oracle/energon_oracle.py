"""CPU oracle for the padding-free transformer-layer forward.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
file; the product path (the HIP library) never does, and this file imports nothing
from it.  Everything is NumPy fp64 (plus scipy's erf), written for reading, not speed.

What the method computes (Sec. 4.3, "Distributed Redundant Computation
Elimination"): the tokens of a padded batch are gathered into one dense matrix,
the position-wise operations run on that matrix, and the padded layout is rebuilt.
A linear layer treats every token vector on its own, so this removal changes no
valid token's value: the method's result IS the ordinary padded layer forward,
restricted to the valid positions.  The oracle is therefore that plain definition:
a pre-LayerNorm decoder block (Sec. 2.2: an attention module made of a pair of
linear layers around multi-head attention with a causal mask, then an MLP module
made of a pair of linear layers) evaluated at ALL B*S positions, pads included,
with pad rows set to zero at the very end.

Readings the paper leaves open, fixed here (the same ones the HIP path follows):
  * pre-LN block, residual around each module, no LayerNorm after the stack;
  * right padding: valid tokens of sequence b sit at positions 0 .. len[b]-1;
  * query i may attend key j iff j <= i and j < len[b];
  * LayerNorm: biased variance over the H features, eps inside the square root;
  * GeLU in its exact erf form; softmax scale 1/sqrt(d);
  * weights stored [out, in]; w_qkv rows are Q | K | V, head-major inside each;
  * a missing out-proj / FC2 bias (None) means "no bias": the row-split shard of
    Sec. 4.1.3 keeps only its partial sum, the cross-GPU accumulation is left out;
  * rebuilt pad rows are exact zeros; packed order is batch-major, then position.

Pins (tests/test_oracle_*.py): brute-force unbatched runs, padding invariance,
hand-computed one-token/one-head values, position-0 closed form, uniform-attention
closed form, identity block with zero output weights, per-stage agreement with
textbook library routines, and (for the paper's padded attention path) round trips,
closed-form indices and agreement with the variable-length attention on valid tokens; for
the LayerNorm-folded linear, the identity against layer_norm + linear, a hand-computed 2x2
case and the rounding rule for its column sums; for the generation step, agreement with the
last row of the whole-sequence forward at every position, the one-key closed form and a
hand-computed two-key case; for the embedding and last-row gathers, closed-form indices.
No function here is "parity unpinned".
"""
import numpy as np
from scipy.special import erf as _erf


# --------------------------------------------------------------------------- packing
def pack_indices(lengths, S):
    """Compaction of the valid-token mask (Sec. 4.3, removing padding).

    The mask over the row-major [B, S] grid is m[b, s] = (s < len[b]).  Its exclusive
    prefix sum gives every valid token its packed row; here that is written out as:
    cu[b] = number of valid tokens before sequence b, idx[t] = flat padded position
    of packed row t.  Returns (cu int32 [B+1], idx int32 [T])."""
    lengths = np.asarray(lengths, dtype=np.int64)
    B = lengths.shape[0]
    mask = np.zeros((B, S), dtype=bool)
    for b in range(B):
        if lengths[b] < 0 or lengths[b] > S:
            raise ValueError("length out of range")
        for s in range(S):
            mask[b, s] = s < lengths[b]
    flat = mask.reshape(-1)
    excl = np.cumsum(flat) - flat          # exclusive prefix sum of the 0/1 mask
    T = int(flat.sum())
    idx = np.empty(T, dtype=np.int32)
    for p in range(B * S):
        if flat[p]:
            idx[excl[p]] = p
    cu = np.zeros(B + 1, dtype=np.int32)
    for b in range(B):
        cu[b + 1] = cu[b] + lengths[b]
    return cu, idx


def pack(x_pad, lengths):
    """Remove padding: [B, S, H] -> [T, H] in batch-major, position order."""
    B, S, H = x_pad.shape
    _, idx = pack_indices(lengths, S)
    return x_pad.reshape(B * S, H)[idx].copy()


def unpack(x_packed, lengths, S):
    """Rebuild padding: [T, H] -> [B, S, H]; pad rows are zero."""
    B = len(lengths)
    H = x_packed.shape[1]
    _, idx = pack_indices(lengths, S)
    out = np.zeros((B * S, H), dtype=x_packed.dtype)
    out[idx] = x_packed
    return out.reshape(B, S, H)



# ----------------------------------------------------- LayerNorm folded into the next linear
# The fusion the paper credits to the comparison system (Sec. 5.5: LayerNorm, the QKV
# contractions and the bias in one kernel), in the algebraic form the HIP path uses.  With
# mu, r = row mean and 1/sqrt(var + eps) of x:
#   linear(layer_norm(x), W, b) = r * (x @ Wf^T - mu * c) + bf,
#   Wf = W * gamma (per input feature),  c = Wf summed over the input features,  bf = b + W @ beta.
# The definition of the result stays linear(layer_norm(x, ...), W, b); these two functions
# state the pieces the fused kernels exchange, so that each piece can be compared on its own.
def row_stats(x, eps):
    """(mean, 1/sqrt(biased variance + eps)) of every row."""
    mu = x.mean(axis=-1)
    var = ((x - mu[:, None]) ** 2).mean(axis=-1)
    return mu, 1.0 / np.sqrt(var + eps)


def fold_layer_norm(w, b, gamma, beta, round_weights=None):
    """(Wf, c, bf) as above.  `round_weights`, if given, is applied to Wf before c is summed:
    the identity must hold for the weights the contraction really uses, so a 16-bit Wf has its
    column sums taken after the rounding."""
    wf = w * gamma[None, :]
    if round_weights is not None:
        wf = round_weights(wf)
    c = wf.sum(axis=1)
    bf = w @ beta + (0.0 if b is None else b)
    return wf, c, bf


def linear_ln_folded(x, wf, c, bf, mu, r):
    """r * (x @ Wf^T - mu * c) + bf, the right-hand side of the identity."""
    return r[:, None] * (x @ wf.T - mu[:, None] * c[None, :]) + bf[None, :]

# --------------------------------------------------------------------------- stages
def layer_norm(x, gamma, beta, eps):
    """Per-row normalisation over the last axis (biased variance)."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * gamma + beta


def gelu(z):
    return 0.5 * z * (1.0 + _erf(z / np.sqrt(2.0)))


def linear(x, w, b):
    """y = x @ w^T (+ b); w is [out, in]."""
    y = x @ w.T
    if b is not None:
        y = y + b
    return y


def masked_causal_attention(q, k, v, length, n_heads, head_dim):
    """Multi-head attention for ONE sequence laid out [S, A] (A = nh*d), evaluated at
    every one of the S positions.  Query i sees the key set
    J(i) = { j : j <= i and j < length }; an empty set (length 0) gives a zero row."""
    S = q.shape[0]
    out = np.zeros_like(q)
    scale = 1.0 / np.sqrt(float(head_dim))
    j = np.arange(S)
    for i in range(S):
        J = j[(j <= i) & (j < length)]          # allowed keys of query i
        if J.size == 0:
            continue
        for h in range(n_heads):
            c0, c1 = h * head_dim, (h + 1) * head_dim
            s = (k[J, c0:c1] @ q[i, c0:c1]) * scale
            p = np.exp(s - s.max())
            p = p / p.sum()
            out[i, c0:c1] = p @ v[J, c0:c1]
    return out


# ------------------------------------------------- the paper's own attention path
# Sec. 4.3 keeps the attention core padded: padding is rebuilt in front of it and removed
# behind it, each fused with the head transpose ("two kernels that fuse the transpose and
# pad operations").  These three functions are that path written out as plain index maps;
# on valid tokens it must equal the variable-length attention above (tests pin that).
def rebuild_qkv_heads(qkv_packed, lengths, S, n_heads, head_dim):
    """[T, 3A] packed rows (Q | K | V, head-major inside each third) -> q, k, v, each
    [B, nh, S, d]:  q[b, h, s, :] = qkv_packed[cu[b]+s, h*d:(h+1)*d] for s < len[b],
    zeros at the pad positions (k, v likewise from the second and last third)."""
    qkv_packed = np.asarray(qkv_packed, dtype=np.float64)
    lengths = np.asarray(lengths, dtype=np.int64)
    B, A = lengths.shape[0], n_heads * head_dim
    out = np.zeros((3, B, n_heads, S, head_dim), dtype=np.float64)
    t = 0
    for b in range(B):
        for s_ in range(int(lengths[b])):
            row = qkv_packed[t]
            for which in range(3):
                for h in range(n_heads):
                    c0 = which * A + h * head_dim
                    out[which, b, h, s_, :] = row[c0:c0 + head_dim]
            t += 1
    return out[0], out[1], out[2]


def padded_attention_heads(q, k, v, lengths):
    """Attention of every (sequence, head) over all S positions of the padded layout
    [B, nh, S, d], with the key set J(i) = { j : j <= i and j < len[b] } (causal and
    key-padding mask); a query with no allowed key (len[b] = 0) gives a zero row."""
    q, k, v = (np.asarray(a, dtype=np.float64) for a in (q, k, v))
    B, nh, S, d = q.shape
    out = np.zeros_like(q)
    scale = 1.0 / np.sqrt(float(d))
    j = np.arange(S)
    for b in range(B):
        for h in range(nh):
            for i in range(S):
                J = j[(j <= i) & (j < int(lengths[b]))]
                if J.size == 0:
                    continue
                s_ = (k[b, h, J] @ q[b, h, i]) * scale
                p_ = np.exp(s_ - s_.max())
                out[b, h, i] = (p_ / p_.sum()) @ v[b, h, J]
    return out


def remove_padding_heads(o_pad, lengths):
    """[B, nh, S, d] -> packed [T, A]:  out[cu[b]+s, h*d:(h+1)*d] = o_pad[b, h, s, :]
    for s < len[b] (the inverse transpose, fused with the removal of padding)."""
    o_pad = np.asarray(o_pad, dtype=np.float64)
    B, nh, S, d = o_pad.shape
    T = int(np.sum(lengths))
    out = np.zeros((T, nh * d), dtype=np.float64)
    t = 0
    for b in range(B):
        for s_ in range(int(lengths[b])):
            for h in range(nh):
                out[t, h * d:(h + 1) * d] = o_pad[b, h, s_, :]
            t += 1
    return out


def layer_forward_padded(x_pad, lengths, p, n_heads, head_dim, eps=1e-5, stages=None):
    """One pre-LN decoder block on the padded batch [B, S, H]; every position is
    computed (pads too), nothing is zeroed here.  If `stages` is a dict it receives
    the intermediates (u, qkv, attn, y1, w, m), each [B, S, .]."""
    x_pad = np.asarray(x_pad, dtype=np.float64)
    B, S, H = x_pad.shape
    A = n_heads * head_dim
    f = lambda a: None if a is None else np.asarray(a, dtype=np.float64)
    p = {k_: f(v_) for k_, v_ in p.items()}
    y = np.empty_like(x_pad)
    keep = {k_: [] for k_ in ("u", "qkv", "attn", "y1", "w", "m")}
    for b in range(B):
        x = x_pad[b]
        u = layer_norm(x, p["ln1_g"], p["ln1_b"], eps)
        qkv = linear(u, p["w_qkv"], p["b_qkv"])
        q, k, v = qkv[:, 0:A], qkv[:, A:2 * A], qkv[:, 2 * A:3 * A]
        attn = masked_causal_attention(q, k, v, int(lengths[b]), n_heads, head_dim)
        y1 = x + linear(attn, p["w_o"], p["b_o"])
        w = layer_norm(y1, p["ln2_g"], p["ln2_b"], eps)
        m = gelu(linear(w, p["w_fc1"], p["b_fc1"]))
        y[b] = y1 + linear(m, p["w_fc2"], p["b_fc2"])
        for name, val in (("u", u), ("qkv", qkv), ("attn", attn), ("y1", y1), ("w", w), ("m", m)):
            keep[name].append(val)
    if stages is not None:
        for name, vals in keep.items():
            stages[name] = np.stack(vals)
    return y


def zero_pad_rows(y_pad, lengths):
    out = y_pad.copy()
    for b in range(out.shape[0]):
        out[b, int(lengths[b]):, :] = 0.0
    return out


def stack_forward(x_pad, lengths, layer_params, n_heads, head_dim, eps=1e-5, stages=None):
    """L blocks applied in turn to the padded batch, then pad rows set to zero: the
    result the pack -> L x layer -> unpack pipeline must reproduce.  `stages`, if
    given, receives the LAST layer's intermediates."""
    y = np.asarray(x_pad, dtype=np.float64)
    for li, p in enumerate(layer_params):
        st = stages if (stages is not None and li == len(layer_params) - 1) else None
        y = layer_forward_padded(y, lengths, p, n_heads, head_dim, eps, st)
    return zero_pad_rows(y, lengths)

# ------------------------------------------------- one generation step on cached keys / values
# The paper describes the decoder block (Sec. 2.2: causal mask) and its forward over a batch of
# sequences of different lengths (Sec. 4.3), not token-by-token generation.  The step below is
# what that definition implies: under a causal mask the rows of K and V that earlier tokens
# produced never change, so the block's output for a token appended at position p is row p of the
# block applied to the whole sequence, and it needs from the earlier tokens only their K and V
# rows (the cache).  Each sequence of the batch has its own cache length: nothing is padded.
def decode_attention(q_new, k_new, v_new, k_cache, v_cache, n_heads, head_dim):
    """One sequence, one new token.  q_new, k_new, v_new [A]; k_cache, v_cache [p, A] (rows of the
    p earlier tokens, p may be 0).  The query attends the p cached keys and its own key."""
    A = n_heads * head_dim
    keys = np.concatenate([k_cache.reshape(-1, A), k_new[None, :]], axis=0)
    vals = np.concatenate([v_cache.reshape(-1, A), v_new[None, :]], axis=0)
    out = np.empty(A, dtype=np.float64)
    for h in range(n_heads):
        sl = slice(h * head_dim, (h + 1) * head_dim)
        s = keys[:, sl] @ q_new[sl] / np.sqrt(head_dim)
        e = np.exp(s - s.max())
        out[sl] = (e / e.sum()) @ vals[:, sl]
    return out


def decode_layer(x_new, caches, p, n_heads, head_dim, eps=1e-5):
    """One pre-LN decoder block for one new token per sequence.  x_new [B, H]; caches[b] =
    (k_cache [p_b, A], v_cache [p_b, A]).  Returns (y [B, H], k_new [B, A], v_new [B, A]); the
    caller appends k_new[b], v_new[b] to sequence b's cache."""
    x_new = np.asarray(x_new, dtype=np.float64)
    f = lambda a: None if a is None else np.asarray(a, dtype=np.float64)
    p = {k_: f(v_) for k_, v_ in p.items()}
    A = n_heads * head_dim
    u = layer_norm(x_new, p["ln1_g"], p["ln1_b"], eps)
    qkv = linear(u, p["w_qkv"], p["b_qkv"])
    q, k_new, v_new = qkv[:, 0:A], qkv[:, A:2 * A], qkv[:, 2 * A:3 * A]
    attn = np.stack([decode_attention(q[b], k_new[b], v_new[b], np.asarray(caches[b][0], dtype=np.float64),
                                      np.asarray(caches[b][1], dtype=np.float64), n_heads, head_dim)
                     for b in range(x_new.shape[0])])
    y1 = x_new + linear(attn, p["w_o"], p["b_o"])
    w = layer_norm(y1, p["ln2_g"], p["ln2_b"], eps)
    m = gelu(linear(w, p["w_fc1"], p["b_fc1"]))
    return y1 + linear(m, p["w_fc2"], p["b_fc2"]), k_new, v_new


# ------------------------------------------------------------- the two ends of the model
def embed_packed(ids, lengths, wte, wpe):
    """Token + position embedding on the packed layout: row t of the result belongs to position
    t - cu[b] of its sequence b (Sec. 2.2 mentions the embedding layer only by name; learned
    absolute positions as in the GPT models the paper runs)."""
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    out = np.empty((int(cu[-1]), wte.shape[1]), dtype=np.float64)
    for b in range(len(lengths)):
        for i in range(int(lengths[b])):
            out[cu[b] + i] = wte[ids[cu[b] + i]] + wpe[i]
    return out


def last_token_rows(x_packed, lengths):
    """Row of the last valid token of every sequence (what the next-token logits are computed
    from); a sequence of length 0 gives a zero row."""
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    out = np.zeros((len(lengths), x_packed.shape[1]), dtype=np.float64)
    for b in range(len(lengths)):
        if lengths[b] > 0:
            out[b] = x_packed[cu[b + 1] - 1]
    return out


def cache_from_packed(qkv_packed, lengths, S_cap, A, fill=0.0):
    """K and V of a prefill laid out as the generation step reads them: [B, S_cap, A] each, row i of
    sequence b = columns A..2A / 2A..3A of its packed row cu[b] + i; other rows keep `fill`."""
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    B = len(lengths)
    k = np.full((B, S_cap, A), fill, dtype=np.float64)
    v = np.full((B, S_cap, A), fill, dtype=np.float64)
    for b in range(B):
        for i in range(min(int(lengths[b]), S_cap)):
            k[b, i] = qkv_packed[cu[b] + i, A:2 * A]
            v[b, i] = qkv_packed[cu[b] + i, 2 * A:3 * A]
    return k, v
