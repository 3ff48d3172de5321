"""GPU parity for one generation step on cached keys / values, for the few-row linear kernel that
serves it, and for the two ends of the model (packed embedding, last-token rows); through the C ABI
against the CPU fp64 oracle.  Integer / byte work (the cache append, the gathers) is bit-exact;
floating point at the tolerances of test_gpu_parity.py.
"""
import numpy as np
import pytest
import torch

from oracle import energon_oracle as orc
from paper_2209_02341_amd import binding as E
from paper_2209_02341_amd import harness as hz
from paper_2209_02341_amd import workloads as wl
import math

from test_gpu_parity import TOL, assert_close, layer_noise, recipe_logit_rms

pytestmark = pytest.mark.gpu


# ------------------------------------------------------------------ few-row linear (M <= 64)
SKINNY_CASES = [
    # M, N, K, dtype: every row-tile count (1, 2, 4), ragged M, K with fewer slabs than wavefronts
    # (64, 192), an uneven split over the 4 wavefronts (640 = 10 slabs, 576 = 9), one column block
    (1, 32, 64, wl.BF16), (7, 96, 192, wl.BF16), (16, 256, 640, wl.BF16), (17, 64, 1024, wl.BF16),
    (32, 1536, 5120, wl.BF16), (33, 128, 2048, wl.BF16), (64, 512, 4096, wl.BF16), (50, 320, 20480, wl.BF16),
    (5, 64, 576, wl.F16), (32, 256, 5120, wl.F16),
]


@pytest.mark.parametrize("M,N,K,dtype", SKINNY_CASES)
@pytest.mark.parametrize("epi", [E.EPI_BIAS, E.EPI_BIAS_GELU, E.EPI_BIAS_RESIDUAL])
def test_linear_few_rows(M, N, K, dtype, epi):
    rng = np.random.default_rng(M * 7 + N + K + epi)
    x = wl.round_to_dtype(rng.standard_normal((M, K)), dtype)
    w = wl.round_to_dtype(rng.standard_normal((N, K)) / np.sqrt(K), dtype)
    b = wl.round_to_dtype(rng.standard_normal(N) * 0.5, dtype)
    r = wl.round_to_dtype(rng.standard_normal((M, N)), dtype)
    for bias in (b, None):
        xd, wd, bd, rd = (hz.to_device(a, dtype) for a in (x, w, bias, r))
        yd = torch.full((M + 1, N), 3.0, dtype=xd.dtype, device="cuda")
        E.energon_linear(xd, wd, bd, rd if epi == E.EPI_BIAS_RESIDUAL else None, yd, epi)
        ref = orc.linear(x.astype(np.float64), w.astype(np.float64), None if bias is None else bias.astype(np.float64))
        if epi == E.EPI_BIAS_GELU:
            ref = orc.gelu(ref)
        if epi == E.EPI_BIAS_RESIDUAL:
            ref = ref + r
        out = hz.to_host(yd)
        assert_close(out[:M], ref, dtype, f"few-row linear epi={epi}")
        assert np.all(out[M] == 3.0), "row past M was written"
        yd2 = torch.empty_like(yd)
        E.energon_linear(xd, wd, bd, rd if epi == E.EPI_BIAS_RESIDUAL else None, yd2, epi)
        assert torch.equal(yd[:M].view(torch.int16), yd2[:M].view(torch.int16)), "not deterministic"


def test_linear_few_rows_residual_in_place():
    M, N, K, dtype = 32, 512, 1024, wl.BF16
    rng = np.random.default_rng(11)
    x = wl.round_to_dtype(rng.standard_normal((M, K)), dtype)
    w = wl.round_to_dtype(rng.standard_normal((N, K)) / np.sqrt(K), dtype)
    r = wl.round_to_dtype(rng.standard_normal((M, N)), dtype)
    xd, wd, rd = (hz.to_device(a, dtype) for a in (x, w, r))
    E.energon_linear(xd, wd, None, rd, rd, E.EPI_BIAS_RESIDUAL)
    assert_close(hz.to_host(rd), x.astype(np.float64) @ w.astype(np.float64).T + r, dtype, "in-place residual")


# ------------------------------------------------------------------ attention of one step
DEC_ATTN_CASES = [
    # cached lengths, S_cap, heads, head_dim, dtype
    ([0, 1, 5, 63, 64, 65, 200], 256, 2, 128, wl.BF16),
    ([0, 3, 15, 16, 17, 127, 128, 129, 300], 301, 3, 64, wl.BF16),
    ([511], 512, 2, 128, wl.BF16),
    ([7, 0, 40], 64, 2, 128, wl.F16),
    ([33, 100], 128, 4, 64, wl.F16),
]


@pytest.mark.parametrize("lens,S_cap,nh,d,dtype", DEC_ATTN_CASES)
def test_decode_attention_and_cache_append(lens, S_cap, nh, d, dtype):
    rng = np.random.default_rng(sum(lens) + nh + d)
    B, A = len(lens), nh * d
    qkv = wl.round_to_dtype(rng.standard_normal((B, 3 * A)), dtype)
    kc = wl.round_to_dtype(rng.standard_normal((B, S_cap, A)), dtype)
    vc = wl.round_to_dtype(rng.standard_normal((B, S_cap, A)), dtype)
    for b in range(B):                      # what lies beyond a sequence's length must never matter
        kc[b, lens[b]:] = 1e4
        vc[b, lens[b]:] = -1e4
    qd, kd, vd = (hz.to_device(a, dtype) for a in (qkv, kc, vc))
    k_before, v_before = kd.clone(), vd.clone()
    lens_d = torch.tensor(lens, dtype=torch.int32, device="cuda")
    out = torch.empty((B, A), dtype=qd.dtype, device="cuda")
    E.energon_decode_attention(qd, kd, vd, lens_d, nh, d, out)
    got = hz.to_host(out)
    q64 = qkv.astype(np.float64)
    for b in range(B):
        p = lens[b]
        ref = orc.decode_attention(q64[b, :A], q64[b, A:2 * A], q64[b, 2 * A:], kc[b, :p].astype(np.float64),
                                   vc[b, :p].astype(np.float64), nh, d)
        assert_close(got[b][None, :], ref[None, :], dtype, f"decode attention seq {b} (cached {p})")
    # the append: row lens[b] of each cache now holds the new k / v bit for bit, nothing else moved
    kw, vw = k_before.clone(), v_before.clone()
    for b in range(B):
        kw[b, lens[b]] = qd[b, A:2 * A]
        vw[b, lens[b]] = qd[b, 2 * A:]
    assert torch.equal(kd.view(torch.int16), kw.view(torch.int16))
    assert torch.equal(vd.view(torch.int16), vw.view(torch.int16))


def test_decode_attention_full_cache_does_not_write():
    nh, d, S_cap, dtype = 2, 64, 8, wl.BF16
    A = nh * d
    rng = np.random.default_rng(3)
    qkv = wl.round_to_dtype(rng.standard_normal((1, 3 * A)), dtype)
    kc = wl.round_to_dtype(rng.standard_normal((1, S_cap, A)), dtype)
    vc = wl.round_to_dtype(rng.standard_normal((1, S_cap, A)), dtype)
    qd, kd, vd = (hz.to_device(a, dtype) for a in (qkv, kc, vc))
    guard_k, guard_v = kd.clone(), vd.clone()
    out = torch.empty((1, A), dtype=qd.dtype, device="cuda")
    E.energon_decode_attention(qd, kd, vd, torch.tensor([S_cap], dtype=torch.int32, device="cuda"), nh, d, out)
    assert torch.equal(kd.view(torch.int16), guard_k.view(torch.int16))
    assert torch.equal(vd.view(torch.int16), guard_v.view(torch.int16))
    q64 = qkv.astype(np.float64)
    ref = orc.decode_attention(q64[0, :A], q64[0, A:2 * A], q64[0, 2 * A:], kc[0].astype(np.float64),
                               vc[0].astype(np.float64), nh, d)
    assert_close(hz.to_host(out), ref[None, :], dtype, "decode attention on a full cache")


# ------------------------------------------------------------------ the step through a layer
class DecodeState:
    """Caches of L layers for B sequences plus the buffers of a step."""

    def __init__(self, w: wl.Workload, B: int, S_cap: int, layers):
        self.cfg = hz.layer_config(w.hidden, w.n_heads, w.head_dim, w.ffn, w.dtype, w.ln_eps)
        tdt = {wl.BF16: torch.bfloat16, wl.F16: torch.float16}[w.dtype]
        A = w.n_heads * w.head_dim
        self.layers = layers
        self.k = [torch.zeros((B, S_cap, A), dtype=tdt, device="cuda") for _ in layers]
        self.v = [torch.zeros((B, S_cap, A), dtype=tdt, device="cuda") for _ in layers]
        self.lens = torch.zeros(B, dtype=torch.int32, device="cuda")
        self.ws = torch.empty(E.energon_decode_workspace_bytes(self.cfg, B), dtype=torch.uint8, device="cuda")
        self.buf = [torch.empty((B, w.hidden), dtype=tdt, device="cuda") for _ in range(2)]

    def step(self, x):
        """x [B, H] device -> output of the last layer; appends to every layer's cache."""
        host = self.lens.cpu().numpy()
        src = x
        for i, layer in enumerate(self.layers):
            dst = self.buf[i & 1]
            E.energon_decode_layer_forward(self.cfg, layer.struct, src, dst, self.lens, host, self.k[i], self.v[i], self.ws)
            src = dst
        self.lens += 1
        return src


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F16])
def test_decode_steps_follow_the_whole_sequence_forward(dtype):
    """Prefill nothing; feed three sequences token by token through two layers.  At every position the
    step's output must match that row of the oracle's whole-sequence forward (sequences that have
    ended keep being fed a dummy token, their rows are ignored)."""
    w = wl.Workload("dec", dtype, 2, 256, 4, 64, 512, 3, 12, "uniform", 0, 12)
    lens = np.array([12, 5, 9], dtype=np.int32)
    x = wl.sample_x(w)
    layers = [wl.sample_layer(w, 0), wl.sample_layer(w, 1)]
    ref = orc.stack_forward(x, lens, layers, w.n_heads, w.head_dim, w.ln_eps)
    dev = [hz.DeviceLayer(p, dtype) for p in layers]
    st = DecodeState(w, 3, 16, dev)
    xd = hz.to_device(x, dtype)
    for pos in range(int(lens.max())):
        y = hz.to_host(st.step(xd[:, pos].contiguous()))
        live = [b for b in range(3) if pos < lens[b]]
        assert_close(y[live], ref[live, pos], dtype, f"decode step at position {pos}", **layer_noise(2, recipe_logit_rms(w.hidden)))


def test_decode_after_packed_prefill_matches_oracle():
    """The packed prefill fills nothing by itself; build the caches from its QKV stage, then one step."""
    dtype = wl.BF16
    w = wl.Workload("dec2", dtype, 1, 512, 4, 128, 1024, 4, 40, "uniform", 0, 40)
    lens = np.array([40, 0, 17, 1], dtype=np.int32)
    S = 41
    x_full = wl.round_to_dtype(np.random.default_rng(2).standard_normal((4, S, w.hidden)), dtype)
    p = wl.sample_layer(w, 0)
    A = w.attn_width
    # oracle: whole-sequence forward over lens + 1 tokens; the step must reproduce row lens[b]
    ref = orc.layer_forward_padded(x_full, lens + 1, p, w.n_heads, w.head_dim, w.ln_eps)
    # GPU prefill over the first lens[b] tokens, caches from its QKV stage
    cfg = hz.layer_config(w.hidden, w.n_heads, w.head_dim, w.ffn, dtype, w.ln_eps)
    layer = hz.DeviceLayer(p, dtype)
    run = hz.PackedRun(cfg, 4, S, int(lens.sum()))
    run.forward(hz.to_device(x_full, dtype), lens, [layer])
    qkv = run.stage(E.WS_QKV, 3 * A)
    kc = torch.zeros((4, S, A), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    cu = np.concatenate([[0], np.cumsum(lens)])
    for b in range(4):
        kc[b, :lens[b]] = qkv[cu[b]:cu[b + 1], A:2 * A]
        vc[b, :lens[b]] = qkv[cu[b]:cu[b + 1], 2 * A:]
    x_new = hz.to_device(np.stack([x_full[b, lens[b]] for b in range(4)]), dtype)
    y = torch.empty_like(x_new)
    ws = torch.empty(E.energon_decode_workspace_bytes(cfg, 4), dtype=torch.uint8, device="cuda")
    lens_d = torch.tensor(lens, dtype=torch.int32, device="cuda")
    E.energon_decode_layer_forward(cfg, layer.struct, x_new, y, lens_d, lens, kc, vc, ws)
    want = np.stack([ref[b, lens[b]] for b in range(4)])
    assert_close(hz.to_host(y), want, dtype, "step after a packed prefill", **layer_noise(1, recipe_logit_rms(w.hidden)))


@pytest.mark.timeout(600)
def test_decode_step_full_size_13b_shape():
    """The benchmark's generation workload at full size: 32 sequences, caches of the prefill
    workload's lengths, one layer of the 13B shape (the four contractions in the few-row kernel);
    the oracle checks four sequences (shortest, two in the middle, longest)."""
    w = wl.WORKLOADS["gpt13b_bf16"]
    lens = wl.sample_lengths(w)
    lens = np.minimum(lens, w.max_len - 1).astype(np.int32)
    B, A, S_cap = w.batch, w.attn_width, w.max_len
    rng = np.random.default_rng(9)
    p = wl.sample_layer(w, 0)
    kc = wl.round_to_dtype(rng.standard_normal((B, S_cap, A)), w.dtype)
    vc = wl.round_to_dtype(rng.standard_normal((B, S_cap, A)), w.dtype)
    x = wl.round_to_dtype(rng.standard_normal((B, w.hidden)), w.dtype)
    cfg = hz.layer_config(w.hidden, w.n_heads, w.head_dim, w.ffn, w.dtype, w.ln_eps)
    layer = hz.DeviceLayer(p, w.dtype)
    xd, kd, vd = (hz.to_device(a, w.dtype) for a in (x, kc, vc))
    y = torch.empty_like(xd)
    ws = torch.empty(E.energon_decode_workspace_bytes(cfg, B), dtype=torch.uint8, device="cuda")
    E.energon_decode_layer_forward(cfg, layer.struct, xd, y, torch.tensor(lens, dtype=torch.int32, device="cuda"),
                                   lens, kd, vd, ws)
    order = np.argsort(lens)
    picks = [int(order[0]), int(order[B // 3]), int(order[2 * B // 3]), int(order[-1])]
    caches = [(kc[b, :lens[b]], vc[b, :lens[b]]) for b in picks]
    ref, k_new, v_new = orc.decode_layer(x[picks], caches, p, w.n_heads, w.head_dim, w.ln_eps)
    got = hz.to_host(y)
    # cached keys are unit normal here, queries come from the layer: logit rms = sqrt(hidden) * 0.02
    assert_close(got[picks], ref, w.dtype, "13B-shape generation step, sampled sequences",
                 **layer_noise(1, math.sqrt(w.hidden) * 0.02))
    for i, b in enumerate(picks):
        assert_close(hz.to_host(kd[b, lens[b]])[None, :], k_new[i][None, :], w.dtype, "appended k", stages=2)
        assert_close(hz.to_host(vd[b, lens[b]])[None, :], v_new[i][None, :], w.dtype, "appended v", stages=2)
    assert np.all(np.isfinite(got))


def test_decode_layer_rejects_a_full_cache_given_host_lengths():
    w = wl.Workload("dec3", wl.BF16, 1, 128, 2, 64, 256, 2, 4, "uniform", 0, 4)
    cfg = hz.layer_config(w.hidden, w.n_heads, w.head_dim, w.ffn, w.dtype, w.ln_eps)
    layer = hz.DeviceLayer(wl.sample_layer(w, 0), w.dtype)
    x = torch.zeros((2, 128), dtype=torch.bfloat16, device="cuda")
    y = torch.empty_like(x)
    kc = torch.zeros((2, 4, 128), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(E.energon_decode_workspace_bytes(cfg, 2), dtype=torch.uint8, device="cuda")
    lens = np.array([1, 4], dtype=np.int32)
    with pytest.raises(E.EnergonError) as e:
        E.energon_decode_layer_forward(cfg, layer.struct, x, y, torch.tensor(lens, device="cuda"), lens, kc, kc.clone(), ws)
    assert e.value.status == -3


# ------------------------------------------------------------------ the two ends of the model
@pytest.mark.parametrize("dtype", [wl.BF16, wl.F16])
def test_embed_packed_and_last_rows(dtype):
    rng = np.random.default_rng(4)
    lens = np.array([5, 0, 130, 1, 64], dtype=np.int32)
    V, P, H = 1000, 160, 264
    T = int(lens.sum())
    ids = rng.integers(0, V, T).astype(np.int32)
    wte = wl.round_to_dtype(rng.standard_normal((V, H)), dtype)
    wpe = wl.round_to_dtype(rng.standard_normal((P, H)) * 0.1, dtype)
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32), device="cuda")
    wted, wped = hz.to_device(wte, dtype), hz.to_device(wpe, dtype)
    x = torch.full((T + 1, H), 3.0, dtype=wted.dtype, device="cuda")
    E.energon_embed_packed(torch.tensor(ids, device="cuda"), cu, wted, wped, x[:T])
    ref = orc.embed_packed(ids, lens, wte.astype(np.float64), wpe.astype(np.float64))
    got = hz.to_host(x)
    # one rounding of an exact fp32 sum: equal to the rounded oracle value
    assert np.array_equal(got[:T], wl.round_to_dtype(ref, dtype).astype(np.float64))
    assert np.all(got[T] == 3.0)
    last = torch.full((len(lens) + 1, H), 3.0, dtype=wted.dtype, device="cuda")
    E.energon_last_token_rows(x[:T], cu, last[:len(lens)])
    assert np.array_equal(hz.to_host(last)[:len(lens)], orc.last_token_rows(got[:T], lens))
    assert np.all(hz.to_host(last)[len(lens)] == 3.0)


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F16])
def test_decode_layer_with_split_contraction(dtype):
    """A long FFN (10240 = 160 slabs) with few output columns: the FC2 contraction of the step is cut
    over 4 workgroups along K and finished by the second kernel.  Also run-to-run identical."""
    w = wl.Workload("dec_split", dtype, 1, 256, 4, 64, 10240, 5, 24, "uniform", 0, 24)
    lens = np.array([0, 23, 7, 1, 12], dtype=np.int32)
    rng = np.random.default_rng(21)
    p = wl.sample_layer(w, 0)
    A, B, S_cap = w.attn_width, 5, 24
    kc = wl.round_to_dtype(rng.standard_normal((B, S_cap, A)), dtype)
    vc = wl.round_to_dtype(rng.standard_normal((B, S_cap, A)), dtype)
    x = wl.round_to_dtype(rng.standard_normal((B, w.hidden)), dtype)
    cfg = hz.layer_config(w.hidden, w.n_heads, w.head_dim, w.ffn, dtype, w.ln_eps)
    layer = hz.DeviceLayer(p, dtype)
    ws = torch.empty(E.energon_decode_workspace_bytes(cfg, B), dtype=torch.uint8, device="cuda")
    assert ws.numel() > E.energon_workspace_bytes(cfg, B), "no room for partial sums was planned"
    outs = []
    for _ in range(2):
        xd, kd, vd = (hz.to_device(a, dtype) for a in (x, kc, vc))
        y = torch.empty_like(xd)
        E.energon_decode_layer_forward(cfg, layer.struct, xd, y, torch.tensor(lens, device="cuda"), lens, kd, vd, ws)
        outs.append(y)
    ref, _, _ = orc.decode_layer(x, [(kc[b, :lens[b]], vc[b, :lens[b]]) for b in range(B)], p, w.n_heads, w.head_dim, w.ln_eps)
    assert_close(hz.to_host(outs[0]), ref, dtype, "step with a split FC2", **layer_noise(1, math.sqrt(w.hidden) * 0.02))
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))


def test_cache_fill_bit_exact():
    rng = np.random.default_rng(8)
    lens = np.array([5, 0, 70, 1, 33], dtype=np.int32)
    A, S_cap, dtype = 192, 64, wl.BF16           # one sequence is longer than the cache
    T = int(lens.sum())
    qkv = wl.round_to_dtype(rng.standard_normal((T, 3 * A)), dtype)
    qd = hz.to_device(qkv, dtype)
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32), device="cuda")
    kc = torch.full((5, S_cap, A), 7.0, dtype=qd.dtype, device="cuda")
    vc = torch.full((5, S_cap, A), 7.0, dtype=qd.dtype, device="cuda")
    E.energon_cache_fill(qd, cu, kc, vc)
    k_ref, v_ref = orc.cache_from_packed(qkv.astype(np.float64), lens, S_cap, A, fill=7.0)
    assert np.array_equal(hz.to_host(kc), k_ref) and np.array_equal(hz.to_host(vc), v_ref)


def test_prompt_then_two_generation_steps_end_to_end():
    """A small GPT through the whole C ABI: packed embedding -> 2 layers on the packed prompt ->
    caches from each layer's QKV stage -> last-token rows -> final LayerNorm -> logits; then two
    generation steps with given next tokens (embedding at the cached position, 2 layers on the
    caches, final LayerNorm, logits).  The oracle recomputes every set of logits from scratch with
    the whole-sequence forward on the extended sequences."""
    dtype = wl.BF16
    V, P, H, nh, d, F, L = 512, 64, 256, 4, 64, 512, 2
    A = nh * d
    rng = np.random.default_rng(12)
    w = wl.Workload("e2e", dtype, L, H, nh, d, F, 4, 24, "uniform", 1, 24)
    lens = np.array([9, 1, 17, 5], dtype=np.int32)
    B, steps = 4, 2
    ids_all = [rng.integers(0, V, lens[b] + steps).astype(np.int32) for b in range(B)]   # prompt + forced tokens
    wte = wl.round_to_dtype(rng.standard_normal((V, H)) * 0.5, dtype)
    wpe = wl.round_to_dtype(rng.standard_normal((P, H)) * 0.1, dtype)
    w_lm = wl.round_to_dtype(rng.standard_normal((V, H)) / np.sqrt(H), dtype)
    lnf_g = wl.round_to_dtype(1 + 0.2 * rng.standard_normal(H), dtype)
    lnf_b = wl.round_to_dtype(0.1 * rng.standard_normal(H), dtype)
    layers = [wl.sample_layer(w, l) for l in range(L)]

    def oracle_logits(cur_lens):
        ids = np.concatenate([ids_all[b][:cur_lens[b]] for b in range(B)])
        xp = orc.embed_packed(ids, cur_lens, wte.astype(np.float64), wpe.astype(np.float64))
        y = orc.stack_forward(orc.unpack(xp, cur_lens, int(cur_lens.max())), cur_lens, layers, nh, d, w.ln_eps)
        last = orc.last_token_rows(orc.pack(y, cur_lens), cur_lens)
        return orc.linear(orc.layer_norm(last, lnf_g.astype(np.float64), lnf_b.astype(np.float64), w.ln_eps),
                          w_lm.astype(np.float64), None)

    # ---- GPU: prompt
    cfg = hz.layer_config(H, nh, d, F, dtype, w.ln_eps)
    dev = [hz.DeviceLayer(p, dtype) for p in layers]
    wted, wped, wlmd, gd, bd = (hz.to_device(a, dtype) for a in (wte, wpe, w_lm, lnf_g, lnf_b))
    T = int(lens.sum())
    S_cap = 32
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32), device="cuda")
    ids_prompt = torch.tensor(np.concatenate([ids_all[b][:lens[b]] for b in range(B)]), device="cuda")
    bufs = [torch.empty((T, H), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    E.energon_embed_packed(ids_prompt, cu, wted, wped, bufs[0])
    ws = torch.empty(E.energon_workspace_bytes(cfg, T), dtype=torch.uint8, device="cuda")
    qkv_off = E.energon_workspace_layout(cfg, T)[E.WS_QKV]
    kc = [torch.zeros((B, S_cap, A), dtype=torch.bfloat16, device="cuda") for _ in range(L)]
    vc = [torch.zeros((B, S_cap, A), dtype=torch.bfloat16, device="cuda") for _ in range(L)]
    for i, layer in enumerate(dev):
        E.energon_layer_forward(cfg, layer.struct, bufs[i & 1], bufs[(i + 1) & 1], T, cu, lens, int(lens.max()), ws)
        qkv = ws[qkv_off: qkv_off + T * 3 * A * 2].view(torch.bfloat16).view(T, 3 * A)
        E.energon_cache_fill(qkv, cu, kc[i], vc[i])
    hidden = bufs[L & 1]
    last = torch.empty((B, H), dtype=torch.bfloat16, device="cuda")
    E.energon_last_token_rows(hidden, cu, last)

    def logits_of(rows):
        normed = torch.empty_like(rows)
        E.energon_layernorm(rows, gd, bd, normed, w.ln_eps)
        out = torch.empty((B, V), dtype=torch.bfloat16, device="cuda")
        E.energon_linear(normed, wlmd, None, None, out, E.EPI_BIAS)
        return hz.to_host(out)

    # embedding (1), L layers, final LayerNorm and logits (2)
    noise = dict(stages=7 * L + 3, logit_rms=recipe_logit_rms(H), attn_stages=L)
    assert_close(logits_of(last), oracle_logits(lens), dtype, "logits after the prompt", **noise)

    # ---- GPU: generation steps with the given next tokens
    cache_lens = torch.tensor(lens, dtype=torch.int32, device="cuda")
    dws = torch.empty(E.energon_decode_workspace_bytes(cfg, B), dtype=torch.uint8, device="cuda")
    xb = [torch.empty((B, H), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    cur = lens.copy()
    for s in range(steps):
        nxt = torch.tensor([ids_all[b][cur[b]] for b in range(B)], dtype=torch.int32, device="cuda")
        E.energon_embed_at(nxt, cache_lens, wted, wped, xb[0])
        for i, layer in enumerate(dev):
            E.energon_decode_layer_forward(cfg, layer.struct, xb[i & 1], xb[(i + 1) & 1], cache_lens, cur, kc[i], vc[i], dws)
        cache_lens += 1
        cur = cur + 1
        assert_close(logits_of(xb[L & 1]), oracle_logits(cur), dtype, f"logits after generation step {s + 1}", **noise)


def test_generation_steps_replayed_from_a_hip_graph():
    """The step reads its lengths from device memory and copies nothing from the host, so a whole
    step (2 layers + advancing the lengths) can be captured once and replayed.  Every replay is
    checked against the same step done eagerly, with eager work between the replays."""
    dtype = wl.BF16
    w = wl.Workload("dec_graph", dtype, 2, 256, 4, 64, 512, 3, 16, "uniform", 0, 16)
    layers = [wl.sample_layer(w, 0), wl.sample_layer(w, 1)]
    dev = [hz.DeviceLayer(p, dtype) for p in layers]
    B, S_cap, A = 3, 16, w.attn_width
    rng = np.random.default_rng(5)
    xs = [hz.to_device(wl.round_to_dtype(rng.standard_normal((B, w.hidden)), dtype), dtype) for _ in range(4)]
    start = np.array([0, 5, 2], dtype=np.int32)

    def fresh():
        st = DecodeState(w, B, S_cap, dev)
        st.lens.copy_(torch.tensor(start, device="cuda"))
        g = torch.Generator(device="cuda").manual_seed(1)
        for i in range(2):
            st.k[i].copy_(torch.randn((B, S_cap, A), device="cuda", generator=g).to(torch.bfloat16))
            st.v[i].copy_(torch.randn((B, S_cap, A), device="cuda", generator=g).to(torch.bfloat16))
        return st

    def body(st, x_in):
        src = x_in
        for i, layer in enumerate(st.layers):
            E.energon_decode_layer_forward(st.cfg, layer.struct, src, st.buf[i & 1], st.lens, None, st.k[i], st.v[i], st.ws)
            src = st.buf[i & 1]
        st.lens += 1
        return src

    eager = fresh()
    want = [body(eager, x).clone() for x in xs]

    st = fresh()
    x_static = torch.empty_like(xs[0])
    x_static.copy_(xs[0])
    side = torch.cuda.Stream()                  # warm-up off the default stream, as capture requires
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        body(st, x_static)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    st = fresh()                                # undo the warm-up's append and length change
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        out_static = body(st, x_static)
    st2_lens_after_capture = st.lens.clone()    # capture itself must not have run the step
    assert torch.equal(st2_lens_after_capture.cpu(), torch.tensor(start))
    for i, x in enumerate(xs):
        x_static.copy_(x)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_static.view(torch.int16), want[i].view(torch.int16)), f"replay {i} differs from eager"
        _ = (xs[0].float() @ xs[0].float().T).sum().item()   # unrelated eager work and a sync between replays
    assert torch.equal(st.lens.cpu(), torch.tensor(start + len(xs)))
    for i in range(2):
        assert torch.equal(st.k[i].view(torch.int16), eager.k[i].view(torch.int16))
        assert torch.equal(st.v[i].view(torch.int16), eager.v[i].view(torch.int16))


def test_decode_layer_batch_above_the_few_row_kernel():
    """96 sequences: more rows than the few-row kernel takes, few enough that the tiled kernel would
    leave most CUs idle; with the step's scratch its K is cut over workgroups (QKV, out-proj, FC1
    and FC2 all qualify at this shape).  Against the oracle, and run-to-run identical."""
    dtype = wl.BF16
    w = wl.Workload("dec_b96", dtype, 1, 2048, 16, 128, 8192, 96, 24, "uniform", 0, 24)
    rng = np.random.default_rng(31)
    B, S_cap, A = 96, 24, w.attn_width
    lens = rng.integers(0, S_cap, B).astype(np.int32)
    p = wl.sample_layer(w, 0)
    kc = wl.round_to_dtype(rng.standard_normal((B, S_cap, A)), dtype)
    vc = wl.round_to_dtype(rng.standard_normal((B, S_cap, A)), dtype)
    x = wl.round_to_dtype(rng.standard_normal((B, w.hidden)), dtype)
    cfg = hz.layer_config(w.hidden, w.n_heads, w.head_dim, w.ffn, dtype, w.ln_eps)
    layer = hz.DeviceLayer(p, dtype)
    ws = torch.empty(E.energon_decode_workspace_bytes(cfg, B), dtype=torch.uint8, device="cuda")
    assert ws.numel() > E.energon_workspace_bytes(cfg, B), "no room for partial sums was planned"
    outs = []
    for _ in range(2):
        xd, kd, vd = (hz.to_device(a, dtype) for a in (x, kc, vc))
        y = torch.empty_like(xd)
        E.energon_decode_layer_forward(cfg, layer.struct, xd, y, torch.tensor(lens, device="cuda"), lens, kd, vd, ws)
        outs.append(y)
    ref, _, _ = orc.decode_layer(x, [(kc[b, :lens[b]], vc[b, :lens[b]]) for b in range(B)], p, w.n_heads, w.head_dim, w.ln_eps)
    assert_close(hz.to_host(outs[0]), ref, dtype, "step at batch 96", **layer_noise(1, math.sqrt(w.hidden) * 0.02))
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))
