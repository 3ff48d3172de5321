"""GPU parity of the paper's own attention path (Sec. 4.3): rebuild padding + head transpose,
padded attention core, inverse transpose + remove padding; each through the C ABI against the
oracle.  The two layout kernels are bit-exact; the attention core is held to the bf16 bar."""
import numpy as np
import pytest
import torch

from oracle import energon_oracle as orc
from paper_2209_02341_amd import binding as E
from paper_2209_02341_amd import harness as hz
from paper_2209_02341_amd import workloads as wl
from test_gpu_parity import assert_close, layer_noise, recipe_logit_rms

pytestmark = pytest.mark.gpu

CASES = [
    # lengths, S, nh, d
    ([5, 0, 1, 64, 65, 130], 130, 2, 64), ([128, 16, 77], 128, 3, 128), ([300, 7], 320, 1, 128),
    ([0, 0], 9, 2, 64), ([513, 200, 128, 127], 640, 2, 128), ([17], 17, 5, 64),
]


def _bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy()


@pytest.mark.parametrize("lengths,S,nh,d", CASES)
def test_rebuild_and_remove_are_bit_exact(lengths, S, nh, d):
    lens = np.asarray(lengths, dtype=np.int32)
    B, T, A = len(lens), int(lens.sum()), nh * d
    rng = np.random.default_rng(S + nh)
    qkv = wl.round_to_dtype(rng.standard_normal((max(T, 1), 3 * A)), wl.BF16)[:T]
    cu_ref, _ = orc.pack_indices(lens, S)
    qd = hz.to_device(qkv if T else np.zeros((1, 3 * A), np.float32), wl.BF16)[:T]
    cud = torch.from_numpy(cu_ref).cuda()
    pads = [torch.full((B, nh, S, d), 9.0, dtype=torch.bfloat16, device="cuda") for _ in range(3)]
    E.energon_rebuild_qkv(qd, cud, B, S, nh, d, *pads)
    ref = orc.rebuild_qkv_heads(qkv, lens, S, nh, d)
    for got, want in zip(pads, ref):
        assert np.array_equal(_bits(got), _bits(torch.from_numpy(want.astype(np.float32)).to(torch.bfloat16)))
    # inverse transpose + remove padding, on a tensor with non-zero pads (they must not be read into the result)
    o = torch.randn((B, nh, S, d), generator=torch.Generator().manual_seed(3)).to(torch.bfloat16).cuda()
    out = torch.full((T + 1, A), 4.0, dtype=torch.bfloat16, device="cuda")
    E.energon_remove_attn_padding(o, cud, out[:T])
    want = orc.remove_padding_heads(o.float().cpu().numpy(), lens)
    assert np.array_equal(_bits(out[:T]), _bits(torch.from_numpy(want.astype(np.float32)).to(torch.bfloat16)))
    assert torch.all(out[T] == 4.0)


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F16])
@pytest.mark.parametrize("lengths,S,nh,d", CASES)
def test_padded_attention_core(lengths, S, nh, d, dtype):
    lens = np.asarray(lengths, dtype=np.int32)
    B, T, A = len(lens), int(lens.sum()), nh * d
    rng = np.random.default_rng(S * 7 + d)
    qkv = wl.round_to_dtype(rng.standard_normal((T, 3 * A)), dtype)
    q, k, v = orc.rebuild_qkv_heads(qkv, lens, S, nh, d)
    cu_ref, _ = orc.pack_indices(lens, S)
    cud = torch.from_numpy(cu_ref).cuda()
    qd, kd, vd = (hz.to_device(a, dtype) for a in (q, k, v))
    od = torch.full((B, nh, S, d), 5.0, dtype=qd.dtype, device="cuda")
    E.energon_attention_padded(qd, kd, vd, cud, od)
    got = hz.to_host(od)
    ref = orc.padded_attention_heads(q, k, v, lens)
    assert_close(got, ref, dtype, "padded attention", stages=2)   # all S positions, pad queries included
    for b in range(B):
        if lens[b] == 0:
            assert not got[b].any()


@pytest.mark.parametrize("name", ["small_bf16", "small_f16"])
def test_drce_layer_equals_oracle_and_variable_length_layer(name):
    w = wl.WORKLOADS[name]
    lens, x, layers = wl.sample_lengths(w), wl.sample_x(w), [wl.sample_layer(w, 0)]
    lens = lens.copy(); lens[1] = 0
    cfg = hz.layer_config(w.hidden, w.n_heads, w.head_dim, w.ffn, w.dtype, w.ln_eps)
    B, S, T = w.batch, w.max_len, int(lens.sum())
    run = hz.PackedRun(cfg, B, S, T)
    layer = hz.DeviceLayer(layers[0], w.dtype)
    xd = hz.to_device(x, w.dtype)
    assert E.energon_pack(xd, lens, run.x_packed, run.cu, run.idx) == T
    E.energon_layer_forward(cfg, layer.struct, run.x_packed, run.y_packed, T, run.cu, lens, S, run.workspace)
    y_var = run.y_packed.clone()
    padws = torch.empty(E.energon_drce_workspace_bytes(cfg, B, S), dtype=torch.uint8, device="cuda")
    ms = E.energon_layer_forward_drce(cfg, layer.struct, run.x_packed, run.y_packed, T, run.cu, lens, S,
                                      run.workspace, padws, timed=True)
    assert set(ms) == set(E.STAGE_NAMES) and all(v >= 0 for v in ms.values())
    E.energon_layer_forward_drce(cfg, layer.struct, run.x_packed, run.y_packed, T, run.cu, lens, S, run.workspace, padws)
    torch.cuda.synchronize()
    ref = orc.pack(orc.stack_forward(x, lens, layers, w.n_heads, w.head_dim, w.ln_eps), lens)
    noise = layer_noise(1, recipe_logit_rms(w.hidden))
    assert_close(hz.to_host(run.y_packed), ref, w.dtype, "drce layer vs oracle", **noise)
    # two GPU results that share everything up to the attention stage: its two roundings and the four stages after it, twice
    assert_close(hz.to_host(run.y_packed), hz.to_host(y_var).astype(np.float64), w.dtype, "drce vs variable-length",
                 tol=4e-3 if w.dtype == wl.BF16 else 1e-3, stages=12)
