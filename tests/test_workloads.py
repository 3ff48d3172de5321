"""Seeded input generators: shapes, ranges, bf16 rounding and the parameter count the
paper quotes for one GPT-3 layer (Sec. 4.4: 1.812e9 parameters at hidden 12288)."""
import numpy as np
import torch

from paper_2209_02341_amd import workloads as wl


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(4096).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38], np.float32)])
    bits = wl.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), ref.view(torch.int16).numpy())
    assert np.array_equal(wl.bf16_bits_to_f32(bits), ref.float().numpy())


def test_lengths_in_range_and_reproducible():
    for w in wl.WORKLOADS.values():
        a, b = wl.sample_lengths(w, 0), wl.sample_lengths(w, 0)
        assert np.array_equal(a, b) and a.dtype == np.int32 and a.shape == (w.batch,)
        assert a.min() >= w.len_lo and a.max() <= w.len_hi <= w.max_len
    assert np.all(wl.sample_lengths(wl.WORKLOADS["heavy_pad_control_bf16"]) == 2048)
    frac = wl.sample_lengths(wl.WORKLOADS["heavy_pad_bf16"]).sum() / (64 * 2048)
    assert 0.08 < frac < 0.25          # "about 85 % padding"


def test_shard_parameter_count():
    w = wl.WORKLOADS["gpt175b_tp8_shard_bf16"]
    per_shard = 4 * w.hidden * w.attn_width + 2 * w.hidden * w.ffn
    assert abs(per_shard * 8 - 1.812e9) / 1.812e9 < 1e-3


def test_small_workload_tensors():
    w = wl.WORKLOADS["tiny_f32"]
    x = wl.sample_x(w, 0)
    assert x.shape == (4, 32, 256) and x.dtype == np.float32
    assert np.array_equal(wl.sample_x(w, 0, seqs=[2])[0], x[2])
    p = wl.sample_layer(w, 0)
    assert p["w_qkv"].shape == (768, 256) and p["w_fc2"].shape == (256, 1024)
    assert abs(p["w_fc1"].std() - 0.02) < 2e-3 and np.all(p["ln1_g"] == 1)
    w2 = wl.WORKLOADS["small_bf16"]
    q = wl.sample_layer(w2, 0)["w_o"]
    assert np.array_equal(q, wl.round_to_dtype(q, wl.BF16))
