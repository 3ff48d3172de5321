"""A stack whose weights stay in pinned host memory and reach the GPU one layer ahead of their use, on a
second stream (the one-GPU form of the paper's asynchronous layer prefetch, Sec. 4.4): the result must be
bit-identical to the same stack on resident weights, and match the oracle."""
import numpy as np
import pytest
import torch

from oracle import energon_oracle as orc
from paper_2209_02341_amd import binding as E
from paper_2209_02341_amd import harness as hz
from paper_2209_02341_amd import workloads as wl
from test_gpu_parity import assert_close, layer_noise, recipe_logit_rms

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.contiguous().view(torch.int16)


@pytest.mark.parametrize("name,L,bias", [("small_bf16", 3, True), ("small_f16", 2, True), ("small_bf16", 1, False)])
def test_streamed_stack_equals_resident_stack_and_oracle(name, L, bias):
    base = wl.WORKLOADS[name]
    w = wl.Workload("streamed", base.dtype, L, base.hidden, base.n_heads, base.head_dim, base.ffn, base.batch,
                    base.max_len, "uniform", 0, base.max_len)
    lens = np.array([base.max_len, 0, 17, 1, 64, 33, 128, 5][: base.batch], dtype=np.int32)
    x = wl.sample_x(w)
    layers = [wl.sample_layer(w, l) for l in range(L)]
    if not bias:
        for p in layers:
            p["b_o"] = None
            p["b_fc2"] = None
    cfg = hz.layer_config(w.hidden, w.n_heads, w.head_dim, w.ffn, w.dtype, w.ln_eps)
    T = int(lens.sum())
    run = hz.PackedRun(cfg, w.batch, w.max_len, T)
    xd = hz.to_device(x, w.dtype)
    # resident weights, every layer in place
    dev_layers = [hz.DeviceLayer(p, w.dtype) for p in layers]
    assert E.energon_pack(xd, lens, run.x_packed, run.cu, run.idx) == T
    for layer in dev_layers:
        E.energon_layer_forward(cfg, layer.struct, run.x_packed, run.x_packed, T, run.cu, lens, w.max_len, run.workspace)
    resident = run.x_packed.clone()
    # the same weights in pinned host memory
    host_layers, keep = [], []
    for layer in dev_layers:
        pinned = {k: (None if v is None else v.cpu().pin_memory()) for k, v in layer.tensors.items()}
        keep.append(pinned)
        host_layers.append(E.make_weights(pinned))
    nbytes = E.energon_layer_weights_bytes(cfg)
    slots = [torch.full((nbytes,), 0x5a, dtype=torch.uint8, device="cuda") for _ in range(2)]
    copy_stream = torch.cuda.Stream()
    for _ in range(2):   # twice: the second call starts while the slots still hold the last layers
        assert E.energon_pack(xd, lens, run.x_packed, run.cu, run.idx) == T
        E.energon_stack_forward_streamed(cfg, host_layers, run.x_packed, T, run.cu, lens, w.max_len, run.workspace,
                                         slots[0], slots[1], copy_stream.cuda_stream)
        torch.cuda.synchronize()
        assert torch.equal(_bits(run.x_packed[:T]), _bits(resident[:T]))
    ref = orc.pack(orc.stack_forward(x, lens, layers, w.n_heads, w.head_dim, w.ln_eps), lens)
    assert_close(hz.to_host(run.x_packed[:T]), ref, w.dtype, f"streamed stack of {L}",
                 **layer_noise(L, recipe_logit_rms(w.hidden)))


def test_streamed_stack_rejects_bad_arguments():
    w = wl.WORKLOADS["small_bf16"]
    cfg = hz.layer_config(w.hidden, w.n_heads, w.head_dim, w.ffn, w.dtype, w.ln_eps)
    lens = np.array([4] * w.batch, dtype=np.int32)
    T = int(lens.sum())
    run = hz.PackedRun(cfg, w.batch, w.max_len, T)
    layer = hz.DeviceLayer(wl.sample_layer(w, 0), w.dtype)
    host = E.make_weights({k: (None if v is None else v.cpu().pin_memory()) for k, v in layer.tensors.items()})
    nbytes = E.energon_layer_weights_bytes(cfg)
    slots = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(2)]
    cs = torch.cuda.Stream()
    cur = torch.cuda.current_stream().cuda_stream
    with pytest.raises(E.EnergonError) as e:   # one stream for both: nothing could overlap
        E.energon_stack_forward_streamed(cfg, [host], run.x_packed, T, run.cu, lens, w.max_len, run.workspace, slots[0],
                                         slots[1], cur, stream=cur)
    assert e.value.status == -6
    with pytest.raises(E.EnergonError) as e:
        E.energon_stack_forward_streamed(cfg, [host], run.x_packed, T, run.cu, lens, w.max_len, run.workspace,
                                         slots[0][:nbytes - 256], slots[1], cs.cuda_stream)
    assert e.value.status == -4
    with pytest.raises(E.EnergonError) as e:
        E.energon_stack_forward_streamed(cfg, [host], run.x_packed, T, run.cu, lens, w.max_len, run.workspace, slots[0],
                                         slots[0], cs.cuda_stream)
    assert e.value.status == -5
