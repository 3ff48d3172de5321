"""A whole step of the padding-free path (pack, the layers, unpack; Sec. 4.3) recorded into a HIP graph and
replayed: the path enqueues kernels only, so a serving loop can submit a step with one call.  Every replay,
on new input contents and with unrelated eager work and a synchronisation between replays, must equal the
eager step bit for bit; one replay is also compared with the oracle."""
import numpy as np
import pytest
import torch

from oracle import energon_oracle as orc
from paper_2209_02341_amd import harness as hz
from paper_2209_02341_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["small_bf16", "small_f16"])
def test_step_replayed_from_a_hip_graph(name):
    w = wl.WORKLOADS[name]
    lens = wl.sample_lengths(w, 3)
    lens[1] = 0                                   # an empty sequence inside the batch
    T = int(lens.sum())
    layers = [wl.sample_layer(w, l, 3) for l in range(2)]
    dev = [hz.DeviceLayer(p, w.dtype) for p in layers]
    cfg = hz.layer_config(w.hidden, w.n_heads, w.head_dim, w.ffn, w.dtype, w.ln_eps)
    xs = [wl.sample_x(w, 10 + i) for i in range(3)]
    xs_dev = [hz.to_device(x, w.dtype) for x in xs]

    eager = hz.PackedRun(cfg, w.batch, w.max_len, T)
    want = [eager.forward(x, lens, dev).clone() for x in xs_dev]

    run = hz.PackedRun(cfg, w.batch, w.max_len, T)
    x_static = torch.empty_like(xs_dev[0])
    x_static.copy_(xs_dev[0])
    graph = run.capture_forward(x_static, lens, dev)
    bits = torch.int16
    for i, x in enumerate(xs_dev):
        x_static.copy_(x)
        run.y_padded.fill_(7.0)                   # a replay must rewrite every element, pads included
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(run.y_padded.view(bits), want[i].view(bits)), f"replay {i} differs from the eager step"
        _ = (xs_dev[0].float().sum() * 2).item()  # unrelated eager work and a sync between replays

    # and the last replay against the oracle, at the tolerance of the layer tests
    ref = orc.stack_forward(xs[-1], lens, layers, w.n_heads, w.head_dim, w.ln_eps)
    got = hz.to_host(run.y_padded).astype(np.float64)
    tol = {wl.BF16: 1e-2, wl.F16: 2.5e-3}[w.dtype]
    assert np.abs(got - ref).max() <= 2 * tol * np.abs(ref).max()   # two layers
    pad = np.arange(w.max_len)[None, :] >= lens[:, None]
    assert np.all(got[pad] == 0.0)
