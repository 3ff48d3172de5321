"""Device-side plumbing shared by the GPU tests, the smoke check and the benchmark:
uploading a synthetic workload, allocating the buffers the C ABI wants, and calling
pack -> L x layer_forward -> unpack.  torch is used for device memory only."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as E
from . import workloads as wl


def to_device(a: np.ndarray | None, dtype: str, device="cuda"):
    """fp32 host array (already rounded to `dtype`) -> device tensor of that dtype."""
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == wl.BF16:
        bits = wl.f32_to_bf16_bits(a)
        return torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16)
    if dtype == wl.F16:
        return torch.from_numpy(a.astype(np.float16)).to(device)
    return torch.from_numpy(a).to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    """device tensor -> fp64 host array (exact)."""
    return t.detach().float().cpu().numpy().astype(np.float64)


def layer_config(hidden, n_heads, head_dim, ffn, dtype: str, eps=1e-5) -> E.LayerConfig:
    code = {wl.BF16: E.BF16, wl.F16: E.F16, wl.F32: E.F32}[dtype]
    return E.LayerConfig(hidden, n_heads, head_dim, ffn, eps, code)


class DeviceLayer:
    """One layer's parameters on the device plus the pointer struct handed to the library."""

    def __init__(self, params: dict, dtype: str, device="cuda"):
        self.tensors = {k: to_device(v, dtype, device) for k, v in params.items()}
        self.struct = E.make_weights(self.tensors)


class FoldedDeviceLayer:
    """A DeviceLayer with both LayerNorms folded into the linears that follow them, by the
    library's own fold kernel; the struct is what energon_layer_forward_ln_folded takes."""

    def __init__(self, layer: DeviceLayer):
        t = layer.tensors
        self.tensors = {k: t.get(k) for k in ("w_o", "b_o", "w_fc2", "b_fc2")}
        for name, w, b, g, beta in (("qkv", "w_qkv", "b_qkv", "ln1_g", "ln1_b"),
                                    ("fc1", "w_fc1", "b_fc1", "ln2_g", "ln2_b")):
            N = t[w].shape[0]
            wf = torch.empty_like(t[w])
            c = torch.empty(N, dtype=torch.float32, device=wf.device)
            bf = torch.empty(N, dtype=torch.float32, device=wf.device)
            E.energon_fold_layernorm(t[w], t.get(b), t[g], t[beta], wf, c, bf)
            self.tensors["wf_" + name], self.tensors["c_" + name], self.tensors["bf_" + name] = wf, c, bf
        self.struct = E.make_folded_weights(self.tensors)


class PackedRun:
    """Buffers for one batch: packed activations (ping/pong), cu_seqlens, token_idx, workspace."""

    def __init__(self, cfg: E.LayerConfig, B: int, S: int, capacity_tokens: int, device="cuda"):
        tdt = {E.BF16: torch.bfloat16, E.F16: torch.float16, E.F32: torch.float32}[cfg.dtype]
        cap = max(int(capacity_tokens), 1)
        self.cfg, self.B, self.S = cfg, B, S
        self.x_packed = torch.empty((cap, cfg.hidden), dtype=tdt, device=device)
        self.y_packed = torch.empty((cap, cfg.hidden), dtype=tdt, device=device)
        self.cu = torch.empty(B + 1, dtype=torch.int32, device=device)
        self.idx = torch.empty(cap, dtype=torch.int32, device=device)
        self.ws_bytes = E.energon_workspace_bytes(cfg, cap)
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)
        self.y_padded = torch.empty((B, S, cfg.hidden), dtype=tdt, device=device)
        self.T = 0

    def forward(self, x_padded: torch.Tensor, lengths: np.ndarray, layers: list) -> torch.Tensor:
        """pack once, every layer on the packed rows, unpack once; returns y_padded."""
        cfg = self.cfg
        self.T = T = E.energon_pack(x_padded, lengths, self.x_packed, self.cu, self.idx)
        src, dst = self.x_packed, self.y_packed
        for layer in layers:
            E.energon_layer_forward(cfg, layer.struct, src, dst, T, self.cu, lengths, self.S, self.workspace)
            src, dst = dst, src
        self.last_packed = src
        E.energon_unpack(src, self.cu, T, self.y_padded)
        return self.y_padded

    def capture_forward(self, x_padded: torch.Tensor, lengths: np.ndarray, layers: list) -> "torch.cuda.CUDAGraph":
        """forward() recorded once into a HIP graph: replay() reruns pack, the layers and unpack on whatever
        x_padded holds then, for the SAME lengths (they are part of the pack launch's arguments), and
        leaves the result in y_padded.  The path enqueues kernels only (batches of up to 896 sequences), so
        nothing in it is refused by a capture.  One eager run on a side stream first: what the library sets
        once per process (kernel attributes) must not happen inside the capture."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            self.forward(x_padded, lengths, layers)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.forward(x_padded, lengths, layers)
        return graph

    def forward_folded(self, x_padded: torch.Tensor, lengths: np.ndarray, layers: list) -> torch.Tensor:
        """forward() on FoldedDeviceLayers: the first layer takes its row statistics itself, every
        later one gets them from the epilogue of the layer before."""
        cfg = self.cfg
        self.T = T = E.energon_pack(x_padded, lengths, self.x_packed, self.cu, self.idx)
        if not hasattr(self, "stats"):
            cap = self.x_packed.shape[0]
            self.stats = [torch.empty((cap, 2), dtype=torch.float32, device=self.x_packed.device) for _ in range(2)]
        src, dst = self.x_packed, self.y_packed
        for i, layer in enumerate(layers):
            E.energon_layer_forward_ln_folded(cfg, layer.struct, src, dst, T, self.cu, lengths, self.S,
                                              self.workspace, stats_in=self.stats[i & 1] if i else None,
                                              stats_out=self.stats[(i + 1) & 1] if i + 1 < len(layers) else None)
            src, dst = dst, src
        self.last_packed = src
        E.energon_unpack(src, self.cu, T, self.y_padded)
        return self.y_padded

    def stage(self, which: int, cols: int) -> torch.Tensor:
        """View of one intermediate of the last layer run, [T, cols]."""
        off = E.energon_workspace_layout(self.cfg, self.T)[which]
        esz = self.x_packed.element_size()
        flat = self.workspace[off: off + self.T * cols * esz]
        return flat.view(self.x_packed.dtype).view(self.T, cols)
