#!/usr/bin/env python3
"""Benchmark of the packed (padding-free) transformer-layer forward on one MI355X.

One step = the whole hot path on one synthetic batch: pack (length scan + gather), L layer
forwards on the packed rows, unpack (scatter + zero fill).  Inputs are resident in HBM before
the timed region.  Prints ONE JSON line:
  value      effective (non-pad) tokens/s per layer forward = T * L / step time
  roofline   the bf16 MFMA GEMM kernel (the dominant kernel): algorithmic flops of the four
             GEMMs of a layer / their launch durations, measured with HIP events recorded on
             the launch stream between the stages (energon_layer_forward_profiled)
  padded     the same library run with every position treated as valid (no elimination)
  paper_attention_path  the layer with the attention stage done the paper's way (padded core
             between a rebuild-padding and a remove-padding transpose kernel)
  ln_folded  the same step with both LayerNorms folded into the contractions that follow them
  decode     one generation step (one new token per sequence on cached keys / values of the
             batch's lengths) through the same L layers: bound by streaming the weights and the
             cache from HBM once; algorithmic bytes / time against the HBM peak
  streamed_weights  the same step with the L layers' weights kept in pinned host memory and fetched one
             layer ahead on a second stream (the paper's asynchronous layer prefetch, one-GPU form), next to
             the copies alone: bound by the host link
  hip_graph_replay  the same step recorded once into a HIP graph and replayed: one submission per step
             instead of a launch per kernel (`value` stays the launch-per-kernel figure)
  other_workloads  the tensor-parallel shard and the heavy-padding workload (each packed and padded:
             the speed-up against the row ratio) and the zero-padding control (whole step against the
             layers alone: what pack + unpack cost when there is nothing to remove), a few steps each
  cpu_baseline  the CPU oracle timed on a bounded sample of whole sequences, one layer
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA (fp16: the same)
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
# Bytes per GEMM launch at the L2 -> fabric boundary (mean of the four GEMMs of a layer, the second
# kernels of the two launches that cut tiles included), from the rocprofv3 FETCH_SIZE / WRITE_SIZE
# runs summarised in profiles/bench_gpt13b_bf16_hbm_traffic.md.
GEMM_TRAFFIC_BYTES = {"gpt13b_bf16": 2481e6}


def measure_other_workload(name, steps, warmup, seed, log):
    """Packed and padded step of another workload (fewer steps than the headline): ms/step, effective
    tokens/s per layer, algorithmic TFLOP/s, share of the bf16 MFMA peak, speed-up over the padded path
    against the row ratio; for the padded run also the layers alone (no pack / unpack), which is the
    zero-padding control: every length = S, packing is the identity permutation."""
    import torch
    from paper_2209_02341_amd import binding as E
    from paper_2209_02341_amd import harness as hz
    from paper_2209_02341_amd import workloads as wl

    w = wl.WORKLOADS[name]
    L, H, A, F, B, S = w.layers, w.hidden, w.attn_width, w.ffn, w.batch, w.max_len
    lens = wl.sample_lengths(w, seed)
    T = int(lens.sum())
    x_dev = hz.to_device(wl.sample_x(w, seed), w.dtype)
    dev_layers = [hz.DeviceLayer(wl.sample_layer(w, l, seed), w.dtype) for l in range(L)]
    cfg = hz.layer_config(H, w.n_heads, w.head_dim, F, w.dtype, w.ln_eps)

    def timed(fn, n, nwarm):
        for _ in range(nwarm):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    def flops(lengths):
        t = float(lengths.sum())
        return L * (t * (8.0 * H * A + 4.0 * H * F) + 2.0 * A * float(np.sum(lengths.astype(np.float64) * (lengths + 1))))

    out = {"valid_tokens": T, "rows_padded": B * S, "rows_ratio": B * S / T}
    run = hz.PackedRun(cfg, B, S, T)
    ms = timed(lambda: run.forward(x_dev, lens, dev_layers), steps, warmup)
    stage = {k: 0.0 for k in E.STAGE_NAMES}
    n_prof = 3
    for _ in range(n_prof):
        src, dst = run.x_packed, run.y_packed
        for layer in dev_layers:
            for k, v in E.energon_layer_forward_profiled(cfg, layer.struct, src, dst, T, run.cu, lens, S, run.workspace).items():
                stage[k] += v / (L * n_prof)
            src, dst = dst, src
    tf = flops(lens) / (ms * 1e-3) / 1e12
    # the same step submitted as one HIP graph (what a serving loop would do where a step is a dozen short launches)
    graph = run.capture_forward(x_dev, lens, dev_layers)
    ms_graph = timed(graph.replay, steps, warmup)
    tf_graph = flops(lens) / (ms_graph * 1e-3) / 1e12
    del graph
    out["packed"] = {"ms_per_step": ms, "value": T * L / (ms * 1e-3), "tflops": tf,
                     "pct_bf16_mfma_peak": 100.0 * tf / PEAK_BF16_TFLOPS, "stage_ms_per_layer": stage,
                     "hip_graph_replay": {"ms_per_step": ms_graph, "value": T * L / (ms_graph * 1e-3), "tflops": tf_graph,
                                          "pct_bf16_mfma_peak": 100.0 * tf_graph / PEAK_BF16_TFLOPS}}
    del run
    torch.cuda.empty_cache()
    full = np.full(B, S, dtype=np.int32)
    run_p = hz.PackedRun(cfg, B, S, B * S)
    n_pad = max(2, steps // 2)
    ms_pad = timed(lambda: run_p.forward(x_dev, full, dev_layers), n_pad, 1)

    def layers_only():
        src, bufs = x_dev.view(B * S, H), (run_p.y_packed, run_p.x_packed)
        for i, layer in enumerate(dev_layers):
            E.energon_layer_forward(cfg, layer.struct, src, bufs[i & 1], B * S, run_p.cu, full, S, run_p.workspace)
            src = bufs[i & 1]

    ms_layers = timed(layers_only, n_pad, 1)
    tf_pad = flops(full) / (ms_pad * 1e-3) / 1e12
    out["padded"] = {"ms_per_step": ms_pad, "value": T * L / (ms_pad * 1e-3),
                     "speedup_packed_over_padded": ms_pad / ms}
    out["zero_padding_control"] = {
        "what": "every length = S: pack + layers + unpack against the layers alone on the padded tensor",
        "ms_per_step": ms_pad, "ms_layers_only": ms_layers, "pack_unpack_share": (ms_pad - ms_layers) / ms_pad,
        "tflops": tf_pad, "pct_bf16_mfma_peak": 100.0 * tf_pad / PEAK_BF16_TFLOPS}
    log(f"[bench] {name}: T={T} of {B * S} rows; packed {ms:.3f} ms/step = {tf:.0f} TFLOP/s "
        f"({100.0 * tf / PEAK_BF16_TFLOPS:.1f} %; as one HIP graph {ms_graph:.3f} ms = {100.0 * tf_graph / PEAK_BF16_TFLOPS:.1f} %), padded {ms_pad:.3f} ms -> {ms_pad / ms:.2f}x at row ratio {B * S / T:.2f}; "
        f"control: layers alone {ms_layers:.3f} ms, pack + unpack {100.0 * (ms_pad - ms_layers) / ms_pad:.2f} % of the step")
    del run_p, x_dev, dev_layers
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gpt13b_bf16")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-padded", action="store_true")
    ap.add_argument("--no-paper-path", action="store_true")
    ap.add_argument("--no-ln-folded", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true")
    ap.add_argument("--no-streamed-weights", action="store_true")
    ap.add_argument("--cpu-sample-seqs", type=int, default=16)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2209_02341_amd import binding as E
    from paper_2209_02341_amd import harness as hz
    from paper_2209_02341_amd import workloads as wl

    E.lib()  # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    w = wl.WORKLOADS[args.workload]
    L, H, A, F, B, S = w.layers, w.hidden, w.attn_width, w.ffn, w.batch, w.max_len
    esz = 4 if w.dtype == wl.F32 else 2
    lens = wl.sample_lengths(w, args.seed)
    T = int(lens.sum())
    log = lambda *a: print(*a, file=sys.stderr, flush=True)
    log(f"[bench] workload {w.name}: B={B} S={S} H={H} heads={w.n_heads}x{w.head_dim} F={F} L={L} "
        f"T={T} ({T / (B * S):.1%} valid)")

    x_host = wl.sample_x(w, args.seed)
    x_dev = hz.to_device(x_host, w.dtype)
    host_layers = []
    dev_layers = []
    for l in range(L):
        p = wl.sample_layer(w, l, args.seed)
        dev_layers.append(hz.DeviceLayer(p, w.dtype))
        host_layers.append(p if l == 0 else None)   # the CPU sample uses layer 0 only
    log("[bench] inputs resident on the GPU")
    cfg = hz.layer_config(H, w.n_heads, w.head_dim, F, w.dtype, w.ln_eps)

    def time_steps(run, lengths, steps, warmup, folded=None):
        # wall clock over exactly `steps` steps between two synchronisations; per-step durations from
        # HIP events on the launch stream (for the median and the minimum)
        if folded is not None:
            fwd = lambda: run.forward_folded(x_dev, lengths, folded)
        else:
            fwd = lambda: run.forward(x_dev, lengths, dev_layers)
        for _ in range(warmup):
            fwd()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        marks[0].record()
        for i in range(steps):
            fwd()
            marks[i + 1].record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / steps * 1e3
        per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
        return wall, per_step[len(per_step) // 2], per_step[0]

    run = hz.PackedRun(cfg, B, S, T)
    ms_step, ms_step_median, ms_step_min = time_steps(run, lens, args.steps, args.warmup)
    ms_layer = ms_step / L
    value = T / (ms_layer * 1e-3)
    gemm_flops_layer = T * (8.0 * H * A + 4.0 * H * F)
    # x and W read once, y written once, residual read once (out-proj, FC2)
    gemm_bytes_layer = esz * (T * (H + 3 * A) + 3.0 * A * H + T * (A + 2 * H) + H * A + T * (H + F) + F * H
                              + T * (F + 2 * H) + H * F)
    attn_flops_layer = 2.0 * A * float(np.sum(lens.astype(np.float64) * (lens + 1)))
    flops_layer = gemm_flops_layer + attn_flops_layer
    tflops = flops_layer / (ms_layer * 1e-3) / 1e12
    log(f"[bench] packed: {ms_step:.3f} ms/step (median {ms_step_median:.3f}, min {ms_step_min:.3f}), "
        f"{value:,.0f} tokens/s/layer, {tflops:.1f} TFLOP/s")

    # ---- the same step recorded once into a HIP graph and replayed (one submission per step) ----
    graph = run.capture_forward(x_dev, lens, dev_layers)
    for _ in range(args.warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    ms_graph = (time.perf_counter() - t0) / args.steps * 1e3
    del graph
    log(f"[bench] as one HIP graph per step: {ms_graph:.3f} ms/step")

    # ---- per-stage durations (HIP events on the launch stream), same kernels, same buffers ----
    stage_ms = {k: 0.0 for k in E.STAGE_NAMES}
    n_prof = max(1, min(args.steps, 10))
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    for _ in range(n_prof):
        E.energon_pack(x_dev, lens, run.x_packed, run.cu, run.idx)
        src, dst = run.x_packed, run.y_packed
        for layer in dev_layers:
            ms = E.energon_layer_forward_profiled(cfg, layer.struct, src, dst, T, run.cu, lens, S, run.workspace)
            for k, v in ms.items():
                stage_ms[k] += v
            src, dst = dst, src
        E.energon_unpack(src, run.cu, T, run.y_padded)
    n_layer_calls = n_prof * L
    stage_ms = {k: v / n_layer_calls for k, v in stage_ms.items()}
    # pack and unpack: launches back to back between one pair of events each (a single launch between
    # two events would be timed with the gap that the host needs to submit it)
    n_copy = 10
    torch.cuda.synchronize()
    ev[0].record()
    for _ in range(n_copy):
        E.energon_pack(x_dev, lens, run.x_packed, run.cu, run.idx)
    ev[1].record()
    for _ in range(n_copy):
        E.energon_unpack(run.x_packed, run.cu, T, run.y_padded)
    ev[2].record()
    torch.cuda.synchronize()
    pack_ms = ev[0].elapsed_time(ev[1]) / n_copy
    unpack_ms = ev[1].elapsed_time(ev[2]) / n_copy
    gemm_ms = sum(stage_ms[k] for k in ("qkv", "out", "fc1", "fc2"))
    gemm_tflops = gemm_flops_layer / (gemm_ms * 1e-3) / 1e12
    gbs = lambda nbytes, ms: nbytes / (ms * 1e-3) / 1e9 if ms > 0 else None
    hbm = {
        "pack_GBs": gbs(2.0 * T * H * esz, pack_ms),
        "unpack_GBs": gbs((T + B * S) * H * esz, unpack_ms),
        "layernorm_GBs": gbs(2.0 * T * H * esz * 2, stage_ms["ln1"] + stage_ms["ln2"]),
        "peak_GBs": PEAK_HBM_GBS,
    }
    stage_tflops = {
        "qkv": 2.0 * T * 3 * A * H / (stage_ms["qkv"] * 1e9), "out": 2.0 * T * H * A / (stage_ms["out"] * 1e9),
        "fc1": 2.0 * T * F * H / (stage_ms["fc1"] * 1e9), "fc2": 2.0 * T * H * F / (stage_ms["fc2"] * 1e9),
        "attn": attn_flops_layer / (stage_ms["attn"] * 1e9),
    }
    log(f"[bench] stages (ms/layer): " + ", ".join(f"{k}={v:.3f}" for k, v in stage_ms.items()) +
        f"; pack={pack_ms:.3f} unpack={unpack_ms:.3f}; GEMMs {gemm_tflops:.1f} TFLOP/s")

    # ---- the paper's own attention path (Sec. 4.3): rebuild padding + transpose, padded attention
    # core, remove padding + transpose, in place of the variable-length attention; same other stages ----
    paper_path = None
    if w.dtype != wl.F32 and not args.no_paper_path:
        padws = torch.empty(E.energon_drce_workspace_bytes(cfg, B, S), dtype=torch.uint8, device="cuda")
        acc = {k: 0.0 for k in E.STAGE_NAMES}
        n_rep = max(1, min(args.steps, 5))
        for _ in range(n_rep):
            src, dst = run.x_packed, run.y_packed
            for layer in dev_layers:
                ms = E.energon_layer_forward_drce(cfg, layer.struct, src, dst, T, run.cu, lens, S, run.workspace,
                                                  padws, timed=True)
                for k, v in ms.items():
                    acc[k] += v
                src, dst = dst, src
        acc = {k: v / (n_rep * L) for k, v in acc.items()}
        paper_path = {"attention_stage_ms_per_layer": acc["attn"], "layer_ms": sum(acc.values()),
                      "variable_length_attention_ms_per_layer": stage_ms["attn"],
                      "variable_length_layer_ms": sum(stage_ms.values()),
                      "what": "rebuild padding + head transpose, padded causal attention over all S positions, "
                              "inverse transpose + remove padding"}
        log(f"[bench] paper's attention path: {acc['attn']:.3f} ms/layer for the attention stage "
            f"(variable-length: {stage_ms['attn']:.3f}); layer {sum(acc.values()):.3f} vs {sum(stage_ms.values()):.3f} ms")
        del padws

    # ---- LayerNorm folded into the QKV and FC1 contractions (Sec. 5.5's fusion, algebraic form):
    # same step, folded weights, no normalised activation written, row statistics from the
    # residual epilogues ----
    ln_folded = None
    if w.dtype != wl.F32 and not args.no_ln_folded:
        folded_layers = [hz.FoldedDeviceLayer(d) for d in dev_layers]
        ms_f, ms_f_median, ms_f_min = time_steps(run, lens, args.steps, min(args.warmup, 2), folded=folded_layers)
        ln_folded = {"ms_per_step": ms_f, "ms_per_step_median": ms_f_median, "ms_per_step_min": ms_f_min,
                     "value": T / (ms_f / L * 1e-3), "speedup_over_unfused": ms_step / ms_f,
                     "unfused_layernorm_ms_per_layer": stage_ms["ln1"] + stage_ms["ln2"]}
        log(f"[bench] LayerNorm folded: {ms_f:.3f} ms/step (median {ms_f_median:.3f}) vs {ms_step:.3f} unfused "
            f"({ms_step / ms_f:.3f}x)")
        del folded_layers

    # ---- one generation step on cached keys / values (HBM-bound): every sequence has as many cached
    # tokens as it has valid tokens in the batch above; the lengths are not advanced between the
    # timed steps, so every step does the same work ----
    decode = None
    if w.dtype != wl.F32 and not args.no_decode and B <= 64:
        tdt = x_dev.dtype
        s_cap = S + 8
        kc = [torch.randn((B, s_cap, A), device="cuda", dtype=torch.float32).to(tdt) for _ in range(L)]
        vc = [torch.randn((B, s_cap, A), device="cuda", dtype=torch.float32).to(tdt) for _ in range(L)]
        x_new = x_dev[:, 0].contiguous()
        bufs = [torch.empty_like(x_new) for _ in range(2)]
        lens_d = torch.tensor(lens, dtype=torch.int32, device="cuda")
        dws = torch.empty(E.energon_decode_workspace_bytes(cfg, B), dtype=torch.uint8, device="cuda")

        def decode_step():
            src = x_new
            for i, layer in enumerate(dev_layers):
                E.energon_decode_layer_forward(cfg, layer.struct, src, bufs[i & 1], lens_d, lens if i == 0 else None,
                                               kc[i], vc[i], dws)
                src = bufs[i & 1]

        for _ in range(3):
            decode_step()
        n_dec = max(5, args.steps)
        d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        d0.record()
        for _ in range(n_dec):
            decode_step()
        d1.record()
        torch.cuda.synchronize()
        ms_dec = d0.elapsed_time(d1) / n_dec
        weight_bytes = esz * L * (3.0 * A * H + H * A + 2.0 * F * H)
        kv_bytes = esz * L * 2.0 * A * float(lens.sum())
        decode = {"ms_per_step": ms_dec, "value": B / (ms_dec * 1e-3), "unit": "generated tokens/s (batch of %d)" % B,
                  "layers": L, "cached_tokens": int(lens.sum()),
                  "roofline": {"bound": "hbm", "achieved": (weight_bytes + kv_bytes) / (ms_dec * 1e-3) / 1e9,
                               "peak": PEAK_HBM_GBS, "unit": "GB/s",
                               "frac": (weight_bytes + kv_bytes) / (ms_dec * 1e-3) / 1e9 / PEAK_HBM_GBS,
                               "algorithmic_bytes_per_step": weight_bytes + kv_bytes,
                               "what": "weights read once + cached K and V rows read once"}}
        log(f"[bench] generation step: {ms_dec * 1e3:.0f} us for {L} layers at batch {B} "
            f"({decode['roofline']['achieved']:.0f} GB/s algorithmic, {B / (ms_dec * 1e-3):,.0f} tokens/s)")
        del kc, vc, dws

    # ---- weights streamed from pinned host memory, one layer ahead, on a second stream (Sec. 4.4) ----
    streamed = None
    if w.dtype != wl.F32 and not args.no_streamed_weights:
        pinned = [{k: (None if v is None else v.cpu().pin_memory()) for k, v in d.tensors.items()} for d in dev_layers]
        host_structs = [E.make_weights(p) for p in pinned]
        slot_bytes = E.energon_layer_weights_bytes(cfg)
        slots = [torch.empty(slot_bytes, dtype=torch.uint8, device="cuda") for _ in range(2)]
        copy_stream = torch.cuda.Stream()

        def streamed_step():
            E.energon_pack(x_dev, lens, run.x_packed, run.cu, run.idx)
            E.energon_stack_forward_streamed(cfg, host_structs, run.x_packed, T, run.cu, lens, S, run.workspace,
                                             slots[0], slots[1], copy_stream.cuda_stream)
            E.energon_unpack(run.x_packed, run.cu, T, run.y_padded)

        def copies_only():
            with torch.cuda.stream(copy_stream):
                for i, p in enumerate(pinned):
                    for k, v in p.items():
                        if v is not None:
                            dev_layers[i].tensors[k].copy_(v, non_blocking=True)

        def timed_ms(fn, n):
            fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / n * 1e3

        n_s = max(2, min(args.steps, 4))
        ms_streamed = timed_ms(streamed_step, n_s)
        ms_copies = timed_ms(copies_only, n_s)
        wbytes = float(slot_bytes) * L
        # copy-bound here: the pipeline's floor is all the copies plus the last layer's compute, which nothing follows
        ms_floor = ms_copies + ms_step / L
        streamed = {"ms_per_step": ms_streamed, "ms_copies_alone": ms_copies, "ms_resident_weights": ms_step,
                    "ms_one_after_the_other": ms_copies + ms_step, "ms_pipeline_floor": ms_floor,
                    "weight_bytes_per_step": wbytes, "host_link_GBs": wbytes / (ms_copies * 1e-3) / 1e9,
                    "what": "layer l+1's weights copied host-pinned -> device on a second stream while layer l computes"}
        log(f"[bench] weights streamed from pinned host memory: {ms_streamed:.2f} ms/step; copies alone {ms_copies:.2f} ms "
            f"({streamed['host_link_GBs']:.1f} GB/s), resident weights {ms_step:.2f} ms; one after the other "
            f"{ms_copies + ms_step:.2f} ms, floor of the pipeline {ms_floor:.2f} ms")
        del pinned, host_structs, slots

    # ---- padded (no-elimination) path: same library, every position valid ----
    padded = None
    if not args.no_padded:
        full = np.full(B, S, dtype=np.int32)
        del run
        torch.cuda.empty_cache()
        run_p = hz.PackedRun(cfg, B, S, B * S)
        ms_pad, _, _ = time_steps(run_p, full, max(2, args.steps // 2), min(args.warmup, 2))
        padded = {"ms_per_step": ms_pad, "value": T / (ms_pad / L * 1e-3), "rows": B * S,
                  "speedup_packed_over_padded": ms_pad / ms_step, "rows_ratio": B * S / T}
        log(f"[bench] padded: {ms_pad:.3f} ms/step -> packed is {ms_pad / ms_step:.2f}x faster "
            f"(row ratio {B * S / T:.2f})")
        del run_p
        torch.cuda.empty_cache()

    # ---- the other large workloads: tensor-parallel shard, heavy padding, zero-padding control ----
    others = None
    if not args.no_other_workloads and args.workload == "gpt13b_bf16":
        del x_dev, dev_layers
        torch.cuda.empty_cache()
        others = {name: measure_other_workload(name, max(3, args.steps // 4), 2, args.seed, log)
                  for name in ("gpt175b_tp8_shard_bf16", "heavy_pad_bf16")}

    # ---- CPU oracle on a bounded sample: whole sequences near the median length, one layer ----
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import energon_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            threads = max([d.get("num_threads", 1) for d in threadpool_info()] or [1])
        except Exception:
            threads = os.cpu_count()
        order = np.argsort(np.abs(lens - np.median(lens)))
        picks = np.sort(order[: args.cpu_sample_seqs])
        sub_len = lens[picks]
        s_sub = int(sub_len.max())
        t0 = time.perf_counter()
        orc.stack_forward(x_host[picks][:, :s_sub], sub_len, [host_layers[0]], w.n_heads, w.head_dim, w.ln_eps)
        dt = time.perf_counter() - t0
        cpu = {"value": float(sub_len.sum()) / dt, "unit": "tokens/s per layer forward", "cores": int(threads),
               "kind": "oracle", "seconds": dt,
               "sample": f"{len(picks)} whole sequences nearest the median length "
                         f"({int(sub_len.sum())} valid tokens, padded to {s_sub}), one layer at full layer shape, "
                         f"NumPy fp64"}
        log(f"[bench] cpu oracle sample: {dt:.1f} s -> {cpu['value']:.1f} tokens/s/layer on {threads} threads")

    out = {
        "metric": "effective (non-pad) tokens/s per layer forward",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "ms_per_step_median": ms_step_median, "ms_per_step_min": ms_step_min,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "layers": L, "hidden": H, "heads": w.n_heads, "head_dim": w.head_dim,
                   "ffn": F, "batch": B, "max_len": S, "valid_tokens": T, "valid_fraction": T / (B * S),
                   "step": "pack + L x layer_forward + unpack"},
        "ms_per_layer": ms_layer, "tflops": tflops, "pct_bf16_mfma_peak": 100.0 * tflops / PEAK_BF16_TFLOPS,
        "roofline": {"bound": "mfma", "kernel": "gemm_mfma_sched_kernel", "achieved": gemm_tflops,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": gemm_tflops / PEAK_BF16_TFLOPS,
                     "traffic": GEMM_TRAFFIC_BYTES.get(w.name),
                     "algorithmic_bytes_per_launch": gemm_bytes_layer / 4,
                     "launches_per_layer": 4, "avg_launch_ms": gemm_ms / 4,
                     "flops_per_launch": gemm_flops_layer / 4},
        "stage_ms_per_layer": stage_ms, "stage_tflops": stage_tflops,
        "pack_ms": pack_ms, "unpack_ms": unpack_ms, "hbm": hbm,
        "padded": padded, "paper_attention_path": paper_path, "ln_folded": ln_folded, "decode": decode,
        "hip_graph_replay": {"ms_per_step": ms_graph, "value": T * L / (ms_graph * 1e-3)},
        "streamed_weights": streamed, "other_workloads": others, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
