"""Per-layer cost table and layer-wise plan: the model-profiler / discovery-phase part of the
strategy selector (paper, section 3 "Model Profiler" and "Dynamic Strategy Selector"), built on
what this library can measure on one GPU.

A strategy for a layer is a pair (tp_attn, tp_ffn) of tensor-parallel degrees on a group of
`gpus` devices; the rest of the group is data parallel, so with a global batch of `global_batch`
samples per step a tensor-parallel group of degree d handles ``global_batch * d / gpus`` samples.
For every candidate the table holds, per GPU:

  compute   gx_layer_fwd + gx_layer_bwd of the attention half at its micro-batch and of the
            feed-forward half at its micro-batch, timed on the GPU (single-phase calls), or, without
            a GPU, model FLOPs over an assumed rate;
  memory    optimizer and parameter state (gx_strategy_cost) + the activations the forward pass
            keeps (gx_layer_saved_bytes, exact);
  comm      gx_strategy_cost's ring model, NOT measured (one GPU here), at `link_gbps`.

Shard sizes, state bytes, communication and hand-over times and FLOP counts are computed by the
library (gx_strategy_cost, checked against a plain definition in the tests); this module only
applies the candidate rules, times the kernels and marshals the table into gx_plan_search.
The communication model, the candidate rules and the objective are this repository's reading: the
paper names the search but prints no cost model.
"""
from __future__ import annotations

import argparse
import json
from dataclasses import dataclass

from . import binding as gx
from .inputs import LayerShape


@dataclass(frozen=True)
class Model:
    hidden: int
    heads: int
    ffn: int
    seq: int
    layers: int
    dtype: str = "bf16"


def candidates(model: Model, gpus: int, global_batch: int):
    """Decision rules that build the candidate set: power-of-two degrees that divide the group,
    the heads (attention) or the FFN width, and leave every data-parallel replica at least one
    whole sample (global_batch * d / gpus an integer >= 1)."""
    def ok(d, width):
        return gpus % d == 0 and width % d == 0 and (global_batch * d) % gpus == 0 and global_batch * d >= gpus
    degs = [d for d in (1, 2, 4, 8, 16, 32, 64) if d <= gpus]
    return [(a, f) for a in degs if ok(a, model.heads) for f in degs if ok(f, model.ffn)]


def measure_half(model: Model, degree: int, micro_batch: int, phase: str, reps: int = 5):
    """Milliseconds of gx_layer_fwd + gx_layer_bwd of one half at one shard shape, on cuda:0."""
    import torch
    from .inputs import rank_params, activations
    from .runtime import DeviceLayer, to_device
    shape = LayerShape(model.hidden, model.heads, model.ffn, degree if phase == "attn" else 1,
                       degree if phase == "mlp" else 1, 0, model.seq, micro_batch, model.dtype)
    layer = DeviceLayer(shape, rank_params(shape, case=60))
    x, dy = (to_device(t, model.dtype) for t in activations(shape, case=60))

    def once():
        layer.forward(x, phase)
        layer.backward(x, dy, phase)
    once()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        once()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def cost_table(model: Model, gpus: int, global_batch: int, link_gbps: float = 150.0, measure: bool = True,
               assumed_tflops: float = 900.0):
    """One row per candidate strategy: times in ms per step per layer, memory in bytes per GPU.
    Sizes, communication times and FLOP counts come from gx_strategy_cost; compute times are
    measured here (or, with measure=False, FLOPs over an assumed rate)."""
    dt = gx.GX_BF16 if model.dtype == "bf16" else gx.GX_F32
    cache = {}

    def half(phase, d, mb, flops):
        key = (phase, d)
        if key not in cache:
            cfg = gx.make_cfg(model.hidden, model.heads, model.ffn, d if phase == "attn" else 1,
                              d if phase == "mlp" else 1, 0, model.seq, mb, dt,
                              gx.GX_PHASE_ATTN if phase == "attn" else gx.GX_PHASE_MLP)
            if gx.layer_validate(cfg) != gx.GX_OK:
                cache[key] = None
            else:
                ms = measure_half(model, d, mb, phase) if measure else flops / (assumed_tflops * 1e9)
                cache[key] = dict(compute_ms=ms, saved_bytes=gx.layer_saved_bytes(cfg))
        return cache[key]

    rows = []
    for a, f in candidates(model, gpus, global_batch):
        st, c = gx.strategy_cost(model.hidden, model.heads, model.ffn, model.seq, dt, gpus, global_batch, a, f,
                                 link_gbps, check=False)
        if st != gx.GX_OK:
            continue
        ha = half("attn", a, c.micro_batch_attn, c.flops_attn)
        hf = half("mlp", f, c.micro_batch_ffn, c.flops_ffn)
        if ha is None or hf is None:
            continue
        compute = ha["compute_ms"] + hf["compute_ms"]
        comm = c.tp_comm_ms + c.dp_comm_ms
        saved = ha["saved_bytes"] + hf["saved_bytes"]
        rows.append(dict(tp_attn=a, tp_ffn=f, micro_batch_attn=c.micro_batch_attn, micro_batch_ffn=c.micro_batch_ffn,
                         compute_ms=compute, comm_ms=comm, time_ms=compute + comm, switch_ms=c.switch_ms,
                         tflops_per_gpu=(c.flops_attn + c.flops_ffn) / (compute * 1e9),
                         state_bytes=c.state_bytes, saved_bytes=saved, mem_bytes=c.state_bytes + saved))
    return rows


def switch_table(rows):
    """Cost of handing a layer's output to the next layer: the strategy's switch_ms when this
    layer's feed-forward degree differs from the next layer's attention degree, else 0."""
    return [[0.0 if r1["tp_ffn"] == r2["tp_attn"] or r1 is r2 else r1["switch_ms"] for r2 in rows] for r1 in rows]


def plan(model: Model, rows, gpus: int, global_batch: int, budget_bytes: float, link_gbps: float = 150.0,
         quantum_bytes: float = 64 * 2 ** 20):
    """gx_plan_search over identical layers; returns (status, per-layer rows, result)."""
    time = [[r["time_ms"] for r in rows]] * model.layers
    mem = [[float(r["mem_bytes"]) for r in rows]] * model.layers
    sw = switch_table(rows)
    st, choice, res = gx.plan_search(time, mem, sw, budget=budget_bytes, quantum=quantum_bytes, check=False)
    return st, [rows[c] for c in choice] if st == gx.GX_OK else [], res


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--hidden", type=int, default=4096)
    ap.add_argument("--heads", type=int, default=32)
    ap.add_argument("--ffn", type=int, default=16384)
    ap.add_argument("--seq", type=int, default=2048)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--gpus", type=int, default=8, help="size of the tensor x data parallel group being planned")
    ap.add_argument("--global-batch", type=int, default=16)
    ap.add_argument("--budget-gib", type=float, default=200.0, help="memory per GPU available to the layers")
    ap.add_argument("--link-gbps", type=float, default=150.0, help="per-link bandwidth of the communication model")
    ap.add_argument("--no-measure", action="store_true", help="FLOP model instead of GPU timing")
    ap.add_argument("--json", action="store_true")
    a = ap.parse_args()
    model = Model(a.hidden, a.heads, a.ffn, a.seq, a.layers)
    rows = cost_table(model, a.gpus, a.global_batch, a.link_gbps, measure=not a.no_measure)
    st, chosen, res = plan(model, rows, a.gpus, a.global_batch, a.budget_gib * 2 ** 30, a.link_gbps)
    if a.json:
        print(json.dumps(dict(rows=rows, status=st, plan=[(r["tp_attn"], r["tp_ffn"]) for r in chosen],
                              total_ms=res.total_ms, total_mem_bytes=res.total_mem_bytes)))
        return
    print(f"# per-layer cost table: hidden {a.hidden}, heads {a.heads}, ffn {a.ffn}, seq {a.seq}, group of {a.gpus} GPUs, "
          f"global batch {a.global_batch}, compute {'FLOP model' if a.no_measure else 'measured on this GPU'}, "
          f"communication modelled at {a.link_gbps:g} GB/s per link")
    print(f"{'tp_attn':>7} {'tp_ffn':>6} {'mb_attn':>7} {'mb_ffn':>6} {'compute_ms':>10} {'comm_ms':>8} {'time_ms':>8} "
          f"{'TFLOP/s/GPU':>11} {'state_GiB':>9} {'saved_GiB':>9}")
    for r in rows:
        print(f"{r['tp_attn']:>7} {r['tp_ffn']:>6} {r['micro_batch_attn']:>7} {r['micro_batch_ffn']:>6} "
              f"{r['compute_ms']:>10.3f} {r['comm_ms']:>8.3f} {r['time_ms']:>8.3f} {r['tflops_per_gpu']:>11.0f} "
              f"{r['state_bytes'] / 2 ** 30:>9.3f} {r['saved_bytes'] / 2 ** 30:>9.3f}")
    if st != gx.GX_OK:
        print(f"# plan: {gx.status_str(st)} (budget {a.budget_gib:g} GiB per GPU for {a.layers} layers)")
        return
    runs, prev = [], None
    for r in chosen:
        key = (r["tp_attn"], r["tp_ffn"])
        if key == prev:
            runs[-1][1] += 1
        else:
            runs.append([key, 1])
        prev = key
    print(f"# plan for {a.layers} layers under {a.budget_gib:g} GiB per GPU: "
          + ", ".join(f"{n} x (tp_attn {k[0]}, tp_ffn {k[1]})" for k, n in runs)
          + f"; {res.total_ms:.2f} ms per step, {res.total_mem_bytes / 2 ** 30:.1f} GiB, "
          f"{res.pruned} candidates pruned, largest frontier {res.frontier_peak}")


if __name__ == "__main__":
    main()
