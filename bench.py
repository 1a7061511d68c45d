#!/usr/bin/env python3
"""Benchmark of the co-batched heterogeneous-rank LoRA delta on one MI355X.

Default workload (the configuration the metric is quoted on): a decode co-batch at the Llama-3-8B
q_proj shape, 4096 -> 4096, 256 tokens (one per request), 128 resident adapters with ranks balanced
over {8,16,32,64,128}, request -> adapter Zipf(1.1), bf16.  One step is one pass of the whole hot path
for that batch through the q_proj of all 32 layers: one lora_segments_rebuild (host grouping + table
upload) followed by 32 lora_apply calls (shrink + expand), each on its own layer's pool, x and y.
The 32 layers touch about 1.9 GB per step, far more than the 256 MB last-level cache, so every
apply streams its weights from HBM, as it does in a real decode step.

value = token-deltas per second = tokens * projections per step / step time, inputs resident in HBM.

--workload selects the other configurations' shapes (prefill segments, one projection of the mixed
stack batch, the rank-skew batch) for profiling the same path; their weights and x are random bf16
filled on the device, and the parity spot check against the oracle runs for the default only.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0

# Figures that only a profiler run can give (HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE,
# the rate of a kernel that only reads) live in profiles/measured.json, beside the summaries that quote
# them: counters cannot be read from inside this process.  Keys of "traffic_bytes": "<workload>|<launch phase>".
MEASURED_PATH = os.path.join(ROOT, "profiles", "measured.json")


def load_measured() -> dict:
    with open(MEASURED_PATH) as f:
        return json.load(f)


class Hip:
    """The few HIP runtime calls the benchmark needs for events on the launch stream."""

    def __init__(self):
        self.rt = ctypes.CDLL("libamdhip64.so")

    # hipEventDisableSystemFence: a timing event without the system-scope release (cache write-back
    # and invalidate) it otherwise performs between the two kernels it separates
    EVENT_FLAGS = 0x20000000

    def event(self) -> ctypes.c_void_p:
        e = ctypes.c_void_p()
        rc = self.rt.hipEventCreateWithFlags(ctypes.byref(e), ctypes.c_uint(self.EVENT_FLAGS))
        assert rc == 0, f"hipEventCreateWithFlags -> {rc}"
        return e

    def record(self, e, stream) -> None:
        rc = self.rt.hipEventRecord(e, ctypes.c_void_p(int(stream.cuda_stream) or None))
        assert rc == 0, f"hipEventRecord -> {rc}"

    def elapsed_ms(self, a, b) -> float:
        ms = ctypes.c_float()
        rc = self.rt.hipEventElapsedTime(ctypes.byref(ms), a, b)
        assert rc == 0, f"hipEventElapsedTime -> {rc}"
        return float(ms.value)

    def destroy(self, e):
        self.rt.hipEventDestroy(e)


def pick_workload(spec: str, wl, tp: str = None):
    """-> (batch, description, default projections per step, seeded host weights?)"""
    if "@r" in spec:
        # <workload>@r<rank>: the same routing with every adapter at one rank (what a placement that
        # groups adapters by rank gives a server; the operating points of the placement what-if)
        import dataclasses
        base, rank = spec.split("@r")
        b, description, layers, _ = pick_workload(base, wl, tp)
        ranks = np.full_like(b.ranks, int(rank))
        b = dataclasses.replace(b, name=f"{b.name}_r{int(rank)}", ranks=ranks, scales=wl._scales_for(ranks))
        return b, f"{description}; every adapter at rank {int(rank)}", layers, False
    if tp:
        # one GPU's shard of a tensor-parallel layer: a column-parallel layer keeps A_a and holds
        # out/N columns of B_a, a row-parallel layer holds in/N rows of A_a and all of B_a (its v is
        # what the ranks would sum before the expand; that exchange needs other GPUs and is not run)
        import dataclasses
        n, kind = tp.split(":")
        n = int(n)
        b, description, layers, seeded = pick_workload(spec, wl)
        in_f, out_f = (b.in_features, b.out_features // n) if kind == "col" else (b.in_features // n, b.out_features)
        if kind not in ("col", "row") or in_f % 64 or out_f % 128 or n < 1:
            raise SystemExit(f"--tp {tp}: want <N>:col or <N>:row with in/N a multiple of 64, out/N of 128")
        b = dataclasses.replace(b, name=f"{b.name}_tp{n}{kind}", in_features=in_f, out_features=out_f)
        return b, f"{description}; tensor-parallel shard 1/{n} ({kind}): {in_f}->{out_f}", layers, seeded
    parts = spec.split(":")
    kind = parts[0]
    if kind == "groups":
        # groups:<in>x<out>:<count>x<tokens>[r<rank>]+...   e.g. groups:4096x4096:1x40r64+960x1
        in_f, out_f = (int(v) for v in parts[1].split("x"))
        groups = []
        for g in parts[2].split("+"):
            body, _, rank = g.partition("r")
            count, tokens = (int(v) for v in body.split("x"))
            groups.append((count, tokens, int(rank) if rank else 0))
        b = wl.groups_batch(in_f, out_f, groups)
        return (b, f"groups {parts[2]} (count x tokens, one adapter each), {in_f}->{out_f}, T={b.T}", 4, False)
    if kind == "cfg1" and len(parts) > 1:
        # cfg1:<in>x<out>: the same routing on another projection shape
        in_f, out_f = (int(v) for v in parts[1].split("x"))
        return (wl.cfg1_decode(layer=0, in_features=in_f, out_features=out_f), f"cfg1's routing (T=256, 128 adapters ranks "
                f"{{8,16,32,64,128}}, Zipf(1.1)) on {in_f}->{out_f}", 32, False)
    if kind == "cfg1":
        return (wl.cfg1_decode(layer=0), "cfg1 decode co-batch, Llama-3-8B q_proj 4096->4096, T=256, 128 adapters "
                "ranks {8,16,32,64,128}, Zipf(1.1)", 32, True)
    if kind == "cfg2":
        shape = int(parts[1]) if len(parts) > 1 else 0
        b = wl.cfg2_prefill(shape)
        return (b, f"cfg2 prefill segments, {b.in_features}->{b.out_features}, 32 requests, T={b.T}, ranks "
                "{8,16,32,64,128}", 4, False)
    if kind == "cfg3":
        proj = int(parts[1]) if len(parts) > 1 else 0
        scale = float(parts[2]) if len(parts) > 2 else 1.0       # prompt lengths times this (smaller chunks)
        b = wl.cfg3_stack(layer=0, projection=proj, length_scale=scale)
        tag = "" if scale == 1.0 else f" (prompt lengths x {scale:g})"
        return (b, f"cfg3 mixed batch, {wl.CFG3_PROJECTIONS[proj][0]}_proj {b.in_features}->{b.out_features}, "
                f"8 prefills{tag} + 384 decode tokens, T={b.T}, 256 adapters", 8, False)
    if kind == "cfg4":
        shape = int(parts[1]) if len(parts) > 1 else 0
        split = (parts[2] if len(parts) > 2 else "1to1").replace("to", ":")
        only = int(parts[3]) if len(parts) > 3 else None
        b = wl.cfg4_skew(shape, split, only_class=only)
        tag = "" if only is None else f", only rank-{(8, 256)[only]} tokens routed"
        return (b, f"cfg4 rank skew, {b.in_features}->{b.out_features}, T=512 split {split} between rank 8 and "
                f"rank 256 (32 adapters each){tag}", 8, False)
    raise SystemExit(f"unknown workload {spec!r}")


def run_projections(args, torch, L, wl, dev, stream, hip) -> int:
    """Projections of one layer that read the same x, fused into one lora_apply_multi per layer or run
    as separate lora_apply calls on the column blocks of the same y.  Weights and x are device-random."""
    outs = {"qkv": (4096, 1024, 1024), "gateup": (14336, 14336), "q": (4096,)}[args.projections]
    b0, description, default_layers, _ = pick_workload(args.workload, wl)
    assert b0.in_features == 4096, "--projections uses the routing of cfg1 or cfg3:0 (in_features 4096)"
    nl = args.layers or (32 if b0.T <= 1024 else 4)
    T, in_f, P = b0.T, 4096, len(outs)
    sizes = [L.lora_pool_bytes(in_f, o, b0.ranks, b0.scales) for o in outs]
    starts = np.concatenate([[0], np.cumsum([(n + 4095) // 4096 * 4096 for n in sizes])])
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    arenas, pools, xs, ys = [], [], [], []
    for l in range(nl):
        arena = torch.empty(int(starts[-1]), dtype=torch.uint8, device=dev)
        arena.view(torch.bfloat16).normal_(0.0, 0.02, generator=g)
        arenas.append(arena)
        layer_pools = []
        for q, o in enumerate(outs):
            pool = L.lora_pool_create(in_f, o, b0.ranks, b0.scales, arena[int(starts[q]): int(starts[q]) + sizes[q]])
            for a in range(b0.n_adapters):
                L.lora_pool_mark_resident(pool, a)
            layer_pools.append(pool)
        pools.append(layer_pools)
        xs.append(torch.empty(T, in_f, dtype=torch.bfloat16, device=dev).normal_(0.0, 1.0, generator=g))
        ys.append(torch.zeros(T, sum(outs), dtype=torch.bfloat16, device=dev))
    if args.separate:
        segs = [L.lora_segments_build(pools[0][q], b0.token_adapter, stream=stream) for q in range(P)]
        ws = torch.empty(max(max(L.lora_apply_workspace_bytes(pools[0][q], segs[q]) for q in range(P)), 256),
                         dtype=torch.uint8, device=dev)
        cols = np.concatenate([[0], np.cumsum(outs)])

        def step():
            for q in range(P):
                L.lora_segments_rebuild(segs[q], b0.token_adapter, stream=stream)
            for l in range(nl):
                for q in range(P):
                    L.lora_apply(pools[l][q], segs[q], xs[l], ys[l][:, int(cols[q]): int(cols[q + 1])], ws,
                                 stream=stream, ldy=sum(outs))
    else:
        seg = L.lora_segments_build_multi(pools[0], b0.token_adapter, stream=stream)
        ws = torch.empty(max(L.lora_apply_workspace_bytes(pools[0][0], seg), 256), dtype=torch.uint8, device=dev)

        def step():
            L.lora_segments_rebuild(seg, b0.token_adapter, stream=stream)
            for l in range(nl):
                L.lora_apply_multi(pools[l], seg, xs[l], ys[l], ws, stream=stream)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    n_act = int((b0.token_adapter >= 0).sum())
    act = b0.token_adapter >= 0
    rsum = int(b0.ranks[b0.token_adapter[act]].astype(np.int64).sum())
    r8 = (b0.ranks.astype(np.int64) + 7) // 8 * 8
    wsum = int(r8[b0.used_adapters()].sum())
    # x once per layer when fused, once per projection otherwise; weights, y and v as ever
    per_layer = sum(2 * wsum * (in_f + o) + 4 * n_act * o + 4 * rsum for o in outs)
    per_layer += 2 * n_act * in_f * (P if args.separate else 1)
    us_per_layer = dt / args.steps / nl * 1e6
    out = {
        "metric": "LoRA-delta tokens/s + achieved HBM GB/s (decode) / MFMA util (prefill), mixed ranks",
        "value": n_act * P * nl / (dt / args.steps), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{description}; projections {args.projections} {outs} of {nl} layers, "
                               + ("one lora_apply each" if args.separate else "one lora_apply_multi per layer"),
                   "tokens": T, "active_tokens": n_act, "projections": P, "layers_per_step": nl,
                   "us_per_layer": us_per_layer, "algorithmic_bytes_per_layer": per_layer},
        "roofline": {"bound": "hbm", "kernel": "all launches of a layer", "achieved": per_layer / us_per_layer / 1e3,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": per_layer / us_per_layer / 1e3 / HBM_PEAK_GBS,
                     "traffic": None},
        "cpu_baseline": None,
    }
    print(json.dumps(out))
    return 0


def run_layer(args, torch, L, wl, dev, stream, hip) -> dict:
    """All seven adapted projections of Llama-3-8B layers on one routing (cfg1's or cfg3's): per layer
    q|k|v in one lora_apply_multi (they share x), o, gate|up in one lora_apply_multi, down.  Each
    projection has its own x and y (no base model here, so nothing flows from one to the next).
    Weights and x are device-random; `value` counts a token once per layer it has passed."""
    b0, description, _, _ = pick_workload(args.workload, wl)
    assert b0.in_features == 4096, "--projections layer uses the routing of cfg1 or cfg3:0"
    groups = [(4096, (4096, 1024, 1024)), (4096, (4096,)), (4096, (14336, 14336)), (14336, (4096,))]
    # the routing is planned once per step, as in a model of 32 layers; the mixed batch's pools of 32
    # layers would not leave room for x and y, so it runs 8 layers per step
    nl = args.layers or (32 if args.workload == "cfg1" else 8)
    T = b0.T
    n_slots = min(nl, 32 if T <= 1024 else 4)
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    layers = []
    for l in range(nl):
        applies = []
        for in_f, outs in groups:
            sizes = [L.lora_pool_bytes(in_f, o, b0.ranks, b0.scales) for o in outs]
            starts = np.concatenate([[0], np.cumsum([(n + 4095) // 4096 * 4096 for n in sizes])])
            arena = torch.empty(int(starts[-1]), dtype=torch.uint8, device=dev)
            arena.view(torch.bfloat16).normal_(0.0, 0.02, generator=g)
            pools = []
            for q, o in enumerate(outs):
                pool = L.lora_pool_create(in_f, o, b0.ranks, b0.scales, arena[int(starts[q]): int(starts[q]) + sizes[q]])
                for a in range(b0.n_adapters):
                    L.lora_pool_mark_resident(pool, a)
                pools.append(pool)
            # x and y of a projection group: the layers take turns on a few copies (each far larger than the
            # caches when the batch is), the pools are all distinct
            slot = l % n_slots
            if l < n_slots:
                x = torch.empty(T, in_f, dtype=torch.bfloat16, device=dev).normal_(0.0, 1.0, generator=g)
                y = torch.zeros(T, sum(outs), dtype=torch.bfloat16, device=dev)
            else:
                x, y = layers[slot][len(applies)][2:4]
            applies.append((arena, pools, x, y))
        layers.append(applies)
    # one segment object per apply of a layer; every layer's pools are spaced alike, so they serve all layers
    segs, wss = [], []
    for arena, pools, x, y in layers[0]:
        seg = (L.lora_segments_build_multi(pools, b0.token_adapter, stream=stream) if len(pools) > 1
               else L.lora_segments_build(pools[0], b0.token_adapter, stream=stream))
        segs.append(seg)
        wss.append(torch.empty(max(L.lora_apply_workspace_bytes(pools[0], seg), 256), dtype=torch.uint8, device=dev))

    def step():
        for seg in segs:
            L.lora_segments_rebuild(seg, b0.token_adapter, stream=stream)
        for applies in layers:
            for (arena, pools, x, y), seg, ws in zip(applies, segs, wss):
                if len(pools) > 1:
                    L.lora_apply_multi(pools, seg, x, y, ws, stream=stream)
                else:
                    L.lora_apply(pools[0], seg, x, y, ws, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    step_ev = [hip.event() for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    hip.record(step_ev[0], stream)
    for k in range(args.steps):
        step()
        hip.record(step_ev[k + 1], stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    step_ms = np.array([hip.elapsed_ms(step_ev[k], step_ev[k + 1]) for k in range(args.steps)])
    for e in step_ev:
        hip.destroy(e)
    for seg in segs:
        L.lora_segments_check(seg, stream=stream)
    act = b0.token_adapter >= 0
    n_act = int(act.sum())
    rsum = int(b0.ranks[b0.token_adapter[act]].astype(np.int64).sum())
    r8 = (b0.ranks.astype(np.int64) + 7) // 8 * 8
    wsum = int(r8[b0.used_adapters()].sum())
    per_layer = 0
    for in_f, outs in groups:
        per_layer += 2 * n_act * in_f + sum(2 * wsum * (in_f + o) + 4 * n_act * o + 4 * rsum for o in outs)
    us_per_layer = dt / args.steps / nl * 1e6
    out = {
        "metric": "LoRA-delta tokens/s + achieved HBM GB/s (decode) / MFMA util (prefill), mixed ranks",
        "value": n_act * nl / (dt / args.steps), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3, "ms_per_step_median": float(np.median(step_ms)),
        "ms_per_step_min": float(step_ms.min()), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{description}; all seven projections of {nl} Llama-3-8B layers per step "
                               "(q|k|v and gate|up as lora_apply_multi, o and down as lora_apply)",
                   "tokens": T, "active_tokens": n_act, "layers_per_step": nl, "us_per_layer": us_per_layer,
                   "algorithmic_bytes_per_layer": per_layer,
                   "tokens_per_s_through_32_layers": n_act / (32 * us_per_layer * 1e-6)},
        "roofline": {"bound": "hbm", "kernel": "all launches of a layer", "achieved": per_layer / us_per_layer / 1e3,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": per_layer / us_per_layer / 1e3 / HBM_PEAK_GBS,
                     "traffic": None},
        "cpu_baseline": None,
    }
    for seg in segs:
        L.lora_segments_destroy(seg)
    for applies in layers:
        for _arena, pools, _x, _y in applies:
            for p_ in pools:
                L.lora_pool_destroy(p_)
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--layers", type=int, default=None,
                    help="projections per step (default: 32 for cfg1, fewer for the larger workloads)")
    ap.add_argument("--workload", default="cfg1",
                    help="cfg1 (default, the benchmark line) | cfg2:<shape 0..2> | cfg3:<projection 0..6>[:<prompt length scale>] | "
                         "cfg4:<shape 0..2>:<9to1|1to1|1to9>[:<0|1> only that rank class] | groups:<in>x<out>:<count>x<tokens>[r<rank>]+...; "
                         "any of them with @r<rank> appended: "
                         "every adapter at that rank")
    ap.add_argument("--plan", default=None, metavar="NAME=VALUE[,...]",
                    help="fields of lora_plan_options_t for the timed object, e.g. heavy_k_cut_max_units=0,whole_k_max_in=16384 "
                         "(a planner rule measured on the other side of its threshold)")
    ap.add_argument("--tp", default=None, metavar="N:col|N:row",
                    help="time one GPU's shard of the workload's projection under N-way tensor parallelism: "
                         "col = out_features/N columns of B (column-parallel layer), row = in_features/N rows of A "
                         "(row-parallel layer; the sum of v over the ranks is not part of the run)")
    ap.add_argument("--fused", action="store_true", help="single-launch lora_apply (decode-sized batches)")
    ap.add_argument("--mixed-form", choices=("merged", "two-streams", "one-stream"), default="merged",
                    help="how a mixed batch (token-heavy and decode-sized groups) is launched: two launches that "
                         "hold both kinds of unit (default), four launches with the decode-sized pair on a side "
                         "stream, or four launches on one stream")
    ap.add_argument("--whole-k-limit", type=int, default=None,
                    help="planning knob lora_set_whole_k_limit (default: the library's, 1024; 0 = always k-slices)")
    ap.add_argument("--projections", default=None,
                    help="several projections that share x in one pass, e.g. qkv or gateup (Llama-3-8B shapes), with "
                         "the routing of --workload cfg1 or cfg3:0; add --separate to run them one lora_apply each; "
                         "`layer`: all seven projections of a layer (q|k|v, o, gate|up, down)")
    ap.add_argument("--separate", action="store_true")
    ap.add_argument("--concurrent-loads", type=int, default=0,
                    help="adapters (ones the batch does not use) loaded into the step's pools on a second stream "
                         "per step, while the applies run")
    ap.add_argument("--padded-control", action="store_true",
                    help="control run: every adapter stored at the largest rank of the pool, zero-padded (the "
                         "layout whose cost the paper's motivation measures); same batch, same results")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="budget of the oracle timing leg")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true",
                    help="only the headline workload (the default run also times the other configurations)")
    ap.add_argument("--wg-clocks", action="store_true",
                    help="per-work-group device clocks of one apply of --workload, by rank class: when each class's "
                         "first work group starts and its last one ends in either launch.  Needs the measurement "
                         "build of the library: python -m paper_2511_22880_amd.build --clocks, then "
                         "LORA_GFX950_LIB=<repo>/paper_2511_22880_amd/liblora_gfx950_clocks.so")
    ap.add_argument("--linear", action="store_true",
                    help="the adapted layer in one pass (lora_linear: base GEMM with the delta in its epilogue) on "
                         "--workload, beside `base GEMM (torch.matmul), then lora_apply` on the same inputs")
    ap.add_argument("--two-launches", action="store_true",
                    help="decode batches as a shrink launch and an expand launch (lora_set_decode_single_launch(0))")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2511_22880_amd import binding as L
    from paper_2511_22880_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream()
    hip = Hip()
    if args.fused:
        L.lora_set_fused_apply(True)
    if args.two_launches:
        L.lora_set_decode_single_launch(False)
    if args.whole_k_limit is not None:
        L.lora_set_whole_k_limit(args.whole_k_limit)
    L.lora_set_merged_launches(args.mixed_form == "merged")
    L.lora_set_side_stream(args.mixed_form != "one-stream")

    if args.wg_clocks:
        return run_wg_clocks(args, torch, L, wl, dev, stream)
    if args.linear:
        print(json.dumps(run_linear(args, torch, L, wl, dev, stream, hip)))
        return 0
    if args.projections == "layer":
        print(json.dumps(run_layer(args, torch, L, wl, dev, stream, hip)))
        return 0
    if args.projections:
        return run_projections(args, torch, L, wl, dev, stream, hip)

    out, err = run_workload(args, torch, L, wl, dev, stream, hip, args.workload, args.layers, args.steps, args.warmup,
                            not args.no_cpu_baseline)
    headline = (args.workload == "cfg1" and not (args.tp or args.fused or args.padded_control or args.concurrent_loads
                                                 or args.whole_k_limit is not None or args.two_launches))
    if headline and not args.no_secondary:
        out["secondary"] = run_secondary(args, torch, L, wl, dev, stream, hip)
    print(json.dumps(out))
    if err is not None:
        assert err <= 5e-3, f"parity spot check failed: {err}"
    return 0


def run_wg_clocks(args, torch, L, wl, dev, stream) -> int:
    """One apply of the workload with every work group's wall clock (100 MHz) at its entry and its end,
    grouped by the rank of the unit's adapter: per class and launch, the first start, the median and
    the last end, in microseconds from the apply's first work group."""
    b0, description, _, _ = pick_workload(args.workload, wl, args.tp)
    T, in_f, out_f = b0.T, b0.in_features, b0.out_features
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    n_rot = 4
    nbytes = L.lora_pool_bytes(in_f, out_f, b0.ranks, b0.scales)
    arenas = [torch.empty(nbytes, dtype=torch.uint8, device=dev) for _ in range(n_rot)]
    pools = []
    for a in arenas:
        a.view(torch.bfloat16).normal_(0.0, 0.02, generator=g)
        pools.append(L.lora_pool_create(in_f, out_f, b0.ranks, b0.scales, a))
        for k in range(b0.n_adapters):
            L.lora_pool_mark_resident(pools[-1], k)
    xs = [torch.empty(T, in_f, dtype=torch.bfloat16, device=dev).normal_(0.0, 1.0, generator=g) for _ in range(n_rot)]
    ys = [torch.zeros(T, out_f, dtype=torch.bfloat16, device=dev) for _ in range(n_rot)]
    seg = L.lora_segments_build(pools[0], b0.token_adapter, stream=stream)
    info = L.lora_segments_info(seg)
    ws = torch.empty(max(L.lora_apply_workspace_bytes(pools[0], seg), 256), dtype=torch.uint8, device=dev)
    for _ in range(3):
        for l in range(n_rot):
            L.lora_apply(pools[l], seg, xs[l], ys[l], ws, stream=stream)
    torch.cuda.synchronize()
    E_BASE, SLOTS = 32768, 65536
    buf = torch.zeros(SLOTS * 8, dtype=torch.int64, device=dev)
    L.lora_debug_clock_buffer(buf, SLOTS)
    for l in range(n_rot):     # the last apply's clocks stay (the pools before it keep the caches cold)
        L.lora_apply(pools[l], seg, xs[l], ys[l], ws, stream=stream)
    torch.cuda.synchronize()
    L.lora_debug_clock_buffer(None, 0)
    h = buf.cpu().numpy().reshape(SLOTS, 8)
    ex = L.lora_segments_export(seg)
    rank_of_seg = b0.ranks[ex["seg_adapter"]]
    rows = []
    heavy_seg = np.zeros(len(rank_of_seg), dtype=bool)
    if info["single_launch"]:
        lu = L.lora_segments_export_launch_units(seg)
        n = info["launch_work_groups"]
        t0 = h[:n, 0][h[:n, 0] > 0].min()
        lists = [("one launch, by the shrink unit's rank", lu["shrink"], h[:n]),]
    else:
        units = L.lora_segments_export_units(seg)
        ns, ne = len(units["shrink"]), len(units["expand"])
        # The export holds the decode-sized groups' list first and the token-heavy groups' list behind it; a
        # launch that holds both runs the token-heavy list first.  (Token-heavy: 32 tokens or more in a batch
        # of 1024 or more, the planner's default; such a group's expand units are in the second list up to
        # rank 128; places that only pad the token-heavy shrink list have segment -1.)
        seg_ntok = np.diff(ex["seg_start"])
        heavy_seg = (seg_ntok >= 32) & (int(seg_ntok.sum()) >= 1024)

        def launch_order(ulist, second):
            n_first = next((k for k, u in enumerate(ulist) if second(u)), len(ulist))
            return np.concatenate([ulist[n_first:], ulist[:n_first]]) if 0 < n_first < len(ulist) else ulist

        shrink_list = launch_order(units["shrink"], lambda u: u[0] < 0 or heavy_seg[u[0]])
        expand_list = launch_order(units["expand"], lambda u: heavy_seg[u[0]] and rank_of_seg[u[0]] <= 128)
        t0 = h[:ns, 0][h[:ns, 0] > 0].min()
        lists = [("shrink launch", shrink_list, h[:ns]), ("expand launch", expand_list, h[E_BASE:E_BASE + ne])]
    for name, ulist, clk in lists:
        # classes: the adapter's rank, and whether the unit's group is token-heavy
        for r, heavy in [(r, h) for r in sorted(set(int(v) for v in rank_of_seg)) for h in (False, True)]:
            sel = np.array([u[2] > 0 and rank_of_seg[u[0]] == r and bool(heavy_seg[u[0]]) == heavy for u in ulist]) & \
                (clk[:, 0] > 0) & (clk[:, 4] > 0)
            if not sel.any():
                continue
            start, end = (clk[sel, 0] - t0) * 0.01, (clk[sel, 4] - t0) * 0.01
            rows.append({"launch": name, "rank": r, "token_heavy_units": heavy, "work_groups": int(sel.sum()),
                         "first_start_us": float(start.min()),
                         "median_start_us": float(np.median(start)), "median_duration_us": float(np.median(end - start)),
                         "max_duration_us": float((end - start).max()), "duration_deciles_us": [round(float(v), 1) for v in
                         np.percentile(end - start, [10, 30, 50, 70, 90])], "last_end_us": float(end.max())})
            if name == "shrink launch" and (clk[sel, 1] > 0).any() and (clk[sel, 1] < 10 ** 7).all():
                # token tiles above rank 32: of the duration, the part between the top of a pass and its barrier's exit
                rows[-1]["median_wait_for_x_us"] = float(np.median(clk[sel, 1]) * 0.01)
    out = {"workload": description, "tokens": T, "single_launch": bool(info["single_launch"]),
           "clock": "wall clock of the device, 100 MHz; microseconds from the first work group's entry",
           "per_class": rows}
    if info["single_launch"]:
        # the one-launch decode kernel also records where a work group stands inside its two halves
        n = info["launch_work_groups"]
        t0 = h[:n, 0][h[:n, 0] > 0].min()
        points = {}
        for slot, name in ((0, "entry"), (1, "shrink loop done (wavefront 0)"), (7, "v stored (behind the work group's barrier)"),
                           (2, "stores of v acknowledged, counter bumped"), (3, "tile's v seen by the expand unit"), (4, "end")):
            v = h[:n, slot]
            v = v[v > 0]
            if len(v):
                points[name] = {k: round(float(q), 2) for k, q in
                                zip(("p10", "median", "p90", "last"), (np.percentile(v, [10, 50, 90, 100]) - t0) * 0.01)}
        out["points_us"] = points
    print(json.dumps(out))
    return 0


def run_linear(args, torch, L, wl, dev, stream, hip) -> dict:
    """y = x W + delta for every token of the workload: lora_linear against torch.matmul followed by
    lora_apply, and against lora_linear on a pool whose batch uses no adapter (the GEMM alone)."""
    b0, description, _, _ = pick_workload(args.workload, wl, args.tp)
    T, in_f, out_f = b0.T, b0.in_features, b0.out_features
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    nl = args.layers or 4
    nbytes = L.lora_pool_bytes(in_f, out_f, b0.ranks, b0.scales)
    arenas, pools, wts, wps, xs, ys = [], [], [], [], [], []
    for l in range(nl):
        a = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        a.view(torch.bfloat16).normal_(0.0, 0.02, generator=g)
        arenas.append(a)
        pools.append(L.lora_pool_create(in_f, out_f, b0.ranks, b0.scales, a))
        for k in range(b0.n_adapters):
            L.lora_pool_mark_resident(pools[-1], k)
        wt = torch.empty(out_f, in_f, dtype=torch.bfloat16, device=dev).normal_(0.0, 0.02, generator=g)
        wp = torch.empty(in_f * out_f * 2, dtype=torch.uint8, device=dev)
        L.lora_linear_pack_weight(wt, in_f, out_f, wp, stream=stream)
        wts.append(wt)
        wps.append(wp)
        xs.append(torch.empty(T, in_f, dtype=torch.bfloat16, device=dev).normal_(0.0, 1.0, generator=g))
        ys.append(torch.empty(T, out_f, dtype=torch.bfloat16, device=dev))
    seg = L.lora_segments_build(pools[0], b0.token_adapter, stream=stream)
    none = L.lora_segments_build(pools[0], np.full(T, -1, dtype=np.int32), stream=stream)
    ws = torch.empty(max(L.lora_apply_workspace_bytes(pools[0], seg), 256), dtype=torch.uint8, device=dev)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        ev = [hip.event() for _ in range(args.steps + 1)]
        hip.record(ev[0], stream)
        for k in range(args.steps):
            fn()
            hip.record(ev[k + 1], stream)
        torch.cuda.synchronize()
        ms = np.array([hip.elapsed_ms(ev[k], ev[k + 1]) for k in range(args.steps)]) / nl
        for e in ev:
            hip.destroy(e)
        return float(np.median(ms) * 1e3), float(ms.min() * 1e3)

    def fused():
        for l in range(nl):
            L.lora_linear(pools[l], seg, xs[l], wps[l], ys[l], ws, stream=stream)

    def gemm_alone():
        for l in range(nl):
            L.lora_linear(pools[l], none, xs[l], wps[l], ys[l], ws, stream=stream)

    def separate():
        for l in range(nl):
            torch.matmul(xs[l], wts[l].t(), out=ys[l])
            L.lora_apply(pools[l], seg, xs[l], ys[l], ws, stream=stream)

    def library_gemm():
        for l in range(nl):
            torch.matmul(xs[l], wts[l].t(), out=ys[l])

    res = {name: timed(fn) for name, fn in (("lora_linear", fused), ("lora_linear without adapters", gemm_alone),
                                            ("torch.matmul then lora_apply", separate), ("torch.matmul", library_gemm))}
    # the two paths agree (same inputs; different summation orders and one rounding more in the separate path)
    fused()
    y_f = ys[0].float().clone()
    separate()
    torch.cuda.synchronize()
    rel = float(((y_f - ys[0].float()).norm(dim=1) / ys[0].float().norm(dim=1).clamp_min(1e-30)).max())
    n_act = int((b0.token_adapter >= 0).sum())
    gemm_flops = 2.0 * T * in_f * out_f
    flops = gemm_flops + b0.flops()
    us = res["lora_linear"][0]
    return {"workload": description + "; adapted layer y = x W + delta, median us per layer over "
                        f"{args.steps} steps of {nl} layers", "tokens": T, "active_tokens": n_act,
            "us_per_layer": {k: {"median": v[0], "min": v[1]} for k, v in res.items()},
            "flops_per_layer": flops, "lora_linear_TFLOPs": flops / (us * 1e-6) / 1e12,
            "lora_linear_mfma_frac": flops / (us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "torch_matmul_TFLOPs": gemm_flops / (res["torch.matmul"][0] * 1e-6) / 1e12,
            "delta_cost_us": {"in the epilogue (lora_linear minus the same kernel without adapters)":
                              res["lora_linear"][0] - res["lora_linear without adapters"][0],
                              "as lora_apply behind the library GEMM": res["torch.matmul then lora_apply"][0] - res["torch.matmul"][0]},
            "max_row_rel_l2_between_the_two_paths": rel}


def brief(out: dict) -> dict:
    """The part of a workload's result that goes into the headline line's `secondary` list."""
    r, c = out["roofline"], out["config"]
    return {"workload": c["workload"], "tokens": c["tokens"], "projections_per_step": c.get("projections_per_step"),
            "tokens_per_s": out["value"], "ms_per_step": out["ms_per_step"],
            "ms_per_step_median": out["ms_per_step_median"], "ms_per_step_min": out["ms_per_step_min"],
            "shrink_launch_us": r.get("shrink_launch_us"), "expand_launch_us": r.get("expand_launch_us"),
            "single_launch": c.get("single_launch_apply"),
            "algorithmic_bytes_per_apply": c.get("algorithmic_bytes_per_apply", c.get("algorithmic_bytes_per_layer")),
            "apply_GBps": r.get("apply_GBps", r.get("achieved")), "frac_of_hbm_peak": r.get("apply_frac", r.get("frac")),
            "mfma_useful_frac": r.get("apply_mfma_frac"), "dominant": r.get("kernel"), "dominant_frac": r.get("frac")}


def run_secondary(args, torch, L, wl, dev, stream, hip) -> list:
    """The other configurations, timed in the same run: the three prefill shapes, the mixed batch on
    q_proj and through all seven projections of 32 layers, the rank-skew batch."""
    import gc
    res = []
    for spec, nl, steps in (("cfg2:0", 4, 10), ("cfg2:1", 4, 10), ("cfg2:2", 4, 10), ("cfg3:0", 8, 10),
                            ("cfg4:0:1to1", 8, 20)):
        out, _ = run_workload(args, torch, L, wl, dev, stream, hip, spec, nl, steps, 2, False)
        res.append(brief(out))
        gc.collect()
        torch.cuda.empty_cache()
    sub = argparse.Namespace(**vars(args))
    sub.workload, sub.layers, sub.steps, sub.warmup = "cfg3:0", 32, 3, 1
    res.append(brief(run_layer(sub, torch, L, wl, dev, stream, hip)))
    gc.collect()
    torch.cuda.empty_cache()
    # the adapted layer y = x W + delta in one GEMM (MFMA-bound: its roofline is the bf16 MFMA peak)
    sub = argparse.Namespace(**vars(args))
    sub.workload, sub.layers, sub.steps, sub.warmup = "cfg2:0", 4, 10, 2
    lin = run_linear(sub, torch, L, wl, dev, stream, hip)
    res.append({"workload": lin["workload"], "tokens": lin["tokens"], "us_per_layer": lin["us_per_layer"],
                "roofline": {"bound": "mfma", "achieved": lin["lora_linear_TFLOPs"], "peak": 2500.0, "unit": "TFLOP/s",
                             "frac": lin["lora_linear_mfma_frac"], "traffic": None},
                "delta_cost_us": lin["delta_cost_us"]})
    gc.collect()
    torch.cuda.empty_cache()
    return res


def run_workload(args, torch, L, wl, dev, stream, hip, workload, layers, steps, warmup, cpu_baseline):
    """One workload through lora_segments_rebuild + lora_apply on each of `layers` pools per step.
    Returns (the result object, parity spot check or None)."""
    measured = load_measured()
    b0, description, default_layers, seeded = pick_workload(workload, wl, args.tp)
    nl = layers or default_layers
    T, in_f, out_f = b0.T, b0.in_features, b0.out_features

    # ---- pools: one arena per projection of the step (distinct memory, so nothing is served from cache)
    pool_ranks = np.full_like(b0.ranks, b0.ranks.max()) if args.padded_control else b0.ranks
    nbytes = L.lora_pool_bytes(in_f, out_f, pool_ranks, b0.scales)
    arenas = [torch.zeros(nbytes, dtype=torch.uint8, device=dev) for _ in range(nl)]
    pools = [L.lora_pool_create(in_f, out_f, pool_ranks, b0.scales, a) for a in arenas]
    A = [None] * b0.n_adapters
    B = [None] * b0.n_adapters
    if seeded:
        # layer 0 from the seeded host generator, the other layers device copies of its packed arena
        for a in range(b0.n_adapters):
            A[a], B[a] = b0.adapter_bits(a)
            Ap, Bp = A[a], B[a]
            if args.padded_control:
                Ap = np.zeros((in_f, int(pool_ranks[a])), dtype=np.uint16)
                Bp = np.zeros((int(pool_ranks[a]), out_f), dtype=np.uint16)
                Ap[:, :A[a].shape[1]] = A[a]
                Bp[:B[a].shape[0]] = B[a]
            L.lora_pool_load(pools[0], a, Ap, Bp, stream=stream)
        for l in range(1, nl):
            arenas[l].copy_(arenas[0])
        xs_bits = [wl.cfg1_decode(layer=l).x_bits() for l in range(nl)]
        xs = [torch.from_numpy(xb.view(np.int16)).to(dev).view(torch.bfloat16) for xb in xs_bits]
    else:
        g = torch.Generator(device=dev)
        g.manual_seed(0)
        for l in range(nl):
            arenas[l].view(torch.bfloat16).normal_(0.0, 0.02, generator=g)
        xs = [torch.empty(T, in_f, dtype=torch.bfloat16, device=dev).normal_(0.0, 1.0, generator=g) for _ in range(nl)]
    for l in range(0 if not seeded else 1, nl):
        for a in range(b0.n_adapters):
            L.lora_pool_mark_resident(pools[l], a)
    ys = [torch.zeros(T, out_f, dtype=torch.bfloat16, device=dev) for _ in range(nl)]

    plan = None
    if getattr(args, "plan", None):
        plan = L.plan_options(**{k: int(v) for k, v in (kv.split("=") for kv in args.plan.split(","))})
    seg = L.lora_segments_build(pools[0], b0.token_adapter, stream=stream, options=plan)
    info = L.lora_segments_info(seg)
    ws = torch.empty(max(L.lora_apply_workspace_bytes(pools[0], seg), 256), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    # adapters that arrive while batches run: device-resident row-major sources of adapters the batch
    # does not use, packed into the pools by lora_pool_load on a stream of their own
    copy_stream, load_src, load_bytes, load_count = None, [], 0, [0]
    if args.concurrent_loads > 0:
        copy_stream = torch.cuda.Stream()
        unused = [a for a in range(b0.n_adapters) if a not in set(int(u) for u in b0.used_adapters())]
        assert unused, "every adapter is used by the batch"
        for a in unused[:16]:
            r = int(b0.ranks[a])
            load_src.append((a, torch.empty(in_f, r, dtype=torch.bfloat16, device=dev).normal_(0.0, 0.02),
                             torch.empty(r, out_f, dtype=torch.bfloat16, device=dev).normal_(0.0, 0.02)))

    def step():
        nonlocal load_bytes
        L.lora_segments_rebuild(seg, b0.token_adapter, stream=stream)
        for l in range(nl):
            L.lora_apply(pools[l], seg, xs[l], ys[l], ws, stream=stream)
        for _ in range(args.concurrent_loads):
            a, As, Bs = load_src[load_count[0] % len(load_src)]
            L.lora_pool_load(pools[load_count[0] % nl], a, As, Bs, stream=copy_stream)
            load_count[0] += 1
            load_bytes += 2 * int(b0.ranks[a]) * (in_f + out_f)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    load_bytes = 0
    step_ev = [hip.event() for _ in range(steps + 1)]
    t0 = time.perf_counter()
    hip.record(step_ev[0], stream)
    for k in range(steps):
        step()
        hip.record(step_ev[k + 1], stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    step_ms = np.array([hip.elapsed_ms(step_ev[k], step_ev[k + 1]) for k in range(steps)])
    for e in step_ev:
        hip.destroy(e)
    L.lora_segments_check(seg, stream=stream)
    load_bytes_per_step = load_bytes / steps
    ms_per_step = dt / steps * 1e3
    n_act = int((b0.token_adapter >= 0).sum())
    value = n_act * nl / (dt / steps)

    # ---- per-phase durations, live, with HIP events on the launch stream around the launches of the
    # same steps (shrink launches | expand launches; a fused apply is one launch).  The events sit
    # between back-to-back launches, so they also see the dispatch of a launch, which a kernel trace leaves out.
    n_prof_steps = max(1, min(steps, 10))
    evs = [[(hip.event(), hip.event(), hip.event()) for _ in range(nl)] for _ in range(n_prof_steps)]
    for s in range(n_prof_steps):
        L.lora_segments_rebuild(seg, b0.token_adapter, stream=stream)
        for l in range(nl):
            e = evs[s][l]
            L.lora_profile_next_apply(e[0], e[1], e[2])
            L.lora_apply(pools[l], seg, xs[l], ys[l], ws, stream=stream)
    torch.cuda.synchronize()
    shrink_us = np.array([[hip.elapsed_ms(e[0], e[1]) * 1e3 for e in row] for row in evs])
    expand_us = np.array([[hip.elapsed_ms(e[1], e[2]) * 1e3 for e in row] for row in evs])
    for row in evs:
        for e in row:
            for h in e:
                hip.destroy(h)

    # ---- algorithmic bytes per launch: adapter weights once, x once, y read + write, v write + read
    wbytes = b0.weight_bytes_touched()
    act = b0.token_adapter >= 0
    rsum = int(b0.ranks[b0.token_adapter[act]].astype(np.int64).sum())
    shrink_bytes = wbytes * in_f // (in_f + out_f) + 2 * n_act * in_f + 4 * rsum
    expand_bytes = wbytes * out_f // (in_f + out_f) + 4 * n_act * out_f + 4 * rsum
    one_launch = bool(args.fused) or bool(info["single_launch"])
    if one_launch:
        dom, dom_us, dom_bytes = "one launch", float(shrink_us.mean()), shrink_bytes + expand_bytes
    elif expand_us.mean() >= shrink_us.mean():
        dom, dom_us, dom_bytes = "expand launch", float(expand_us.mean()), expand_bytes
    else:
        dom, dom_us, dom_bytes = "shrink launch", float(shrink_us.mean()), shrink_bytes
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9
    traffic = measured["traffic_bytes"].get(f"{workload}|{dom}")
    dom_kernel = measured["phase_kernels"].get(f"{workload}|{dom}")
    if args.whole_k_limit is not None or args.padded_control or args.fused:
        traffic = dom_kernel = None      # the carried figures belong to the default plan
    # (one launch: both events of the hook follow that launch, so the first interval is the whole apply and
    # the second one the gap between two event records)
    apply_us = float(shrink_us.mean()) if one_launch else float(shrink_us.mean() + expand_us.mean())

    # ---- parity spot check of one layer against the oracle (not timed; seeded workload only)
    err = None
    if seeded:
        import oracle
        lchk = nl - 1
        ys[lchk].zero_()
        L.lora_apply(pools[lchk], seg, xs[lchk], ys[lchk], ws, stream=stream)
        torch.cuda.synchronize()
        yb = ys[lchk].view(torch.int16).cpu().numpy().view(np.uint16)
        rows = np.arange(0, T, 8, dtype=np.int32)
        y_ref = oracle.lora_apply(xs_bits[lchk], b0.token_adapter, b0.ranks, b0.scales, A, B, rows=rows)
        yg = wl.bf16_bits_to_f64(yb[rows])
        err = float((np.linalg.norm(yg - y_ref, axis=1) / np.linalg.norm(y_ref, axis=1)).max())

    # ---- the oracle as it stands, timed on this host's cores on a bounded sample of the workload
    cpu = None
    if seeded and cpu_baseline:
        import oracle
        n_done, t_cpu = 0, 0.0
        while t_cpu < args.cpu_seconds:
            xb = xs_bits[n_done % nl]
            t1 = time.perf_counter()
            oracle.lora_apply(xb, b0.token_adapter, b0.ranks, b0.scales, A, B)
            t_cpu += time.perf_counter() - t1
            n_done += 1
        cpu = {"value": T * n_done / t_cpu, "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
               "sample": f"{n_done} full-layer deltas of the same 256-token batch ({t_cpu:.1f} s of fp64 oracle)"}

    out = {
        "metric": "LoRA-delta tokens/s + achieved HBM GB/s (decode) / MFMA util (prefill), mixed ranks",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "ms_per_step_median": float(np.median(step_ms)), "ms_per_step_min": float(step_ms.min()), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": description, "projections_per_step": nl, "tokens": T, "active_tokens": n_act,
                   "distinct_adapters": info["n_segments"], "shrink_units": info["n_shrink_units"],
                   "expand_units": info["n_expand_units"], "k_slices": info["n_k_slices"],
                   "algorithmic_bytes_per_apply": shrink_bytes + expand_bytes,
                   "flops_per_apply": b0.flops(), "single_launch_apply": one_launch, "mixed_form": args.mixed_form,
                   "padded_control": bool(args.padded_control), "concurrent_loads_per_step": args.concurrent_loads,
                   "adapter_bytes_loaded_per_step": load_bytes_per_step, "weight_bytes_read_per_apply": info["weight_bytes"],
                   "parity_max_row_rel_l2": err},
        "roofline": {"bound": "hbm", "kernel": dom if dom_kernel is None else f"{dom}: {dom_kernel}", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     # context: what a kernel that only reads gets from HBM on this chip (1 GB read once by 256 to
                     # 1024 work groups, 8 x 16-byte loads per lane in flight: 6.1 TB/s, measured)
                     "measured_read_ceiling_GBps": measured["read_ceiling_GBps"],
                     "frac_of_measured_read_ceiling": achieved / measured["read_ceiling_GBps"],
                     "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_us": dom_us,
                     "shrink_launch_us": float(shrink_us.mean()), "expand_launch_us": None if one_launch else float(expand_us.mean()),
                     "apply_us": apply_us, "apply_GBps": (shrink_bytes + expand_bytes) / (apply_us * 1e-6) / 1e9,
                     "apply_frac": (shrink_bytes + expand_bytes) / (apply_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                     "apply_mfma_frac": b0.flops() / (apply_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
        "cpu_baseline": cpu,
    }
    for p in pools:
        L.lora_pool_destroy(p)
    L.lora_segments_destroy(seg)
    return out, err


if __name__ == "__main__":
    sys.exit(main())
