#!/usr/bin/env python3
"""Benchmark of the mixed-precision delta linear hot path on one MI355X.

Workloads (`--workload`), all synthetic and seeded (inputs/synth.py), every input resident in HBM before the
timed region:

  c4  (default; the configuration the headline metric is quoted on) the seven linear shapes of one Mistral-7B
      block, 16 experts resident, a decode batch of 64 tokens (`--tokens` for larger batches) routed Zipf(1.1),
      2-bit codes, 64 fp16 salient input channels.  One step = one pass of the batch through all seven linears:
      four library calls, because layers that read the same activations share one (mes_delta_linear_multi):
      [q, k, v], [o], [gate, up], [down].  `--unfused` issues seven single calls.
  c2  q_proj 4096 x 4096, 3 experts, 48 tokens routed 16/16/16; one call per step, rotating over 14 independent
      copies of the weights so that every call streams from HBM and not from the 256 MB on-die cache.
  c3  the three MLP shapes, 3 experts, one 512-token prompt per expert (1536 tokens), 128 salient channels: the
      one-product path, priced against the bf16 matrix-core peak with 2 T d_out d_in flops per call.
  c5  a stack of `--layers` (32) blocks of all seven shapes, 16 experts resident (base bf16 plus packed deltas,
      about 45 GB at 2 bits), a mixed batch of 256 decode tokens and 4 x 1024 prompt tokens; also timed on the
      decode tokens alone and on the prompt tokens alone.
  step  learning the step sizes: loss and straight-through gradient of one MLP matrix per call (512 tokens).
  swap  on-demand swapping of q_proj deltas from pinned host memory (32 experts, 16 device slots).

Protocol: `--warmup` untimed steps, then `--repeats` timed regions of exactly `--steps` steps each, every region
bracketed by events and a device synchronisation on both sides; `ms_per_step` and `value` come from the MEDIAN
region.  A token = one row of x through all the linears of the workload.

Prints ONE JSON line.  `roofline` prices the dominant kernel with ALGORITHMIC bytes (or flops) per launch over
its average duration, measured with HIP events that the library records on the kernel's own stream right around
it; `cpu_baseline` times the fp64 oracle on a bounded sample of the same workload on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X published HBM3E peak
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 matrix-core peak
COPY_PROBE_BYTES = 1 << 30
FUSED_GROUPS = [["q_proj", "k_proj", "v_proj"], ["o_proj"], ["gate_proj", "up_proj"], ["down_proj"]]


def algorithmic_bytes(d_in, d_out, k, bits, n_active, T):
    """Bytes the method must move for one call: base once, each ACTIVE expert's compact codes, fp16
    salient columns, steps and indices, plus x in and y out.  Padding, codes stored at salient
    columns and workspace traffic are not credited."""
    base = 2 * d_out * d_in
    per_expert = d_out * (d_in - k) * bits // 8 + 2 * d_out * k + 4 * d_out + 4 * k
    return base + n_active * per_expert + 2 * T * d_in + 2 * T * d_out


def credited_flops(d_in, d_out, seg, long_min):
    """Flops of one call: the two products of Eq. 4 (4 T d_out d_in) for streamed tokens; a segment that takes the
    one-product path does one product per token and is credited 2 T d_out d_in."""
    f = 0
    for a, b in zip(seg[:-1], seg[1:]):
        f += (2 if b - a >= long_min else 4) * (b - a) * d_out * d_in
    return f


def write_traffic(args):
    """HBM bytes per k_delta_linear launch from hardware counters.  Each counter's reading for the streaming
    kernel is scaled by the same counter's reading for k_copy_probe, which moves a known number of bytes."""
    import csv
    import glob

    def mean_by_kernel(folder, counter):
        files = glob.glob(os.path.join(folder, "**", "*counter_collection.csv"), recursive=True)
        assert files, f"no counter_collection.csv under {folder}"
        acc = {}
        for r in csv.DictReader(open(files[0])):
            if r["Counter_Name"] != counter:
                continue
            for key in ("k_delta_linear", "k_copy_probe"):
                if key in r["Kernel_Name"]:
                    acc.setdefault(key, []).append(float(r["Counter_Value"]))
        assert "k_delta_linear" in acc and "k_copy_probe" in acc, f"{counter}: kernels missing in {files[0]}"
        return {k: (sum(v) / len(v), len(v)) for k, v in acc.items()}

    fetch = mean_by_kernel(args.traffic_from[0], "FETCH_SIZE")
    write = mean_by_kernel(args.traffic_from[1], "WRITE_SIZE")
    f_scale = COPY_PROBE_BYTES / fetch["k_copy_probe"][0]      # bytes per counter unit, from the copy kernel
    w_scale = COPY_PROBE_BYTES / write["k_copy_probe"][0]
    rd = fetch["k_delta_linear"][0] * f_scale
    wr = write["k_delta_linear"][0] * w_scale
    key = f"{args.workload}_b{args.bits}"
    path = os.path.join(ROOT, "profiles", "traffic.json")
    table = json.load(open(path)) if os.path.exists(path) else {}
    table[key] = {"bytes_per_launch": int(rd + wr), "read_bytes_per_launch": int(rd), "write_bytes_per_launch": int(wr),
                  "launches": fetch["k_delta_linear"][1], "fetch_bytes_per_unit": round(f_scale, 3),
                  "write_bytes_per_unit": round(w_scale, 3), "copy_probe_bytes": COPY_PROBE_BYTES,
                  "unfused": bool(args.unfused)}
    json.dump(table, open(path, "w"), indent=1, sort_keys=True)
    print(json.dumps({key: table[key]}))


def timed_regions(step, steps, warmup, repeats):
    """`warmup` untimed steps, then `repeats` regions of exactly `steps` steps; returns the regions' ms per step."""
    import torch
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    out, walls = [], []
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        for i in range(steps):
            step(i)
        ev1.record()
        torch.cuda.synchronize()
        walls.append((time.perf_counter() - t0) * 1e3 / steps)
        out.append(ev0.elapsed_time(ev1) / steps)
    return out, walls


def host_cores():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] or [1]))
    except Exception:
        return os.cpu_count() or 1


class Sampler:
    """What the oracle leg needs of one linear: a seeded sample of its output channels, kept on the host."""

    def __init__(self, seed):
        import torch
        self.g = torch.Generator().manual_seed(seed)
        self.items = []

    def add(self, wl, layer_index, n_rows, grid):
        import torch
        rows = torch.sort(torch.randperm(wl.d_out, generator=self.g)[:n_rows]).values
        rd = rows.to(wl.w_base.device)
        self.items.append(dict(name=wl.name, rows=rows, layer=layer_index, w=wl.w_base[rd].double().cpu().numpy(),
                               x=wl.x.double().cpu().numpy(), deltas=[ex.delta[rd].cpu().numpy() for ex in wl.experts],
                               sidx=[ex.salient_idx.numpy() for ex in wl.experts], seg=list(wl.seg_offsets), bits=wl.bits,
                               d_out=wl.d_out, d_in=wl.d_in, grid=grid))

    def run(self, outputs):
        """Times the oracle on the samples; returns (seconds, fraction of the workload's multiply-adds covered,
        relative Frobenius error and worst element-wise distance in bf16 ulps of the HIP outputs)."""
        import numpy as np
        from oracle import mes_oracle as O
        prepared = []
        for s in self.items:           # offline compression of the sampled rows is not part of the timed oracle work
            exs = []
            for d, si in zip(s["deltas"], s["sidx"]):
                c, st, sal = O.quantize(d, si, s["bits"], s["grid"])
                exs.append(dict(codes=c, step=st, salient=sal, salient_idx=si, bits=s["bits"], grid=s["grid"]))
            prepared.append(exs)
        t0 = time.perf_counter()
        refs = [O.delta_linear(s["x"], s["w"], exs, s["seg"]) for s, exs in zip(self.items, prepared)]
        t_cpu = time.perf_counter() - t0
        num = den = 0.0
        for s, ref in zip(self.items, refs):
            yg = outputs[s["layer"]][:, s["rows"].to(outputs[s["layer"]].device)].double().cpu().numpy()
            num += float(((yg - ref) ** 2).sum())
            den += float((ref ** 2).sum())
        covered = sum(len(s["rows"]) * s["d_in"] for s in self.items)
        return t_cpu, covered, (num / den) ** 0.5


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--repeats", type=int, default=7, help="timed regions of --steps steps; the median is reported")
    ap.add_argument("--workload", default="c4", choices=["c4", "c2", "c3", "c5", "step", "swap"])
    ap.add_argument("--bits", type=int, default=2)
    ap.add_argument("--k", type=int, default=None, help="salient fp16 input channels per expert (default: the workload's)")
    ap.add_argument("--tokens", type=int, default=None, help="c4: decode tokens per batch (default 64); step: calibration tokens")
    ap.add_argument("--layers", type=int, default=32, help="c5: blocks in the stack")
    ap.add_argument("--grid", default="sym", choices=["sym", "eq1"], help="quantisation grid (eq1 needs bits >= 2)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sample-frac", type=int, default=0, help="oracle leg: 1/N of the output channels (default 2 for c4)")
    ap.add_argument("--breakdown", action="store_true", help="also report every call's kernel time (stderr and JSON)")
    ap.add_argument("--unfused", action="store_true", help="c4: seven single-layer calls per step instead of four")
    ap.add_argument("--mlp-act", default="none", choices=["none", "fused", "separate"],
                    help="c4: also form h = SiLU(gate) * up, inside the gate+up call (mes_delta_linear_gated) or by a separate "
                         "elementwise kernel after it (no oracle leg in these modes)")
    ap.add_argument("--graph", action="store_true",
                    help="c4: capture one step as a HIP graph and replay it in the timed region (outputs checked against eager)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="after the measurements run the library's plain copy kernel on 1 GiB (counter calibration)")
    ap.add_argument("--traffic-from", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"),
                    help="no GPU work: read the counter CSVs of two `rocprofv3 --pmc` runs of this script with "
                         "--copy-probe (FETCH_SIZE, then WRITE_SIZE) and write profiles/traffic.json")
    args = ap.parse_args()
    if args.traffic_from:
        write_traffic(args)
        return
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU; --gpus must be 1 (nothing here uses a second GPU).", file=sys.stderr)
        sys.exit(2)
    defaults = {"c4": (200, 20), "c2": (280, 28), "c3": (20, 3), "c5": (2, 1), "step": (20, 3), "swap": (200, 10)}
    if args.steps is None:
        args.steps = defaults[args.workload][0]
    if args.warmup is None:
        args.warmup = defaults[args.workload][1]

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    run = {"c4": bench_decode, "c2": bench_decode, "c3": bench_prefill, "c5": bench_stack, "step": bench_step,
           "swap": bench_swap}[args.workload]
    out = run(args)
    print(json.dumps(out))


def base_record(args, metric, value, unit, ms_per_step, regions, walls, dtype="bf16"):
    return {
        "metric": metric, "value": value, "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "timing": {"repeats": len(regions), "statistic": "median", "ms_per_step_regions": [round(r, 5) for r in regions],
                   "host_wall_ms_per_step": round(statistics.median(walls), 5)},
    }


# ------------------------------------------------------------------------------------------------ c4 / c2

def bench_decode(args):
    import torch

    import paper_2406_09041_amd as mes
    from inputs import synth

    dev = "cuda:0"
    grid = mes.GRID_EQ1 if args.grid == "eq1" else mes.GRID_SYM
    c4 = args.workload == "c4"
    k = 64 if args.k is None else args.k
    n_tokens = args.tokens or 64
    if c4:
        names = [n for n, _, _ in synth.MISTRAL7B_LINEARS]
        makers = [(n, lambda n=n: synth.config4_linear(n, device=dev, bits=args.bits, k=k, n_tokens=n_tokens)) for n in names]
        sample_frac, copies = args.sample_frac or 2, 1
    else:
        # 48 MB per call fits the 256 MB on-die cache: rotate over independent copies so every call streams from HBM
        copies = 14
        makers = [(f"q_proj#{c}", lambda c=c: synth.config2(device=dev, copy=c)) for c in range(copies)]
        sample_frac = args.sample_frac or 8
    layers, sampler, T = [], Sampler(4242), None
    for name, make in makers:
        wl = make()
        T = wl.x.shape[0]
        w_t = mes.mes_pack_base(wl.w_base)
        packed = [mes.mes_pack_delta(ex.delta, ex.salient_idx if wl.k else None, wl.bits, grid) for ex in wl.experts]
        lin = mes.DeltaLinear(w_t, packed, T)
        y = torch.empty((T, wl.d_out), dtype=torch.bfloat16, device=dev)
        n_active = sum(1 for e in range(len(packed)) if wl.seg_offsets[e + 1] > wl.seg_offsets[e])
        layers.append(dict(name=name, lin=lin, x=wl.x, seg=wl.seg_offsets, y=y, d_in=wl.d_in, d_out=wl.d_out, k=wl.k,
                           bits=wl.bits, n_active=n_active,
                           bytes=algorithmic_bytes(wl.d_in, wl.d_out, wl.k, wl.bits, n_active, T)))
        if not args.no_cpu_baseline and (c4 or not sampler.items):
            sampler.add(wl, len(layers) - 1, max(wl.d_out // sample_frac, 16), grid)
        del wl
    torch.cuda.synchronize()
    # ---- the calls of one step
    if c4 and not args.unfused:
        index = {L["name"]: i for i, L in enumerate(layers)}
        groups = [[index[n] for n in g] for g in FUSED_GROUPS]        # layers that read the same activations share a call
    else:
        groups = [[i] for i in range(len(layers))]
    calls = []
    for g_ in groups:
        Ls = [layers[i] for i in g_]
        if len(Ls) == 1:
            L = Ls[0]
            calls.append(dict(name=L["name"], bytes=L["bytes"], ys=[L["y"]], run=(lambda L=L: L["lin"](L["x"], L["seg"], L["y"]))))
        elif args.mlp_act == "fused" and [L["name"] for L in Ls] == ["gate_proj", "up_proj"]:
            g_, u_ = Ls
            gated = mes.DeltaLinearGated(g_["lin"].w, g_["lin"].experts, u_["lin"].w, u_["lin"].experts, T)
            h = torch.empty((T, g_["d_out"]), dtype=torch.bfloat16, device=dev)
            nbytes = g_["bytes"] + u_["bytes"] - 2 * T * g_["d_in"] - 2 * T * g_["d_out"]   # x read once, one output
            calls.append(dict(name="SiLU(gate_proj)*up_proj", bytes=nbytes, ys=[h],
                              run=(lambda gated=gated, L0=g_, h=h: gated(L0["x"], L0["seg"], h))))
        else:
            assert all(torch.equal(L["x"], Ls[0]["x"]) and L["seg"] == Ls[0]["seg"] for L in Ls), \
                "fused layers must read the same activations and routing"
            fused = mes.DeltaLinearMulti([(L["lin"].w, L["lin"].experts) for L in Ls], T)
            ys = [L["y"] for L in Ls]
            nbytes = sum(L["bytes"] for L in Ls) - (len(Ls) - 1) * 2 * T * Ls[0]["d_in"]   # the shared activations are read once
            run = (lambda fused=fused, L0=Ls[0], ys=ys: fused(L0["x"], L0["seg"], ys))
            if args.mlp_act == "separate" and [L["name"] for L in Ls] == ["gate_proj", "up_proj"]:
                h = torch.empty_like(ys[0])

                def run(fused=fused, L0=Ls[0], ys=ys, h=h):
                    fused(L0["x"], L0["seg"], ys)
                    torch.mul(torch.nn.functional.silu(ys[0]), ys[1], out=h)
            calls.append(dict(name="+".join(L["name"] for L in Ls), bytes=nbytes, ys=ys, run=run))
    calls_per_step = len(calls) if c4 else 1

    def one_step(i):
        if c4:
            for c in calls:
                c["run"]()
        else:
            calls[i % copies]["run"]()

    step_fn, graph = one_step, None
    if args.graph:
        # One step captured as a HIP graph and replayed: same kernels, same arguments, launch overhead paid once.
        # The library never synchronises, allocates or clears memory in these calls, so they can be captured; the
        # replayed outputs are compared bit for bit with the eager ones, with eager work in between.
        assert c4, "--graph replays the whole c4 step"
        one_step(0)
        torch.cuda.synchronize()
        eager = [[y.clone() for y in c["ys"]] for c in calls]
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            one_step(0)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            one_step(0)
        for _ in range(3):
            for c in calls:
                for y in c["ys"]:
                    y.fill_(0)
            graph.replay()
            torch.cuda.synchronize()
            for c, ref in zip(calls, eager):
                for y, r in zip(c["ys"], ref):
                    assert torch.equal(y, r), "graph replay differs from the eager result"
            one_step(0)                                   # eager work between the replays
            torch.cuda.synchronize()
        step_fn = lambda i: graph.replay()
    regions, walls = timed_regions(step_fn, args.steps, args.warmup, args.repeats)
    ms_per_step = statistics.median(regions)

    # ---- roofline of the dominant kernel: the library records HIP events on the call's own stream right around
    # k_delta_linear.  The same step sequence is replayed (caches in the same state); every call is read back before
    # the next one is issued, because an event recorded while earlier kernels are still running is stamped early.
    n_steps_timed = max(5, min(25, args.steps))
    timer = mes.KernelTimer()
    kernel_us = [0.0] * len(calls)
    plan = []
    for r in range(n_steps_timed):
        for ci, c in (enumerate(calls) if c4 else [(r % copies, calls[r % copies])]):
            timer.arm()
            c["run"]()
            kernel_us[ci] += timer.elapsed_us()
            plan.append(ci)
    n_launches = len(plan)
    step_bytes = sum(c["bytes"] for c in calls) if c4 else calls[0]["bytes"]
    launch_bytes = step_bytes / calls_per_step
    launch_us = sum(kernel_us) / n_launches
    achieved = launch_bytes / (launch_us * 1e-6) / 1e9

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath) and n_tokens == 64 and k == 64 and grid == mes.GRID_SYM and not args.unfused:
        try:
            traffic = json.load(open(tpath)).get(f"{args.workload}_b{args.bits}", {}).get("bytes_per_launch")
        except Exception:
            traffic = None

    breakdown = None
    if args.breakdown and c4:
        breakdown = {c["name"]: dict(kernel_us=round(kernel_us[ci] / n_steps_timed, 2), MB=round(c["bytes"] / 1e6, 2),
                                     GBs=round(c["bytes"] / (kernel_us[ci] / n_steps_timed) / 1e3, 1)) for ci, c in enumerate(calls)}
        print("breakdown:", json.dumps(breakdown), file=sys.stderr)

    if args.copy_probe:
        src = torch.empty(COPY_PROBE_BYTES, dtype=torch.uint8, device=dev).random_(0, 256)
        dst = torch.empty_like(src)
        for _ in range(3):
            mes.mes_copy_probe(dst, src)
        torch.cuda.synchronize()
        del src, dst

    cpu_baseline = parity = None
    if not args.no_cpu_baseline and args.mlp_act == "none":
        one_step(0)
        torch.cuda.synchronize()
        t_cpu, covered, parity = sampler.run([L["y"] for L in layers])
        total = sum(L["d_out"] * L["d_in"] for L in layers) if c4 else layers[0]["d_out"] * layers[0]["d_in"]
        cpu_baseline = dict(value=round(T / (t_cpu * total / covered), 2), unit="tokens/s", cores=host_cores(), kind="oracle",
                            sample=f"fp64 numpy oracle on a seeded 1/{sample_frac} sample of the output channels of "
                                   f"{'each of the 7 linears' if c4 else 'one q_proj copy'}, all {T} tokens and all experts "
                                   f"({t_cpu:.2f} s of CPU work), scaled linearly by rows (extrapolated)")

    whole_gbs = step_bytes / (ms_per_step * 1e-3) / 1e9
    out = base_record(args, "tokens/s + achieved HBM GB/s, 16-expert Mistral-7B-shape decode delta linear",
                      round(T / (ms_per_step * 1e-3), 1), "tokens/s", ms_per_step, regions, walls)
    out["config"] = {
        "workload": (f"c4: 7 Mistral-7B linear shapes of one block, 16 experts, {T} decode tokens, Zipf(1.1) routing, "
                     f"{args.bits}-bit codes ({args.grid} grid), {k} fp16 salient channels") if c4 else
                    f"c2: Mistral-7B q_proj 4096x4096, 3 experts, 48 decode tokens 16/16/16, 2-bit, 64 salient; {copies} rotating copies",
        "tokens": T, "experts": 16 if c4 else 3, "bits": args.bits, "calls_per_step": calls_per_step,
        "graph_replay": bool(args.graph), "mlp_act": args.mlp_act, "fused_calls": [c["name"] for c in calls] if c4 else None,
        "active_experts": layers[0]["n_active"]}
    out["roofline"] = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "kernel": "k_delta_linear",
                       "algorithmic_bytes_per_launch": int(launch_bytes), "avg_launch_us": round(launch_us, 3),
                       "launches_timed": n_launches,
                       "whole_step": {"algorithmic_bytes": int(step_bytes), "GBs": round(whole_gbs, 1),
                                      "frac": round(whole_gbs / HBM_PEAK_GBS, 4),
                                      "note": "all kernels of a step (preparation, streaming, split reduction) over the median step time"}}
    out["cpu_baseline"] = cpu_baseline
    out["parity_rel_fro_vs_oracle_sample"] = None if parity is None else float(f"{parity:.3e}")
    if breakdown:
        out["breakdown"] = breakdown
    return out


# ------------------------------------------------------------------------------------------------ c3

def bench_prefill(args):
    import torch

    import paper_2406_09041_amd as mes
    from inputs import synth

    dev = "cuda:0"
    grid = mes.GRID_EQ1 if args.grid == "eq1" else mes.GRID_SYM
    long_min = mes.binding.lib.mes_long_segment_tokens()
    sampler = Sampler(4343)
    calls, T = [], None
    for which in ("gate_proj", "up_proj", "down_proj"):
        wl = synth.config3(which, bits=args.bits, device=dev)
        T = wl.x.shape[0]
        w_t = mes.mes_pack_base(wl.w_base)
        packed = [mes.mes_pack_delta(ex.delta, ex.salient_idx, wl.bits, grid) for ex in wl.experts]
        lin = mes.DeltaLinear(w_t, packed, T)
        y = torch.empty((T, wl.d_out), dtype=torch.bfloat16, device=dev)
        calls.append(dict(name=which, y=y, flops=credited_flops(wl.d_in, wl.d_out, wl.seg_offsets, long_min),
                          bytes=algorithmic_bytes(wl.d_in, wl.d_out, wl.k, wl.bits, 3, T),
                          run=(lambda lin=lin, wl=wl, y=y: lin(wl.x, wl.seg_offsets, y))))
        if not args.no_cpu_baseline:
            sampler.add(wl, len(calls) - 1, args.sample_frac and wl.d_out // args.sample_frac or 64, grid)
        del wl
    torch.cuda.synchronize()

    def one_step(i):
        for c in calls:
            c["run"]()
    regions, walls = timed_regions(one_step, args.steps, args.warmup, args.repeats)
    ms_per_step = statistics.median(regions)
    n_steps_timed = max(5, min(20, args.steps))
    timer = mes.KernelTimer()
    kernel_us = [0.0] * len(calls)
    for r in range(n_steps_timed):
        for ci, c in enumerate(calls):
            timer.arm()
            c["run"]()
            kernel_us[ci] += timer.elapsed_us()       # read back before the next call is issued
    step_flops = sum(c["flops"] for c in calls)
    launch_us = sum(kernel_us) / (n_steps_timed * len(calls))
    achieved = step_flops / len(calls) / (launch_us * 1e-6) / 1e12
    breakdown = {c["name"]: dict(kernel_us=round(kernel_us[ci] / n_steps_timed, 2),
                                 TFLOPs=round(c["flops"] / (kernel_us[ci] / n_steps_timed * 1e-6) / 1e12, 1))
                 for ci, c in enumerate(calls)}
    cpu_baseline = parity = None
    if not args.no_cpu_baseline:
        t_cpu, covered, parity = sampler.run([c["y"] for c in calls])
        total = sum(d_out * d_in for _, d_in, d_out in synth.MISTRAL7B_LINEARS[4:])
        cpu_baseline = dict(value=round(T / (t_cpu * total / covered), 2), unit="tokens/s", cores=host_cores(), kind="oracle",
                            sample=f"fp64 numpy oracle on 64 seeded output channels of each of the 3 matrices, all {T} tokens "
                                   f"({t_cpu:.2f} s of CPU work), scaled linearly by rows (extrapolated)")
    whole = step_flops / (ms_per_step * 1e-3) / 1e12
    out = base_record(args, "tokens/s + bf16 MFMA utilisation, Mistral-7B MLP prefill delta linear (3 experts x 512 tokens)",
                      round(T / (ms_per_step * 1e-3), 1), "tokens/s", ms_per_step, regions, walls)
    out["config"] = {"workload": f"c3: gate/up 4096->14336 and down 14336->4096, 3 experts, 3 x 512 prompt tokens, "
                                 f"{args.bits}-bit codes ({args.grid} grid), 128 fp16 salient channels; one call per matrix",
                     "tokens": T, "experts": 3, "bits": args.bits, "calls_per_step": len(calls)}
    out["roofline"] = {"bound": "mfma", "achieved": round(achieved, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                       "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None, "kernel": "k_prefill_fused",
                       "algorithmic_flops_per_launch": int(step_flops / len(calls)), "avg_launch_us": round(launch_us, 3),
                       "launches_timed": n_steps_timed * len(calls),
                       "flops_rule": "2 T d_out d_in per call: the one-product path multiplies once per token",
                       "whole_step": {"TFLOPs": round(whole, 1), "frac": round(whole / MFMA_BF16_PEAK_TFLOPS, 4)}}
    out["cpu_baseline"] = cpu_baseline
    out["parity_rel_fro_vs_oracle_sample"] = None if parity is None else float(f"{parity:.3e}")
    out["breakdown"] = breakdown
    return out


# ------------------------------------------------------------------------------------------------ c5

def bench_stack(args):
    import torch

    import paper_2406_09041_amd as mes
    from inputs import synth

    dev = "cuda:0"
    grid = mes.GRID_EQ1 if args.grid == "eq1" else mes.GRID_SYM
    long_min = mes.binding.lib.mes_long_segment_tokens()
    k = 64 if args.k is None else args.k
    E = 16
    parts = {p: synth.config5_routing(p) for p in ("mixed", "decode", "prefill")}
    T = parts["mixed"][-1]
    shapes = {n: (di, do) for n, di, do in synth.MISTRAL7B_LINEARS}
    # one activation batch per input width, shared by every layer (the shapes do not chain); the decode tokens of every
    # expert come first in its segment, so the sub-batches are gathered rows of the mixed batch
    xs = {w: synth.normal((T, w), 1.0, synth.seed_for(5, 0, 0, 3 + 16 * i), dev, torch.bfloat16) for i, w in enumerate((4096, 14336))}
    sub_rows = {}
    for p in ("decode", "prefill"):
        rows = []
        for e in range(E):
            lo, hi = parts["mixed"][e], parts["mixed"][e + 1]
            n_dec = parts["decode"][e + 1] - parts["decode"][e]
            rows += list(range(lo, lo + n_dec)) if p == "decode" else list(range(lo + n_dec, hi))
        sub_rows[p] = torch.tensor(rows, dtype=torch.long, device=dev)
    xpart = {"mixed": xs}
    for p in ("decode", "prefill"):
        xpart[p] = {w: xs[w][sub_rows[p]].contiguous() for w in xs}
    # workspaces, one per call shape, shared by all layers (the calls are stream-ordered)
    ws = {}
    for g in FUSED_GROUPS:
        d_in, d_outs = shapes[g[0]][0], [shapes[n][1] for n in g]
        nbytes = mes.DeltaLinearMulti.workspace_bytes(d_in, d_outs, T)
        ws["+".join(g)] = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    ys = {p: {n: torch.empty((parts[p][-1], do), dtype=torch.bfloat16, device=dev) for n, (di, do) in shapes.items()} for p in parts}
    t_setup = time.perf_counter()
    stack, sampler = [], Sampler(4545)
    resident = 0
    for layer in range(args.layers):
        packed_layer = {}
        for n, (d_in, d_out) in shapes.items():
            wl = synth.config5_linear(n, layer=layer, bits=args.bits, device=dev, k=k)
            wl.x = xs[d_in]                                   # the shared batch (same routing, see config5_routing)
            w_t = mes.mes_pack_base(wl.w_base)
            packed = [mes.mes_pack_delta(ex.delta, ex.salient_idx if k else None, args.bits, grid) for ex in wl.experts]
            packed_layer[n] = (w_t, packed)
            resident += w_t.numel() + sum(p.codes.numel() + 4 * p.step.numel() + (p.salient.numel() if p.salient is not None else 0) for p in packed)
            if not args.no_cpu_baseline and layer < 2:
                sampler.add(wl, (layer, n), 128, grid)
            del wl
        calls = []
        for g in FUSED_GROUPS:
            fused = mes.DeltaLinearMulti([packed_layer[n] for n in g], T, workspace=ws["+".join(g)])
            calls.append((g, fused))
        stack.append(calls)
        if layer % 4 == 3:
            print(f"c5: layer {layer + 1}/{args.layers} packed ({resident / 1e9:.1f} GB resident, "
                  f"{time.perf_counter() - t_setup:.0f} s)", file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    keep = {}

    def make_step(p):
        seg = parts[p]

        def step(i, capture=None):
            for li, calls in enumerate(stack):
                for g, fused in calls:
                    outs = [ys[p][n] for n in g]
                    fused(xpart[p][shapes[g[0]][0]], seg, outs)
                    if capture is not None and li in capture:
                        for n in g:
                            keep[(li, n)] = ys[p][n].clone()
        return step

    results = {}
    n_act = {p: sum(1 for e in range(E) if parts[p][e + 1] > parts[p][e]) for p in parts}
    for p in ("mixed", "decode", "prefill"):
        step = make_step(p)
        regions, walls = timed_regions(step, args.steps, args.warmup, args.repeats if p == "mixed" else max(3, args.repeats // 2))
        ms = statistics.median(regions)
        Tp = parts[p][-1]
        nbytes = args.layers * sum(algorithmic_bytes(di, do, k, args.bits, n_act[p], Tp) for di, do in shapes.values())
        flops = args.layers * sum(credited_flops(di, do, parts[p], long_min) for di, do in shapes.values())
        results[p] = dict(tokens=Tp, ms_per_step=round(ms, 4), tokens_per_s=round(Tp / (ms * 1e-3), 1), active_experts=n_act[p],
                          regions=[round(r, 4) for r in regions], walls=walls,
                          algorithmic_GB=round(nbytes / 1e9, 3), hbm_GBs=round(nbytes / (ms * 1e-3) / 1e9, 1),
                          hbm_frac=round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                          credited_TFLOP=round(flops / 1e12, 3), TFLOPs=round(flops / (ms * 1e-3) / 1e12, 1),
                          mfma_frac=round(flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4))
        print(f"c5 {p}: {json.dumps({k_: v for k_, v in results[p].items() if k_ != 'walls'})}", file=sys.stderr, flush=True)
    cpu_baseline = parity = None
    if not args.no_cpu_baseline:
        make_step("mixed")(0, capture={0, 1})
        torch.cuda.synchronize()
        t_cpu, covered, parity = sampler.run(keep)
        total = args.layers * sum(di * do for di, do in shapes.values())
        cpu_baseline = dict(value=round(T / (t_cpu * total / covered), 3), unit="tokens/s", cores=host_cores(), kind="oracle",
                            sample=f"fp64 numpy oracle on 128 seeded output channels of each of the 7 linears of the first "
                                   f"{min(2, args.layers)} layers, all {T} tokens of the mixed batch ({t_cpu:.2f} s of CPU work), "
                                   f"scaled linearly by rows and layers (extrapolated)")
    m = results["mixed"]
    out = base_record(args, "tokens/s, 32-layer stack of Mistral-7B-shaped delta linears, mixed decode + prefill batch",
                      m["tokens_per_s"], "tokens/s", m["ms_per_step"], m["regions"], m.pop("walls"))
    for p in ("decode", "prefill"):
        results[p].pop("walls")
    out["config"] = {"workload": f"c5: {args.layers} layers x 7 Mistral-7B linear shapes, 16 experts resident, mixed batch of 256 decode "
                                 f"tokens + 4 x 1024 prompt tokens, Zipf(1.1) routing per query, {args.bits}-bit codes ({args.grid} grid), "
                                 f"{k} fp16 salient channels; 4 fused calls per layer",
                     "tokens": T, "experts": E, "bits": args.bits, "layers": args.layers, "calls_per_step": 4 * args.layers,
                     "resident_GB": round(resident / 1e9, 2), "segments": [b - a for a, b in zip(parts["mixed"][:-1], parts["mixed"][1:])]}
    out["roofline"] = {"bound": "mfma", "achieved": m["TFLOPs"], "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                       "frac": m["mfma_frac"], "traffic": None, "kernel": "whole step (k_prefill_fused dominates)",
                       "flops_rule": "2 T d_out d_in for tokens of segments on the one-product path, 4 T d_out d_in for streamed tokens",
                       "sub_batches": {"mixed": m, "decode_only": results["decode"], "prefill_only": results["prefill"]}}
    out["cpu_baseline"] = cpu_baseline
    out["parity_rel_fro_vs_oracle_sample"] = None if parity is None else float(f"{parity:.3e}")
    return out


# ------------------------------------------------------------------------------------------------ step-size learning

def bench_step(args):
    import numpy as np
    import torch

    import paper_2406_09041_amd as mes
    from inputs import synth

    dev = "cuda:0"
    gridv = 1 if args.grid == "eq1" else 0
    tokens = args.tokens or 512
    k = 8 if args.k is None else args.k
    shrink = 0.6                       # step = 0.6 x the max-abs step, so that a few per cent of the weights clamp
    z = 2.0 ** (args.bits - 1) - (0.5 if gridv == 0 else 1.0)
    shapes = {"gate_proj": (4096, 14336), "up_proj": (4096, 14336), "down_proj": (14336, 4096)}
    calls = []
    for i, (which, (d_in, d_out)) in enumerate(shapes.items()):
        ex = synth.make_delta(d_in, d_out, k, 0.003, 15.0, synth.seed_for(951, 0, i, 2), dev)
        x = synth.normal((tokens, d_in), 1.0, synth.seed_for(951, 0, i, 3), dev, torch.bfloat16)
        ns = torch.ones(d_in, dtype=torch.bool, device=dev)
        ns[ex.salient_idx.to(dev).long()] = False
        step = (ex.delta[:, ns].abs().amax(dim=1) / max(z, 0.5) * shrink).float().contiguous()
        sg = mes.StepGrad(ex.delta, ex.salient_idx, args.bits, gridv, tokens)
        calls.append(dict(name=which, sg=sg, step=step, x=x, ex=ex, flops=2 * 2.0 * tokens * d_out * d_in,
                          run=(lambda sg=sg, step=step, x=x: sg(step, x))))

    def one_step(i):
        for c in calls:
            c["run"]()
    regions, walls = timed_regions(one_step, args.steps, args.warmup, args.repeats)
    ms_per_step = statistics.median(regions)
    n_timed = max(5, min(20, args.steps))
    timer = mes.KernelTimer()
    kernel_us = [0.0] * len(calls)
    for r in range(n_timed):
        for ci, c in enumerate(calls):
            timer.arm()
            c["run"]()
            kernel_us[ci] += timer.elapsed_us() / n_timed
    flops = sum(c["flops"] for c in calls)
    launch_us = sum(kernel_us) / len(calls)
    achieved = flops / len(calls) / (launch_us * 1e-6) / 1e12
    cpu_baseline = parity = None
    if not args.no_cpu_baseline:
        from oracle import step_oracle as SO
        c = calls[0]
        g = torch.Generator().manual_seed(7)
        rows = torch.sort(torch.randperm(c["ex"].delta.shape[0], generator=g)[:256]).values
        rd = rows.to(dev)
        t0 = time.perf_counter()
        loss_o, grad_o = SO.step_loss_grad(c["ex"].delta[rd].cpu().numpy(), c["x"].double().cpu().numpy(),
                                           c["ex"].salient_idx.numpy(), args.bits, gridv, c["step"][rd].cpu().numpy())
        t_cpu = time.perf_counter() - t0
        loss_g, grad_g = c["sg"](c["step"], c["x"])
        torch.cuda.synchronize()
        gg = grad_g[rd].double().cpu().numpy()
        parity = float(np.linalg.norm(gg - grad_o) / np.linalg.norm(grad_o))
        frac = 256 * 4096 / sum(do * di for di, do in shapes.values())
        cpu_baseline = dict(value=round(tokens / (t_cpu / frac), 2), unit="tokens/s", cores=host_cores(), kind="oracle",
                            sample=f"fp64 numpy oracle (loss and gradient) on 256 seeded output channels of gate_proj, all {tokens} "
                                   f"tokens ({t_cpu:.2f} s of CPU work), scaled linearly by rows to the three matrices (extrapolated)")
    out = base_record(args, "calibration tokens/s + bf16 MFMA utilisation, step-size loss and gradient of the Mistral-7B MLP matrices",
                      round(tokens / (ms_per_step * 1e-3), 1), "tokens/s", ms_per_step, regions, walls)
    out["config"] = {"workload": f"step: loss + straight-through gradient of the step sizes, gate/up/down of one Mistral-7B block, {tokens} "
                                 f"calibration tokens, {args.bits}-bit codes ({args.grid} grid), {k} fp16 salient channels; one call per matrix",
                     "tokens": tokens, "bits": args.bits, "calls_per_step": len(calls)}
    out["roofline"] = {"bound": "mfma", "achieved": round(achieved, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                       "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None, "kernel": "k_step_grad",
                       "algorithmic_flops_per_launch": int(flops / len(calls)), "avg_launch_us": round(launch_us, 3),
                       "flops_rule": "two products of 2 N d_out d_in per call (residual and slope)"}
    out["cpu_baseline"] = cpu_baseline
    out["parity_rel_2norm_grad_vs_oracle_sample"] = parity
    out["breakdown"] = {c["name"]: round(kernel_us[ci], 2) for ci, c in enumerate(calls)}
    return out


# ------------------------------------------------------------------------------------------------ on-demand swapping

def bench_swap(args):
    """One Mistral-7B block (the seven linears, four fused calls) decoding 64-token batches whose experts come from a
    pool: 32 experts' packed deltas in pinned host memory (one blob per expert for the whole block), 20 device slots.
    Three variants of the same step sequence: deltas loaded on demand (a miss stalls the batch), the experts of the
    batch four steps ahead prefetched right after the current batch is enqueued (a sequence keeps its expert and a
    new one is known from its admission on), and every expert resident."""
    import numpy as np
    import torch

    import paper_2406_09041_amd as mes
    from inputs import synth

    dev = "cuda:0"
    n_experts, n_slots, ahead, max_active = 32, 20, 4, 16
    k, bits = 64 if args.k is None else args.k, args.bits
    shapes = [(di, do) for _, di, do in synth.MISTRAL7B_LINEARS]
    names = [n for n, _, _ in synth.MISTRAL7B_LINEARS]
    w_t = [mes.mes_pack_base(synth.normal((do, di), 0.02, 11 + i, dev, torch.bfloat16)) for i, (di, do) in enumerate(shapes)]
    pool = mes.ExpertPool([s[0] for s in shapes], [s[1] for s in shapes], [k] * 7, bits, mes.GRID_SYM, n_slots, n_experts, device=dev)
    resident = []
    for e in range(n_experts):
        pks = []
        for i, (di, do) in enumerate(shapes):
            ex = synth.make_delta(di, do, k, 0.003, 15.0, 5000 + 16 * e + i, dev)
            pks.append(mes.mes_pack_delta(ex.delta, ex.salient_idx if k else None, bits))
            del ex
        pool.register(e, pks)
        resident.append(pks)
    expert_bytes = sum(mes.codes_bytes(di, do, bits) + 4 * do + (mes.salient_bytes(do, k) + 4 * k if k else 0) for di, do in shapes)
    index = {n: i for i, n in enumerate(names)}
    groups = [[index[n] for n in g] for g in FUSED_GROUPS]
    ws = torch.empty(max(mes.DeltaLinearMulti.workspace_bytes(shapes[g[0]][0], [shapes[i][1] for i in g], 64) for g in groups),
                     dtype=torch.uint8, device=dev)
    xs = {di: synth.normal((64, di), 1.0, 12 + di, dev, torch.bfloat16) for di in {s[0] for s in shapes}}
    ys = [torch.empty((64, do), dtype=torch.bfloat16, device=dev) for _, do in shapes]
    # (a) what a miss costs: fill all slots from the host, timed on the compute stream (which waits for the copies)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fills = []
    for rep in range(4):
        ids = [(rep * n_slots + i) % n_experts for i in range(n_slots)]
        before = pool.stats()[1]
        torch.cuda.synchronize()
        ev0.record()
        pool.acquire(ids)
        ev1.record()
        torch.cuda.synchronize()
        missed = pool.stats()[1] - before
        if missed:
            fills.append((missed * expert_bytes / 1e9) / (ev0.elapsed_time(ev1) * 1e-3))
    # (b) decode steps.  A query is routed once and keeps its expert while it decodes: the batch holds 64 sequences,
    # every step `churn` of them finish and as many new ones (experts drawn Zipf(1.1) over all registered experts)
    # take their places.  A draw that would put more than 16 experts into one batch is repeated.
    rng = np.random.default_rng(3)
    p = 1.0 / np.arange(1, n_experts + 1) ** 1.1
    p /= p.sum()
    churn = 2
    seqs = list(rng.choice(n_experts, size=64, p=p))
    while len(set(seqs)) > max_active:
        seqs[int(rng.integers(64))] = int(rng.choice(n_experts, p=p))
    batches = []
    for _ in range(args.steps):
        for _ in range(churn):
            pos = int(rng.integers(64))
            while True:
                e = int(rng.choice(n_experts, p=p))
                if len(set(seqs[:pos] + [e] + seqs[pos + 1:])) <= max_active:
                    break
            seqs[pos] = e
        uniq, counts = np.unique(np.asarray(seqs), return_counts=True)
        batches.append((uniq.tolist(), [0] + np.cumsum(counts).tolist()))

    def run_calls(desc_of, seg):
        T = seg[-1]
        for g in groups:
            mes.mes_delta_linear_multi_descriptors([w_t[i] for i in g], [desc_of(i) for i in g], xs[shapes[g[0]][0]][:T], seg, ws,
                                                   [ys[i][:T] for i in g])

    def swap_step(i, prefetch):
        ids, seg = batches[i % len(batches)]
        desc = pool.acquire(ids)
        run_calls(lambda l: desc[l], seg)
        if prefetch:
            # a new sequence is known when it is admitted, a few steps before it joins the decoding batch (its prompt
            # is processed first): its expert is requested `ahead` steps early.  One expert takes about three steps'
            # time to cross the host link.
            pool.prefetch(batches[(i + ahead) % len(batches)][0])

    res_desc = {}

    def resident_step(i):
        ids, seg = batches[i % len(batches)]
        key = i % len(batches)
        if key not in res_desc:
            res_desc[key] = [(mes.binding.mes_delta * len(ids))(*[resident[e][l].descriptor() for e in ids]) for l in range(7)]
        run_calls(lambda l: res_desc[key][l], seg)

    results = {}
    for name, fn in (("on_demand", lambda i: swap_step(i, False)), ("prefetch", lambda i: swap_step(i, True))):
        h0, m0, b0 = pool.stats()
        regions, walls = timed_regions(fn, args.steps, args.warmup, max(3, args.repeats // 2))
        h1, m1, b1 = pool.stats()
        n_calls = args.warmup + args.steps * len(regions)
        results[name] = dict(ms_per_step=round(statistics.median(regions), 4), regions=[round(r, 4) for r in regions],
                             hit_rate=round((h1 - h0) / max(h1 - h0 + m1 - m0, 1), 4),
                             MB_copied_per_step=round((b1 - b0) / n_calls / 1e6, 3), walls=walls)
    res_regions, _ = timed_regions(resident_step, args.steps, args.warmup, max(3, args.repeats // 2))
    ms_res = statistics.median(res_regions)
    best = results["prefetch"]
    out = base_record(args, "tokens/s, one Mistral-7B block decoding with on-demand swapping of the deltas from pinned host memory "
                            "(next batch prefetched)", round(64 / (best["ms_per_step"] * 1e-3), 1), "tokens/s", best["ms_per_step"],
                      best["regions"], best.pop("walls"))
    results["on_demand"].pop("walls")
    out["config"] = {"workload": f"swap: the 7 linears of a Mistral-7B block (4 fused calls), {bits}-bit, {k} salient, {n_experts} experts in "
                                 f"pinned host memory (one blob per expert), {n_slots} device slots, 64 decoding sequences that keep their "
                                 f"expert, {churn} of them replaced per step by new Zipf(1.1)-routed ones, LRU over requests, prefetch {ahead} steps ahead",
                     "tokens": 64, "expert_MB": round(expert_bytes / 1e6, 3)}
    out["roofline"] = {"bound": "pcie", "achieved": round(best["MB_copied_per_step"] / best["ms_per_step"], 2), "peak": None, "unit": "GB/s",
                       "frac": None, "traffic": None, "kernel": "host-to-device copies of missed experts (one per expert)",
                       "fill_GBs": [round(f, 1) for f in fills]}
    out["swap"] = {"on_demand": results["on_demand"], "prefetch": results["prefetch"], "ms_per_step_all_resident": round(ms_res, 4)}
    out["cpu_baseline"] = None
    return out


if __name__ == "__main__":
    main()
