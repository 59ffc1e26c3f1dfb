#!/usr/bin/env python3
"""Benchmark of the mixed-precision delta linear hot path on one MI355X.

Workload (config "c4", the one the headline metric is quoted on): the seven linear shapes of one
Mistral-7B block, 16 experts resident, a decode batch of 64 tokens routed Zipf(1.1), 2-bit
non-salient codes, 64 fp16 salient input channels.  One "step" = one pass of that batch through
all seven linears: four library calls, because layers that read the same activations share one
(mes_delta_linear_multi): [q, k, v], [o], [gate, up], [down].  `--unfused` issues seven single calls.
A token = one row of x through all seven.

Prints ONE JSON line.  `value` is tokens/s with every input already resident in HBM.
`roofline` prices the hot kernel against the HBM peak with ALGORITHMIC bytes; `cpu_baseline`
times the fp64 oracle on a bounded sample of the same workload on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E peak


def algorithmic_bytes(d_in, d_out, k, bits, n_active, T):
    """Bytes the method must move for one call: base once, each ACTIVE expert's compact codes, fp16
    salient columns, steps and indices, plus x in and y out.  Padding, codes stored at salient
    columns and workspace traffic are not credited."""
    base = 2 * d_out * d_in
    per_expert = d_out * (d_in - k) * bits // 8 + 2 * d_out * k + 4 * d_out + 4 * k
    return base + n_active * per_expert + 2 * T * d_in + 2 * T * d_out


COPY_PROBE_BYTES = 1 << 30


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="c4", choices=["c4", "c2"])
    ap.add_argument("--bits", type=int, default=2)
    ap.add_argument("--k", type=int, default=64, help="salient fp16 input channels per expert (c4 only)")
    ap.add_argument("--grid", default="sym", choices=["sym", "eq1"], help="quantisation grid (eq1 needs bits >= 2)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sample-frac", type=int, default=0, help="oracle leg: 1/N of the output channels (default 2 for c4)")
    ap.add_argument("--breakdown", action="store_true", help="also time every call on its own (stderr)")
    ap.add_argument("--unfused", action="store_true", help="seven single-layer calls per step instead of four")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step as a HIP graph and replay it in the timed region (outputs checked against eager)")
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

    import numpy as np
    import torch

    import paper_2406_09041_amd as mes
    from inputs import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)

    # ---------------------------------------------------------------- build the workload in HBM
    layers = []          # one entry per mes_delta_linear call of a step
    samples = []         # what the oracle leg needs (a seeded sample of output channels), kept on the host
    g = torch.Generator().manual_seed(4242)
    if args.workload == "c4":
        names = [n for n, _, _ in synth.MISTRAL7B_LINEARS]
        wls = [(n, lambda n=n: synth.config4_linear(n, device=dev, bits=args.bits, k=args.k)) for n in names]
        sample_frac = 2
        copies = 1
    else:
        # 48 MB per call fits the 256 MB Infinity Cache: rotate over independent copies so every call streams from HBM
        copies = 14
        wls = [(f"q_proj#{c}", lambda c=c: synth.config2(device=dev, copy=c)) for c in range(copies)]
        sample_frac = 8
    T = None
    for name, make in wls:
        wl = make()
        T = wl.x.shape[0]
        w_t = mes.mes_pack_base(wl.w_base)
        grid = mes.GRID_EQ1 if args.grid == "eq1" else mes.GRID_SYM
        packed = [mes.mes_pack_delta(ex.delta, ex.salient_idx, wl.bits, grid) for ex in wl.experts]
        lin = mes.DeltaLinear(w_t, packed, T)
        y = torch.empty((T, wl.d_out), dtype=torch.bfloat16, device=dev)
        n_active = sum(1 for e in range(len(packed)) if wl.seg_offsets[e + 1] > wl.seg_offsets[e])
        layers.append(dict(name=name, lin=lin, x=wl.x, seg=wl.seg_offsets, y=y, d_in=wl.d_in, d_out=wl.d_out,
                           k=wl.k, bits=wl.bits, n_active=n_active,
                           bytes=algorithmic_bytes(wl.d_in, wl.d_out, wl.k, wl.bits, n_active, T)))
        if not args.no_cpu_baseline and (args.workload == "c4" or len(samples) == 0):
            rows = torch.sort(torch.randperm(wl.d_out, generator=g)[: max(wl.d_out // (args.sample_frac or sample_frac), 16)]).values
            rd = rows.to(dev)
            samples.append(dict(name=name, rows=rows, layer=len(layers) - 1,
                                w=wl.w_base[rd].double().cpu().numpy(), x=wl.x.double().cpu().numpy(),
                                deltas=[ex.delta[rd].cpu().numpy() for ex in wl.experts],
                                sidx=[ex.salient_idx.numpy() for ex in wl.experts], seg=wl.seg_offsets,
                                bits=wl.bits, d_out=wl.d_out))
        del wl
    torch.cuda.synchronize()
    # ---------------------------------------------------------------- the calls of one step
    if args.workload == "c4" and not args.unfused:
        groups = [[0, 1, 2], [3], [4, 5], [6]]          # layers that read the same activations share a call
    else:
        groups = [[i] for i in range(len(layers))]
    calls = []
    for g_ in groups:
        Ls = [layers[i] for i in g_]
        if len(Ls) == 1:
            L = Ls[0]
            calls.append(dict(name=L["name"], bytes=L["bytes"], ys=[L["y"]],
                              run=(lambda L=L: L["lin"](L["x"], L["seg"], L["y"]))))
        else:
            assert all(torch.equal(L["x"], Ls[0]["x"]) and L["seg"] == Ls[0]["seg"] for L in Ls), \
                "fused layers must read the same activations and routing"
            fused = mes.DeltaLinearMulti([(L["lin"].w, L["lin"].experts) for L in Ls], T)
            ys = [L["y"] for L in Ls]
            # the shared activations are read (and credited) once
            nbytes = sum(L["bytes"] for L in Ls) - (len(Ls) - 1) * 2 * T * Ls[0]["d_in"]
            calls.append(dict(name="+".join(L["name"] for L in Ls), bytes=nbytes, ys=ys,
                              run=(lambda fused=fused, L0=Ls[0], ys=ys: fused(L0["x"], L0["seg"], ys))))
    calls_per_step = len(calls) if args.workload == "c4" else 1

    def one_step(i):
        if args.workload == "c4":
            for c in calls:
                c["run"]()
        else:
            calls[i % copies]["run"]()

    # ---------------------------------------------------------------- timed region
    for i in range(args.warmup):
        one_step(i)
    torch.cuda.synchronize()
    graph = None
    if args.graph:
        # One step captured as a HIP graph and replayed: same kernels, same arguments, launch overhead paid once.
        # The library never synchronises, allocates or clears memory in these calls, so they can be captured; the
        # replayed outputs are compared bit for bit with the eager ones below, with eager work in between.
        assert args.workload == "c4", "--graph replays the whole c4 step"
        eager = [[y.clone() for y in (c.get("ys") or [])] for c in calls]
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
                for y in (c.get("ys") or []):
                    y.fill_(0)
            graph.replay()
            torch.cuda.synchronize()
            for c, ref in zip(calls, eager):
                for y, r in zip(c.get("ys") or [], ref):
                    assert torch.equal(y, r), "graph replay differs from the eager result"
            one_step(0)                                   # eager work between the replays
            torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_wall0 = time.perf_counter()
    ev0.record()
    for i in range(args.steps):
        if graph is not None:
            graph.replay()
        else:
            one_step(i)
    ev1.record()
    torch.cuda.synchronize()
    t_wall = time.perf_counter() - t_wall0
    ms_total = ev0.elapsed_time(ev1)
    ms_per_step = ms_total / args.steps
    tokens_per_s = T * args.steps / (ms_total * 1e-3)

    # ---------------------------------------------------------------- roofline of the dominant kernel
    # The library records HIP events on the call's own stream right around its streaming kernel
    # (k_delta_linear); the same step sequence is replayed so that the caches are in the same state.
    timer = mes.KernelTimer()
    reps = max(10, min(50, args.steps))
    kernel_us = [0.0] * len(calls)
    for r in range(reps):
        for ci, c in enumerate(calls if args.workload == "c4" else [calls[r % copies]]):
            timer.arm()
            c["run"]()
            kernel_us[ci if args.workload == "c4" else 0] += timer.elapsed_us()
    n_launches = reps * calls_per_step
    step_bytes = sum(c["bytes"] for c in calls) if args.workload == "c4" else calls[0]["bytes"]
    launch_bytes = step_bytes / calls_per_step
    launch_us = sum(kernel_us) / n_launches
    achieved = launch_bytes / (launch_us * 1e-6) / 1e9

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(f"{args.workload}_b{args.bits}", {}).get("bytes_per_launch")
        except Exception:
            traffic = None

    breakdown = None
    if args.breakdown and args.workload == "c4":
        breakdown = {c["name"]: dict(kernel_us=round(kernel_us[ci] / reps, 2), MB=round(c["bytes"] / 1e6, 2),
                                     GBs=round(c["bytes"] / (kernel_us[ci] / reps) / 1e3, 1)) for ci, c in enumerate(calls)}
        print("breakdown:", json.dumps(breakdown), file=sys.stderr)

    if args.copy_probe:
        src = torch.empty(COPY_PROBE_BYTES, dtype=torch.uint8, device=dev).random_(0, 256)
        dst = torch.empty_like(src)
        for _ in range(3):
            mes.mes_copy_probe(dst, src)
        torch.cuda.synchronize()
        del src, dst

    # ---------------------------------------------------------------- oracle leg (baseline only)
    cpu_baseline = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import mes_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        prepared = []
        for s in samples:           # offline compression of the sampled rows is not part of the timed oracle work
            exs = []
            for d, si in zip(s["deltas"], s["sidx"]):
                og = O.GRID_EQ1 if args.grid == "eq1" else O.GRID_SYM
                c, st, sal = O.quantize(d, si, s["bits"], og)
                exs.append(dict(codes=c, step=st, salient=sal, salient_idx=si, bits=s["bits"], grid=og))
            prepared.append(exs)
        t0 = time.perf_counter()
        refs = [O.delta_linear(s["x"], s["w"], exs, s["seg"]) for s, exs in zip(samples, prepared)]
        t_cpu = time.perf_counter() - t0
        # scale the sampled rows to the full step: every linear was sampled at the same fraction of its rows
        frac = sum(len(s["rows"]) * s["x"].shape[1] for s in samples) / sum(s["d_out"] * s["x"].shape[1] for s in samples)
        cpu_tokens_per_s = T / (t_cpu / frac)
        num = den = 0.0
        for s, ref in zip(samples, refs):
            yg = layers[s["layer"]]["y"][:, s["rows"].to(dev)].double().cpu().numpy()
            num += float(((yg - ref) ** 2).sum())
            den += float((ref ** 2).sum())
        parity = (num / den) ** 0.5
        cpu_baseline = dict(value=round(cpu_tokens_per_s, 2), unit="tokens/s", cores=int(cores), kind="oracle",
                            sample=f"fp64 numpy oracle on a seeded 1/{sample_frac} sample of the output channels of "
                                   f"{'each of the 7 linears' if args.workload == 'c4' else 'one q_proj copy'}, all {T} tokens "
                                   f"and all experts ({t_cpu:.2f} s of CPU work), scaled linearly by rows (extrapolated)")

    out = {
        "metric": "tokens/s + achieved HBM GB/s, 16-expert Mistral-7B-shape decode delta linear",
        "value": round(tokens_per_s, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": ("c4: 7 Mistral-7B linear shapes of one block, 16 experts, 64 decode tokens, Zipf(1.1) routing, "
                                f"{args.bits}-bit codes ({args.grid} grid), {args.k} fp16 salient channels") if args.workload == "c4" else
                               "c2: Mistral-7B q_proj 4096x4096, 3 experts, 48 decode tokens 16/16/16, 2-bit, 64 salient; "
                               f"{copies} rotating copies",
                   "tokens": T, "experts": 16 if args.workload == "c4" else 3, "bits": args.bits,
                   "calls_per_step": calls_per_step, "graph_replay": bool(args.graph), "fused_calls": [c["name"] for c in calls] if args.workload == "c4" else None,
                   "active_experts": layers[0]["n_active"]},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "kernel": "k_delta_linear", "algorithmic_bytes_per_launch": int(launch_bytes),
                     "avg_launch_us": round(launch_us, 3), "launches_timed": n_launches,
                     "whole_call_GBs": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1)},
        "cpu_baseline": cpu_baseline,
        "parity_rel_fro_vs_oracle_sample": None if parity is None else float(f"{parity:.3e}"),
        "host_wall_ms_per_step": round(t_wall / args.steps * 1e3, 5),
    }
    if breakdown:
        out["breakdown"] = breakdown
    print(json.dumps(out))


if __name__ == "__main__":
    main()
