#!/usr/bin/env python3
"""Measures on-demand swapping (mes_pool_*) on one MI355X: what a miss costs and what a decode step costs when the
experts a batch routes to are not all resident.

Workload: the Mistral-7B q_proj shape (4096 x 4096), 2-bit codes, 64 fp16 salient channels; N experts registered
in pinned host memory, 16 device slots; decode batches of 64 tokens whose experts are drawn Zipf(1.1) over all N
experts (synthetic, seeded).  Prints one JSON object.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--experts", type=int, default=32)
    ap.add_argument("--slots", type=int, default=16)
    ap.add_argument("--steps", type=int, default=200)
    args = ap.parse_args()
    import numpy as np
    import torch

    import paper_2406_09041_amd as mes
    from inputs import synth

    dev = "cuda:0"
    d_in = d_out = 4096
    k, bits = 64, 2
    w = synth.normal((d_out, d_in), 0.02, 11, dev, torch.bfloat16)
    w_t = mes.mes_pack_base(w)
    pool = mes.ExpertPool(d_in, d_out, k, bits, mes.GRID_SYM, args.slots, args.experts, device=dev)
    resident = []
    for e in range(args.experts):
        ex = synth.make_delta(d_in, d_out, k, 0.003, 15.0, 5000 + e, dev)
        pk = mes.mes_pack_delta(ex.delta, ex.salient_idx, bits)
        pool.register(e, pk)
        resident.append(pk)
    ws = mes.make_workspace(d_in, d_out, 64, torch.device(dev))
    expert_bytes = mes.codes_bytes(d_in, d_out, bits) + 4 * d_out + mes.salient_bytes(d_out, k) + 4 * k

    # (a) what a miss costs: fill all slots from the host, timed on the compute stream (which waits for the copies)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fills = []
    for rep in range(5):
        ids = [(rep * args.slots + i) % args.experts for i in range(args.slots)]
        if rep and args.experts < 2 * args.slots:          # make sure they all miss
            ids = [(ids[0] + args.slots + i) % args.experts for i in range(args.slots)]
        before = pool.stats()[1]
        torch.cuda.synchronize()
        ev0.record()
        pool.acquire(ids)
        ev1.record()
        torch.cuda.synchronize()
        missed = pool.stats()[1] - before
        if missed:
            fills.append((missed * expert_bytes / 1e9) / (ev0.elapsed_time(ev1) * 1e-3))
    # (b) decode steps with Zipf routing over all registered experts
    rng = np.random.default_rng(3)
    p = 1.0 / np.arange(1, args.experts + 1) ** 1.1
    p /= p.sum()
    x = synth.normal((64, d_in), 1.0, 12, dev, torch.bfloat16)
    y = torch.empty((64, d_out), dtype=torch.bfloat16, device=dev)
    batches = []
    for _ in range(args.steps):
        ids = np.sort(rng.choice(args.experts, size=64, p=p))
        uniq, counts = np.unique(ids, return_counts=True)
        uniq, counts = uniq[: args.slots], counts[: args.slots]     # a batch can use at most `slots` experts
        batches.append((uniq.tolist(), [0] + np.cumsum(counts).tolist()))

    def run(swap: bool):
        h0, m0, b0 = pool.stats()
        torch.cuda.synchronize()
        ev0.record()
        for ids, seg in batches:
            xs = x[: seg[-1]]
            if swap:
                desc = pool.acquire(ids)
                mes.mes_delta_linear_descriptors(w_t, desc, xs, seg, ws, y[: seg[-1]])
            else:
                mes.mes_delta_linear(w_t, [resident[e] for e in ids], xs, seg, y[: seg[-1]], ws)
        ev1.record()
        torch.cuda.synchronize()
        h1, m1, b1 = pool.stats()
        return ev0.elapsed_time(ev1) / len(batches), h1 - h0, m1 - m0, b1 - b0

    run(True)
    ms_swap, hits, misses, nbytes = run(True)
    run(False)
    ms_res, _, _, _ = run(False)
    print(json.dumps({
        "shape": [d_out, d_in], "bits": bits, "k": k, "experts_registered": args.experts, "slots": args.slots,
        "expert_MB": round(expert_bytes / 1e6, 3),
        "fill_GBs": [round(f, 1) for f in fills],
        "decode_ms_per_step_all_resident": round(ms_res, 4),
        "decode_ms_per_step_swapping": round(ms_swap, 4),
        "hit_rate": round(hits / max(hits + misses, 1), 4),
        "MB_copied_per_step": round(nbytes / len(batches) / 1e6, 3),
    }))


if __name__ == "__main__":
    main()
