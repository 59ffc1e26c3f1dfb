#!/usr/bin/env python3
"""Measures larger decode batches on one MI355X: the Mistral-7B MLP matrices of the headline workload (16 experts,
Zipf-routed tokens, 2-bit codes, 64 fp16 salient channels; synthetic, seeded) at 64 to 512 tokens per batch, as the
fused gate+up call and the down call.  The streaming kernel takes 64 tokens per launch and re-reads the base weights
for each; a launch reads only the code streams of the experts its 64 tokens belong to (tokens are sorted by expert),
so the per-token cost falls as the batch grows.  Prints one JSON object; times are per call.
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
    ap.add_argument("--bits", type=int, default=2)
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--tokens", type=int, nargs="+", default=[64, 128, 256, 512])
    args = ap.parse_args()
    import torch

    import paper_2406_09041_amd as mes
    from inputs import synth

    dev = "cuda:0"
    out = {"bits": args.bits, "calls": {}}
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for call in (("gate_proj", "up_proj"), ("down_proj",)):
        res = {}
        for T in args.tokens:
            wls = [synth.config4_linear(w, device=dev, n_tokens=T, bits=args.bits) for w in call]
            x, seg = wls[0].x, wls[0].seg_offsets
            tiled = [mes.mes_pack_base(w.w_base) for w in wls]
            packed = [[mes.mes_pack_delta(ex.delta, ex.salient_idx, w.bits) for ex in w.experts] for w in wls]
            ys = [torch.empty((T, w.d_out), dtype=torch.bfloat16, device=dev) for w in wls]
            row = {"largest_segment": max(b - a for a, b in zip(seg[:-1], seg[1:]))}
            for name in ("streaming",):
                lin = mes.DeltaLinearMulti(list(zip(tiled, packed)), T)
                for _ in range(2):
                    lin(x, seg, ys)
                torch.cuda.synchronize()
                ev0.record()
                for _ in range(args.reps):
                    lin(x, seg, ys)
                ev1.record()
                torch.cuda.synchronize()
                ms = ev0.elapsed_time(ev1) / args.reps
                row[name] = {"ms_per_call": round(ms, 4), "tokens_per_s": round(T / (ms * 1e-3))}
                print(f"{'+'.join(call)} T={T} {name}: {ms:.4f} ms", file=sys.stderr, flush=True)
                del lin
            res[str(T)] = row
            del wls, tiled, packed, ys
            torch.cuda.empty_cache()
        out["calls"]["+".join(call)] = res
    print(json.dumps(out))


if __name__ == "__main__":
    main()
