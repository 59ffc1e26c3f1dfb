#!/usr/bin/env python3
"""Measures the long-segment (prefill) path on one MI355X: the three MLP shapes of a Mistral-7B block, 3 experts
with one 512-token sequence each (1536 tokens), 128 fp16 salient channels, 2- or 3-bit codes (synthetic, seeded).
For every matrix: time per call on the one-product path (W + Delta~ formed in registers, one fused kernel) and, for
comparison, on the streaming path (a workspace without the extra room), tokens/s, and the fraction of the dense
bf16 matrix-core peak reached, with 2 T d_out d_in flops per call (one product per token).  Prints one JSON object.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--bits", type=int, default=2)
    ap.add_argument("--reps", type=int, default=10)
    args = ap.parse_args()
    import torch

    import paper_2406_09041_amd as mes
    from inputs import synth

    dev = "cuda:0"
    out = {"bits": args.bits, "tokens": 1536, "experts": 3, "matrices": {}}
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for which in ("gate_proj", "up_proj", "down_proj"):
        wl = synth.config3(which, bits=args.bits, device=dev)
        T = wl.x.shape[0]
        w_t = mes.mes_pack_base(wl.w_base)
        packed = [mes.mes_pack_delta(ex.delta, ex.salient_idx, wl.bits) for ex in wl.experts]
        y = torch.empty((T, wl.d_out), dtype=torch.bfloat16, device=dev)
        res = {}
        for name, max_tokens in (("one_product", T), ("streaming", 64)):
            lin = mes.DeltaLinear(w_t, packed, max_tokens)
            for _ in range(2):
                lin(wl.x, wl.seg_offsets, y)
            torch.cuda.synchronize()
            ev0.record()
            for _ in range(args.reps):
                lin(wl.x, wl.seg_offsets, y)
            ev1.record()
            torch.cuda.synchronize()
            ms = ev0.elapsed_time(ev1) / args.reps
            flops = 2.0 * T * wl.d_out * wl.d_in
            res[name] = {"ms_per_call": round(ms, 4), "tokens_per_s": round(T / (ms * 1e-3)),
                         "TFLOPs": round(flops / (ms * 1e-3) / 1e12, 1),
                         "frac_of_bf16_mfma_peak": round(flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}
            del lin
        out["matrices"][which] = res
        del wl, w_t, packed, y
        torch.cuda.empty_cache()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
