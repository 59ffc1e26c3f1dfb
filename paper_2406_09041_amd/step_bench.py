#!/usr/bin/env python3
"""Measures mes_step_grad on one MI355X: the MLP matrices of a Mistral-7B block, one mini-batch of calibration
tokens (4 sequences of 128 tokens, Section 5), 8 fp16 salient channels, 2-bit codes (synthetic, seeded).

Per matrix: time per call (host clock over whole calls, all helper kernels included), the duration of the kernel
that does the two contractions (HIP events recorded by the library around it, on its stream), the fraction of the
dense bf16 matrix-core peak it reaches with 2 products x 2 n_tokens d_out d_in flops per call, and the bytes of
delta it streams per second.  Prints one JSON object.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0
SHAPES = {"gate_proj": (4096, 14336), "up_proj": (4096, 14336), "down_proj": (14336, 4096)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--bits", type=int, default=2)
    ap.add_argument("--grid", type=int, default=0)
    ap.add_argument("--tokens", type=int, default=512)
    ap.add_argument("--k", type=int, default=8)
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--shrink", type=float, default=0.6, help="step = shrink x max-abs step (below 1: some weights clamp)")
    ap.add_argument("--matrices", nargs="+", default=list(SHAPES))
    args = ap.parse_args()
    import torch

    import paper_2406_09041_amd as mes
    from inputs import synth

    dev = "cuda:0"
    out = {"bits": args.bits, "grid": args.grid, "tokens": args.tokens, "k": args.k, "matrices": {}}
    timer = mes.KernelTimer()
    z = 2.0 ** (args.bits - 1) - (0.5 if args.grid == 0 else 1.0)
    for i, which in enumerate(args.matrices):
        d_in, d_out = SHAPES[which]
        ex = synth.make_delta(d_in, d_out, args.k, 0.003, 15.0, synth.seed_for(951, 0, i, 2), dev)
        x = synth.normal((args.tokens, d_in), 1.0, synth.seed_for(951, 0, i, 3), dev, torch.bfloat16)
        ns = torch.ones(d_in, dtype=torch.bool, device=dev)
        ns[ex.salient_idx.to(dev).long()] = False
        step = (ex.delta[:, ns].abs().amax(dim=1) / max(z, 0.5) * args.shrink).float().contiguous()
        sg = mes.StepGrad(ex.delta, ex.salient_idx, args.bits, args.grid, args.tokens)
        for _ in range(3):
            sg(step, x)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.reps):
            sg(step, x)
        torch.cuda.synchronize()
        ms_call = (time.perf_counter() - t0) * 1e3 / args.reps
        us = []
        for _ in range(args.reps):
            timer.arm()
            sg(step, x)
            us.append(timer.elapsed_us())
        k_us = sum(us) / len(us)
        flops = 2 * 2.0 * args.tokens * d_out * d_in
        out["matrices"][which] = {
            "ms_per_call": round(ms_call, 4), "k_step_grad_us": round(k_us, 1),
            "TFLOPs": round(flops / (k_us * 1e-6) / 1e12, 1),
            "frac_of_bf16_mfma_peak": round(flops / (k_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "delta_GBps": round(4.0 * d_out * d_in / (k_us * 1e-6) / 1e9, 1),
            "tokens_per_s": round(args.tokens / (ms_call * 1e-3))}
        print(f"{which}: {ms_call:.4f} ms per call, kernel {k_us:.1f} us", file=sys.stderr, flush=True)
        del ex, x, sg, step
        torch.cuda.empty_cache()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
