"""Seeded synthetic inputs for the mixed-precision delta linear layer.

This module only draws random tensors and routing tables with the shapes, value
distributions and structure of the workloads (Mistral-7B-shaped linears, a few
outlier input channels in every expert's delta, equal-split or Zipf routing).
It holds none of the method's arithmetic: no quantisation, no packing, no
matmul.  Both the CPU oracle's tests and the HIP path's tests/benchmarks take
their inputs from here, so the two sides see identical data.

Everything is produced as torch tensors in the storage type the method reads
(bf16 activations and base weights, fp32 deltas) so that promotion to fp64 for
the oracle is exact.

Synthetic stand-in: the paper's own workloads are fine-tuned Mistral-7B /
LLaMA-2-13B checkpoints and their calibration sets; neither is available, so
deltas are Gaussian with a few input channels scaled up (the structure the
paper's Figure 1 shows: some input channels of the delta have a much larger
range than the rest).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import torch

BASE_SEED = 20240609

# (name, d_in, d_out) of the seven linear layers of one Mistral-7B block.
MISTRAL7B_LINEARS = (
    ("q_proj", 4096, 4096),
    ("k_proj", 4096, 1024),
    ("v_proj", 4096, 1024),
    ("o_proj", 4096, 4096),
    ("gate_proj", 4096, 14336),
    ("up_proj", 4096, 14336),
    ("down_proj", 14336, 4096),
)


def seed_for(config_id: int, layer: int = 0, expert: int = 0, stream: int = 0) -> int:
    """One integer seed per (config, layer, expert, stream)."""
    return BASE_SEED + config_id * 1000 + layer * 16 + expert + stream * 100003


def _gen(seed: int, device: str) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def normal(shape, std: float, seed: int, device: str = "cpu", dtype=torch.float32) -> torch.Tensor:
    """N(0, std^2) samples drawn in fp32, then cast to `dtype` (round-to-nearest-even)."""
    g = _gen(seed, device)
    t = torch.empty(shape, dtype=torch.float32, device=device)
    t.normal_(0.0, 1.0, generator=g)
    if std != 1.0:
        t.mul_(std)
    return t if dtype == torch.float32 else t.to(dtype)


def salient_columns(d_in: int, k: int, seed: int) -> torch.Tensor:
    """k distinct input-channel indices, ascending, int32 (always drawn on the CPU)."""
    if k == 0:
        return torch.empty(0, dtype=torch.int32)
    g = _gen(seed, "cpu")
    perm = torch.randperm(d_in, generator=g)[:k]
    return torch.sort(perm).values.to(torch.int32)


def zipf_expert_ids(n_tokens: int, n_experts: int, s: float, seed: int) -> torch.Tensor:
    """iid expert ids with P(rank r) proportional to r^-s, rank r <-> expert r-1; int64, unsorted."""
    g = _gen(seed, "cpu")
    ranks = torch.arange(1, n_experts + 1, dtype=torch.float64)
    p = ranks.pow(-s)
    p = p / p.sum()
    return torch.multinomial(p, n_tokens, replacement=True, generator=g)


def segments_from_ids(expert_ids: torch.Tensor, n_experts: int):
    """Stable sort of tokens by expert id.

    Returns (perm, seg_offsets): `perm[i]` is the original position of the token
    now at row i; tokens of expert e occupy rows seg_offsets[e]..seg_offsets[e+1].
    """
    perm = torch.sort(expert_ids, stable=True).indices
    counts = torch.bincount(expert_ids, minlength=n_experts)
    off = torch.zeros(n_experts + 1, dtype=torch.int64)
    off[1:] = torch.cumsum(counts, 0)
    return perm, [int(v) for v in off]


def equal_segments(n_tokens: int, n_experts: int) -> List[int]:
    base, rem = divmod(n_tokens, n_experts)
    off = [0]
    for e in range(n_experts):
        off.append(off[-1] + base + (1 if e < rem else 0))
    return off


@dataclass
class ExpertDelta:
    """One expert's uncompressed delta for one linear layer."""
    delta: torch.Tensor          # [d_out, d_in] fp32
    salient_idx: torch.Tensor    # [k] int32 ascending (CPU) -- the planted outlier channels


@dataclass
class LinearWorkload:
    name: str
    d_in: int
    d_out: int
    w_base: torch.Tensor                 # [d_out, d_in] bf16
    experts: List[ExpertDelta]
    x: torch.Tensor                      # [T, d_in] bf16, rows already sorted by expert
    seg_offsets: List[int]               # len E+1
    bits: int = 2
    k: int = 0
    meta: dict = field(default_factory=dict)


def make_delta(d_in: int, d_out: int, k: int, std: float, outlier_scale: float,
               seed: int, device: str = "cpu") -> ExpertDelta:
    """Gaussian delta with k randomly chosen input channels (columns) scaled by `outlier_scale`."""
    d = normal((d_out, d_in), std, seed, device)
    idx = salient_columns(d_in, k, seed + 7)
    if k:
        d[:, idx.to(device=device, dtype=torch.long)] *= outlier_scale
    return ExpertDelta(delta=d, salient_idx=idx)


def make_linear(name: str, d_in: int, d_out: int, n_experts: int, seg_offsets: Sequence[int],
                k: int, bits: int, config_id: int, layer: int = 0, *,
                base_std: float = 0.02, delta_std: float = 0.003, outlier_scale: float = 15.0,
                x_std: float = 1.0, device: str = "cpu", shape_id: int = 0,
                x_id: Optional[int] = None) -> LinearWorkload:
    """One linear layer's worth of synthetic data for `n_experts` experts.  Layers given the same `x_id`
    (and input width) draw the same activations."""
    T = int(seg_offsets[-1])
    sid = shape_id * 16
    w_base = normal((d_out, d_in), base_std, seed_for(config_id, layer, 0, 1 + sid), device, torch.bfloat16)
    experts = [make_delta(d_in, d_out, k, delta_std, outlier_scale,
                          seed_for(config_id, layer, e, 2 + sid), device) for e in range(n_experts)]
    x = normal((T, d_in), x_std, seed_for(config_id, layer, 0, 3 + (sid if x_id is None else 16 * x_id)), device, torch.bfloat16)
    return LinearWorkload(name, d_in, d_out, w_base, experts, x, list(map(int, seg_offsets)), bits, k,
                          {"config_id": config_id, "layer": layer})


# --- the configurations the benchmarks and parity tests name -------------------------------------

def config1(device: str = "cpu") -> LinearWorkload:
    """256x256, 1 expert, 4 tokens, 8 outlier channels (x20), 2-bit."""
    return make_linear("c1", 256, 256, 1, [0, 4], 8, 2, 1, delta_std=0.002, outlier_scale=20.0, device=device)


def config2(device: str = "cpu", copy: int = 0) -> LinearWorkload:
    """Mistral-7B q_proj shape, 3 experts, 48 decode tokens routed 16/16/16, 64 outlier channels (x15)."""
    return make_linear("c2_q_proj", 4096, 4096, 3, [0, 16, 32, 48], 64, 2, 2, layer=copy, device=device)


def config3(which: str = "gate_proj", bits: int = 2, device: str = "cpu") -> LinearWorkload:
    """Mistral-7B MLP shape, 3 experts, prefill of 3 x 512 tokens, 128 outlier channels."""
    shapes = {n: (i, di, do) for i, (n, di, do) in enumerate(MISTRAL7B_LINEARS)}
    sid, d_in, d_out = shapes[which]
    return make_linear(f"c3_{which}", d_in, d_out, 3, [0, 512, 1024, 1536], 128, bits, 3,
                       device=device, shape_id=sid)


def config4_routing(n_tokens: int = 64, n_experts: int = 16, layer: int = 0):
    """Zipf(s=1.1) expert ids for a decode batch, turned into sorted segments."""
    ids = zipf_expert_ids(n_tokens, n_experts, 1.1, seed_for(4, layer, 0, 9))
    return segments_from_ids(ids, n_experts)


def config4_linear(which: str, device: str = "cpu", layer: int = 0, n_tokens: int = 64,
                   n_experts: int = 16, bits: int = 2, k: int = 64) -> LinearWorkload:
    """One of the seven Mistral-7B linear shapes, 16 experts, Zipf-routed decode batch.  The shapes do not
    chain, so every layer of one input width reads the same fixed activations (one batch 4096 wide for six
    of them, one 14336 wide for down_proj)."""
    shapes = {n: (i, di, do) for i, (n, di, do) in enumerate(MISTRAL7B_LINEARS)}
    sid, d_in, d_out = shapes[which]
    _, off = config4_routing(n_tokens, n_experts, layer)
    return make_linear(f"c4_{which}", d_in, d_out, n_experts, off, k, bits, 4, layer=layer,
                       device=device, shape_id=sid, x_id=(0 if d_in == 4096 else 1))


def config5_routing(part: str = "mixed", n_decode: int = 256, n_prefill: int = 4,
                    prefill_len: int = 1024, n_experts: int = 16):
    """Routing of the mixed batch of the 32-layer configuration: `n_decode` decode tokens with iid Zipf(1.1) expert
    ids and `n_prefill` prompt sequences of `prefill_len` tokens, each sequence routed as a whole to one
    Zipf-drawn expert; tokens sorted by expert (an expert's decode tokens first, then its sequences).  The
    method routes a query to one expert MODEL, so every layer of the stack sees this same routing.
    part = "decode" / "prefill" keeps only that kind of token, with the same draws.  Returns seg_offsets."""
    dec = zipf_expert_ids(n_decode, n_experts, 1.1, seed_for(5, 0, 0, 9))
    pre = zipf_expert_ids(n_prefill, n_experts, 1.1, seed_for(5, 0, 0, 10))
    counts = torch.zeros(n_experts, dtype=torch.int64)
    if part in ("mixed", "decode"):
        counts += torch.bincount(dec, minlength=n_experts)
    if part in ("mixed", "prefill"):
        counts += prefill_len * torch.bincount(pre, minlength=n_experts)
    off = [0]
    for c in counts.tolist():
        off.append(off[-1] + int(c))
    return off


def config5_linear(which: str, layer: int = 0, bits: int = 2, device: str = "cpu", part: str = "mixed",
                   k: int = 64, n_experts: int = 16) -> LinearWorkload:
    """One linear of one layer of the 32-layer stack: a Mistral-7B shape, 16 experts, the mixed batch of
    config5_routing (256 decode tokens + 4 x 1024 prompt tokens).  Weights and deltas depend on (layer, shape,
    expert); the activations only on the input width, so layers of one width read one batch."""
    shapes = {n: (i, di, do) for i, (n, di, do) in enumerate(MISTRAL7B_LINEARS)}
    sid, d_in, d_out = shapes[which]
    off = config5_routing(part, n_experts=n_experts)
    return make_linear(f"c5_{which}_L{layer}", d_in, d_out, n_experts, off, k, bits, 5, layer=layer,
                       device=device, shape_id=sid, x_id=(0 if d_in == 4096 else 1))


def small_case(d_in: int, d_out: int, seg_offsets: Sequence[int], k: int, bits: int,
               seed: int = 0, device: str = "cpu", **kw) -> LinearWorkload:
    """Free-form small case for parity tests (ragged shapes, empty segments, ...)."""
    return make_linear("small", d_in, d_out, len(seg_offsets) - 1, seg_offsets, k, bits,
                       config_id=900 + seed, device=device, **kw)
