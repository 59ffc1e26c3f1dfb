"""The entry point that allocates nothing (mes_delta_linear_noalloc: scratch in a device-resident static array)
against mes_delta_linear with a caller-owned workspace: same kernels, so the outputs must agree bit for bit, on two
calls in a row that share the array, the second with a smaller input; the first is also checked against the oracle."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2406_09041_amd as mes
from inputs import synth
from oracle import mes_oracle as O

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(d_in, d_out, seg, k, bits, seed):
    wl = synth.small_case(d_in, d_out, seg, k, bits, seed=seed)
    w_t = mes.mes_pack_base(wl.w_base.to(DEV))
    ge = [mes.mes_pack_delta(ex.delta.to(DEV), ex.salient_idx, bits) for ex in wl.experts]
    return wl, w_t, ge


def test_noalloc_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    big = _case(4096, 320, [0, 7, 30, 31, 50, 61, 90], 64, 2, 71)       # several column splits, two token groups
    small = _case(520, 72, [0, 3, 3, 20], 5, 3, 72)                      # smaller, other bit width, an empty expert
    outs = []
    for wl, w_t, ge in (big, small):
        x = wl.x.to(DEV)
        y_ws = mes.mes_delta_linear(w_t, ge, x, wl.seg_offsets)
        y_na = torch.full((x.shape[0] + 2, wl.d_out), 7.0, dtype=torch.bfloat16, device=DEV)   # two canary rows
        mes.mes_delta_linear_noalloc(w_t, ge, x, wl.seg_offsets, y_na[: x.shape[0]])
        outs.append((wl, y_ws, y_na))
    torch.cuda.synchronize()
    for wl, y_ws, y_na in outs:
        T = wl.x.shape[0]
        assert torch.equal(y_na[:T].view(torch.int16), y_ws.view(torch.int16))
        assert torch.all(y_na[T:] == 7.0)
    wl, y_ws, y_na = outs[0]
    oe = []
    for ex in wl.experts:
        c, s, sal = O.quantize(ex.delta.numpy(), ex.salient_idx.numpy(), wl.bits)
        oe.append(dict(codes=c, step=s, salient=sal, salient_idx=ex.salient_idx.numpy(), bits=wl.bits, grid=O.GRID_SYM))
    y_ref = O.delta_linear(wl.x.double().numpy(), wl.w_base.double().numpy(), oe, wl.seg_offsets)
    err = np.linalg.norm(y_na[: wl.x.shape[0]].double().cpu().numpy() - y_ref) / np.linalg.norm(y_ref)
    assert err <= 5e-3


def test_noalloc_rejects_what_does_not_fit_and_takes_an_empty_batch():
    wl, w_t, ge = _case(520, 72, [0, 3, 3, 20], 5, 3, 72)
    y = torch.empty((0, wl.d_out), dtype=torch.bfloat16, device=DEV)
    mes.mes_delta_linear_noalloc(w_t, ge, wl.x.to(DEV)[:0], [0, 0, 0, 0], y)
    assert mes.binding.lib.mes_noalloc_scratch_bytes() == 64 << 20
