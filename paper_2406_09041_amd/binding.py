"""Thin ctypes binding over libmes.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels.  PyTorch is used for device
memory (tensors own every buffer) and for the current HIP stream.  There is no CPU
fallback: if libmes.so is missing the import fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("MES_LIBRARY") or os.path.join(_HERE, "libmes.so")   # MES_LIBRARY: another build of the same library

MES_OK = 0
GRID_SYM, GRID_EQ1 = 0, 1
STEP_GIVEN, STEP_MAXABS, STEP_MEANABS = 0, 1, 2
MAX_EXPERTS = 64

STATUS_NAMES = {0: "MES_OK", 1: "MES_ERR_NULL", 2: "MES_ERR_SHAPE", 3: "MES_ERR_BITS", 4: "MES_ERR_SALIENT",
                5: "MES_ERR_SEGMENTS", 6: "MES_ERR_ALIGN", 7: "MES_ERR_WORKSPACE", 8: "MES_ERR_DEVICE"}

EXPORTS = ["mes_base_bytes", "mes_codes_bytes", "mes_salient_bytes", "mes_pack_workspace_bytes",
           "mes_select_workspace_bytes", "mes_linear_workspace_bytes", "mes_last_error", "mes_layout_version",
           "mes_pack_base", "mes_unpack_base", "mes_select_salient", "mes_pack_delta", "mes_unpack_delta",
           "mes_delta_linear", "mes_linear_multi_workspace_bytes",
           "mes_delta_linear_multi", "mes_time_next_call", "mes_copy_probe", "mes_pool_slot_bytes", "mes_pool_create",
           "mes_pool_destroy", "mes_pool_register", "mes_pool_acquire", "mes_pool_slot_of", "mes_pool_stats",
           "mes_pool_slot_layout", "mes_pool_multi_slot_bytes", "mes_pool_create_multi", "mes_pool_linear_offset",
           "mes_pool_register_blob", "mes_pool_acquire_multi", "mes_pool_prefetch", "mes_pool_prefetched",
           "mes_gated_workspace_bytes", "mes_delta_linear_gated",
           "mes_step_grad_workspace_bytes", "mes_step_grad", "mes_step_adamw", "mes_noalloc_scratch_bytes",
           "mes_delta_linear_noalloc", "mes_long_segment_tokens"]


class MesError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


class mes_delta(ctypes.Structure):
    _fields_ = [("d_in", ctypes.c_int32), ("d_out", ctypes.c_int32), ("k", ctypes.c_int32),
                ("bits", ctypes.c_int32), ("grid", ctypes.c_int32), ("layout_version", ctypes.c_int32),
                ("codes", ctypes.c_void_p), ("step", ctypes.c_void_p), ("salient", ctypes.c_void_p),
                ("salient_idx", ctypes.c_void_p)]


class mes_linear(ctypes.Structure):
    _fields_ = [("w_base_tiled", ctypes.c_void_p), ("experts", ctypes.POINTER(mes_delta)), ("y", ctypes.c_void_p)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = ctypes.CDLL(LIB_PATH)
    c_int, c_sz, vp = ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p
    lib.mes_base_bytes.restype = c_sz
    lib.mes_base_bytes.argtypes = [c_int, c_int]
    lib.mes_codes_bytes.restype = c_sz
    lib.mes_codes_bytes.argtypes = [c_int, c_int, c_int]
    lib.mes_salient_bytes.restype = c_sz
    lib.mes_salient_bytes.argtypes = [c_int, c_int]
    lib.mes_pack_workspace_bytes.restype = c_sz
    lib.mes_pack_workspace_bytes.argtypes = []
    lib.mes_select_workspace_bytes.restype = c_sz
    lib.mes_select_workspace_bytes.argtypes = [c_int, c_int, c_int]
    lib.mes_linear_workspace_bytes.restype = c_sz
    lib.mes_linear_workspace_bytes.argtypes = [c_int, c_int, c_int]
    lib.mes_last_error.restype = ctypes.c_char_p
    lib.mes_last_error.argtypes = []
    lib.mes_layout_version.restype = c_int
    lib.mes_layout_version.argtypes = []
    lib.mes_pack_base.restype = c_int
    lib.mes_pack_base.argtypes = [vp, c_int, c_int, vp, vp]
    lib.mes_unpack_base.restype = c_int
    lib.mes_unpack_base.argtypes = [vp, c_int, c_int, vp, vp]
    lib.mes_select_salient.restype = c_int
    lib.mes_select_salient.argtypes = [vp, vp, c_int, c_int, c_int, c_int, c_int, c_int, c_int, vp, vp, vp, c_sz, vp]
    lib.mes_pack_delta.restype = c_int
    lib.mes_pack_delta.argtypes = [vp, c_int, c_int, vp, c_int, c_int, c_int, c_int, vp, vp, vp, vp, vp, c_sz, vp]
    lib.mes_unpack_delta.restype = c_int
    lib.mes_unpack_delta.argtypes = [ctypes.POINTER(mes_delta), vp, vp, vp]
    lib.mes_delta_linear.restype = c_int
    lib.mes_delta_linear.argtypes = [vp, ctypes.POINTER(mes_delta), c_int, vp, c_int,
                                     ctypes.POINTER(ctypes.c_int32), vp, vp, c_sz, vp]
    lib.mes_long_segment_tokens.restype = c_int
    lib.mes_long_segment_tokens.argtypes = []
    lib.mes_noalloc_scratch_bytes.restype = c_sz
    lib.mes_noalloc_scratch_bytes.argtypes = []
    lib.mes_delta_linear_noalloc.restype = c_int
    lib.mes_delta_linear_noalloc.argtypes = [vp, ctypes.POINTER(mes_delta), c_int, vp, c_int,
                                             ctypes.POINTER(ctypes.c_int32), vp, vp]
    lib.mes_linear_multi_workspace_bytes.restype = c_sz
    lib.mes_linear_multi_workspace_bytes.argtypes = [c_int, ctypes.POINTER(ctypes.c_int32), c_int, c_int]
    lib.mes_delta_linear_multi.restype = c_int
    lib.mes_delta_linear_multi.argtypes = [ctypes.POINTER(mes_linear), c_int, c_int, vp, c_int,
                                           ctypes.POINTER(ctypes.c_int32), vp, c_sz, vp]
    lib.mes_time_next_call.restype = c_int
    lib.mes_time_next_call.argtypes = [vp, vp]
    lib.mes_step_grad_workspace_bytes.restype = c_sz
    lib.mes_step_grad_workspace_bytes.argtypes = [c_int, c_int, c_int]
    lib.mes_step_grad.restype = c_int
    lib.mes_step_grad.argtypes = [vp, c_int, c_int, vp, c_int, c_int, c_int, vp, vp, c_int, vp, vp, vp, c_sz, vp]
    lib.mes_step_adamw.restype = c_int
    lib.mes_step_adamw.argtypes = [vp, vp, vp, vp, c_int, c_int, ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                   ctypes.c_float, ctypes.c_float, vp]
    lib.mes_copy_probe.restype = c_int
    lib.mes_copy_probe.argtypes = [vp, vp, c_sz, vp]
    lib.mes_pool_slot_bytes.restype = c_sz
    lib.mes_pool_slot_bytes.argtypes = [c_int, c_int, c_int, c_int]
    lib.mes_pool_create.restype = c_int
    lib.mes_pool_create.argtypes = [c_int, c_int, c_int, c_int, c_int, c_int, c_int, vp, c_sz, c_int, ctypes.POINTER(vp)]
    lib.mes_pool_destroy.restype = None
    lib.mes_pool_destroy.argtypes = [vp]
    lib.mes_pool_register.restype = c_int
    lib.mes_pool_register.argtypes = [vp, c_int, vp, vp, vp, vp]
    lib.mes_pool_acquire.restype = c_int
    lib.mes_pool_acquire.argtypes = [vp, ctypes.POINTER(ctypes.c_int32), c_int, ctypes.POINTER(mes_delta), vp, vp]
    lib.mes_pool_slot_of.restype = c_int
    lib.mes_pool_slot_of.argtypes = [vp, c_int]
    lib.mes_gated_workspace_bytes.restype = c_sz
    lib.mes_gated_workspace_bytes.argtypes = [c_int, c_int, c_int]
    lib.mes_delta_linear_gated.restype = c_int
    lib.mes_delta_linear_gated.argtypes = [vp, ctypes.POINTER(mes_delta), vp, ctypes.POINTER(mes_delta), c_int, vp, c_int,
                                           ctypes.POINTER(ctypes.c_int32), vp, vp, c_sz, vp]
    i32p = ctypes.POINTER(ctypes.c_int32)
    lib.mes_pool_slot_layout.restype = c_sz
    lib.mes_pool_slot_layout.argtypes = [c_int, c_int, c_int, c_int, ctypes.POINTER(c_sz)]
    lib.mes_pool_multi_slot_bytes.restype = c_sz
    lib.mes_pool_multi_slot_bytes.argtypes = [c_int, i32p, i32p, i32p, c_int]
    lib.mes_pool_create_multi.restype = c_int
    lib.mes_pool_create_multi.argtypes = [c_int, i32p, i32p, i32p, c_int, c_int, c_int, c_int, vp, c_sz, c_int, ctypes.POINTER(vp)]
    lib.mes_pool_linear_offset.restype = c_sz
    lib.mes_pool_linear_offset.argtypes = [vp, c_int]
    lib.mes_pool_register_blob.restype = c_int
    lib.mes_pool_register_blob.argtypes = [vp, c_int, vp]
    lib.mes_pool_acquire_multi.restype = c_int
    lib.mes_pool_acquire_multi.argtypes = [vp, i32p, c_int, ctypes.POINTER(mes_delta), vp, vp]
    lib.mes_pool_prefetch.restype = c_int
    lib.mes_pool_prefetch.argtypes = [vp, i32p, c_int, ctypes.POINTER(c_int), vp]
    lib.mes_pool_prefetched.restype = ctypes.c_uint64
    lib.mes_pool_prefetched.argtypes = [vp]
    lib.mes_pool_stats.restype = c_int
    lib.mes_pool_stats.argtypes = [vp, ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint64)]
    return lib


lib = _load()


def _check(status: int) -> None:
    if status != MES_OK:
        raise MesError(status, lib.mes_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(device) -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def base_bytes(d_in, d_out): return lib.mes_base_bytes(d_in, d_out)
def codes_bytes(d_in, d_out, bits): return lib.mes_codes_bytes(d_in, d_out, bits)
def salient_bytes(d_out, k): return lib.mes_salient_bytes(d_out, k)
def linear_workspace_bytes(d_in, d_out, max_tokens): return lib.mes_linear_workspace_bytes(d_in, d_out, max_tokens)


def mes_pack_base(w: torch.Tensor) -> torch.Tensor:
    """w: bf16 [d_out, d_in] on the GPU -> tiled base (uint8 tensor of mes_base_bytes)."""
    assert w.dtype == torch.bfloat16 and w.is_cuda and w.is_contiguous()
    d_out, d_in = w.shape
    out = torch.empty(base_bytes(d_in, d_out), dtype=torch.uint8, device=w.device)
    _check(lib.mes_pack_base(_ptr(w), d_in, d_out, _ptr(out), _stream(w.device)))
    return out


def mes_copy_probe(dst: torch.Tensor, src: torch.Tensor) -> None:
    """Plain copy kernel of known traffic (src.nbytes read, as many written); see mes_copy_probe in mes_bench.h."""
    assert dst.is_cuda and src.is_cuda and dst.is_contiguous() and src.is_contiguous() and dst.nbytes == src.nbytes
    _check(lib.mes_copy_probe(_ptr(dst), _ptr(src), src.nbytes, _stream(src.device)))


def mes_unpack_base(w_tiled: torch.Tensor, d_in: int, d_out: int) -> torch.Tensor:
    out = torch.empty((d_out, d_in), dtype=torch.bfloat16, device=w_tiled.device)
    _check(lib.mes_unpack_base(_ptr(w_tiled), d_in, d_out, _ptr(out), _stream(w_tiled.device)))
    return out


@dataclass
class PackedDelta:
    """Device buffers of one expert's compressed delta (see include/mes.h for the layouts)."""
    d_in: int
    d_out: int
    k: int
    bits: int
    grid: int
    codes: torch.Tensor                  # uint8 [mes_codes_bytes]
    step: torch.Tensor                   # fp32 [d_out]
    salient: Optional[torch.Tensor]      # uint8 [mes_salient_bytes] or None
    salient_idx: Optional[torch.Tensor]  # int32 [k] or None

    def descriptor(self) -> mes_delta:
        return mes_delta(self.d_in, self.d_out, self.k, self.bits, self.grid, lib.mes_layout_version(),
                         self.codes.data_ptr(), self.step.data_ptr(),
                         self.salient.data_ptr() if self.salient is not None else None,
                         self.salient_idx.data_ptr() if self.salient_idx is not None else None)


def mes_pack_delta(delta: torch.Tensor, salient_idx: Optional[torch.Tensor], bits: int, grid: int = GRID_SYM,
                   step_policy: int = STEP_MAXABS, step_in: Optional[torch.Tensor] = None) -> PackedDelta:
    """delta: fp32 [d_out, d_in] on the GPU; salient_idx: int32 [k] ascending (any device) or None."""
    assert delta.dtype == torch.float32 and delta.is_cuda and delta.is_contiguous()
    dev = delta.device
    d_out, d_in = delta.shape
    k = 0 if salient_idx is None else int(salient_idx.numel())
    sidx = None if k == 0 else salient_idx.to(device=dev, dtype=torch.int32).contiguous()
    codes = torch.empty(max(codes_bytes(d_in, d_out, bits), 16), dtype=torch.uint8, device=dev)
    step = torch.empty(d_out, dtype=torch.float32, device=dev)
    sal = None if k == 0 else torch.empty(salient_bytes(d_out, k), dtype=torch.uint8, device=dev)
    ws = torch.empty(lib.mes_pack_workspace_bytes(), dtype=torch.uint8, device=dev)
    if step_in is not None:
        step_in = step_in.to(device=dev, dtype=torch.float32).contiguous()
    _check(lib.mes_pack_delta(_ptr(delta), d_in, d_out, _ptr(sidx), k, bits, grid, step_policy, _ptr(step_in),
                              _ptr(codes), _ptr(step), _ptr(sal), _ptr(ws), ws.numel(), _stream(dev)))
    return PackedDelta(d_in, d_out, k, bits, grid, codes, step, sal, sidx)


def mes_unpack_delta(p: PackedDelta, want_codes: bool = True, want_delta: bool = True):
    dev = p.codes.device
    dh = torch.empty((p.d_out, p.d_in), dtype=torch.float32, device=dev) if want_delta else None
    cd = torch.empty((p.d_out, p.d_in), dtype=torch.uint8, device=dev) if want_codes else None
    desc = p.descriptor()
    _check(lib.mes_unpack_delta(ctypes.byref(desc), _ptr(dh), _ptr(cd), _stream(dev)))
    return dh, cd


def mes_select_salient(delta: torch.Tensor, x_calib: torch.Tensor, bits: int, grid: int, k: int,
                       step_policy: int = STEP_MAXABS, want_scores: bool = False):
    """Eq. 2 selection.  Returns idx int32 [k] ascending (and the fp64 scores [d_in] if asked)."""
    assert delta.dtype == torch.float32 and x_calib.dtype == torch.float32 and delta.is_cuda and x_calib.is_cuda
    dev = delta.device
    d_out, d_in = delta.shape
    n = x_calib.shape[0]
    idx = torch.empty(max(k, 1), dtype=torch.int32, device=dev)
    score = torch.empty(d_in, dtype=torch.float64, device=dev) if want_scores else None
    ws = torch.empty(max(lib.mes_select_workspace_bytes(n, d_in, d_out), 16), dtype=torch.uint8, device=dev)
    _check(lib.mes_select_salient(_ptr(delta.contiguous()), _ptr(x_calib.contiguous()), n, d_in, d_out, bits, grid,
                                  step_policy, k, _ptr(idx), _ptr(score), _ptr(ws), ws.numel(), _stream(dev)))
    idx = idx[:k]
    return (idx, score) if want_scores else idx


class StepGrad:
    """Marshalled arguments of mes_step_grad for one delta matrix (workspace and outputs allocated once)."""

    def __init__(self, delta: torch.Tensor, salient_idx: Optional[torch.Tensor], bits: int, grid: int = GRID_SYM,
                 max_tokens: int = 512):
        assert delta.dtype == torch.float32 and delta.is_cuda and delta.is_contiguous()
        self.delta, self.bits, self.grid = delta, bits, grid
        self.d_out, self.d_in = delta.shape
        self.k = 0 if salient_idx is None else int(salient_idx.numel())
        self.sidx = None if self.k == 0 else salient_idx.to(device=delta.device, dtype=torch.int32).contiguous()
        self.max_tokens = max_tokens
        n = max(lib.mes_step_grad_workspace_bytes(self.d_in, self.d_out, max_tokens), 16)
        self.ws = torch.empty(n, dtype=torch.uint8, device=delta.device)
        self.loss = torch.empty(self.d_out, dtype=torch.float32, device=delta.device)
        self.grad = torch.empty(self.d_out, dtype=torch.float32, device=delta.device)

    def __call__(self, step: torch.Tensor, x: torch.Tensor):
        """step fp32 [d_out], x bf16 [n_tokens, d_in] -> (loss [d_out], grad [d_out]), overwritten by the next call."""
        assert step.dtype == torch.float32 and x.dtype == torch.bfloat16 and x.shape[0] <= self.max_tokens
        _check(lib.mes_step_grad(_ptr(self.delta), self.d_in, self.d_out, _ptr(self.sidx), self.k, self.bits, self.grid,
                                 _ptr(step), _ptr(x), x.shape[0], _ptr(self.loss), _ptr(self.grad), _ptr(self.ws),
                                 self.ws.numel(), _stream(self.delta.device)))
        return self.loss, self.grad


def mes_step_adamw(step: torch.Tensor, grad: torch.Tensor, m: torch.Tensor, v: torch.Tensor, t: int, lr: float,
                   beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8, weight_decay: float = 0.01) -> None:
    """One in-place AdamW update of the step vector (and of the moments m, v)."""
    _check(lib.mes_step_adamw(_ptr(step), _ptr(grad), _ptr(m), _ptr(v), step.numel(), t, lr, beta1, beta2, eps,
                              weight_decay, _stream(step.device)))


def make_workspace(d_in: int, d_out: int, max_tokens: int, device) -> torch.Tensor:
    """Allocates a mes_delta_linear workspace (scratch: its contents do not matter)."""
    n = max(linear_workspace_bytes(d_in, d_out, max_tokens), 16)
    return torch.empty(n, dtype=torch.uint8, device=device)


class DeltaLinear:
    """Marshalled arguments of mes_delta_linear for one layer (descriptor array built once)."""

    def __init__(self, w_base_tiled: torch.Tensor, experts: Sequence[PackedDelta], max_tokens: int = 64,
                 workspace: Optional[torch.Tensor] = None):
        self.w = w_base_tiled
        self.experts = list(experts)
        self.E = len(self.experts)
        self.d_in, self.d_out = self.experts[0].d_in, self.experts[0].d_out
        self.desc = (mes_delta * self.E)(*[e.descriptor() for e in self.experts])
        self.ws = workspace if workspace is not None else make_workspace(self.d_in, self.d_out, max_tokens, w_base_tiled.device)

    def __call__(self, x: torch.Tensor, seg_offsets: Sequence[int], y: Optional[torch.Tensor] = None) -> torch.Tensor:
        T = x.shape[0]
        if y is None:
            y = torch.empty((T, self.d_out), dtype=torch.bfloat16, device=x.device)
        seg = (ctypes.c_int32 * (self.E + 1))(*seg_offsets)
        _check(lib.mes_delta_linear(_ptr(self.w), self.desc, self.E, _ptr(x), T, seg, _ptr(y), _ptr(self.ws),
                                    self.ws.numel(), _stream(x.device)))
        return y


def mes_delta_linear(w_base_tiled, experts, x, seg_offsets, y=None, workspace=None):
    return DeltaLinear(w_base_tiled, experts, x.shape[0], workspace)(x, seg_offsets, y)


def mes_delta_linear_noalloc(w_base_tiled: torch.Tensor, experts: Sequence[PackedDelta], x: torch.Tensor,
                             seg_offsets: Sequence[int], y: torch.Tensor) -> torch.Tensor:
    """mes_delta_linear_noalloc: the scratch is the library's device-resident static array; y is the caller's."""
    E, T = len(experts), x.shape[0]
    desc = (mes_delta * E)(*[e.descriptor() for e in experts])
    seg = (ctypes.c_int32 * (E + 1))(*seg_offsets)
    _check(lib.mes_delta_linear_noalloc(_ptr(w_base_tiled), desc, E, _ptr(x), T, seg, _ptr(y), _stream(x.device)))
    return y


def mes_delta_linear_descriptors(w_base_tiled: torch.Tensor, desc, x: torch.Tensor, seg_offsets: Sequence[int],
                                 workspace: torch.Tensor, y: Optional[torch.Tensor] = None) -> torch.Tensor:
    """mes_delta_linear on a ready ctypes array of mes_delta (e.g. what ExpertPool.acquire returns)."""
    E, T, d_out = len(desc), x.shape[0], desc[0].d_out
    if y is None:
        y = torch.empty((T, d_out), dtype=torch.bfloat16, device=x.device)
    seg = (ctypes.c_int32 * (E + 1))(*seg_offsets)
    _check(lib.mes_delta_linear(_ptr(w_base_tiled), desc, E, _ptr(x), T, seg, _ptr(y), _ptr(workspace),
                                workspace.numel(), _stream(x.device)))
    return y


def mes_delta_linear_multi_descriptors(ws_tiled: Sequence[torch.Tensor], descs: Sequence, x: torch.Tensor,
                                       seg_offsets: Sequence[int], workspace: torch.Tensor,
                                       ys: Optional[Sequence[torch.Tensor]] = None):
    """mes_delta_linear_multi on ready ctypes arrays of mes_delta, one per layer (e.g. what a layer-spanning
    ExpertPool.acquire returns)."""
    n, E, T = len(descs), len(descs[0]), x.shape[0]
    if ys is None:
        ys = [torch.empty((T, d[0].d_out), dtype=torch.bfloat16, device=x.device) for d in descs]
    lin = (mes_linear * n)(*[mes_linear(ws_tiled[l].data_ptr(), descs[l], ys[l].data_ptr()) for l in range(n)])
    seg = (ctypes.c_int32 * (E + 1))(*seg_offsets)
    _check(lib.mes_delta_linear_multi(lin, n, E, _ptr(x), T, seg, _ptr(workspace), workspace.numel(), _stream(x.device)))
    return list(ys)


class DeltaLinearMulti:
    """Marshalled arguments of mes_delta_linear_multi: several layers that read the same activations and routing."""

    def __init__(self, layers: Sequence, max_tokens: int = 64, workspace: Optional[torch.Tensor] = None):
        """layers: sequence of (w_base_tiled, [PackedDelta per expert]).  workspace: a workspace of at
        least workspace_bytes(...) bytes to share between calls that are stream-ordered, or None to allocate one."""
        self.ws_tiled = [w for w, _ in layers]
        self.experts = [list(ex) for _, ex in layers]
        self.n = len(layers)
        self.E = len(self.experts[0])
        self.d_in = self.experts[0][0].d_in
        self.d_out = [ex[0].d_out for ex in self.experts]
        self.desc = [(mes_delta * self.E)(*[e.descriptor() for e in ex]) for ex in self.experts]
        dev = self.ws_tiled[0].device
        d = (ctypes.c_int32 * self.n)(*self.d_out)
        nbytes = max(lib.mes_linear_multi_workspace_bytes(self.d_in, d, self.n, max_tokens), 16)
        if workspace is not None:
            assert workspace.numel() >= nbytes
            self.ws = workspace
        else:
            self.ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)

    @staticmethod
    def workspace_bytes(d_in: int, d_outs: Sequence[int], max_tokens: int) -> int:
        d = (ctypes.c_int32 * len(d_outs))(*d_outs)
        return max(lib.mes_linear_multi_workspace_bytes(d_in, d, len(d_outs), max_tokens), 16)

    def __call__(self, x: torch.Tensor, seg_offsets: Sequence[int], ys: Optional[Sequence[torch.Tensor]] = None):
        T = x.shape[0]
        if ys is None:
            ys = [torch.empty((T, d), dtype=torch.bfloat16, device=x.device) for d in self.d_out]
        lin = (mes_linear * self.n)(*[mes_linear(self.ws_tiled[l].data_ptr(), self.desc[l], ys[l].data_ptr())
                                      for l in range(self.n)])
        seg = (ctypes.c_int32 * (self.E + 1))(*seg_offsets)
        _check(lib.mes_delta_linear_multi(lin, self.n, self.E, _ptr(x), T, seg, _ptr(self.ws), self.ws.numel(),
                                          _stream(x.device)))
        return list(ys)


class DeltaLinearGated:
    """Marshalled arguments of mes_delta_linear_gated: h = SiLU(gate layer) * (up layer), one pass, one output."""

    def __init__(self, w_gate_tiled, gate_experts, w_up_tiled, up_experts, max_tokens: int = 64,
                 workspace: Optional[torch.Tensor] = None):
        self.w_gate, self.w_up = w_gate_tiled, w_up_tiled
        self.gate, self.up = list(gate_experts), list(up_experts)
        self.E = len(self.gate)
        self.d_in, self.d_out = self.gate[0].d_in, self.gate[0].d_out
        self.gate_desc = (mes_delta * self.E)(*[e.descriptor() for e in self.gate])
        self.up_desc = (mes_delta * self.E)(*[e.descriptor() for e in self.up])
        nbytes = max(lib.mes_gated_workspace_bytes(self.d_in, self.d_out, max_tokens), 16)
        self.ws = workspace if workspace is not None else torch.empty(nbytes, dtype=torch.uint8, device=w_gate_tiled.device)
        assert self.ws.numel() >= nbytes

    def __call__(self, x: torch.Tensor, seg_offsets: Sequence[int], h: Optional[torch.Tensor] = None) -> torch.Tensor:
        T = x.shape[0]
        if h is None:
            h = torch.empty((T, self.d_out), dtype=torch.bfloat16, device=x.device)
        seg = (ctypes.c_int32 * (self.E + 1))(*seg_offsets)
        _check(lib.mes_delta_linear_gated(_ptr(self.w_gate), self.gate_desc, _ptr(self.w_up), self.up_desc, self.E, _ptr(x), T,
                                          seg, _ptr(h), _ptr(self.ws), self.ws.numel(), _stream(x.device)))
        return h


class ExpertPool:
    """On-demand swapping (mes_pool_* in mes.h): a device arena of `n_slots` slots and one pinned host blob per
    registered expert.  d_in, d_out, k: ints for a pool over one linear layer, or equally long sequences for a pool
    whose slots hold an expert's deltas of several layers (a miss is one copy either way)."""

    def __init__(self, d_in, d_out, k, bits: int, grid: int, n_slots: int, n_experts: int,
                 device="cuda:0", dry_run: bool = False):
        self.single = isinstance(d_in, int)
        as_list = lambda v: [int(v)] if isinstance(v, int) else [int(a) for a in v]
        self.d_in, self.d_out, self.k = as_list(d_in), as_list(d_out), as_list(k)
        self.n_linears = len(self.d_in)
        assert len(self.d_out) == self.n_linears and len(self.k) == self.n_linears
        self.bits, self.grid = bits, grid
        self.n_slots = n_slots
        arr = lambda v: (ctypes.c_int32 * self.n_linears)(*v)
        self.slot_bytes = lib.mes_pool_multi_slot_bytes(self.n_linears, arr(self.d_in), arr(self.d_out), arr(self.k), bits)
        if dry_run:
            self.arena, arena_ptr = None, 256          # any aligned non-null address: a dry-run pool never touches it
        else:
            self.arena = torch.empty(self.slot_bytes * n_slots, dtype=torch.uint8, device=device)
            arena_ptr = self.arena.data_ptr()
            self.copy_stream = torch.cuda.Stream(device=device)
        self.device = device
        self.dry_run = dry_run
        self.host = {}                                  # expert -> pinned host blob (kept alive here)
        h = ctypes.c_void_p()
        _check(lib.mes_pool_create_multi(self.n_linears, arr(self.d_in), arr(self.d_out), arr(self.k), bits, grid, n_slots,
                                         n_experts, arena_ptr, self.slot_bytes * n_slots, int(dry_run), ctypes.byref(h)))
        self.handle = h
        # where each linear's buffers sit inside a slot / blob
        self.offsets = []
        for l in range(self.n_linears):
            off = (ctypes.c_size_t * 4)()
            lib.mes_pool_slot_layout(self.d_in[l], self.d_out[l], self.k[l], bits, off)
            base = lib.mes_pool_linear_offset(self.handle, l)
            self.offsets.append([base + int(o) for o in off])

    def register(self, expert: int, packed) -> None:
        """packed: a PackedDelta (single-linear pool) or one per linear.  Builds the expert's blob in pinned host
        memory and registers it."""
        packed = [packed] if self.single and not isinstance(packed, (list, tuple)) else list(packed)
        assert len(packed) == self.n_linears
        blob = torch.zeros(self.slot_bytes, dtype=torch.uint8, pin_memory=True)
        for l, pk in enumerate(packed):
            for off, t in zip(self.offsets[l], (pk.codes, pk.step, pk.salient, pk.salient_idx)):
                if t is None or t.numel() == 0:
                    continue
                raw = t.contiguous().view(torch.uint8).reshape(-1)
                blob[off: off + raw.numel()].copy_(raw)
        if expert in self.host and not self.dry_run:
            # a copy out of the blob this one replaces may still be in flight
            self.copy_stream.synchronize()
        _check(lib.mes_pool_register_blob(self.handle, expert, blob.data_ptr()))
        self.host[expert] = blob

    def register_raw(self, expert: int, codes: int, step: int, salient: int, sidx: int) -> None:
        _check(lib.mes_pool_register(self.handle, expert, codes, step, salient, sidx))

    def _streams(self):
        if self.dry_run:
            return None, None
        return self.copy_stream.cuda_stream, _stream(torch.device(self.device))

    def acquire(self, experts: Sequence[int]):
        """Makes `experts` resident; returns the ctypes array of their descriptors (valid until the next acquire):
        [n] for a single-linear pool, else a list with one such array per linear."""
        n = len(experts)
        ids = (ctypes.c_int32 * n)(*experts)
        out = (mes_delta * (n * self.n_linears))()
        cs, ks = self._streams()
        _check(lib.mes_pool_acquire_multi(self.handle, ids, n, out, cs, ks))
        if self.single:
            return out
        size = ctypes.sizeof(mes_delta) * n
        return [(mes_delta * n).from_buffer(out, l * size) for l in range(self.n_linears)]   # views: `out` stays alive with them

    def prefetch(self, experts: Sequence[int]) -> int:
        """Starts loading the experts that are not resident into slots the latest acquire did not hand out; returns
        how many copies were started."""
        n = len(experts)
        ids = (ctypes.c_int32 * n)(*experts)
        loaded = ctypes.c_int(0)
        cs, _ = self._streams()
        _check(lib.mes_pool_prefetch(self.handle, ids, n, ctypes.byref(loaded), cs))
        return loaded.value

    def slot_of(self, expert: int) -> int:
        return lib.mes_pool_slot_of(self.handle, expert)

    def stats(self):
        h, m, b = ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_uint64()
        _check(lib.mes_pool_stats(self.handle, ctypes.byref(h), ctypes.byref(m), ctypes.byref(b)))
        return h.value, m.value, b.value

    def prefetched(self) -> int:
        return lib.mes_pool_prefetched(self.handle)

    def __del__(self):
        if getattr(self, "handle", None):
            lib.mes_pool_destroy(self.handle)
            self.handle = None


class KernelTimer:
    """HIP events recorded by the library around its dominant kernel (mes_time_next_call in mes_bench.h): `n` pairs,
    so that a whole sequence of calls can be timed without a synchronisation in between."""

    def __init__(self, n: int = 1):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.pairs = []
        for _ in range(n):
            pair = (ctypes.c_void_p(), ctypes.c_void_p())
            for ev in pair:
                if self.hip.hipEventCreate(ctypes.byref(ev)) != 0:
                    raise RuntimeError("hipEventCreate failed")
            self.pairs.append(pair)

    def arm(self, i: int = 0) -> None:
        """The next timed library call of this thread records pair i."""
        _check(lib.mes_time_next_call(self.pairs[i][0], self.pairs[i][1]))

    def elapsed_us(self, i: int = 0) -> float:
        start, stop = self.pairs[i]
        if self.hip.hipEventSynchronize(stop) != 0:
            raise RuntimeError("hipEventSynchronize failed")
        ms = ctypes.c_float()
        if self.hip.hipEventElapsedTime(ctypes.byref(ms), start, stop) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return ms.value * 1e3
