"""CPU-only checks of the C-ABI library: it loads, exports what include/mes.h declares, its size
functions agree with the layout specification, and every argument error is caught on the host
(before any HIP call), so none of these needs a GPU."""
import ctypes
import os
import re

import pytest

import paper_2406_09041_amd.binding as B
from oracle import mes_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
lib = B.lib
FAKE = 0x10000          # a non-null, 16-byte aligned address that is never dereferenced on the host
ODD = 0x10004           # misaligned


def test_every_declared_symbol_is_exported():
    declared = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        declared |= set(re.findall(r"\b(mes_[a-z_]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.mes_layout_version() == 3


def test_size_functions_match_the_layout_specification():
    for d_in, d_out, k in [(256, 256, 8), (4096, 4096, 64), (14336, 4096, 128), (4096, 14336, 64), (264, 72, 5), (8, 4, 0)]:
        po, pi, pk = O.padded_dims(d_out, d_in, k)
        assert lib.mes_base_bytes(d_in, d_out) == po * pi * 2
        for bits in (1, 2, 3, 4):
            assert lib.mes_codes_bytes(d_in, d_out, bits) == O.codes_bytes(d_in, d_out, bits)
        assert lib.mes_salient_bytes(d_out, k) == po * pk * 2
        assert lib.mes_linear_workspace_bytes(d_in, d_out, 64) >= po // 16 * 4
    assert lib.mes_codes_bytes(4096, 4096, 5) == 0
    assert lib.mes_base_bytes(0, 4) == 0


def _status(call):
    st = call()
    return st, lib.mes_last_error().decode()


def test_pack_base_argument_errors():
    st, msg = _status(lambda: lib.mes_pack_base(None, 64, 64, FAKE, None))
    assert st == 1 and "null" in msg
    assert lib.mes_pack_base(FAKE, 0, 64, FAKE, None) == 2
    assert lib.mes_pack_base(FAKE, 60, 64, FAKE, None) == 2        # d_in % 8
    assert lib.mes_pack_base(FAKE, 64, 62, FAKE, None) == 2        # d_out % 4
    assert lib.mes_pack_base(ODD, 64, 64, FAKE, None) == 6


def test_pack_delta_argument_errors():
    def call(delta=FAKE, d_in=64, d_out=64, sidx=FAKE, k=4, bits=2, grid=0, pol=1, step_in=None, codes=FAKE,
             step=FAKE, sal=FAKE, ws=FAKE, wsb=256):
        return lib.mes_pack_delta(delta, d_in, d_out, sidx, k, bits, grid, pol, step_in, codes, step, sal, ws, wsb, None)
    assert call(delta=None) == 1
    assert call(bits=0) == 3 and call(bits=5) == 3
    assert call(bits=1, grid=1) == 3                               # Eq. 1 grid has no 1-bit form
    assert call(grid=2) == 3
    assert call(pol=2, bits=2) == 3                                # MEANABS is the binary scale
    assert call(pol=0, step_in=None) == 1                          # GIVEN needs step_in
    assert call(k=-1) == 4 and call(k=65) == 4
    assert call(sidx=None) == 1 and call(sal=None) == 1
    assert call(codes=ODD) == 6
    assert call(ws=None) == 7 and call(wsb=8) == 7
    assert call(d_in=-8) == 2


def test_select_argument_errors():
    def call(delta=FAKE, xc=FAKE, n=4, d_in=64, d_out=64, bits=2, grid=0, pol=1, k=4, idx=FAKE, score=None, ws=FAKE, wsb=1 << 20):
        return lib.mes_select_salient(delta, xc, n, d_in, d_out, bits, grid, pol, k, idx, score, ws, wsb, None)
    assert call(xc=None) == 1
    assert call(n=0) == 2
    assert call(pol=0) == 3                                        # selection never takes a given step
    assert call(k=65) == 4
    assert call(idx=None) == 1
    assert call(wsb=16) == 7


def _desc(**kw):
    d = dict(d_in=64, d_out=64, k=4, bits=2, grid=0, layout_version=3, codes=FAKE, step=FAKE, salient=FAKE, salient_idx=FAKE)
    d.update(kw)
    return B.mes_delta(**d)


def _linear(descs, T, seg, w=FAKE, x=FAKE, y=FAKE, ws=FAKE, wsb=1 << 30):
    arr = (B.mes_delta * len(descs))(*descs)
    segc = (ctypes.c_int32 * len(seg))(*seg)
    return lib.mes_delta_linear(w, arr, len(descs), x, T, segc, y, ws, wsb, None)


def test_delta_linear_argument_errors():
    d = _desc()
    assert _linear([d], 4, [0, 4], w=None) == 1
    assert _linear([d], 4, [1, 4]) == 5                            # must start at 0
    assert _linear([d, d], 4, [0, 3, 2]) == 5                      # decreasing
    assert _linear([d, d], 4, [0, 2, 3]) == 5                      # must end at T
    assert _linear([d], -1, [0, -1]) == 2
    assert _linear([d, _desc(k=8)], 4, [0, 2, 4]) == 2             # experts must agree
    assert _linear([d, _desc(bits=3)], 4, [0, 2, 4]) == 2
    assert _linear([_desc(bits=5)], 4, [0, 4]) == 3
    assert _linear([_desc(layout_version=7)], 4, [0, 4]) == 2
    assert _linear([_desc(codes=None)], 4, [0, 4]) == 1
    assert _linear([_desc(salient_idx=None)], 4, [0, 4]) == 1
    assert _linear([_desc(step=ODD)], 4, [0, 4]) == 6
    assert _linear([d], 4, [0, 4], x=ODD) == 6
    assert _linear([d], 4, [0, 4], ws=None) == 7
    assert _linear([d], 4, [0, 4], wsb=4) == 7
    assert "workspace needs" in lib.mes_last_error().decode()
    # T = 0 is a no-op that never touches a pointer
    assert _linear([d], 0, [0, 0], w=None, x=None, y=None, ws=None, wsb=0) == 0
    arr = (B.mes_delta * 1)(d)
    assert lib.mes_delta_linear(FAKE, arr, 65, FAKE, 4, (ctypes.c_int32 * 2)(0, 4), FAKE, FAKE, 1 << 30, None) == 2


def test_delta_linear_multi_argument_errors():
    d = _desc()
    arr = (B.mes_delta * 2)(d, d)
    wide = (B.mes_delta * 2)(_desc(d_out=128), _desc(d_out=128))
    seg = (ctypes.c_int32 * 3)(0, 2, 4)

    def call(layers, n=None, T=4, ws=FAKE, wsb=1 << 30, x=FAKE):
        lin = (B.mes_linear * len(layers))(*layers)
        return lib.mes_delta_linear_multi(lin, len(layers) if n is None else n, 2, x, T, seg, ws, wsb, None)
    ok = B.mes_linear(FAKE, arr, FAKE)
    assert call([ok, B.mes_linear(FAKE, wide, FAKE)], wsb=4) == 7          # two layers of different widths: fine up to the workspace
    assert call([ok], n=0) == 2 and call([ok] * 4) == 2                    # 1 .. MES_MAX_FUSED layers
    assert call([ok, B.mes_linear(None, arr, FAKE)]) == 1
    assert call([ok, B.mes_linear(FAKE, arr, None)]) == 1
    assert call([ok, B.mes_linear(FAKE, arr, ODD)]) == 6
    other_k = (B.mes_delta * 2)(_desc(k=8), _desc(k=8))
    assert call([ok, B.mes_linear(FAKE, other_k, FAKE)]) == 2              # k must agree across layers
    mixed = (B.mes_delta * 2)(_desc(d_out=128), _desc(d_out=64))
    assert call([B.mes_linear(FAKE, mixed, FAKE)]) == 2                    # experts of one layer must agree on d_out
    d2 = (ctypes.c_int32 * 2)(64, 128)
    assert lib.mes_linear_multi_workspace_bytes(64, d2, 2, 64) > lib.mes_linear_workspace_bytes(64, 64, 64)
    assert lib.mes_linear_multi_workspace_bytes(64, d2, 4, 64) == 0


def test_unpack_argument_errors():
    d = _desc()
    assert lib.mes_unpack_delta(ctypes.byref(d), None, None, None) == 1
    assert lib.mes_unpack_delta(None, FAKE, None, None) == 1


def test_noalloc_entry_point_argument_errors():
    """The allocation-free entry point checks its limit on the host, before any GPU call."""
    assert lib.mes_noalloc_scratch_bytes() == 64 << 20
    seg = (ctypes.c_int32 * 2)(0, 4)
    d = _desc()
    assert lib.mes_delta_linear_noalloc(FAKE, None, 1, FAKE, 4, seg, FAKE, None) == 1
    assert lib.mes_delta_linear_noalloc(FAKE, ctypes.byref(d), 0, FAKE, 4, seg, FAKE, None) == 2
    huge = _desc(d_in=1 << 20, d_out=1 << 20)
    assert lib.mes_linear_workspace_bytes(1 << 20, 1 << 20, 1) > lib.mes_noalloc_scratch_bytes()
    assert lib.mes_delta_linear_noalloc(FAKE, ctypes.byref(huge), 1, FAKE, 4, seg, FAKE, None) == 7
    assert b"static array" in lib.mes_last_error()
    for d_in, d_out in [(4096, 4096), (4096, 1024), (4096, 14336), (14336, 4096)]:      # every Mistral-7B shape fits
        assert 0 < lib.mes_linear_workspace_bytes(d_in, d_out, 1) <= lib.mes_noalloc_scratch_bytes()


def test_gated_entry_point_argument_errors_and_workspace_sizes():
    """Host-side validation of mes_delta_linear_gated, and the slices of the streaming workspaces: one 64-token group
    for up to 64 tokens, two up to 128, four above."""
    seg = (ctypes.c_int32 * 2)(0, 4)
    g, u = _desc(), _desc()
    ws = lib.mes_gated_workspace_bytes(g.d_in, g.d_out, 4)
    call = lambda gate=g, up=u, h=FAKE, wsp=FAKE, n=ws: lib.mes_delta_linear_gated(
        FAKE, ctypes.byref(gate) if gate is not None else None, FAKE, ctypes.byref(up) if up is not None else None, 1, FAKE, 4, seg,
        h, wsp, n, None)
    assert call(gate=None) == 1 and call(up=None) == 1 and call(h=None) == 1
    assert call(up=_desc(d_out=g.d_out * 2)) == 2 and b"d_out" in lib.mes_last_error()
    assert call(up=_desc(bits=3)) == 2
    assert call(wsp=None) == 7 and call(n=ws - 1) == 7
    assert lib.mes_gated_workspace_bytes(0, 64, 4) == 0
    one = lib.mes_linear_workspace_bytes(4096, 4096, 64)
    assert lib.mes_linear_workspace_bytes(4096, 4096, 1) == one
    assert lib.mes_linear_workspace_bytes(4096, 4096, 65) == 2 * one == lib.mes_linear_workspace_bytes(4096, 4096, 128)
    assert lib.mes_linear_workspace_bytes(4096, 4096, 129) == 4 * one
    assert lib.mes_linear_workspace_bytes(4096, 4096, 192) > 4 * one            # + the one-product scratch
    g1 = lib.mes_gated_workspace_bytes(4096, 14336, 64)
    assert lib.mes_gated_workspace_bytes(4096, 14336, 256) == 4 * g1


def test_copy_probe_argument_errors():
    lib = B.lib
    assert lib.mes_copy_probe(None, 16, 16, None) == 1
    assert lib.mes_copy_probe(32, 16, 24, None) == 6
    assert lib.mes_copy_probe(32, 24, 16, None) == 6


def test_step_grad_argument_errors_and_workspace_size():
    """Host-side validation of the step-learning entry points (no kernel is launched on any of these paths)."""
    lib = B.lib
    c_f = ctypes.c_float
    assert lib.mes_step_grad_workspace_bytes(0, 64, 8) == 0 and lib.mes_step_grad_workspace_bytes(64, 64, -1) == 0
    # 512 tokens, 4096 -> 14336: activations as fragments (4 MiB) + column mask + 8 token groups of partial sums
    assert lib.mes_step_grad_workspace_bytes(4096, 14336, 512) == 4096 * 512 * 2 + 512 + 8 * 2 * 14336 * 4
    # one token still takes a whole 256-token block of fragments
    assert lib.mes_step_grad_workspace_bytes(128, 64, 1) == 128 * 256 * 2 + 256 + 4 * 2 * 64 * 4
    # few rows: the input channels are split over workgroups (4 x 64 of them here), which leave their accumulator
    # tiles (32 tiles of 16 bytes per thread, 512 multiplying threads) in the workspace
    assert lib.mes_step_grad_workspace_bytes(14336, 4096, 512) == \
        14336 * 512 * 2 + 1792 + 8 * 2 * 4096 * 4 + 4 * 64 * 32 * 512 * 16
    ok = dict(delta=4096, d_in=128, d_out=64, sidx=4096, k=2, bits=2, grid=0, step=4096, x=4096, n=8, loss=4096,
              grad=4096, ws=4096, ws_bytes=1 << 20, stream=None)

    def call(**kw):
        a = {**ok, **kw}
        return lib.mes_step_grad(a["delta"], a["d_in"], a["d_out"], a["sidx"], a["k"], a["bits"], a["grid"], a["step"],
                                 a["x"], a["n"], a["loss"], a["grad"], a["ws"], a["ws_bytes"], a["stream"])

    assert call(delta=None) == 1 and call(loss=None) == 1 and call(x=None) == 1 and call(sidx=None) == 1
    assert call(d_in=100) == 2 and call(n=-1) == 2
    assert call(bits=5) == 3 and call(bits=1, grid=1) == 3
    assert call(k=129) == 4
    assert call(delta=4100) == 6 and call(ws=4104) == 6
    assert call(ws=None) == 7 and call(ws_bytes=100) == 7
    assert b"workspace" in lib.mes_last_error()
    adam = lambda **kw: lib.mes_step_adamw(*[{**dict(s=4096, g=4096, m=4096, v=4096, n=8, t=1, lr=c_f(1e-3),
                                                     b1=c_f(0.9), b2=c_f(0.99), eps=c_f(1e-8), wd=c_f(0.0), st=None), **kw}[k]
                                             for k in ("s", "g", "m", "v", "n", "t", "lr", "b1", "b2", "eps", "wd", "st")])
    assert adam(m=None) == 1 and adam(n=0) == 2 and adam(t=0) == 2 and adam(b1=c_f(1.0)) == 2


def test_no_cpu_fallback_in_the_product_path():
    """The binding and the library sources never import or include the oracle."""
    pkg = os.path.join(ROOT, "paper_2406_09041_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src, os.path.join(dirpath, f)
