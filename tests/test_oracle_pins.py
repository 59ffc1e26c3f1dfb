"""Pins for the CPU oracle: what the paper and the mathematics fix, independent of the oracle itself.

Each test is chosen so that a plausible mistake in oracle/mes_oracle.py (a dropped term, a wrong
sign or index, a transposed operand, an off-by-one level) makes it fail.
"""
import itertools
import math
import os

import numpy as np
import pytest
import torch

from inputs import synth
from oracle import mes_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_sizes.txt")


def _rng(seed):
    return np.random.default_rng(seed)


def _delta(d_out, d_in, seed, k=0, scale=15.0):
    ex = synth.make_delta(d_in, d_out, k, 0.003, scale, 1234 + seed)
    return ex.delta.numpy(), ex.salient_idx.numpy()


# ---------------------------------------------------------------- pack / unpack round trip

@pytest.mark.parametrize("bits", [1, 2, 3, 4])
@pytest.mark.parametrize("shape", [(16, 64), (70, 248), (33, 515), (1, 1), (64, 1031)])
def test_pack_unpack_roundtrip(bits, shape):
    d_out, d_in = shape
    codes = _rng(bits * 100 + d_in).integers(0, 2 ** bits, size=shape, dtype=np.uint8)
    packed = O.pack_codes(codes, bits)
    assert packed.dtype == np.uint32
    assert packed.nbytes == O.codes_bytes(d_in, d_out, bits)
    back = O.unpack_codes(packed, bits, d_out, d_in)
    assert np.array_equal(back, codes)


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_pack_every_bit_is_used_exactly_once(bits):
    """One-hot probes: each (row, column, code bit) lands on its own bit of the packed words, none collide,
    and the place is the one the layout specification gives."""
    seen = set()
    for row in (5, 21):
        for col in range(128):
            for cb in range(bits):
                codes = np.zeros((32, 128), dtype=np.uint8)
                codes[row, col] = 1 << cb
                packed = O.pack_codes(codes, bits)
                assert packed.shape == (1, 4, 64 * bits)         # rows are padded to 64 = four row tiles
                nz = np.argwhere(packed != 0)
                assert len(nz) == 1 and nz[0][0] == 0 and nz[0][1] == row // 16
                widx = int(nz[0][2])
                word = int(packed[0, row // 16, widx])
                assert word & (word - 1) == 0                    # exactly one bit
                bit = word.bit_length() - 1
                g, q, p = col // 32, (col % 32) // 8, col % 8
                lane = 16 * g + row % 16
                if bits == 1 or (bits == 3 and cb == 2):         # one word per lane, bit 4 p + q
                    off = 128 if bits == 3 else 0
                    assert (widx, bit) == (off + lane, 4 * p + q)
                elif bits == 4 and cb >= 2:                      # the second 2-bit block: the high two bits
                    assert (widx, bit) == (128 + 2 * lane + q // 2, 4 * p + 2 * (q % 2) + cb - 2)
                else:                                            # two words per lane, 2-bit fields
                    assert (widx, bit) == (2 * lane + q // 2, 4 * p + 2 * (q % 2) + cb)
                assert (row // 16, widx, bit) not in seen
                seen.add((row // 16, widx, bit))
    assert len(seen) == 2 * 128 * bits


def test_pack_is_chunk_major():
    """All row tiles of one 128-column chunk are contiguous: the block of (chunk c, row tile jt) is packed[c, jt]."""
    codes = np.zeros((64, 384), dtype=np.uint8)
    codes[40, 300] = 3                                           # row tile 2, chunk 2
    packed = O.pack_codes(codes, 2)
    assert packed.shape == (3, 4, 128)
    nz = np.argwhere(packed != 0)
    assert len(nz) == 1 and tuple(nz[0][:2]) == (2, 2)


def test_packed_words_are_fp4_operands():
    """The reason for the 4-bit fields: a 2-bit code u in the low half of a field is the fp4 (E2M1) bit
    pattern of u / 2, a high bit in position 2 of a field is the pattern of 2.  E2M1: sign, two exponent
    bits (bias 1), one mantissa bit; exponent 0 is subnormal (0 or 1/2)."""
    def e2m1(n):
        e, m = (n >> 1) & 3, n & 1
        return (m * 0.5 if e == 0 else (1 + m * 0.5) * 2.0 ** (e - 1)) * (-1 if n & 8 else 1)
    assert [e2m1(u) for u in range(4)] == [0.0, 0.5, 1.0, 1.5]
    assert e2m1(0b0100) == 2.0
    codes = _rng(9).integers(0, 8, size=(16, 128), dtype=np.uint8)
    packed = O.pack_codes(codes, 3)[0, 0]
    low, high = packed[:128].reshape(64, 2), packed[128:]
    for lane in (0, 17, 63):
        row, g = lane % 16, lane // 16
        for q in range(4):
            lo_reg = (int(low[lane, q // 2]) >> (2 * (q % 2))) & 0x33333333
            hi_reg = ((int(high[lane]) << 2) >> q) & 0x44444444
            for p in range(8):
                u = int(codes[row, 32 * g + 8 * q + p])
                assert e2m1((lo_reg >> (4 * p)) & 15) + e2m1((hi_reg >> (4 * p)) & 15) == u / 2
    # b = 4: two 2-bit planes; the high plane counts four times (a block scale of 2^2 in the kernel)
    codes = _rng(10).integers(0, 16, size=(16, 128), dtype=np.uint8)
    packed = O.pack_codes(codes, 4)[0, 0]
    low, high = packed[:128].reshape(64, 2), packed[128:].reshape(64, 2)
    for lane in (3, 30, 62):
        row, g = lane % 16, lane // 16
        for q in range(4):
            lo_reg = (int(low[lane, q // 2]) >> (2 * (q % 2))) & 0x33333333
            hi_reg = (int(high[lane, q // 2]) >> (2 * (q % 2))) & 0x33333333
            for p in range(8):
                u = int(codes[row, 32 * g + 8 * q + p])
                assert e2m1((lo_reg >> (4 * p)) & 15) + 4 * e2m1((hi_reg >> (4 * p)) & 15) == u / 2


def test_pack_padding_and_salient_are_zero_codes():
    codes = np.full((5, 70), 3, dtype=np.uint8)
    codes[:, [3, 17]] = O.SALIENT_MARK
    packed = O.pack_codes(codes, 2)
    back = O.unpack_codes(packed, 2, 64, 128)
    assert back[:5, :70].sum() == 3 * 5 * 68
    assert back[5:].sum() == 0 and back[:, 70:].sum() == 0
    assert back[:5, 3].sum() == 0 and back[:5, 17].sum() == 0


def test_base_and_salient_tiling_roundtrip_and_slot_rule():
    w = _rng(3).integers(0, 65536, size=(70, 100), dtype=np.uint16)
    t = O.pack_base(w)
    assert t.shape == (1, 128 // 16, 4, 64, 8)
    assert np.array_equal(O.unpack_base(t, 70, 100), w)
    # slot rule stated independently: lane = 16 g + r holds W[16 jt + r, 128 c + 32 kb + 8 g + e]
    for (j, i) in [(0, 0), (17, 45), (69, 99), (33, 8)]:
        jt, r, c, kb, g, e = j // 16, j % 16, i // 128, (i % 128) // 32, (i % 32) // 8, i % 8
        assert t[c, jt, kb, 16 * g + r, e] == w[j, i]
    w2 = _rng(5).integers(0, 65536, size=(32, 384), dtype=np.uint16)
    t2 = O.pack_base(w2)
    assert t2.shape == (3, 4, 4, 64, 8) and t2[2, 1, 3, 16 * 2 + 5, 7] == w2[21, 256 + 96 + 16 + 7]
    assert np.array_equal(O.unpack_base(t2, 32, 384), w2)
    s = _rng(4).standard_normal((20, 40)).astype(np.float16)
    ts = O.pack_salient(s)
    assert ts.shape == (4, 2, 64, 8)
    assert np.array_equal(O.unpack_salient(ts, 20, 40).view(np.uint16), s.view(np.uint16))


# ---------------------------------------------------------------- Eq. 1: quantiser

@pytest.mark.parametrize("bits,grid", [(1, O.GRID_SYM), (2, O.GRID_SYM), (3, O.GRID_SYM), (4, O.GRID_SYM),
                                       (2, O.GRID_EQ1), (3, O.GRID_EQ1), (4, O.GRID_EQ1)])
def test_rounding_error_at_most_half_a_step(bits, grid):
    """With the initial step nothing clips, so |w - w_hat| <= s/2 everywhere (Eq. 1)."""
    delta, sidx = _delta(48, 300, bits + 10 * grid, k=8)
    codes, step, sal = O.quantize(delta, sidx, bits, grid, O.STEP_MAXABS)
    ns = O.non_salient_mask(300, sidx)
    w_hat = O.dequantize(codes, step, bits, grid)
    err = np.abs(delta.astype(np.float64) - w_hat)[:, ns]
    bound = step.astype(np.float64)[:, None] / 2 * (1 + 1e-6)
    assert np.all(err <= bound)
    assert err.max() > 0.45 * step.max()          # the bound is tight, not vacuous
    assert codes[:, ns].max() == 2 ** bits - 1 and codes[:, ns].min() == 0 or grid == O.GRID_EQ1


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_eq1_level_set(bits):
    """Eq. 1: integer levels -2^(b-1) .. 2^(b-1)-1; with s = max|X|/(2^(b-1)-1) the row maximum sits on +Q_P."""
    delta, _ = _delta(32, 200, 77 + bits)
    codes, step, _ = O.quantize(delta, [], bits, O.GRID_EQ1, O.STEP_MAXABS)
    lv = codes.astype(np.int64) - 2 ** (bits - 1)
    assert lv.min() >= -(2 ** (bits - 1)) and lv.max() <= 2 ** (bits - 1) - 1
    qp = 2 ** (bits - 1) - 1
    for j in range(32):
        i = np.argmax(np.abs(delta[j]))
        assert abs(lv[j, i]) == qp or (delta[j, i] < 0 and lv[j, i] == -qp)
        assert math.isclose(step[j], np.abs(delta[j]).max() / qp, rel_tol=1e-6)
    # direct restatement of Eq. 1 on one row with python floats
    j = 3
    s = float(step[j])
    for i in range(0, 200, 7):
        r = float(delta[j, i]) / s
        n = math.floor(r)
        frac = r - n
        if frac > 0.5 or (frac == 0.5 and n % 2 == 1):
            n += 1
        n = max(-(2 ** (bits - 1)), min(qp, n))
        assert lv[j, i] == n


def test_sym_levels_are_half_integers_and_match_config_wording():
    """2-bit symmetric, step = rowmax/1.5  ->  levels {-1.5,-0.5,0.5,1.5} * step (the benchmark configs' wording)."""
    delta, _ = _delta(16, 128, 5)
    codes, step, _ = O.quantize(delta, [], 2, O.GRID_SYM, O.STEP_MAXABS)
    for j in range(16):
        assert math.isclose(step[j], np.abs(delta[j]).max() / 1.5, rel_tol=1e-6)
    w_hat = O.dequantize(codes, step, 2, O.GRID_SYM)
    lv = np.unique(np.round(w_hat / step[:, None].astype(np.float64), 6))
    assert set(lv.tolist()) <= {-1.5, -0.5, 0.5, 1.5}
    assert np.all(np.sign(w_hat) == np.where(delta >= 0, 1, -1))


def test_step_excludes_salient_columns():
    delta, sidx = _delta(16, 256, 9, k=8, scale=20.0)
    _, step_ns, _ = O.quantize(delta, sidx, 2)
    _, step_all, _ = O.quantize(delta, [], 2)
    assert np.all(step_all > 3 * step_ns)        # planted x20 columns would otherwise set the step
    ns = O.non_salient_mask(256, sidx)
    assert np.allclose(step_ns, np.abs(delta[:, ns]).max(axis=1) / 1.5, rtol=1e-6)


def test_given_step_clips_and_zero_step_rows():
    delta, _ = _delta(8, 64, 11)
    step_in = np.full(8, 1e-4, dtype=np.float32)
    step_in[2] = 0.0
    step_in[5] = -1.0
    codes, step, _ = O.quantize(delta, [], 2, O.GRID_SYM, O.STEP_GIVEN, step_in)
    assert step[2] == 0 and step[5] == 0
    assert np.all(codes[2] == 2) and np.all(codes[5] == 2)
    w_hat = O.dequantize(codes, step, 2, O.GRID_SYM)
    assert np.all(w_hat[2] == 0)
    s0 = float(step[0])
    err = np.abs(delta.astype(np.float64) - w_hat)
    bound = np.maximum(0.5 * s0, np.abs(delta[0].astype(np.float64)) - 1.5 * s0) * (1 + 1e-9)
    assert np.all(err[0] <= bound)
    assert (np.abs(delta[0]) > 2 * s0).any()          # clipping really happens in this row


def test_salient_columns_reproduced_exactly():
    delta, sidx = _delta(24, 128, 21, k=8)
    codes, step, sal = O.quantize(delta, sidx, 2)
    assert sal.dtype == np.float16 and sal.shape == (24, 8)
    want = torch.from_numpy(delta[:, sidx]).to(torch.float16).numpy()      # library RNE conversion
    assert np.array_equal(sal.view(np.uint16), want.view(np.uint16))
    d16 = delta.astype(np.float16).astype(np.float32)                      # fp16-representable delta
    _, _, sal2 = O.quantize(d16, sidx, 2)
    assert np.array_equal(sal2.astype(np.float32), d16[:, sidx])
    dt = O.compressed_delta(codes, step, sal, sidx, 2, O.GRID_SYM)
    assert np.array_equal(dt[:, sidx], sal.astype(np.float64))
    assert np.all(codes[:, sidx] == O.SALIENT_MARK)


def test_binary_meanabs_is_the_least_squares_scale():
    """XNOR-style binary code: w_hat = alpha sign(w); alpha = mean|w| minimises the squared error."""
    delta, _ = _delta(12, 200, 31)
    codes, step, _ = O.quantize(delta, [], 1, O.GRID_SYM, O.STEP_MEANABS)
    w_hat = O.dequantize(codes, step, 1, O.GRID_SYM)
    assert np.allclose(np.abs(w_hat), np.abs(delta).mean(axis=1, keepdims=True), rtol=1e-6)
    assert np.all(np.sign(w_hat) == np.where(delta >= 0, 1.0, -1.0))
    base = ((delta - w_hat) ** 2).sum(axis=1)
    for f in (0.99, 1.01):
        worse = ((delta - f * w_hat) ** 2).sum(axis=1)
        assert np.all(worse >= base)


def test_invalid_arguments():
    delta, _ = _delta(4, 32, 1)
    with pytest.raises(ValueError):
        O.quantize(delta, [], 1, O.GRID_EQ1)
    with pytest.raises(ValueError):
        O.quantize(delta, [], 5)
    with pytest.raises(ValueError):
        O.quantize(delta, [], 2, O.GRID_SYM, O.STEP_MEANABS)


# ---------------------------------------------------------------- Eq. 4: the linear layer

def _compress(wl, grid=O.GRID_SYM, policy=O.STEP_MAXABS, bits=None):
    bits = bits or wl.bits
    out = []
    for ex in wl.experts:
        c, s, sal = O.quantize(ex.delta.numpy(), ex.salient_idx.numpy(), bits, grid, policy)
        out.append(dict(codes=c, step=s, salient=sal, salient_idx=ex.salient_idx.numpy(), bits=bits, grid=grid))
    return out


def _naive_matmul_T(x, w):
    """Separately written textbook product y[t][j] = sum_i x[t][i] w[j][i] (python floats)."""
    T, n = x.shape
    m = w.shape[0]
    y = np.zeros((T, m))
    for t in range(T):
        for j in range(m):
            acc = 0.0
            for i in range(n):
                acc += float(x[t, i]) * float(w[j, i])
            y[t, j] = acc
    return y


def test_special_cases_reduce_to_dense_products():
    wl = synth.small_case(40, 24, [0, 3, 3, 7], 4, 2, seed=1)     # non-square, one empty segment
    x = wl.x.double().numpy()
    w = wl.w_base.double().numpy()
    # (i) zero step and no salient channels -> the base product alone
    ex0 = []
    for ex in wl.experts:
        c, s, sal = O.quantize(ex.delta.numpy(), [], 2, O.GRID_SYM, O.STEP_GIVEN, np.zeros(24, np.float32))
        ex0.append(dict(codes=c, step=s, salient=sal, salient_idx=[], bits=2, grid=O.GRID_SYM))
    y = O.delta_linear(x, w, ex0, wl.seg_offsets)
    assert np.allclose(y, _naive_matmul_T(x, w), rtol=1e-12, atol=1e-12)
    # (ii) every channel salient -> x (W + fp16(D_e))^T per segment
    allc = np.arange(40, dtype=np.int32)
    exa = []
    for ex in wl.experts:
        c, s, sal = O.quantize(ex.delta.numpy(), allc, 2)
        exa.append(dict(codes=c, step=s, salient=sal, salient_idx=allc, bits=2, grid=O.GRID_SYM))
    y = O.delta_linear(x, w, exa, wl.seg_offsets)
    for e in range(3):
        lo, hi = wl.seg_offsets[e], wl.seg_offsets[e + 1]
        d16 = wl.experts[e].delta.to(torch.float16).double().numpy()
        assert np.allclose(y[lo:hi], _naive_matmul_T(x[lo:hi], w + d16), rtol=1e-12, atol=1e-12)
    # (iv) zero base -> the second term of Eq. 4 alone: x Dtilde^T
    exs = _compress(wl)
    y = O.delta_linear(x, np.zeros_like(w), exs, wl.seg_offsets)
    for e in range(3):
        lo, hi = wl.seg_offsets[e], wl.seg_offsets[e + 1]
        dt = O.compressed_delta(**{k: exs[e][k] for k in ("codes", "step", "salient", "salient_idx", "bits", "grid")})
        assert np.allclose(y[lo:hi], _naive_matmul_T(x[lo:hi], dt), rtol=1e-10, atol=1e-14)
    # full: x (W + Dtilde_e)^T
    y = O.delta_linear(x, w, exs, wl.seg_offsets)
    for e in range(3):
        lo, hi = wl.seg_offsets[e], wl.seg_offsets[e + 1]
        dt = O.compressed_delta(**{k: exs[e][k] for k in ("codes", "step", "salient", "salient_idx", "bits", "grid")})
        assert np.allclose(y[lo:hi], _naive_matmul_T(x[lo:hi], w + dt), rtol=1e-10, atol=1e-13)


def test_identical_experts_make_routing_irrelevant():
    wl = synth.small_case(64, 32, [0, 5, 9, 16], 4, 2, seed=2)
    exs = _compress(wl)
    same = [exs[1]] * 3
    x = wl.x.double().numpy()
    w = wl.w_base.double().numpy()
    a = O.delta_linear(x, w, same, [0, 5, 9, 16])
    b = O.delta_linear(x, w, same, [0, 16, 16, 16])
    c = O.delta_linear(x, w, same, [0, 0, 1, 16])
    assert np.array_equal(a, b) or np.allclose(a, b, rtol=1e-13, atol=0)
    assert np.allclose(a, c, rtol=1e-13, atol=0)


def test_routing_is_per_row_and_batches_split():
    """Permuting tokens together with their segments permutes rows of y; splitting a batch changes nothing."""
    wl = synth.small_case(96, 48, [0, 4, 10, 12], 6, 3, seed=3)
    exs = _compress(wl)
    x = wl.x.double().numpy()
    w = wl.w_base.double().numpy()
    y = O.delta_linear(x, w, exs, wl.seg_offsets)
    # swap experts 0 and 2 (rows and expert order)
    xp = np.concatenate([x[10:12], x[4:10], x[0:4]])
    yp = O.delta_linear(xp, w, [exs[2], exs[1], exs[0]], [0, 2, 8, 12])
    assert np.allclose(yp, np.concatenate([y[10:12], y[4:10], y[0:4]]), rtol=1e-12, atol=1e-15)
    # split into two calls
    y1 = O.delta_linear(x[:7], w, exs, [0, 4, 7, 7])
    y2 = O.delta_linear(x[7:], w, exs, [0, 0, 3, 5])
    assert np.allclose(np.concatenate([y1, y2]), y, rtol=1e-12, atol=1e-15)
    # each expert's rows really use that expert's delta (mis-routing would be off by >> tolerance)
    for e in range(3):
        lo, hi = wl.seg_offsets[e], wl.seg_offsets[e + 1]
        dt = O.compressed_delta(**{k: exs[e][k] for k in ("codes", "step", "salient", "salient_idx", "bits", "grid")})
        assert np.allclose(y[lo:hi], x[lo:hi] @ (w + dt).T, rtol=1e-10, atol=1e-13)
        other = O.compressed_delta(**{k: exs[(e + 1) % 3][k] for k in ("codes", "step", "salient", "salient_idx", "bits", "grid")})
        assert not np.allclose(y[lo:hi], x[lo:hi] @ (w + other).T, rtol=1e-3)


def test_output_error_bound_from_half_step():
    """|y - x (W + D)^T| <= sum_i |x_i| * s_j / 2 over non-salient i, plus the fp16 rounding of salient columns."""
    wl = synth.small_case(128, 40, [0, 6, 11], 8, 2, seed=4)
    exs = _compress(wl)
    x = wl.x.double().numpy()
    w = wl.w_base.double().numpy()
    y = O.delta_linear(x, w, exs, wl.seg_offsets)
    for e in range(2):
        lo, hi = wl.seg_offsets[e], wl.seg_offsets[e + 1]
        d = wl.experts[e].delta.double().numpy()
        exact = x[lo:hi] @ (w + d).T
        ns = O.non_salient_mask(128, exs[e]["salient_idx"])
        l1 = np.abs(x[lo:hi][:, ns]).sum(axis=1)
        sal_err = np.abs(x[lo:hi][:, ~ns]) @ np.abs(d[:, ~ns] - exs[e]["salient"].astype(np.float64)).T
        bound = l1[:, None] * exs[e]["step"].astype(np.float64)[None, :] / 2 * (1 + 1e-6) + sal_err + 1e-12
        assert np.all(np.abs(y[lo:hi] - exact) <= bound)
        assert np.abs(y[lo:hi] - exact).max() > 1e-4      # quantisation error is really there


# ---------------------------------------------------------------- Eq. 2: salient selection

def test_silu_closed_forms_and_the_gated_input():
    """SiLU against what the definition fixes: SiLU(0) = 0, SiLU(v) - SiLU(-v) = v, SiLU(ln 3) = 3/4 ln 3,
    SiLU(v) = v sigmoid(v) via tanh, its derivative at 0 is 1/2, v -> v for large v and -> 0 for large -v without
    overflow; and the gated input is the element-wise product of SiLU of one layer and the other layer, not the
    other way round (a swapped pair fails)."""
    v = np.linspace(-30, 30, 2001)
    assert O.silu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(O.silu(v) - O.silu(-v), v, rtol=0, atol=1e-13)
    np.testing.assert_allclose(O.silu(np.array([np.log(3.0)]))[0], 0.75 * np.log(3.0), rtol=1e-15)
    np.testing.assert_allclose(O.silu(v), v * 0.5 * (1.0 + np.tanh(0.5 * v)), rtol=1e-12, atol=1e-14)   # (1 + tanh cancels for very negative v)
    h = 1e-6
    np.testing.assert_allclose((O.silu(np.array([h]))[0] - O.silu(np.array([-h]))[0]) / (2 * h), 0.5, rtol=1e-9)
    big = O.silu(np.array([800.0, -800.0]))
    assert big[0] == 800.0 and big[1] == 0.0 and np.all(np.isfinite(big))
    # minimum of SiLU: at v with 1 + e^-v (1 + v) ... = 0, value about -0.27846
    assert abs(O.silu(v).min() + 0.2784645) < 1e-4
    rng = np.random.default_rng(5)
    d_in, d_out, T = 24, 6, 5
    x = rng.standard_normal((T, d_in))
    wg, wu = rng.standard_normal((d_out, d_in)), rng.standard_normal((d_out, d_in))
    def expert(seed):
        r = np.random.default_rng(seed)
        return dict(codes=r.integers(0, 4, (d_out, d_in)).astype(np.uint8), step=(0.01 + r.random(d_out)).astype(np.float32),
                    salient=np.zeros((d_out, 0), np.float16), salient_idx=np.zeros(0, np.int32), bits=2, grid=O.GRID_SYM)
    eg, eu = [expert(1), expert(2)], [expert(3), expert(4)]
    seg = [0, 2, 5]
    got = O.gated_mlp_input(x, wg, eg, wu, eu, seg)
    yg, yu = O.delta_linear(x, wg, eg, seg), O.delta_linear(x, wu, eu, seg)
    want = np.empty_like(yg)
    for t in range(T):
        for j in range(d_out):
            want[t, j] = yg[t, j] / (1.0 + np.exp(-yg[t, j])) * yu[t, j]
    np.testing.assert_allclose(got, want, rtol=1e-13)
    assert np.abs(got - O.gated_mlp_input(x, wu, eu, wg, eg, seg)).max() > 1e-3


def test_selection_matches_brute_force_on_tiny_layers():
    for seed, (d_out, d_in, n, k, bits, grid) in enumerate([(6, 10, 5, 3, 2, O.GRID_SYM), (8, 16, 7, 4, 3, O.GRID_EQ1),
                                                            (5, 12, 4, 2, 1, O.GRID_SYM)]):
        delta, _ = _delta(d_out, d_in, 50 + seed, k=2, scale=6.0)
        xc = synth.normal((n, d_in), 1.0, 700 + seed).numpy()
        idx, score = O.select_salient(delta, xc, bits, grid, k)
        # brute force, scalar python, straight from the formula
        codes, step, _ = O.quantize(delta, [], bits, grid)
        z = O.zero_point(bits, grid)
        brute = []
        for i in range(d_in):
            acc = 0.0
            for j in range(d_out):
                dh = (float(codes[j, i]) - z) * float(step[j])
                for t in range(n):
                    r = float(xc[t, i]) * float(delta[j, i]) - float(xc[t, i]) * dh
                    acc += r * r
            brute.append(acc)
        assert np.allclose(score, brute, rtol=1e-12)
        want = sorted(sorted(range(d_in), key=lambda i: (-brute[i], i))[:k])
        assert idx.tolist() == want
        assert idx.dtype == np.int32
        # factorised identity: score_i = (sum_t x_ti^2) * (sum_j (D_ji - Dhat_ji)^2)
        fact = (xc.astype(np.float64) ** 2).sum(0) * ((delta - O.dequantize(codes, step, bits, grid)) ** 2).sum(0)
        assert np.allclose(score, fact, rtol=1e-12)


def test_selection_ties_go_to_the_lower_index_and_activations_matter():
    score = np.array([1.0, 5.0, 5.0, 0.5, 5.0])
    assert O.top_k_ascending(score, 2).tolist() == [1, 2]
    assert O.top_k_ascending(score, 4).tolist() == [0, 1, 2, 4]
    # a channel with zero activation can never be selected ahead of one with error and activation
    delta, _ = _delta(8, 12, 99)
    xc = synth.normal((6, 12), 1.0, 5).numpy()
    xc[:, 4] = 0.0
    idx, score = O.select_salient(delta, xc, 2, O.GRID_SYM, 11)
    assert score[4] == 0.0 and 4 not in idx.tolist()


def test_eq1_grid_recovers_planted_outlier_channels():
    """With Eq. 1's grid (it has a zero level) the planted x15 channels carry the largest reconstruction error."""
    delta, sidx = _delta(64, 96, 123, k=4, scale=15.0)
    xc = synth.normal((128, 96), 1.0, 9).numpy()
    idx, _ = O.select_salient(delta, xc, 2, O.GRID_EQ1, 4)
    assert idx.tolist() == sidx.tolist()


# ---------------------------------------------------------------- Section 4.3: byte accounting vs the paper's printed sizes

def _golden():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split()
                out[k] = float(v)
    return out


MISTRAL = dict(hidden=4096, inter=14336, kv=1024, layers=32, vocab=32000)
LLAMA13 = dict(hidden=5120, inter=13824, kv=5120, layers=40, vocab=32000)


def _arch(a):
    h, f, kv = a["hidden"], a["inter"], a["kv"]
    lin = [(h, h), (h, kv), (h, kv), (h, h), (h, f), (h, f), (f, h)]
    other = 2 * a["vocab"] * h + a["layers"] * 2 * h + h
    return lin, other


def test_model_sizes_match_the_paper():
    g = _golden()
    gib = 2.0 ** 30
    lin, other = _arch(MISTRAL)
    assert sum(di * do for di, do in lin) * 32 == 6_979_321_856
    fp16 = O.model_bytes(lin, 32, other, None) / gib
    assert abs(fp16 - g["fp16_mistral7b_gb"]) <= 0.011
    fixed = O.model_bytes(lin, 32, other, 2, 0) / gib
    assert abs(fixed - g["fixed_2bit_gb"]) <= 0.011
    for k in (8, 16, 32, 64):
        mixed = O.model_bytes(lin, 32, other, 2, k) / gib
        assert abs(mixed - g[f"mixed_2bit_k{k}_gb"]) <= 0.011, (k, mixed)
    # dropping the 16-bit salient columns or counting them twice would move k = 64 by > 0.1
    assert abs(O.model_bytes(lin, 32, other, 2, 64) / gib - O.model_bytes(lin, 32, other, 2, 0) / gib - 0.1435) < 2e-3
    lin13, other13 = _arch(LLAMA13)
    assert abs(O.model_bytes(lin13, 40, other13, None) / gib - g["fp16_llama13b_gb"]) <= 0.02
    assert abs(O.model_bytes(lin13, 40, other13, 2, 8) / gib - g["mixed_llama13b_gb"]) <= 0.02


def test_compression_ratios_match_the_paper():
    g = _golden()
    r3 = O.compression_ratio(g["fp16_mistral7b_gb"], g["mixed_2bit_k8_gb"], g["router_gb"], 3)
    assert abs(r3 - g["ratio_mistral_m3"]) <= 0.006
    r9 = O.compression_ratio(g["fp16_llama13b_gb"], g["mixed_llama13b_gb"], g["router_gb"], 9)
    assert abs(r9 - g["ratio_llama13b_m9"]) <= 0.006
    assert abs(g["fp16_mistral7b_gb"] / g["mixed_2bit_k8_gb"] - g["per_model_compression"]) <= 0.006


def test_layout_bytes_versus_algorithmic_bytes():
    """The stored code matrix is full width (salient columns hold code 0), so it exceeds the algorithmic
    low-bit bytes by exactly the salient columns plus padding."""
    for d_in, d_out, k, bits in [(4096, 4096, 64, 2), (14336, 4096, 128, 3), (4096, 14336, 64, 1)]:
        stored = O.codes_bytes(d_in, d_out, bits)
        alg = d_out * (d_in - k) * bits // 8
        assert stored - alg == d_out * k * bits // 8       # these shapes need no padding
