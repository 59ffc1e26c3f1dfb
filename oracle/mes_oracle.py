"""CPU fp64 oracle for the mixed-precision delta linear layer (ME-Switch serving path).

THIS IS TEST INFRASTRUCTURE.  Only tests, the smoke check and the benchmark's
`cpu_baseline` leg may import it; the product path (the HIP library and its
Python binding) never does, and shares no code with it.

Everything here is the plain definition, in fp64 numpy, in the paper's order:

* Eq. 1 (Preliminaries): uniform quantiser  clamp(round(X / s), -Q_N, Q_P) * s  with
  Q_N = 2^(b-1), Q_P = 2^(b-1) - 1 and s initialised to max|X| / (2^(b-1) - 1); one
  step size per output channel (Section 4.1).  Binary case: sign * scale, XNOR-Net style.
* Section 4.1, "Salient-aware delta selection" (Eq. 2): per input channel i the score
  sum_j || x_i D_ij - x_i Dhat_ij ||^2 ; the k channels with the largest score stay in
  16-bit, every other input channel is quantised to b bits.
* Eq. 4: y = x W_FT ~= x W + x Dtilde, with Dtilde the compressed delta (low-bit
  non-salient channels plus fp16 salient channels).
* Section 4.3, "Model size reduction analysis": total size Psi + M * Psi_tilde + Phi.

Orientation: matrices are stored nn.Linear-style, W[d_out, d_in], y = x W^T; the paper
writes W[m, n] with m input channels.  "Output-channel step" is therefore one step per
ROW, "salient input channel" one COLUMN.

Readings of points the paper leaves open (each is listed again in the design notes):
* grid: SYM (levels (u - (2^b - 1)/2) * s, the benchmark configs' "2-bit symmetric,
  step = rowmax / 1.5") or EQ1 (levels (u - 2^(b-1)) * s, Eq. 1 literally).  Both are
  (u - z) * s with an unsigned code u; only z differs.
* rounding ties: EQ1 uses round-half-to-even; SYM takes floor(t) as the cell index.
* the row maximum that initialises the step runs over NON-salient columns only.
* the 2-norm in Eq. 2 runs over calibration tokens.
* salient columns are stored as fp16 (round-to-nearest-even of the fp32 delta) and are
  NOT part of the low-bit matrix.

Parity pins live in tests/test_oracle_pins.py.  Parity unpinned: the paper prints no
numeric code, index or output value for any worked example, so the pack byte layouts,
the 3-bit plane split and the tie rules are pinned only by round-trip identities,
bounds, closed forms, brute force on tiny inputs and textbook special cases.
"""
from __future__ import annotations

import numpy as np

GRID_SYM = 0
GRID_EQ1 = 1
STEP_GIVEN = 0
STEP_MAXABS = 1
STEP_MEANABS = 2

SALIENT_MARK = 0xFF  # value stored in a logical code matrix at salient columns


# ------------------------------------------------------------------------------------------------
# Eq. 1: the quantisation grid
# ------------------------------------------------------------------------------------------------

def zero_point(bits: int, grid: int) -> float:
    """z in  w_hat = (u - z) * s  for an unsigned code u in [0, 2^b)."""
    if grid == GRID_SYM:
        return 2.0 ** (bits - 1) - 0.5
    if grid == GRID_EQ1:
        return 2.0 ** (bits - 1)
    raise ValueError("grid")


def init_divisor(bits: int, grid: int) -> float:
    """D in  s_init = max|X| / D.  Eq. 1 gives 2^(b-1) - 1; the symmetric grid's top level is 2^(b-1) - 1/2."""
    if grid == GRID_SYM:
        return 2.0 ** (bits - 1) - 0.5
    if grid == GRID_EQ1:
        if bits < 2:
            raise ValueError("Eq. 1 is undefined for b = 1 (divides by 2^0 - 1 = 0)")
        return 2.0 ** (bits - 1) - 1.0
    raise ValueError("grid")


def non_salient_mask(d_in: int, salient_idx) -> np.ndarray:
    m = np.ones(d_in, dtype=bool)
    m[np.asarray(salient_idx, dtype=np.int64)] = False
    return m


def init_step(delta32: np.ndarray, ns_mask: np.ndarray, bits: int, grid: int, policy: int) -> np.ndarray:
    """Per-output-channel step from the delta itself (Eq. 1's initialisation), fp32 [d_out]."""
    a = np.abs(delta32[:, ns_mask]).astype(np.float64)
    if a.shape[1] == 0:
        return np.zeros(delta32.shape[0], dtype=np.float32)
    if policy == STEP_MAXABS:
        return (a.max(axis=1) / init_divisor(bits, grid)).astype(np.float32)
    if policy == STEP_MEANABS:
        if bits != 1:
            raise ValueError("MEANABS is the binary (XNOR-style) scale; bits must be 1")
        # alpha = mean|w| ; in (u - z) * s form with z = 1/2 the step is 2 * alpha.
        # Sequential (ascending column) fp64 accumulation, so the order is defined.
        tot = np.add.accumulate(a, axis=1)[:, -1]
        return (2.0 * (tot / a.shape[1])).astype(np.float32)
    raise ValueError("policy")


def quantize(delta32: np.ndarray, salient_idx, bits: int, grid: int = GRID_SYM,
             policy: int = STEP_MAXABS, step_in: np.ndarray | None = None):
    """Mixed-precision compression of one delta matrix.

    delta32 [d_out, d_in] fp32; salient_idx ascending column indices.
    Returns (codes, step, salient):
      codes   uint8 [d_out, d_in]: unsigned code u at non-salient columns, 0xFF at salient columns
      step    fp32  [d_out]
      salient fp16  [d_out, k]:    delta[:, salient_idx] rounded to fp16 (RNE)
    """
    assert delta32.dtype == np.float32 and delta32.ndim == 2
    if bits not in (1, 2, 3, 4):
        raise ValueError("bits")
    if grid == GRID_EQ1 and bits == 1:
        raise ValueError("Eq. 1 is undefined for b = 1")
    d_out, d_in = delta32.shape
    sidx = np.asarray(salient_idx, dtype=np.int64)
    ns = non_salient_mask(d_in, sidx)
    if policy == STEP_GIVEN:
        step = np.asarray(step_in, dtype=np.float32).copy()
        step[~(step > 0)] = 0.0
    else:
        step = init_step(delta32, ns, bits, grid, policy)
    half = 2 ** (bits - 1)
    s64 = step.astype(np.float64)
    live = s64 > 0
    t = np.zeros(delta32.shape, dtype=np.float64)
    np.divide(delta32.astype(np.float64), s64[:, None], out=t, where=live[:, None])
    if grid == GRID_SYM:
        u = np.clip(np.floor(t) + half, 0, 2 * half - 1)
    else:
        u = np.clip(np.rint(t), -half, half - 1) + half
    u[~live, :] = half               # zero step: the row dequantises to exactly 0 whatever the code
    codes = u.astype(np.uint8)
    codes[:, ~ns] = SALIENT_MARK
    salient = delta32[:, sidx].astype(np.float16)
    return codes, step, salient


def dequantize(codes: np.ndarray, step: np.ndarray, bits: int, grid: int) -> np.ndarray:
    """(u - z) * s in fp64 at non-salient columns, 0 at salient columns."""
    z = zero_point(bits, grid)
    w = (codes.astype(np.float64) - z) * step.astype(np.float64)[:, None]
    w[codes == SALIENT_MARK] = 0.0
    return w


def compressed_delta(codes, step, salient, salient_idx, bits, grid) -> np.ndarray:
    """The matrix Dtilde of Eq. 4 in fp64: dequantised low-bit columns plus fp16 salient columns."""
    w = dequantize(codes, step, bits, grid)
    sidx = np.asarray(salient_idx, dtype=np.int64)
    if sidx.size:
        w[:, sidx] = salient.astype(np.float64)
    return w


# ------------------------------------------------------------------------------------------------
# Eq. 4: the delta linear layer
# ------------------------------------------------------------------------------------------------

def delta_linear(x64: np.ndarray, w_base64: np.ndarray, experts, seg_offsets) -> np.ndarray:
    """y[t] = x[t] W^T + x_ns[t] dequant(Q_e)^T + x_s[t] D_e^T  with e the expert of row t.

    x64 [T, d_in], w_base64 [d_out, d_in]: storage values promoted exactly to fp64.
    experts: sequence of dicts with keys codes, step, salient, salient_idx, bits, grid.
    seg_offsets: rows seg_offsets[e] .. seg_offsets[e+1] belong to expert e.
    """
    T, d_in = x64.shape
    y = x64 @ w_base64.T
    for e, ex in enumerate(experts):
        lo, hi = int(seg_offsets[e]), int(seg_offsets[e + 1])
        if hi <= lo:
            continue
        xs = x64[lo:hi]
        sidx = np.asarray(ex["salient_idx"], dtype=np.int64)
        ns = non_salient_mask(d_in, sidx)
        z = zero_point(ex["bits"], ex["grid"])
        q = ex["codes"][:, ns].astype(np.float64) - z                  # integer / half-integer levels
        y[lo:hi] += (xs[:, ns] @ q.T) * ex["step"].astype(np.float64)[None, :]
        if sidx.size:
            y[lo:hi] += xs[:, sidx] @ ex["salient"].astype(np.float64).T
    return y


# ------------------------------------------------------------------------------------------------
# The gated MLP input of the evaluated models (Section 5: Mistral-7B, LLaMA-2-13B)
# ------------------------------------------------------------------------------------------------

def silu(v: np.ndarray) -> np.ndarray:
    """SiLU(v) = v / (1 + exp(-v)), fp64, written so that large negative v does not overflow."""
    v = np.asarray(v, dtype=np.float64)
    e = np.exp(-np.abs(v))
    return np.where(v >= 0, v / (1.0 + e), v * e / (1.0 + e))


def gated_mlp_input(x64, w_gate64, gate_experts, w_up64, up_experts, seg_offsets) -> np.ndarray:
    """h = SiLU(y_gate) * y_up with y_gate, y_up two Eq. 4 layers over the same rows and routing -- what the down
    projection of a gated MLP block reads.  Nothing is rounded on the way (fp64 throughout)."""
    return silu(delta_linear(x64, w_gate64, gate_experts, seg_offsets)) * delta_linear(x64, w_up64, up_experts, seg_offsets)


# ------------------------------------------------------------------------------------------------
# Eq. 2: salient input-channel selection
# ------------------------------------------------------------------------------------------------

def salient_scores(delta32: np.ndarray, x_calib32: np.ndarray, bits: int, grid: int = GRID_SYM,
                   policy: int = STEP_MAXABS) -> np.ndarray:
    """score_i = sum_t sum_j (x_ti D_ji - x_ti Dhat_ji)^2, Dhat = b-bit quantisation of the whole delta."""
    d_out, d_in = delta32.shape
    codes, step, _ = quantize(delta32, [], bits, grid, policy)
    d = delta32.astype(np.float64)
    dh = dequantize(codes, step, bits, grid)
    x = x_calib32.astype(np.float64)
    score = np.empty(d_in, dtype=np.float64)
    for i in range(d_in):
        a = np.multiply.outer(x[:, i], d[:, i])        # x_ti * D_ji   [n, d_out]
        b = np.multiply.outer(x[:, i], dh[:, i])       # x_ti * Dhat_ji
        r = a - b
        score[i] = np.sum(r * r)
    return score


def top_k_ascending(score: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest scores (ties: lower index wins), returned ascending, int32."""
    order = sorted(range(score.shape[0]), key=lambda i: (-score[i], i))
    return np.array(sorted(order[:k]), dtype=np.int32)


def select_salient(delta32, x_calib32, bits, grid, k, policy: int = STEP_MAXABS):
    score = salient_scores(delta32, x_calib32, bits, grid, policy)
    return top_k_ascending(score, k), score


# ------------------------------------------------------------------------------------------------
# Storage layouts of the library (its own definition; written here from the layout specification,
# not from the kernels).  A "lane slot" is lane = 16 * g + r: r = row inside a 16-row tile,
# g = one of four column groups.
# ------------------------------------------------------------------------------------------------

ROW_PAD = 64
COL_PAD = 128
SAL_PAD = 32


def _ceil_to(n: int, m: int) -> int:
    return (n + m - 1) // m * m


def padded_dims(d_out: int, d_in: int, k: int = 0):
    return _ceil_to(d_out, ROW_PAD), _ceil_to(d_in, COL_PAD), _ceil_to(k, SAL_PAD)


def _tile_16x32(a: np.ndarray) -> np.ndarray:
    """[R, C] (R % 16 == 0, C % 32 == 0) -> [R/16, C/32, 64 lanes, 8]; lane = 16 g + r holds a[16 jt + r, 32 kb + 8 g + 0..7]."""
    R, C = a.shape
    v = a.reshape(R // 16, 16, C // 32, 4, 8)          # jt, r, kb, g, e
    return np.ascontiguousarray(v.transpose(0, 2, 3, 1, 4)).reshape(R // 16, C // 32, 64, 8)


def _untile_16x32(t: np.ndarray) -> np.ndarray:
    njt, nkb = t.shape[0], t.shape[1]
    v = t.reshape(njt, nkb, 4, 16, 8).transpose(0, 3, 1, 2, 4)
    return np.ascontiguousarray(v).reshape(njt * 16, nkb * 32)


def pack_base(w_bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns [d_out, d_in] uint16 -> tiled uint16 [d_in_pad/128, d_out_pad/16, 4, 64, 8], zero padded.

    Chunk-major: all row tiles of one 128-column chunk are contiguous; slot (c, jt, kb, lane, e) with
    lane = 16 g + r holds W[16 jt + r, 128 c + 32 kb + 8 g + e]."""
    d_out, d_in = w_bits.shape
    po, pi, _ = padded_dims(d_out, d_in)
    a = np.zeros((po, pi), dtype=np.uint16)
    a[:d_out, :d_in] = w_bits
    t = _tile_16x32(a)                                   # jt, kb_all, lane, e
    t = t.reshape(po // 16, pi // 128, 4, 64, 8)         # jt, c, kb, lane, e
    return np.ascontiguousarray(t.transpose(1, 0, 2, 3, 4))


def unpack_base(t: np.ndarray, d_out: int, d_in: int) -> np.ndarray:
    nc, njt = t.shape[0], t.shape[1]
    u = np.ascontiguousarray(t.transpose(1, 0, 2, 3, 4)).reshape(njt, nc * 4, 64, 8)
    return _untile_16x32(u)[:d_out, :d_in]


def pack_salient(salient16: np.ndarray) -> np.ndarray:
    """fp16 [d_out, k] -> tiled uint16 (fp16 bits) [d_out_pad/16, k_pad/32, 64, 8], zero padded."""
    d_out, k = salient16.shape
    po, _, pk = padded_dims(d_out, 1, k)
    a = np.zeros((po, pk), dtype=np.uint16)
    a[:d_out, :k] = salient16.view(np.uint16)
    return _tile_16x32(a)


def unpack_salient(t: np.ndarray, d_out: int, k: int) -> np.ndarray:
    return _untile_16x32(t)[:d_out, :k].copy().view(np.float16)


def _nibble_words(field: np.ndarray, width: int) -> np.ndarray:
    """field uint32 [..., 4 q, 8 p] -> words [..., 4 // (4 // width)]: `width`-bit fields, 4 // width of them
    stacked inside each 4-bit field p (element q % (4 // width) at bit offset width * that), word q // (4 // width)."""
    per = 4 // width                       # elements q sharing one word
    lead = field.shape[:-2]
    words = np.zeros(lead + (4 // per,), dtype=np.uint32)
    for q in range(4):
        for p in range(8):
            words[..., q // per] |= field[..., q, p] << np.uint32(4 * p + width * (q % per))
    return words


def _unnibble_words(words: np.ndarray, width: int) -> np.ndarray:
    per = 4 // width
    lead = words.shape[:-1]
    field = np.zeros(lead + (4, 8), dtype=np.uint32)
    for q in range(4):
        for p in range(8):
            field[..., q, p] = (words[..., q // per] >> np.uint32(4 * p + width * (q % per))) & np.uint32((1 << width) - 1)
    return field


def pack_codes(codes: np.ndarray, bits: int) -> np.ndarray:
    """Logical codes uint8 [d_out, d_in] (0xFF = salient) -> uint32 [d_in_pad/128, d_out_pad/16, 64 * bits].

    Blocks of 16 rows x 128 columns, chunk-major (all row tiles of one 128-column chunk are contiguous).
    Lane 16 g + r owns row 16 jt + r and the 32 columns 128 c + 32 g + 8 q + p.  b = 1: one word per lane,
    code at bit 4 p + q.  b = 2: words [lane][w], code of (q, p) in word q // 2 at bits 4 p + 2 (q % 2).
    b = 3: the b = 2 block of the low two bits, then the b = 1 block of the high bit.  b = 4: the b = 2 block of
    the low two bits, then the b = 2 block of the high two bits.  Salient columns, padding columns and padding
    rows store code 0.
    """
    d_out, d_in = codes.shape
    po, pi, _ = padded_dims(d_out, d_in)
    u = np.zeros((po, pi), dtype=np.uint32)
    c = codes.astype(np.uint32)
    c[codes == SALIENT_MARK] = 0
    u[:d_out, :d_in] = c
    v = u.reshape(po // 16, 16, pi // 128, 4, 4, 8)              # jt, r, c, g, q, p
    v = v.transpose(2, 0, 3, 1, 4, 5)                            # c, jt, g, r, q, p
    v = v.reshape(pi // 128, po // 16, 64, 4, 8)                 # c, jt, lane, q, p
    if bits == 1:
        return _nibble_words(v, 1).reshape(pi // 128, po // 16, 64)
    low = _nibble_words(v & np.uint32(3), 2).reshape(pi // 128, po // 16, 128)
    if bits == 2:
        return low
    if bits == 3:
        high = _nibble_words(v >> np.uint32(2), 1).reshape(pi // 128, po // 16, 64)
    else:
        high = _nibble_words(v >> np.uint32(2), 2).reshape(pi // 128, po // 16, 128)
    return np.concatenate([low, high], axis=2)


def unpack_codes(packed: np.ndarray, bits: int, d_out: int, d_in: int) -> np.ndarray:
    """Inverse of pack_codes (salient columns come back as code 0)."""
    nc, njt = packed.shape[0], packed.shape[1]
    if bits == 1:
        v = _unnibble_words(packed.reshape(nc, njt, 64, 1), 1)
    else:
        v = _unnibble_words(packed[:, :, :128].reshape(nc, njt, 64, 2), 2)
        if bits == 3:
            v = v | (_unnibble_words(packed[:, :, 128:].reshape(nc, njt, 64, 1), 1) << np.uint32(2))
        if bits == 4:
            v = v | (_unnibble_words(packed[:, :, 128:].reshape(nc, njt, 64, 2), 2) << np.uint32(2))
    v = v.reshape(nc, njt, 4, 16, 4, 8).transpose(1, 3, 0, 2, 4, 5)   # jt, r, c, g, q, p
    return np.ascontiguousarray(v).reshape(njt * 16, nc * 128)[:d_out, :d_in].astype(np.uint8)


def codes_bytes(d_in: int, d_out: int, bits: int) -> int:
    po, pi, _ = padded_dims(d_out, d_in)
    return po * pi * bits // 8


# ------------------------------------------------------------------------------------------------
# Section 4.3: byte accounting
# ------------------------------------------------------------------------------------------------

def compressed_linear_bits(d_in: int, d_out: int, bits: int, k: int, step_bits: int = 16) -> int:
    """Bits one compressed delta matrix needs: low-bit non-salient columns, 16-bit salient columns, one step per row."""
    return d_out * (d_in - k) * bits + d_out * k * 16 + d_out * step_bits


def model_bytes(linears, n_layers: int, other_fp16_params: int, bits: int | None, k: int = 0,
                step_bits: int = 16) -> float:
    """Size of a transformer whose `linears` [(d_in, d_out), ...] repeat `n_layers` times.

    bits=None: everything fp16.  Otherwise the linears are compressed deltas and the
    remaining parameters (embeddings, head, norms) stay fp16.
    """
    tot_bits = other_fp16_params * 16
    for d_in, d_out in linears:
        if bits is None:
            tot_bits += n_layers * d_in * d_out * 16
        else:
            tot_bits += n_layers * compressed_linear_bits(d_in, d_out, bits, k, step_bits)
    return tot_bits / 8.0


def compression_ratio(psi: float, psi_tilde: float, phi: float, m: int) -> float:
    """M Psi / (Psi + M Psi_tilde + Phi)."""
    return m * psi / (psi + m * psi_tilde + phi)
