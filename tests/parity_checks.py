"""Element-wise comparisons of the HIP path's bf16 output with the fp64 oracle (helpers of the GPU parity tests).

Two bars, both derived from the arithmetic of the path that produced the rows:

* streaming path (exact products of bf16 / fp16 / code operands, fp32 accumulation, ONE rounding of y to bf16):
  the fp32 accumulator differs from the fp64 sum by about 1e-6 of the output scale, so y_gpu can differ from
  bf16_rne(y_oracle) only where the exact value lies that close to a rounding boundary: within 1 bf16 ulp on at
  least 99.9 % of the elements, within 2 ulp on all of them.  The ulp is that of max(|y_oracle|, 2^-6 rms(y_oracle)):
  an element that cancels to nearly zero has an ulp far below the accumulation error and is held to the ulp of a
  small typical value instead.
* one-product path (long segments: the operand bf16(W + Delta~) is rounded once per weight).  Rounding a number
  m 2^e (1 <= m < 2) to 8 significant bits errs uniformly within half a spacing, 2^-8 / m relative; over a
  log-uniform m the mean square of that is (2^-8)^2 c^2 with c^2 = 0.541 / 3 (c = 0.4247).  The error of y_tj is
  therefore a sum of d_in independent terms with standard deviation sigma_tj = 2^-8 c sqrt(sum_i x_ti^2 w_ji^2).
  Every element must lie within 6 sigma_tj + 1 ulp.  The rounding of y itself adds another 2^-8 c |y_tj|, and
  y_tj^2 is sum_i x_ti^2 w_ji^2 on average, so the errors' root mean square is about sqrt(2) sigma; it must stay
  below 1.8 sigma (a systematic error of a few per cent of the delta term is many sigma).
"""
import numpy as np


def bf16_rne(a):
    """fp64 -> nearest bf16 value (8 significant bits, ties to even), returned as fp64."""
    a = np.asarray(a, dtype=np.float64)
    _, e = np.frexp(a)                       # a = m 2^e, 0.5 <= |m| < 1
    q = np.ldexp(1.0, e - 8)
    return np.rint(a / q) * q


def bf16_ulp(a):
    """Spacing of the bf16 grid at |a| (fp64)."""
    _, e = np.frexp(np.asarray(a, dtype=np.float64))
    return np.ldexp(1.0, e - 8)


def ulp_report(y_gpu, y_ref):
    """Distances of y_gpu (fp64 values of bf16 numbers) from bf16_rne(y_ref) in ulps (see the module text)."""
    y_ref = np.asarray(y_ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(y_ref * y_ref))) or 1.0
    ulp = bf16_ulp(np.maximum(np.abs(y_ref), rms / 64.0))
    d = np.abs(y_gpu - bf16_rne(y_ref)) / ulp
    return dict(max_ulps=float(d.max()) if d.size else 0.0,
                within_1ulp=float((d <= 1.0).mean()) if d.size else 1.0,
                exact=float((d == 0.0).mean()) if d.size else 1.0,
                max_abs=float(np.abs(y_gpu - y_ref).max()) if d.size else 0.0)


def assert_streaming_rows(y_gpu, y_ref, what=""):
    r = ulp_report(y_gpu, y_ref)
    assert r["within_1ulp"] >= 0.999 and r["max_ulps"] <= 2.0, (what, r)
    return r


def assert_one_product_rows(y_gpu, y_ref, x64, w_eff64, what=""):
    """x64 [T, d_in], w_eff64 [rows, d_in] = W + Delta~ of the rows' expert (fp64)."""
    sigma = 2.0 ** -8 * np.sqrt(0.541 / 3.0) * np.sqrt((x64 * x64) @ (w_eff64 * w_eff64).T)
    err = np.abs(y_gpu - y_ref)
    rms = float(np.sqrt(np.mean(y_ref * y_ref))) or 1.0
    bound = 6.0 * sigma + bf16_ulp(np.maximum(np.abs(y_ref), rms / 64.0))
    z = err / np.maximum(sigma, 1e-300)
    r = dict(worst=float((err / bound).max()), rms_in_sigma=float(np.sqrt(np.mean(z * z))), max_abs=float(err.max()))
    assert r["worst"] <= 1.0 and r["rms_in_sigma"] <= 1.8, (what, r)
    return r
