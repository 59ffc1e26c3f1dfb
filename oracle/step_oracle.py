"""CPU oracle for learning the quantisation step sizes (TEST INFRASTRUCTURE ONLY: never imported by the product).

What it defines, in fp64 numpy, in the paper's order:

  * the objective of the "Efficient distillation" paragraph of Section 4.1 taken layer-wise: the delta weights are
    frozen, only the per-output-channel step s of Eq. 1 is learned, and the quantised layer is pulled towards the
    full-precision fine-tuned layer on calibration activations X.  The base product x W^T is common to teacher and
    student and cancels, so per output channel j

        r_tj = sum_i x_ti (Dtilde_ji(s_j) - Delta_ji)          Dtilde as in Eq. 4: low-bit columns + fp16 salient
        L_j  = 1/2 sum_t r_tj^2

  * its gradient with the straight-through estimator that Section 3 prescribes for Eq. 1 (the learned-step-size
    rule: the rounding is treated as the identity when differentiating):

        dDhat_ji/ds_j = (u_ji - z) - [Delta_ji / s_j falls inside the grid] * Delta_ji / s_j
        g_j = sum_t r_tj sum_{i not salient} x_ti dDhat_ji/ds_j

    For b = 1 (sign times scale) the code does not depend on s at all, so the slope is u - z everywhere.
    Rows whose step is not positive are not learnable: loss and gradient are reported as 0.

  * one AdamW update of the step vector (decoupled weight decay), the optimiser Section 5 names.

Pinned in tests/test_step_oracle.py against automatic differentiation of the same objective written with the
detach trick, finite differences where the objective is truly differentiable, and a closed form.
"""
from __future__ import annotations

import numpy as np

from . import mes_oracle as O


def ste_slope(delta32: np.ndarray, step: np.ndarray, salient_idx, bits: int, grid: int) -> np.ndarray:
    """d Dhat_ji / d s_j under the straight-through estimator (Section 3), fp64 [d_out, d_in]; 0 at salient
    columns (they are kept in fp16 and do not depend on s) and in rows with a non-positive step."""
    d_out, d_in = delta32.shape
    half = 2 ** (bits - 1)
    z = O.zero_point(bits, grid)
    s = np.asarray(step, dtype=np.float32).astype(np.float64)
    live = s > 0
    v = np.zeros(delta32.shape, dtype=np.float64)
    np.divide(delta32.astype(np.float64), s[:, None], out=v, where=live[:, None])
    if grid == O.GRID_SYM:
        cell = np.floor(v) + half                   # unclamped code
    else:
        cell = np.rint(v) + half
    u = np.clip(cell, 0, 2 * half - 1)
    inside = (cell == u) if bits > 1 else np.zeros_like(v, dtype=bool)
    slope = (u - z) - np.where(inside, v, 0.0)
    slope[~live, :] = 0.0
    slope[:, ~O.non_salient_mask(d_in, salient_idx)] = 0.0
    return slope


def step_loss_grad(delta32: np.ndarray, x: np.ndarray, salient_idx, bits: int, grid: int, step: np.ndarray):
    """Per-output-channel loss L_j and gradient g_j (fp64 [d_out] each) for calibration activations x [N, d_in]."""
    x64 = np.asarray(x, dtype=np.float64)
    s32 = np.asarray(step, dtype=np.float32)
    codes, s_used, salient = O.quantize(delta32, salient_idx, bits, grid, O.STEP_GIVEN, s32)
    dtilde = O.compressed_delta(codes, s_used, salient, salient_idx, bits, grid)
    r = x64 @ (dtilde - delta32.astype(np.float64)).T                    # [N, d_out]
    slope = ste_slope(delta32, s_used, salient_idx, bits, grid)
    p = x64 @ slope.T                                                    # [N, d_out]
    live = s_used.astype(np.float64) > 0
    loss = np.where(live, 0.5 * np.sum(r * r, axis=0), 0.0)
    grad = np.where(live, np.sum(r * p, axis=0), 0.0)
    return loss, grad


def adamw_update(step, grad, m, v, t: int, lr: float, beta1: float, beta2: float, eps: float, weight_decay: float):
    """One AdamW update (decoupled weight decay) of the step vector; t is the 1-based update count.
    Returns (step, m, v) in fp64."""
    s = np.asarray(step, dtype=np.float64)
    g = np.asarray(grad, dtype=np.float64)
    m = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** t)
    v_hat = v / (1.0 - beta2 ** t)
    s = s * (1.0 - lr * weight_decay) - lr * m_hat / (np.sqrt(v_hat) + eps)
    return s, m, v
