"""Pins for oracle/step_oracle.py (no GPU): the step-size objective and its straight-through gradient against
automatic differentiation (the estimator written with the detach trick), finite differences where the objective is
truly differentiable, a closed form, and torch's AdamW."""
import numpy as np
import pytest
import torch

from oracle import mes_oracle as O
from oracle import step_oracle as S


def bf16_values(a):
    return torch.tensor(a, dtype=torch.float32).bfloat16().double().numpy()


def make_case(seed, d_out=12, d_in=40, n_tok=9, k=3, scale=0.02):
    rng = np.random.default_rng(seed)
    delta = (rng.standard_normal((d_out, d_in)) * scale).astype(np.float32)
    x = bf16_values(rng.standard_normal((n_tok, d_in)))
    sidx = np.sort(rng.choice(d_in, size=k, replace=False)) if k else np.zeros(0, dtype=np.int64)
    return delta, x, sidx


def autograd_loss_grad(delta32, x, sidx, bits, grid, step):
    """The same objective through torch autograd: Eq. 1 with the rounding replaced, for differentiation only, by the
    identity (value kept through a detached correction), clamping kept as it is."""
    d = torch.tensor(delta32.astype(np.float64))
    s = torch.tensor(np.asarray(step, dtype=np.float32).astype(np.float64), requires_grad=True)
    xt = torch.tensor(x)
    half = 2 ** (bits - 1)
    v = d / s[:, None]
    if grid == O.GRID_SYM:
        lo, hi = -float(half), float(half)                    # cells [m, m+1), levels m + 1/2, m in [-half, half-1]
        inside = (v >= lo) & (v < hi)
        level_in = v + (torch.floor(v) + 0.5 - v).detach()
        level_out = torch.where(v < lo, torch.full_like(v, lo + 0.5), torch.full_like(v, hi - 0.5))
    else:
        rounded = torch.round(v)                              # half to even, as numpy's rint
        inside = (rounded >= -half) & (rounded <= half - 1)
        level_in = v + (rounded - v).detach()
        level_out = torch.where(rounded < -half, torch.full_like(v, -float(half)), torch.full_like(v, half - 1.0))
    if bits == 1:
        level = torch.where(d >= 0, torch.full_like(v, 0.5), torch.full_like(v, -0.5))
    else:
        level = torch.where(inside, level_in, level_out)
    dhat = level * s[:, None]
    ns = torch.tensor(O.non_salient_mask(delta32.shape[1], sidx))
    sal16 = torch.tensor(delta32.astype(np.float16).astype(np.float64))
    dtilde = torch.where(ns[None, :], dhat, sal16)
    r = xt @ (dtilde - d).T
    loss = 0.5 * (r * r).sum(dim=0)
    loss.sum().backward()
    return loss.detach().numpy(), s.grad.numpy()


@pytest.mark.parametrize("bits,grid", [(1, 0), (2, 0), (3, 0), (4, 0), (2, 1), (3, 1), (4, 1)])
@pytest.mark.parametrize("shrink", [1.0, 0.6, 0.25])
def test_gradient_matches_autograd_of_the_straight_through_objective(bits, grid, shrink):
    """shrink < 1 makes the step smaller than the max-abs one, so a good share of the weights is clamped."""
    delta, x, sidx = make_case(10 * bits + grid)
    ns = O.non_salient_mask(delta.shape[1], sidx)
    step = (O.init_step(delta, ns, bits, grid, O.STEP_MAXABS).astype(np.float64) * shrink).astype(np.float32)
    loss, grad = S.step_loss_grad(delta, x, sidx, bits, grid, step)
    loss_ad, grad_ad = autograd_loss_grad(delta, x, sidx, bits, grid, step)
    np.testing.assert_allclose(loss, loss_ad, rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(grad, grad_ad, rtol=1e-10, atol=1e-18)
    if shrink < 1.0 and bits > 1:
        v = delta / step[:, None]
        half = 2 ** (bits - 1)
        assert (v[:, ns] > (half if grid == O.GRID_SYM else half - 0.5)).any(), "the case was meant to clamp something"


@pytest.mark.parametrize("bits,grid", [(2, 0), (3, 0), (4, 0), (2, 1), (4, 1)])
def test_without_clamping_and_salient_columns_the_gradient_is_twice_the_loss_over_the_step(bits, grid):
    """Inside the grid Dhat - Delta = s * slope, hence r = s p and g = sum r p = 2 L / s."""
    delta, x, sidx = make_case(77 + bits, k=0)
    ns = O.non_salient_mask(delta.shape[1], sidx)
    step = O.init_step(delta, ns, bits, grid, O.STEP_MAXABS)
    if grid == O.GRID_SYM:
        step = np.nextafter(step, np.float32(np.inf))          # the row maximum itself sits on the clamp boundary
    loss, grad = S.step_loss_grad(delta, x, sidx, bits, grid, step)
    np.testing.assert_allclose(grad, 2.0 * loss / step.astype(np.float64), rtol=1e-10)
    assert (grad > 0).all()


@pytest.mark.parametrize("bits,grid", [(1, 0), (2, 0), (3, 1)])
def test_where_every_weight_is_clamped_the_gradient_is_the_true_derivative(bits, grid):
    """With a tiny step every weight is clamped to an end level (for b = 1 the code never depends on s): the
    objective is then a smooth function of s and central differences must agree."""
    delta, x, sidx = make_case(5 + bits, k=2)
    delta[np.abs(delta) < 1e-3] = 1e-3                         # keep every |Delta / s| far beyond the grid
    step = np.full(delta.shape[0], 1e-5 if bits > 1 else 0.03, dtype=np.float32)
    _, grad = S.step_loss_grad(delta, x, sidx, bits, grid, step)
    h = np.float32(2.0 ** -26) if bits > 1 else np.float32(2.0 ** -12)
    up, _ = S.step_loss_grad(delta, x, sidx, bits, grid, step + h)
    dn, _ = S.step_loss_grad(delta, x, sidx, bits, grid, step - h)
    dh = (step + h).astype(np.float64) - (step - h).astype(np.float64)
    np.testing.assert_allclose(grad, (up - dn) / dh, rtol=1e-6)


def test_slope_values_by_hand():
    """b = 2, symmetric grid, s = 1: cells [m, m+1) with levels m + 1/2, m in [-2, 1]."""
    delta = np.array([[0.25, -0.25, 1.75, 2.5, -2.5, -2.0, 0.0]], dtype=np.float32)
    slope = S.ste_slope(delta, np.array([1.0], dtype=np.float32), [], 2, O.GRID_SYM)
    np.testing.assert_allclose(slope[0], [0.25, -0.25, -0.25, 1.5, -1.5, 0.5, 0.5])
    # Eq. 1's grid, s = 1: integer levels -2..1, half to even
    slope = S.ste_slope(delta, np.array([1.0], dtype=np.float32), [], 2, O.GRID_EQ1)
    np.testing.assert_allclose(slope[0], [-0.25, 0.25, 1.0, 1.0, 0.5, 0.0, 0.0])
    # a salient column and a dead row contribute nothing
    slope = S.ste_slope(np.tile(delta, (2, 1)), np.array([1.0, 0.0], dtype=np.float32), [2], 2, O.GRID_SYM)
    assert slope[0, 2] == 0.0 and not slope[1].any()


def test_rows_with_a_nonpositive_step_report_zero():
    delta, x, sidx = make_case(3)
    step = np.full(delta.shape[0], 0.01, dtype=np.float32)
    step[[1, 4]] = [0.0, -1.0]
    loss, grad = S.step_loss_grad(delta, x, sidx, 2, O.GRID_SYM, step)
    assert loss[1] == 0 and grad[1] == 0 and loss[4] == 0 and grad[4] == 0
    assert (loss[[0, 2, 3]] > 0).all()


def test_loss_counts_the_fp16_rounding_of_salient_columns():
    """One row, every column salient: the residual is x times the fp16 rounding error, nothing else."""
    delta = np.array([[0.1, 0.2, 0.3]], dtype=np.float32)
    x = np.array([[1.0, 2.0, 4.0]])
    loss, grad = S.step_loss_grad(delta, x, [0, 1, 2], 2, O.GRID_SYM, np.array([0.1], dtype=np.float32))
    err = delta.astype(np.float16).astype(np.float64) - delta.astype(np.float64)
    assert loss[0] == pytest.approx(0.5 * float(x[0] @ err[0]) ** 2, rel=1e-12)
    assert grad[0] == 0.0


def test_adamw_against_torch():
    rng = np.random.default_rng(0)
    n = 17
    s0 = rng.uniform(0.01, 0.05, n)
    p = torch.tensor(s0.copy(), dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.01)
    s, m, v = s0.copy(), np.zeros(n), np.zeros(n)
    for t in range(1, 6):
        g = rng.standard_normal(n) * 0.1
        p.grad = torch.tensor(g.copy())
        opt.step()
        s, m, v = S.adamw_update(s, g, m, v, t, 3e-3, 0.9, 0.95, 1e-8, 0.01)
        np.testing.assert_allclose(s, p.detach().numpy(), rtol=1e-12)
