"""GPU parity for learning the step sizes (mes_step_grad, mes_step_adamw) through the C-ABI against the fp64 oracle.

Tolerances.  The kernel rounds its two operand matrices (slope D, clamped part C; both O(1)) to bf16 -- relative
error at most 2^-9 per element, about 1.1e-3 rms -- and accumulates in fp32; activations and deltas enter exactly.
The rounding errors are independent across input channels, so r_tj and p_tj each carry an error of about 1.1e-3 of
rho = sqrt(sum_i x_ti^2 e_ji^2), the size of the terms they are summed from (not of the sums themselves, which may
cancel).  Hence the bars: over all rows, relative 2-norm error <= 5e-3; per row, |loss_j - ref| <= 1e-2 sum_t |r| rho_r
and |grad_j - ref| <= 1e-2 sum_t (|r| rho_p + |p| rho_r), the first-order error bounds at about 2^-9 with a margin.
"""
import numpy as np
import pytest
import torch

from inputs import synth
from oracle import mes_oracle as O
from oracle import step_oracle as S

pytestmark = pytest.mark.gpu

try:
    import paper_2406_09041_amd as mes
except ImportError as e:                                  # the product must not silently fall back
    raise RuntimeError("libmes.so is missing: build it (python -c 'import __graft_entry__ as g; g.build()')") from e

DEV = "cuda:0"
TOL_NORM = 5e-3
TOL_ROW = 1e-2


def case(d_in, d_out, n_tok, k, bits, grid, shrink, seed, dead_rows=()):
    ex = synth.make_delta(d_in, d_out, k, 0.003, 15.0, synth.seed_for(950, 0, seed, 2))
    x = synth.normal((n_tok, d_in), 1.0, synth.seed_for(950, 0, seed, 3), "cpu", torch.bfloat16)
    delta = ex.delta.numpy()
    ns = O.non_salient_mask(d_in, ex.salient_idx.numpy())
    pol = O.STEP_MEANABS if bits == 1 else O.STEP_MAXABS
    step = (O.init_step(delta, ns, bits, grid, pol).astype(np.float64) * shrink).astype(np.float32)
    if k == d_in:
        step[:] = 0.01                                    # no non-salient column to take a maximum over
    for j in dead_rows:
        step[j] = 0.0 if j % 2 else -1.0
    return ex, x, step


def run_gpu(ex, x, step, bits, grid, max_tokens=None):
    sg = mes.StepGrad(ex.delta.to(DEV), ex.salient_idx, bits, grid, max_tokens or max(x.shape[0], 1))
    loss, grad = sg(torch.from_numpy(step).to(DEV), x.to(DEV))
    torch.cuda.synchronize()
    return loss.double().cpu().numpy(), grad.double().cpu().numpy()


def check(got, ref, what, scale):
    err = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300)
    assert err <= TOL_NORM, f"{what}: relative 2-norm error {err:.2e}"
    bad = np.abs(got - ref) > TOL_ROW * scale + 1e-6 * (scale.max() if scale.size else 0.0)
    assert not bad.any(), f"{what}: rows {np.nonzero(bad)[0][:8]} off by {np.abs(got - ref)[bad][:4]} vs {ref[bad][:4]}"


def row_scales(delta, sidx, x, step, bits, grid):
    """Per row, the first-order error scales of loss and gradient (see the module docstring)."""
    codes, s_used, sal = O.quantize(delta, sidx, bits, grid, O.STEP_GIVEN, step)
    e = O.compressed_delta(codes, s_used, sal, sidx, bits, grid) - delta.astype(np.float64)
    d = S.ste_slope(delta, s_used, sidx, bits, grid)
    x64 = x.double().numpy()
    r, p = x64 @ e.T, x64 @ d.T
    rho_r, rho_p = np.sqrt((x64 ** 2) @ (e ** 2).T), np.sqrt((x64 ** 2) @ (d ** 2).T)
    live = s_used > 0
    return (np.where(live, (np.abs(r) * rho_r).sum(axis=0), 0.0),
            np.where(live, (np.abs(r) * rho_p + np.abs(p) * rho_r).sum(axis=0), 0.0))


def check_case(ex_delta, sidx, x, step, bits, grid, loss, grad):
    loss_ref, grad_ref = S.step_loss_grad(ex_delta, x.double().numpy(), sidx, bits, grid, step)
    ls, gs = row_scales(ex_delta, sidx, x, step, bits, grid)
    check(loss, loss_ref, "loss", ls)
    check(grad, grad_ref, "grad", gs)


@pytest.mark.parametrize("d_in,d_out,n_tok,k,bits,grid,shrink", [
    (256, 64, 64, 0, 2, 0, 1.0),          # exactly one tile of everything
    (392, 200, 70, 5, 2, 0, 1.0),         # ragged rows, columns and tokens
    (392, 200, 70, 5, 2, 0, 0.5),         # half the max-abs step: many clamped weights
    (640, 132, 300, 17, 3, 0, 0.7),       # two 256-token blocks
    (640, 132, 300, 17, 4, 1, 0.4),       # Eq. 1's grid
    (392, 200, 1, 3, 2, 1, 1.0),          # a single token
    (512, 96, 257, 8, 1, 0, 1.0),         # 1 bit: sign and scale
    (1024, 260, 513, 64, 3, 1, 0.6),
    (136, 4, 9, 136, 2, 0, 1.0),          # every column salient
    (384, 72, 1000, 6, 2, 0, 0.7),        # two 512-token blocks, the second ragged
    (256, 64, 512, 0, 4, 0, 0.5),         # exactly one 512-token block
])
def test_loss_and_gradient_against_the_oracle(d_in, d_out, n_tok, k, bits, grid, shrink):
    ex, x, step = case(d_in, d_out, n_tok, k, bits, grid, shrink, seed=bits + 4 * grid)
    loss, grad = run_gpu(ex, x, step, bits, grid)
    check_case(ex.delta.numpy(), ex.salient_idx.numpy(), x, step, bits, grid, loss, grad)


@pytest.mark.parametrize("seed", range(10))
def test_random_shapes_and_settings(seed):
    """Seeded random cases: shapes that are no multiple of any tile size, every bit width, both grids, any number of
    salient channels, steps from far too wide to far too narrow, a few dead rows, up to 700 tokens (one to three
    token blocks of either kind, split input channels when the rows are few)."""
    rng = np.random.default_rng(2000 + seed)
    d_in = int(rng.integers(1, 150)) * 8
    d_out = int(rng.integers(1, 80)) * 4
    n_tok = int(rng.integers(1, 701))
    bits = int(rng.integers(1, 5))
    grid = int(rng.integers(0, 2)) if bits > 1 else 0
    k = int(rng.integers(0, min(d_in - 8, 40) + 1))
    shrink = float(rng.choice([1.5, 1.0, 0.7, 0.4, 0.2]))
    dead = tuple(int(j) for j in rng.choice(d_out, size=min(3, d_out), replace=False)) if seed % 3 == 0 else ()
    ex, x, step = case(d_in, d_out, n_tok, k, bits, grid, shrink, seed=30 + seed, dead_rows=dead)
    loss, grad = run_gpu(ex, x, step, bits, grid)
    check_case(ex.delta.numpy(), ex.salient_idx.numpy(), x, step, bits, grid, loss, grad)


def test_dead_rows_no_tokens_and_reuse_of_a_larger_workspace():
    ex, x, step = case(264, 72, 40, 4, 2, 0, 0.8, seed=11, dead_rows=(0, 7, 71))
    sg = mes.StepGrad(ex.delta.to(DEV), ex.salient_idx, 2, 0, max_tokens=600)
    sd = torch.from_numpy(step).to(DEV)
    for _ in range(2):                                    # the second call finds the workspace used
        loss, grad = sg(sd, x.to(DEV))
        torch.cuda.synchronize()
        check_case(ex.delta.numpy(), ex.salient_idx.numpy(), x, step, 2, 0, loss.double().cpu().numpy(),
                   grad.double().cpu().numpy())
        assert loss[0] == 0 and grad[7] == 0 and loss[71] == 0
    loss, grad = sg(sd, x[:0].to(DEV))
    torch.cuda.synchronize()
    assert not loss.any() and not grad.any()


def test_results_are_reproducible_bit_for_bit():
    ex, x, step = case(512, 128, 300, 8, 2, 0, 0.7, seed=5)
    a = run_gpu(ex, x, step, 2, 0)
    b = run_gpu(ex, x, step, 2, 0)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_codes_on_cell_boundaries_are_decided_exactly():
    """Weights that are exact multiples of the step sit on the boundary between two cells (symmetric grid) or
    half-way between two levels (Eq. 1's grid): the slope jumps there, so a quotient rounded the wrong way shows."""
    d_in, d_out, n_tok = 128, 64, 32
    rng = np.random.default_rng(3)
    step = (rng.uniform(0.01, 0.03, d_out)).astype(np.float32)
    x = synth.normal((n_tok, d_in), 1.0, 77, "cpu", torch.bfloat16)
    for grid, offset in ((0, 0.0), (1, 0.5)):
        m = rng.integers(-3, 3, size=(d_out, d_in)).astype(np.float64) + offset
        delta = (m * step.astype(np.float64)[:, None]).astype(np.float32)    # the product may round: either side occurs
        delta[:, ::7] = np.float32(-0.0)                                      # a negative zero is a zero
        ex = synth.ExpertDelta(delta=torch.from_numpy(delta), salient_idx=torch.empty(0, dtype=torch.int32))
        loss, grad = run_gpu(ex, x, step, 3, grid)
        check_case(delta, np.zeros(0, dtype=np.int64), x, step, 3, grid, loss, grad)


def test_full_size_rows_sampled():
    """gate_proj of the headline model (4096 -> 14336), 512 calibration tokens (a mini-batch of 4 sequences of 128
    tokens, Section 5), 2 bits, 8 salient channels, in the launch configuration the measurement script times.  Rows
    are independent, so the oracle checks a sample of them exactly."""
    d_in, d_out, n_tok, k, bits = 4096, 14336, 512, 8, 2
    ex = synth.make_delta(d_in, d_out, k, 0.003, 15.0, synth.seed_for(951, 0, 0, 2), DEV)
    x = synth.normal((n_tok, d_in), 1.0, synth.seed_for(951, 0, 0, 3), DEV, torch.bfloat16)
    rows = np.unique(np.concatenate([np.arange(0, 70), np.arange(14336 - 70, 14336),
                                     np.random.default_rng(0).integers(0, d_out, 116)]))
    d_rows = ex.delta[torch.from_numpy(rows).to(DEV)].cpu().numpy()
    ns = O.non_salient_mask(d_in, ex.salient_idx.numpy())
    step_all = (ex.delta[:, torch.from_numpy(ns).to(DEV)].abs().amax(dim=1) / 1.5 * 0.6).float()
    sg = mes.StepGrad(ex.delta, ex.salient_idx, bits, 0, n_tok)
    loss, grad = sg(step_all, x)
    torch.cuda.synchronize()
    step_rows = step_all.cpu().numpy()[rows]
    check_case(d_rows, ex.salient_idx.numpy(), x.cpu(), step_rows, bits, 0, loss.double().cpu().numpy()[rows],
               grad.double().cpu().numpy()[rows])


def test_adamw_against_the_oracle():
    rng = np.random.default_rng(1)
    n = 1000
    s = rng.uniform(0.005, 0.05, n).astype(np.float32)
    sd = torch.from_numpy(s.copy()).to(DEV)
    md, vd = torch.zeros(n, device=DEV), torch.zeros(n, device=DEV)
    s64, m64, v64 = s.astype(np.float64), np.zeros(n), np.zeros(n)
    for t in range(1, 8):
        g = (rng.standard_normal(n) * 0.3).astype(np.float32)
        mes.mes_step_adamw(sd, torch.from_numpy(g).to(DEV), md, vd, t, 1e-3, 0.9, 0.95, 1e-8, 0.01)
        s64, m64, v64 = S.adamw_update(s64, g, m64, v64, t, 1e-3, 0.9, 0.95, 1e-8, 0.01)
    torch.cuda.synchronize()
    np.testing.assert_allclose(sd.cpu().numpy(), s64, rtol=2e-5)
    np.testing.assert_allclose(md.cpu().numpy(), m64, rtol=2e-5, atol=3e-7)      # fp32 sums of terms of size 0.3
    np.testing.assert_allclose(vd.cpu().numpy(), v64, rtol=2e-5, atol=1e-9)


def test_learning_lowers_the_loss():
    """The whole loop on the GPU: 40 rounds of gradient + AdamW from the max-abs step (far too wide for Gaussian
    weights at 2 bits).  The oracle evaluates the objective before and after."""
    ex, x, step = case(512, 128, 256, 0, 2, 0, 1.0, seed=21)
    sg = mes.StepGrad(ex.delta.to(DEV), ex.salient_idx, 2, 0, 256)
    sd = torch.from_numpy(step.copy()).to(DEV)
    md, vd = torch.zeros_like(sd), torch.zeros_like(sd)
    xd = x.to(DEV)
    lr = float(step.mean()) * 0.02
    for t in range(1, 41):
        _, grad = sg(sd, xd)
        mes.mes_step_adamw(sd, grad, md, vd, t, lr, 0.9, 0.95, 1e-8, 0.0)
    torch.cuda.synchronize()
    args = (ex.delta.numpy(), x.double().numpy(), ex.salient_idx.numpy(), 2, 0)
    before, _ = S.step_loss_grad(*args, step)
    after, _ = S.step_loss_grad(*args, sd.cpu().numpy())
    assert after.sum() < 0.8 * before.sum()
    assert (sd > 0).all()
