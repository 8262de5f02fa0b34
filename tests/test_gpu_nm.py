"""GPU parity: dass_score_mask_nm against the float64 oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2405_01943_amd as dass
from paper_2405_01943_amd import synth

from gpu_helpers import bits_equal, first_mismatch, padded, to_np32

pytestmark = pytest.mark.gpu

AXES = [("rows", "rows"), ("cols", "cols"), ("rows", "cols"), ("cols", "rows")]


def _weights(rows, cols, dtype, device, seed, ties=False):
    g = torch.Generator(device="cpu").manual_seed(seed)
    if ties:
        vals = torch.tensor([-0.5, 0.0, 0.25, 0.5, -0.25, 1.0])
        w = vals[torch.randint(0, len(vals), (rows, cols), generator=g)]
    else:
        w = torch.randn((rows, cols), generator=g) * 0.02
    return w.to(dtype).to(device)


def _norms(n, device, seed, ties=False):
    if ties:
        g = torch.Generator(device="cpu").manual_seed(seed + 1)
        vals = torch.tensor([0.0, 1.0, 4.0, 16.0, 2.0])
        return vals[torch.randint(0, len(vals), (n,), generator=g)].to(device)
    return synth.make_norms(n, "cpu", seed).to(device)


def _run_case(gpu_device, rows, cols, dtype, axes, alpha, n_keep, m, seed, ties=False, pad=0,
              with_mask=True):
    norm_axis, group_axis = axes
    W = _weights(rows, cols, dtype, gpu_device, seed, ties)
    if pad:
        W = padded(W, pad)
    nrm = _norms(rows if norm_axis == "rows" else cols, gpu_device, seed, ties)
    want_w, want_mask = oracle.mask_nm(to_np32(W), nrm.cpu().numpy(), norm_axis, group_axis, alpha,
                                       n_keep, m, want_mask=True)
    mask = torch.full((rows, cols // 8), 0xAA, dtype=torch.uint8, device=gpu_device) if with_mask else None
    dass.score_mask_nm(W, nrm, norm_axis, group_axis, alpha, n_keep, m, mask_out=mask)
    torch.cuda.synchronize()
    assert bits_equal(W, want_w), first_mismatch(W, want_w)
    if with_mask:
        assert np.array_equal(mask.cpu().numpy(), want_mask)
    if pad:  # the canary columns right of the view must be untouched
        base = W._base if W._base is not None else W
        assert torch.all(base[:, cols:] == 7.0)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("axes", AXES)
@pytest.mark.parametrize("n_keep,m", [(2, 4), (4, 8), (1, 2), (1, 4), (3, 4), (5, 8), (8, 16), (3, 16)])
def test_nm_small_ragged(gpu_device, dtype, axes, n_keep, m):
    # several row batches and column blocks with ragged tails in both directions
    rows, cols = 16 * 13, 8 * 2 * 131
    alpha = 0.5 if axes[0] == axes[1] else 1.0
    _run_case(gpu_device, rows, cols, dtype, axes, alpha, n_keep, m, seed=m * 10 + n_keep)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("axes", AXES)
@pytest.mark.parametrize("n_keep,m", [(2, 4), (4, 8), (8, 16)])
def test_nm_heavy_ties(gpu_device, dtype, axes, n_keep, m):
    _run_case(gpu_device, 64, 256, dtype, axes, 0.5, n_keep, m, seed=5, ties=True)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("alpha", [0.0, 0.25, 0.5, 0.75, 1.0, 2.0])
def test_nm_alpha_sweep(gpu_device, dtype, alpha):
    _run_case(gpu_device, 96, 512, dtype, ("rows", "rows"), alpha, 2, 4, seed=11)
    _run_case(gpu_device, 96, 512, dtype, ("cols", "cols"), alpha, 4, 8, seed=12)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_nm_leading_dimension_and_no_mask(gpu_device, dtype):
    _run_case(gpu_device, 40, 264, dtype, ("rows", "rows"), 0.5, 2, 4, seed=21, pad=24)
    _run_case(gpu_device, 40, 264, dtype, ("cols", "cols"), 1.0, 2, 4, seed=22, pad=24, with_mask=False)


def test_nm_smallest_shapes(gpu_device):
    for dtype in (torch.float32, torch.bfloat16):
        _run_case(gpu_device, 2, 8, dtype, ("rows", "rows"), 0.5, 1, 2, seed=31)
        _run_case(gpu_device, 1, 8, dtype, ("cols", "cols"), 1.0, 4, 8, seed=32)
        _run_case(gpu_device, 16, 16, dtype, ("cols", "cols"), 1.0, 8, 16, seed=33)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("axes", [("rows", "rows"), ("cols", "cols")])
@pytest.mark.parametrize("n_keep,m", [(1, 2), (2, 4), (4, 8)])
def test_nm_extreme_magnitudes(gpu_device, dtype, axes, n_keep, m):
    """Scores near the bottom and the top of the f32 range (subnormal weights, tiny and huge norms,
    products that underflow or overflow in f32) and exact zeros: the selection must stay exact."""
    rows, cols = 64, 256
    g = torch.Generator(device="cpu").manual_seed(77)
    mant = torch.rand((rows, cols), generator=g) + 1.0
    expo = torch.randint(-140, -100, (rows, cols), generator=g).to(torch.float32)
    W = (mant * torch.exp2(expo)).to(dtype)                       # tiny, partly subnormal
    W[::3] = (mant[::3] * torch.exp2(expo[::3] + 225.0)).to(dtype)  # huge
    W[:, ::5] = 0.0
    W = W * torch.where(torch.rand((rows, cols), generator=g) < 0.5, -1.0, 1.0).to(dtype)
    n = rows if axes[0] == "rows" else cols
    nrm = torch.exp2(torch.randint(-60, 60, (n,), generator=g).to(torch.float32)) * \
        (torch.rand(n, generator=g) + 1.0)
    nrm[::7] = 0.0
    W, nrm = W.to(gpu_device), nrm.to(torch.float32).to(gpu_device)
    for alpha in (0.5, 1.0):
        Wc = W.clone()
        want, want_mask = oracle.mask_nm(to_np32(Wc), nrm.cpu().numpy(), axes[0], axes[1], alpha, n_keep, m,
                                         want_mask=True)
        mask = torch.zeros((rows, cols // 8), dtype=torch.uint8, device=gpu_device)
        dass.score_mask_nm(Wc, nrm, axes[0], axes[1], alpha, n_keep, m, mask_out=mask)
        torch.cuda.synchronize()
        assert bits_equal(Wc, want), first_mismatch(Wc, want)
        assert np.array_equal(mask.cpu().numpy(), want_mask)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("axes", [("rows", "rows"), ("cols", "cols")])
@pytest.mark.parametrize("n_keep,m", [(2, 4), (4, 8)])
def test_nm_near_ties_decided_below_f32_precision(gpu_device, dtype, axes, n_keep, m):
    """Groups whose scores agree to f32 precision and differ only below it: weight k of a group
    is 1 + k/128 and its norm is fl32(P / weight), so all m products are P up to an f32 rounding
    error.  Only a comparison of the exact products ranks them like the oracle."""
    n_groups, lines = 96, 64
    g = torch.Generator(device="cpu").manual_seed(5 * m + (axes[0] == "rows"))
    k = torch.stack([torch.randperm(m, generator=g) for _ in range(n_groups)]).reshape(-1)   # weight index along d_int
    w_line = (1.0 + k.to(torch.float64) / 128.0)                                             # exact in bf16
    P = torch.exp(torch.rand(n_groups, generator=g, dtype=torch.float64) * 8 - 4).repeat_interleave(m)
    nrm = (P / w_line).to(torch.float32)
    sign = torch.where(torch.rand((lines, n_groups * m), generator=g) < 0.5, -1.0, 1.0).to(torch.float64)
    W = (w_line[None, :] * sign)                                                             # [lines, d_int]
    if axes[0] == "rows":
        W = W.t().contiguous()                                                               # groups down the rows
    W = W.to(dtype)
    # the construction does what it says: many pairs inside a group share the f32 product
    p32 = (w_line.to(torch.float32) * nrm).reshape(n_groups, m)
    exact = (w_line * nrm.to(torch.float64)).reshape(n_groups, m)
    same_p = (p32[:, :, None] == p32[:, None, :]) & (exact[:, :, None] != exact[:, None, :])
    assert same_p.any(dim=(1, 2)).float().mean() > 0.5
    want, want_mask = oracle.mask_nm(to_np32(W), nrm.numpy(), axes[0], axes[1], 1.0, n_keep, m, want_mask=True)
    Wg = W.to(gpu_device)
    mask = torch.zeros((Wg.shape[0], Wg.shape[1] // 8), dtype=torch.uint8, device=gpu_device)
    dass.score_mask_nm(Wg, nrm.to(gpu_device), axes[0], axes[1], 1.0, n_keep, m, mask_out=mask)
    torch.cuda.synchronize()
    assert bits_equal(Wg, want), first_mismatch(Wg, want)
    assert np.array_equal(mask.cpu().numpy(), want_mask)


def test_nm_tiny_config_all_three_matrices(gpu_device):
    """Config 'tiny' (f32, d=256, d_int=688): Gate, Up with alpha 0.5 down rows; Down with alpha 1."""
    cfg = synth.CONFIGS["tiny"]
    nrm = synth.make_norms(cfg.d_int, "cpu", 0).to(gpu_device)
    for which, axes, alpha in (("wg", ("rows", "rows"), 0.5), ("wu", ("rows", "rows"), 0.5),
                               ("wd", ("cols", "cols"), 1.0)):
        W = synth.make_weight(cfg, which, "cpu").to(gpu_device)
        want, _ = oracle.mask_nm(to_np32(W), nrm.cpu().numpy(), axes[0], axes[1], alpha, 2, 4)
        dass.score_mask_nm(W, nrm, axes[0], axes[1], alpha, 2, 4)
        torch.cuda.synchronize()
        assert bits_equal(W, want), first_mismatch(W, want)


def test_factor_square_root_is_correctly_rounded(gpu_device):
    """alpha = 0.5 over the f32 range: the factor the kernel uses must be the oracle's.  Observed
    through 1:2 selections built to sit on the decision boundary: sqrt(a) against
    sqrt(b) * (1 + 2^-7) with b = a / (1 + 2^-7)^2, so a 1-ulp difference in a factor flips them."""
    n = 1 << 18
    g = torch.Generator(device="cpu").manual_seed(3)
    a = torch.exp(torch.rand(n, generator=g, dtype=torch.float64) * 60 - 30)
    b = a / (1 + 2.0 ** -7) ** 2
    nrm = torch.stack([a, b], dim=1).reshape(-1).to(torch.float32)
    W = torch.tensor([1.0, 1.0 + 2.0 ** -7]).repeat(n).reshape(1, 2 * n).to(torch.bfloat16)
    want, _ = oracle.mask_nm(to_np32(W), nrm.numpy(), "cols", "cols", 0.5, 1, 2)
    Wg = W.to(gpu_device)
    dass.score_mask_nm(Wg, nrm.to(gpu_device), "cols", "cols", 0.5, 1, 2)
    torch.cuda.synchronize()
    assert bits_equal(Wg, want), first_mismatch(Wg, want)
    kept_first = (want[0, 0::2] != 0).mean()
    assert 0.2 < kept_first < 0.8  # the construction really sits on the decision boundary


def test_nm_argument_errors_leave_data_untouched(gpu_device):
    W = torch.ones((8, 16), dtype=torch.bfloat16, device=gpu_device)
    nrm = torch.ones(16, device=gpu_device)
    with pytest.raises(dass.DassError) as e:
        dass.score_mask_nm(W, nrm, "cols", "cols", 1.0, 2, 3)
    assert e.value.status_name == "DASS_ERR_ARG"
    with pytest.raises(dass.DassError) as e:
        dass.score_mask_nm(W[:, :8], nrm[:8].contiguous(), "cols", "cols", 1.0, 8, 16)
    assert e.value.status_name == "DASS_ERR_SHAPE"
    torch.cuda.synchronize()
    assert torch.all(W == 1)
