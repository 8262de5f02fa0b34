"""GPU parity: dass_input_norms (Eq. 1, the Wanda metric's input-feature norms) against the
float64 oracle, and the Wanda selection end to end."""
import numpy as np
import pytest
import torch

import oracle
import paper_2405_01943_amd as dass
from paper_2405_01943_amd import synth

from gpu_helpers import bits_equal, first_mismatch, padded, to_np32

pytestmark = pytest.mark.gpu

# f32 squares and 512-row block sums, f64 across blocks.  A block sum of n <= 512 non-negative
# terms has rounding errors of 2^-24 relative that add like a random walk: about sqrt(512) 2^-25 =
# 7e-7 of the sum (the worst-case linear bound, 512 * 2^-24 = 3.1e-5, needs every rounding to go the
# same way).  Observed 4.6e-7 at the worst; the tolerance is ten times that.
TOL = 5e-6


def _rel_err(got, want):
    want = np.asarray(want, dtype=np.float64)
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - want) / np.where(want > 0, want, 1.0)))


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("T,d,pad", [(1, 8, 0), (7, 24, 0), (255, 264, 0), (256, 2048, 0), (1000, 2056, 24), (2311, 520, 8)])
def test_input_norms_small_and_ragged(gpu_device, dtype, T, d, pad):
    g = torch.Generator(device="cpu").manual_seed(T * 131 + d)
    X = (torch.randn((T, d), generator=g) * (torch.rand(d, generator=g) * 4 + 0.01)).to(dtype).to(gpu_device)
    if pad:
        X = padded(X, pad)
    sumsq = torch.full((d,), -1.0, device=gpu_device)
    norms = torch.full((d,), -1.0, device=gpu_device)
    dass.input_norms(X, sumsq, norms_out=norms)
    torch.cuda.synchronize()
    want = oracle.input_sumsq(to_np32(X))
    assert _rel_err(sumsq.cpu().numpy(), want) <= TOL
    assert _rel_err(norms.cpu().numpy(), oracle.norms(want)) <= TOL
    if pad:
        base = X._base if X._base is not None else X
        assert torch.all(base[:, d:] == 7.0)


def test_input_norms_chunks_accumulate_and_zero_columns(gpu_device):
    T, d = 1500, 512
    g = torch.Generator(device="cpu").manual_seed(5)
    X = torch.randn((T, d), generator=g)
    X[:, ::7] = 0.0                     # empty features: norm exactly 0
    X = X.to(torch.bfloat16).to(gpu_device)
    sumsq = torch.empty(d, device=gpu_device)
    norms = torch.empty(d, device=gpu_device)
    dass.input_norms(X[:600], sumsq)
    dass.input_norms(X[600:], sumsq, accumulate=True, norms_out=norms)
    torch.cuda.synchronize()
    want = oracle.input_sumsq(to_np32(X))
    assert _rel_err(sumsq.cpu().numpy(), want) <= TOL
    assert torch.all(norms[::7] == 0)
    # deterministic: a second run gives the same bits
    s2 = torch.empty(d, device=gpu_device)
    dass.input_norms(X[:600], s2)
    dass.input_norms(X[600:], s2, accumulate=True)
    torch.cuda.synchronize()
    assert torch.equal(sumsq.view(torch.int32), s2.view(torch.int32))


def test_input_norms_full_size_and_wanda_masks(gpu_device):
    """All 262144 calibration tokens of the LLaMA2-7B-shaped config, then the Wanda selection
    (|W| * ||X_j||, per output, 2:4) on Gate-Proj: masks equal the oracle's bit for bit."""
    cfg = synth.CONFIGS["llama2_7b"]
    dev = gpu_device
    T, d = cfg.tokens, cfg.d
    X = torch.empty((T, d), dtype=cfg.torch_dtype, device=dev)
    for c in range(T // 32768):
        X[c * 32768:(c + 1) * 32768] = synth.make_x(cfg, c, 32768, dev)
    sumsq = torch.empty(d, device=dev)
    norms = torch.empty(d, device=dev)
    dass.input_norms(X, sumsq, norms_out=norms)
    torch.cuda.synchronize()
    want = np.zeros(d, dtype=np.float64)
    for lo in range(0, T, 32768):
        oracle.input_sumsq(to_np32(X[lo:lo + 32768]), out=want)
    err = _rel_err(sumsq.cpu().numpy(), want)
    print(f"\n[input norms, T={T} d={d}] max rel err {err:.2e}", flush=True)
    assert err <= TOL
    assert _rel_err(norms.cpu().numpy(), oracle.norms(want)) <= TOL
    del X
    Wg = synth.make_weight(cfg, "wg", dev)
    W = Wg.clone()
    dass.score_mask_nm(W, norms, "cols", "cols", 1.0, 2, 4)
    torch.cuda.synchronize()
    want_w, _ = oracle.mask_nm(to_np32(Wg), norms.cpu().numpy(), "cols", "cols", 1.0, 2, 4)
    assert bits_equal(W, want_w), first_mismatch(W, want_w)


def test_input_norms_argument_errors(gpu_device):
    X = torch.ones((16, 12), dtype=torch.bfloat16, device=gpu_device)    # 12 features: not a multiple of 8
    with pytest.raises(dass.DassError):
        dass.input_norms(X, torch.zeros(12, device=gpu_device))
    with pytest.raises(TypeError):
        dass.input_norms(torch.ones((16, 16), dtype=torch.bfloat16, device=gpu_device),
                         torch.zeros(8, device=gpu_device))
