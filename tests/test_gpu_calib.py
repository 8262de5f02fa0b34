"""GPU parity: dass_calib_norms against the float64 oracle.

Tolerances (relative, per neuron, on the norm): 2e-3 for bf16 inputs with f32
accumulation (the stated bar); 1e-5 for f32 inputs (f32 FMA accumulation over
d <= a few hundred terms plus an f32 exp is good to ~1e-6).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2405_01943_amd as dass
from paper_2405_01943_amd import synth

from gpu_helpers import to_np32

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-3}
ACTS = ["silu", "gelu_tanh", "gelu_erf", "relu"]


def _rel_err(got: np.ndarray, want: np.ndarray) -> float:
    denom = np.where(want > 0, want, 1.0)
    return float(np.max(np.abs(got.astype(np.float64) - want) / denom))


def _inputs(T, d, I, dtype, device, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    X = torch.randn((T, d), generator=g)
    X[:, :: max(1, d // 3)] *= 20.0
    Wg = torch.randn((I, d), generator=g) * (1.0 / d ** 0.5)
    Wu = torch.randn((I, d), generator=g) * (1.0 / d ** 0.5)
    return [t.to(dtype).to(device) for t in (X, Wg, Wu)]


def _check(X, Wg, Wu, act, device, chunks=None):
    I = Wg.shape[0]
    sumsq = torch.full((I,), 123.0, device=device)       # must be overwritten, not added to
    norms = torch.empty(I, device=device)
    if chunks is None:
        dass.calib_norms(X, Wg, Wu, act, sumsq, accumulate=False, norms_out=norms)
    else:
        lo = 0
        for k, n in enumerate(chunks):
            dass.calib_norms(X[lo:lo + n], Wg, Wu, act, sumsq, accumulate=k > 0,
                             norms_out=norms if k == len(chunks) - 1 else None)
            lo += n
        assert lo == X.shape[0]
    torch.cuda.synchronize()
    want_sumsq = oracle.sumsq(to_np32(X), to_np32(Wg), to_np32(Wu), act)
    want = oracle.norms(want_sumsq)
    tol = TOL[X.dtype]
    assert _rel_err(norms.cpu().numpy(), want) <= tol
    assert _rel_err(np.sqrt(sumsq.cpu().numpy().astype(np.float64)), want) <= tol
    return norms


def test_calib_tiny_config_full(gpu_device):
    """Config 'tiny' in full: f32, d=256, d_int=688, 512 tokens."""
    cfg = synth.CONFIGS["tiny"]
    X = synth.make_x(cfg, 0, cfg.tokens, "cpu").to(gpu_device)
    Wg = synth.make_weight(cfg, "wg", "cpu").to(gpu_device)
    Wu = synth.make_weight(cfg, "wu", "cpu").to(gpu_device)
    _check(X, Wg, Wu, cfg.act, gpu_device)


@pytest.mark.parametrize("act", ACTS)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_calib_activations_ragged_shapes(gpu_device, dtype, act):
    # T, d_int not multiples of any tile; d not a multiple of the K slab
    X, Wg, Wu = _inputs(300, 200, 150, dtype, gpu_device, seed=1)
    _check(X, Wg, Wu, act, gpu_device)


@pytest.mark.parametrize("act", ACTS)
@pytest.mark.parametrize("T,d,I", [(300, 64, 150), (515, 192, 257), (1100, 448, 130)])
def test_calib_pipelined_kernel_every_activation(gpu_device, act, T, d, I):
    """bf16 with d a multiple of 64: the direct-to-LDS kernel (1, 3 and 7 K slabs, so the prologue,
    the steady state and the peeled last slabs all run), ragged T and d_int, every activation's
    norm epilogue, against the oracle; then the same tokens in chunks."""
    X, Wg, Wu = _inputs(T, d, I, torch.bfloat16, gpu_device, seed=11 + d)
    norms = _check(X, Wg, Wu, act, gpu_device)
    assert float(norms.min()) > 0.0          # no trivially dead neuron: the comparison means something
    _check(X, Wg, Wu, act, gpu_device, chunks=[T - 257, 1, 256])


@pytest.mark.parametrize("act", ACTS)
@pytest.mark.parametrize("d", [32, 96, 160, 224, 4128])
def test_calib_other_widths(gpu_device, act, d):
    """bf16 with d a multiple of 32 but not of 64 (and 4128 = 64 * 64 + 32): the register-staged kernel."""
    T, I = (333, 200) if d < 1000 else (270, 140)
    X, Wg, Wu = _inputs(T, d, I, torch.bfloat16, gpu_device, seed=23 + d)
    _check(X, Wg, Wu, act, gpu_device)
    _check(X, Wg, Wu, act, gpu_device, chunks=[T - 100, 100])


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_calib_several_tiles_both_ways(gpu_device, dtype):
    X, Wg, Wu = _inputs(700, 320, 400, dtype, gpu_device, seed=2)
    _check(X, Wg, Wu, "silu", gpu_device)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_calib_chunked_accumulation_matches_one_shot(gpu_device, dtype):
    X, Wg, Wu = _inputs(640, 128, 96, dtype, gpu_device, seed=3)
    one = _check(X, Wg, Wu, "silu", gpu_device)
    many = _check(X, Wg, Wu, "silu", gpu_device, chunks=[256, 1, 127, 256])
    assert torch.allclose(one, many, rtol=1e-5)


def test_calib_state_round_trip_resumes(gpu_device):
    """sumsq saved to the host after some chunks and restored continues the same accumulation."""
    X, Wg, Wu = _inputs(512, 64, 80, torch.bfloat16, gpu_device, seed=4)
    a = torch.zeros(80, device=gpu_device)
    dass.calib_norms(X[:192], Wg, Wu, "silu", a, accumulate=False)
    saved = a.cpu()
    b = saved.to(gpu_device)
    na, nb = torch.empty(80, device=gpu_device), torch.empty(80, device=gpu_device)
    dass.calib_norms(X[192:], Wg, Wu, "silu", a, accumulate=True, norms_out=na)
    dass.calib_norms(X[192:], Wg, Wu, "silu", b, accumulate=True, norms_out=nb)
    torch.cuda.synchronize()
    assert torch.allclose(na, nb, rtol=1e-5)


def test_calib_smallest_shapes_and_strides(gpu_device):
    for dtype, vec in ((torch.float32, 4), (torch.bfloat16, 8)):
        X, Wg, Wu = _inputs(1, vec, 1, dtype, gpu_device, seed=5)
        _check(X, Wg, Wu, "silu", gpu_device)
        # leading dimensions larger than d
        X, Wg, Wu = _inputs(70, 64 + 2 * vec, 33, dtype, gpu_device, seed=6)
        _check(X[:, :64], Wg[:, :64], Wu[:, :64], "gelu_tanh", gpu_device)


def test_calib_dead_neurons_give_zero_norm(gpu_device):
    """ReGLU with a gate row that is negative on every token: norm exactly 0."""
    X = torch.rand((130, 64), device=gpu_device).to(torch.bfloat16)      # all positive
    Wg = -torch.rand((40, 64), device=gpu_device).to(torch.bfloat16)     # all negative
    Wu = torch.randn((40, 64), device=gpu_device).to(torch.bfloat16)
    sumsq = torch.empty(40, device=gpu_device)
    norms = torch.empty(40, device=gpu_device)
    dass.calib_norms(X, Wg, Wu, "relu", sumsq, norms_out=norms)
    torch.cuda.synchronize()
    assert torch.all(norms == 0)
    # half of the neurons alive again: their norms follow the oracle, the others stay exactly 0
    Wg[::2] = -Wg[::2]
    dass.calib_norms(X, Wg, Wu, "relu", sumsq, norms_out=norms)
    torch.cuda.synchronize()
    want = oracle.norms(oracle.sumsq(to_np32(X), to_np32(Wg), to_np32(Wu), "relu"))
    assert np.all(want[1::2] == 0) and np.all(want[::2] > 0)
    assert torch.all(norms[1::2] == 0)
    assert _rel_err(norms.cpu().numpy(), want) <= TOL[torch.bfloat16]


def test_calib_argument_errors(gpu_device):
    X, Wg, Wu = _inputs(16, 64, 8, torch.bfloat16, gpu_device, seed=7)
    sumsq = torch.zeros(8, device=gpu_device)
    lib = dass.load_library()
    import ctypes
    vp = ctypes.c_void_p
    rc = lib.dass_calib_norms(vp(X.data_ptr()), 0, 64, vp(Wg.data_ptr()), vp(Wu.data_ptr()), 64, 64, 8,
                              1, 0, vp(sumsq.data_ptr()), 0, None, None, 0, None)
    assert lib.dass_status_string(rc) == b"DASS_ERR_SHAPE"
    rc = lib.dass_calib_norms(vp(X.data_ptr() + 2), 16, 64, vp(Wg.data_ptr()), vp(Wu.data_ptr()), 64,
                              64, 8, 1, 0, vp(sumsq.data_ptr()), 0, None, None, 0, None)
    assert lib.dass_status_string(rc) == b"DASS_ERR_ALIGN"
