"""GPU integration: pruning MLP blocks one after the other.  Block l is calibrated on the
output of the pruned block l - 1 (dass_mlp_forward); every step is checked against the oracle
fed with the same inputs the GPU step saw: norms within tolerance, 2:4 masks bit for bit,
block output within its rounding bound, compressed Down-Proj bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2405_01943_amd as dass

from gpu_helpers import bits_equal, first_mismatch, to_np32

pytestmark = pytest.mark.gpu


def test_three_blocks_in_sequence(gpu_device):
    dev = gpu_device
    T, d, d_int, blocks = 640, 128, 320, 3
    g = torch.Generator(device="cpu").manual_seed(11)
    X = torch.randn((T, d), generator=g).to(torch.bfloat16).to(dev)
    for b in range(blocks):
        act = ("silu", "gelu_tanh", "relu")[b]
        Wg, Wu = ((torch.randn((d_int, d), generator=g) * 0.2).to(torch.bfloat16).to(dev) for _ in range(2))
        Wd = (torch.randn((d, d_int), generator=g) * 0.2).to(torch.bfloat16).to(dev)
        X32 = to_np32(X)
        # calibration on this block's input
        sumsq = torch.empty(d_int, device=dev)
        norms = torch.empty(d_int, device=dev)
        dass.calib_norms(X, Wg, Wu, act, sumsq, norms_out=norms)
        torch.cuda.synchronize()
        want = oracle.norms(oracle.sumsq(X32, to_np32(Wg), to_np32(Wu), act))
        n32 = norms.cpu().numpy()
        ok = want > 0
        assert float(np.max(np.abs(n32[ok] - want[ok]) / want[ok])) <= 2e-3, f"block {b}: norms"
        # 2:4 masks from the GPU's own f32 norms, oracle handed the same norms
        for W, axis, alpha in ((Wg, "rows", 0.5), (Wu, "rows", 0.5), (Wd, "cols", 1.0)):
            ref, _ = oracle.mask_nm(to_np32(W), n32, axis, axis, alpha, 2, 4)
            dass.score_mask_nm(W, norms, axis, axis, alpha, 2, 4)
            torch.cuda.synchronize()
            assert bits_equal(W, ref), f"block {b} {axis}: {first_mismatch(W, ref)}"
        # storage form of the pruned Down-Proj
        vals = torch.empty((d, d_int // 2), dtype=Wd.dtype, device=dev)
        meta = torch.empty((d, d_int // 8), dtype=torch.uint8, device=dev)
        surplus = torch.zeros(1, dtype=torch.int64, device=dev)
        dass.compress_24(Wd, "cols", vals, meta, surplus)
        # the next block's input
        nxt = torch.empty((T, d), dtype=torch.bfloat16, device=dev)
        dass.mlp_forward(X, Wg, Wu, Wd, act, nxt)
        torch.cuda.synchronize()
        ov, om, _ = oracle.compress_24(to_np32(Wd), "cols")
        assert int(surplus.item()) == 0
        assert np.array_equal(to_np32(vals).view(np.uint32), ov.view(np.uint32)) and np.array_equal(meta.cpu().numpy(), om)
        ref, ab = oracle.mlp_forward(X32, to_np32(Wg), to_np32(Wu), to_np32(Wd), act, want_abs=True)
        err = np.abs(to_np32(nxt).astype(np.float64) - ref) / (2.0 ** -8 * (np.abs(ref) + 1.05 * ab) + 1e-30)
        assert float(err.max()) <= 1.0, f"block {b}: output at {err.max():.2f} of its tolerance"
        X = nxt
