"""GPU parity on seeded random cases: shapes, dtypes, axes, exponents, patterns, quotas, value
distributions (ties, constants, extreme magnitudes, half-pruned inputs), leading dimensions and
mask requests drawn at random; every case compared with the float64 oracle bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2405_01943_amd as dass

from gpu_helpers import bits_equal, first_mismatch, to_np32

pytestmark = pytest.mark.gpu

MODES = ["normal", "normal", "ties", "const", "extreme", "sparse"]
AXES = [("rows", "rows"), ("cols", "cols"), ("rows", "cols"), ("cols", "rows")]
PATTERNS = [(1, 2), (2, 4), (4, 8), (1, 4), (3, 8), (8, 16), (2, 8)]


def _weights(rows, cols, dtype, mode, g):
    if mode == "ties":
        vals = torch.tensor([-0.5, 0.0, 0.25, 0.5, -0.25, 1.0, 0.75])
        w = vals[torch.randint(0, len(vals), (rows, cols), generator=g)]
    elif mode == "const":
        w = torch.full((rows, cols), -0.375)
    elif mode == "extreme":
        mant = torch.rand((rows, cols), generator=g) + 1.0
        expo = torch.randint(-135, 100, (rows, cols), generator=g).to(torch.float32)
        w = mant * torch.exp2(expo) * torch.where(torch.rand((rows, cols), generator=g) < 0.5, -1.0, 1.0)
    else:
        w = torch.randn((rows, cols), generator=g) * 0.02
        if mode == "sparse":
            w[torch.rand((rows, cols), generator=g) < 0.5] = 0.0
    return w.to(dtype)


def _norms(n, mode, g):
    if mode == "ties":
        vals = torch.tensor([0.0, 1.0, 4.0, 16.0, 2.0, 9.0])
        return vals[torch.randint(0, len(vals), (n,), generator=g)]
    if mode == "extreme":
        v = torch.exp2(torch.randint(-70, 70, (n,), generator=g).to(torch.float32)) * (torch.rand(n, generator=g) + 1.0)
        v[::5] = 0.0
        return v
    return torch.exp(0.7 * torch.randn(n, generator=g) + 3.0)


@pytest.mark.parametrize("master_seed", [11, 12, 13])
def test_random_cases_match_the_oracle(gpu_device, master_seed):
    rng = np.random.default_rng(master_seed)
    done = 0
    for case in range(120):
        seed = int(rng.integers(1 << 30))
        g = torch.Generator(device="cpu").manual_seed(seed)
        kind = rng.choice(["unstructured", "nm"])
        dtype = [torch.bfloat16, torch.float32][int(rng.integers(2))]
        mode = str(rng.choice(MODES))
        axes = AXES[int(rng.integers(4))]
        alpha = float(rng.choice([0.0, 0.5, 1.0, 1.0, 0.5, 0.3]))
        big = rng.random() < 0.15
        if axes[1] == "rows":     # lines / groups run down the columns
            rows = int(rng.integers(1100, 5000)) if big else int(rng.integers(1, 40)) * 16 + \
                (int(rng.integers(0, 16)) if kind == "unstructured" else 0)
            cols = 8 * int(rng.integers(1, 30))
        else:
            rows = int(rng.integers(1, 30))
            cols = 16 * int(rng.integers(600, 2600)) if big else 16 * int(rng.integers(1, 60)) + \
                (8 * int(rng.integers(0, 2)) if kind == "unstructured" else 0)
        pad = int(rng.choice([0, 0, 8, 24]))
        W0 = _weights(rows, cols, dtype, mode, g)
        nrm = _norms(rows if axes[0] == "rows" else cols, mode, g).to(torch.float32)
        wide = torch.full((rows, cols + pad), 7.0, dtype=dtype)
        wide[:, :cols] = W0
        W = wide.to(gpu_device)[:, :cols]
        mask = torch.full((rows, cols // 8), 0x33, dtype=torch.uint8, device=gpu_device) if rng.random() < 0.5 else None
        length = rows if axes[1] == "rows" else cols
        what = f"seed {seed} {kind} {dtype} {mode} {axes} alpha {alpha} {rows}x{cols}+{pad}"
        if kind == "unstructured":
            n_prune = int(rng.choice([0, 1, length // 2, length // 3, length - 1, length,
                                      int(rng.integers(0, length + 1))]))
            want, want_mask = oracle.mask_unstructured(to_np32(W0), nrm.numpy(), axes[0], axes[1], alpha, n_prune,
                                                       want_mask=True)
            dass.score_mask_unstructured(W, nrm.to(gpu_device), axes[0], axes[1], alpha, n_prune, mask_out=mask)
            what += f" n_prune {n_prune}"
        else:
            n_keep, m = PATTERNS[int(rng.integers(len(PATTERNS)))]
            if length % m:
                continue
            want, want_mask = oracle.mask_nm(to_np32(W0), nrm.numpy(), axes[0], axes[1], alpha, n_keep, m,
                                             want_mask=True)
            dass.score_mask_nm(W, nrm.to(gpu_device), axes[0], axes[1], alpha, n_keep, m, mask_out=mask)
            what += f" {n_keep}:{m}"
        torch.cuda.synchronize()
        assert bits_equal(W, want), what + ": " + first_mismatch(W, want)
        if mask is not None:
            assert np.array_equal(mask.cpu().numpy(), want_mask), what
        if pad:
            base = W._base if W._base is not None else W
            assert torch.all(base[:, cols:] == 7.0), what
        done += 1
    assert done >= 80
