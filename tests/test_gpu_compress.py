"""GPU parity: dass_compress_24 (kept values + 2-bit position codes of the 2:4 pattern) against
the oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2405_01943_amd as dass
from paper_2405_01943_amd import synth

from gpu_helpers import padded, to_np32

pytestmark = pytest.mark.gpu


def _sparse_matrix(rows, cols, axis, dtype, seed, surplus_groups=0):
    """Random matrix that is 2:4 along `axis`, with a tenth of the kept weights zero as well, a few
    -0 entries, and `surplus_groups` groups left dense."""
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((rows, cols)).astype(np.float32)
    lines = W if axis == "cols" else W.T
    n_groups = lines.shape[1] // 4
    dense = set(map(tuple, rng.integers(0, [lines.shape[0], n_groups], size=(surplus_groups, 2)).tolist()))
    for li in range(lines.shape[0]):
        for g in range(n_groups):
            if (li, g) in dense:
                continue
            lines[li, 4 * g + rng.choice(4, size=2, replace=False)] = 0.0
    W[rng.random(W.shape) < 0.1] = 0.0
    W[(rng.random(W.shape) < 0.02) & (W == 0)] = -0.0
    return torch.from_numpy(W).to(dtype)


def _run(W, axis, dev, pad=0, want_surplus=True):
    rows, cols = W.shape
    Wd = W.to(dev)
    vshape = (rows // 2, cols) if axis == "rows" else (rows, cols // 2)
    mshape = (rows // 4, cols // 2) if axis == "rows" else (rows, cols // 8)
    values = torch.full(vshape, 5.0, dtype=W.dtype, device=dev)
    meta = torch.full(mshape, 0xEE, dtype=torch.uint8, device=dev)
    if pad:
        Wd, values = padded(Wd, pad), padded(values, pad)
        big = torch.full((mshape[0], mshape[1] + 4), 0xEE, dtype=torch.uint8, device=dev)
        meta = big[:, :mshape[1]]
    surplus = torch.zeros(1, dtype=torch.int64, device=dev) if want_surplus else None
    dass.compress_24(Wd, axis, values, meta, surplus)
    torch.cuda.synchronize()
    ov, om, osurplus = oracle.compress_24(to_np32(Wd), axis)
    got_v = to_np32(values)
    assert np.array_equal(got_v.view(np.uint32), ov.view(np.uint32)), "values differ"
    assert np.array_equal(meta.cpu().numpy(), om), "codes differ"
    if want_surplus:
        assert int(surplus.item()) == osurplus
    if pad:
        assert torch.all(values._base[:, vshape[1]:] == 7.0)
        assert torch.all(meta._base[:, mshape[1]:] == 0xEE)
    return osurplus


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("axis", ["cols", "rows"])
@pytest.mark.parametrize("rows,cols,pad", [(4, 8, 0), (8, 16, 0), (36, 1048, 8), (260, 8200, 0), (1028, 2056, 24)])
def test_compress_small_and_ragged(gpu_device, dtype, axis, rows, cols, pad):
    W = _sparse_matrix(rows, cols, axis, dtype, seed=rows * 31 + cols)
    assert _run(W, axis, gpu_device, pad) == 0


@pytest.mark.parametrize("axis", ["cols", "rows"])
def test_compress_counts_dense_groups_and_accumulates(gpu_device, axis):
    W = _sparse_matrix(64, 512, axis, torch.bfloat16, seed=9, surplus_groups=37)
    n = _run(W, axis, gpu_device)
    assert n > 0
    # the counter is added to, and optional
    rows, cols = W.shape
    Wd = W.to(gpu_device)
    vshape = (rows // 2, cols) if axis == "rows" else (rows, cols // 2)
    mshape = (rows // 4, cols // 2) if axis == "rows" else (rows, cols // 8)
    values = torch.empty(vshape, dtype=W.dtype, device=gpu_device)
    meta = torch.empty(mshape, dtype=torch.uint8, device=gpu_device)
    counter = torch.full((1,), 1000, dtype=torch.int64, device=gpu_device)
    dass.compress_24(Wd, axis, values, meta, counter)
    dass.compress_24(Wd, axis, values, meta, counter)
    dass.compress_24(Wd, axis, values, meta, None)
    torch.cuda.synchronize()
    assert int(counter.item()) == 1000 + 2 * n


def test_compress_all_zero_and_dense_matrices(gpu_device):
    for axis in ("cols", "rows"):
        assert _run(torch.zeros((8, 32), dtype=torch.bfloat16), axis, gpu_device) == 0
        assert _run(torch.ones((8, 32), dtype=torch.float32), axis, gpu_device) == 8 * 32 // 4


def test_compress_full_size_after_dass_pruning(gpu_device):
    """LLaMA2-7B-shaped Down-Proj (groups along the columns) and Gate-Proj (along the rows),
    pruned 2:4 by dass_score_mask_nm, compressed, and compared with the oracle at full size;
    decompressing by the format's definition gives the pruned matrix back."""
    cfg = synth.CONFIGS["llama2_7b"]
    dev = gpu_device
    norms = synth.make_norms(cfg.d_int, dev)
    for which, axis, alpha in (("wd", "cols", 1.0), ("wg", "rows", 0.5)):
        W = synth.make_weight(cfg, which, dev)
        dass.score_mask_nm(W, norms, axis, axis, alpha, 2, 4)
        rows, cols = W.shape
        vshape = (rows // 2, cols) if axis == "rows" else (rows, cols // 2)
        mshape = (rows // 4, cols // 2) if axis == "rows" else (rows, cols // 8)
        values = torch.empty(vshape, dtype=W.dtype, device=dev)
        meta = torch.empty(mshape, dtype=torch.uint8, device=dev)
        surplus = torch.zeros(1, dtype=torch.int64, device=dev)
        dass.compress_24(W, axis, values, meta, surplus)
        torch.cuda.synchronize()
        assert int(surplus.item()) == 0
        W32 = to_np32(W)
        ov, om, osurplus = oracle.compress_24(W32, axis)
        assert osurplus == 0
        assert np.array_equal(to_np32(values).view(np.uint32), ov.view(np.uint32))
        m = meta.cpu().numpy()
        assert np.array_equal(m, om)
        # round trip on the host, vectorised from the definition of the format
        v = to_np32(values)
        back = np.zeros_like(W32)
        if axis == "cols":
            codes = np.stack([m & 15, m >> 4], axis=-1).reshape(rows, cols // 4)
            gbase = np.arange(cols // 4)[None, :] * 4
            r = np.arange(rows)[:, None]
            back[r, gbase + (codes & 3)] = v[:, 0::2]
            back[r, gbase + (codes >> 2)] = v[:, 1::2]
        else:
            codes = np.stack([m & 15, m >> 4], axis=-1).reshape(rows // 4, cols)
            gbase = np.arange(rows // 4)[:, None] * 4
            c = np.arange(cols)[None, :]
            back[gbase + (codes & 3), c] = v[0::2, :]
            back[gbase + (codes >> 2), c] = v[1::2, :]
        assert np.array_equal(back, W32)
