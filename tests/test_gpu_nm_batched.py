"""GPU parity: dass_score_mask_nm_batched against the float64 oracle, matrix by matrix and bit for
bit, and against the single-matrix entry point."""
import numpy as np
import pytest
import torch

import oracle
import paper_2405_01943_amd as dass

from gpu_helpers import bits_equal, first_mismatch, padded, to_np32

pytestmark = pytest.mark.gpu


def _layer(d, d_int, dtype, dev, seed):
    """Gate, Up ([d_int, d]), Down ([d, d_int]) and the norms of one synthetic MLP layer."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    mk = lambda r, c: (torch.randn((r, c), generator=g) * 0.02).to(dtype).to(dev)
    norms = (torch.rand(d_int, generator=g) * 30 + 0.01).to(dev)
    return mk(d_int, d), mk(d_int, d), mk(d, d_int), norms


def _check(W, W0, norms, axes, alpha, n_keep, m, mask=None):
    want, want_mask = oracle.mask_nm(to_np32(W0), norms.cpu().numpy(), axes[0], axes[1], alpha, n_keep, m,
                                     want_mask=True)
    assert bits_equal(W, want), first_mismatch(W, want)
    if mask is not None:
        assert np.array_equal(mask.cpu().numpy().reshape(want_mask.shape), want_mask)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("n_keep,m", [(1, 2), (2, 4), (4, 8)])
def test_batched_model_of_five_layers(gpu_device, dtype, n_keep, m):
    """15 matrices in two shapes: two launches; every matrix equals the oracle's."""
    d, d_int = 328, 1384     # ragged against every workgroup width
    layers = [_layer(d, d_int, dtype, gpu_device, 100 + k) for k in range(5)]
    work = [[w.clone() for w in (g, u, dn)] for g, u, dn, _ in layers]
    tasks = []
    for (g, u, dn, nrm), (wg, wu, wd) in zip(layers, work):
        tasks += [(wg, nrm, "rows", "rows", 0.5), (wu, nrm, "rows", "rows", 0.5), (wd, nrm, "cols", "cols", 1.0)]
    dass.score_mask_nm_batched(tasks, n_keep, m)
    torch.cuda.synchronize()
    for (g, u, dn, nrm), (wg, wu, wd) in zip(layers, work):
        _check(wg, g, nrm, ("rows", "rows"), 0.5, n_keep, m)
        _check(wu, u, nrm, ("rows", "rows"), 0.5, n_keep, m)
        _check(wd, dn, nrm, ("cols", "cols"), 1.0, n_keep, m)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("n_keep,m", [(1, 2), (2, 4), (4, 8)])
@pytest.mark.parametrize("d,d_int", [(328, 1384), (1024, 2752), (72, 136)])
def test_batched_one_block(gpu_device, dtype, n_keep, m, d, d_int):
    """Gate, Up and Down of one MLP block (and of two blocks) in one call, Down-Proj first: what
    bench.py's step does; shapes ragged against every workgroup width."""
    for n_blocks in (1, 2):
        layers = [_layer(d, d_int, dtype, gpu_device, 300 + k) for k in range(n_blocks)]
        work = [[w.clone() for w in (g, u, dn)] for g, u, dn, _ in layers]
        tasks = []
        for (g, u, dn, nrm), (wg, wu, wd) in zip(layers, work):
            tasks += [(wd, nrm, "cols", "cols", 1.0), (wg, nrm, "rows", "rows", 0.5), (wu, nrm, "rows", "rows", 0.5)]
        dass.score_mask_nm_batched(tasks, n_keep, m)
        torch.cuda.synchronize()
        for (g, u, dn, nrm), (wg, wu, wd) in zip(layers, work):
            _check(wg, g, nrm, ("rows", "rows"), 0.5, n_keep, m)
            _check(wu, u, nrm, ("rows", "rows"), 0.5, n_keep, m)
            _check(wd, dn, nrm, ("cols", "cols"), 1.0, n_keep, m)


def test_batched_more_matrices_than_one_launch_holds(gpu_device):
    """130 equal matrices: split over two launches (96 + 34); each gets its own norms."""
    rows, cols, n = 64, 136, 130
    g = torch.Generator(device="cpu").manual_seed(7)
    W0 = [(torch.randn((rows, cols), generator=g) * 0.02).to(torch.bfloat16).to(gpu_device) for _ in range(n)]
    nrm = [(torch.rand(cols, generator=g) * 5 + 0.1).to(gpu_device) for _ in range(n)]
    W = [w.clone() for w in W0]
    dass.score_mask_nm_batched([(W[k], nrm[k], "cols", "cols", 1.0) for k in range(n)], 2, 4)
    torch.cuda.synchronize()
    for k in (0, 1, 47, 95, 96, 97, 128, 129):
        _check(W[k], W0[k], nrm[k], ("cols", "cols"), 1.0, 2, 4)
    single = [w.clone() for w in W0]
    for k in range(n):
        dass.score_mask_nm(single[k], nrm[k], "cols", "cols", 1.0, 2, 4)
    torch.cuda.synchronize()
    for k in range(n):
        assert torch.equal(W[k].view(torch.int16), single[k].view(torch.int16)), k


def test_batched_mixed_tasks(gpu_device):
    """Masks, a leading dimension, cross-axis norms, an exponent and a pattern off the one-pass
    path, all in one call: each task equals its single call and the oracle."""
    dev = gpu_device
    g = torch.Generator(device="cpu").manual_seed(9)
    mk = lambda r, c: (torch.randn((r, c), generator=g) * 0.02).to(torch.bfloat16).to(dev)
    nr = lambda n: (torch.rand(n, generator=g) * 9 + 0.05).to(dev)
    specs = [   # rows, cols, axes, alpha, mask?, pad
        (96, 264, ("rows", "rows"), 0.5, True, 0),
        (96, 264, ("rows", "rows"), 0.5, True, 0),
        (96, 264, ("rows", "rows"), 0.5, False, 0),
        (96, 264, ("cols", "cols"), 1.0, False, 24),
        (96, 264, ("cols", "cols"), 1.0, False, 24),
        (96, 264, ("rows", "cols"), 1.0, False, 0),     # Wanda-style: norms of the other axis
        (96, 264, ("cols", "cols"), 0.3, False, 0),     # general path (pow)
        (40, 72, ("cols", "rows"), 0.0, True, 0),
    ]
    W0, W, norms, masks, tasks = [], [], [], [], []
    for rows, cols, axes, alpha, with_mask, pad in specs:
        w0 = mk(rows, cols)
        w = padded(w0.clone(), pad) if pad else w0.clone()
        n = nr(rows if axes[0] == "rows" else cols)
        mask = torch.full((rows, cols // 8), 0x55, dtype=torch.uint8, device=dev) if with_mask else None
        W0.append(w0); W.append(w); norms.append(n); masks.append(mask)
        tasks.append((w, n, axes[0], axes[1], alpha, mask) if with_mask else (w, n, axes[0], axes[1], alpha))
    dass.score_mask_nm_batched(tasks, 2, 4)
    torch.cuda.synchronize()
    for (rows, cols, axes, alpha, with_mask, pad), w0, w, n, mask in zip(specs, W0, W, norms, masks):
        _check(w, w0, n, axes, alpha, 2, 4, mask)
        if pad:
            base = w._base if w._base is not None else w
            assert torch.all(base[:, cols:] == 7.0)
    # 3:8 is not a one-pass pattern: every task runs as its own call
    W2 = [w0.clone() for w0 in W0[:3]]
    dass.score_mask_nm_batched([(W2[k], norms[k], "rows", "rows", 0.5) for k in range(3)], 3, 8)
    torch.cuda.synchronize()
    for k in range(3):
        _check(W2[k], W0[k], norms[k], ("rows", "rows"), 0.5, 3, 8)


def test_batched_error_leaves_every_matrix_untouched(gpu_device):
    W = [torch.ones((8, 16), dtype=torch.bfloat16, device=gpu_device) for _ in range(3)]
    nrm = torch.ones(16, device=gpu_device)
    bad = torch.ones((8, 24), dtype=torch.bfloat16, device=gpu_device)   # 24 columns: not a multiple of 16
    with pytest.raises(dass.DassError) as e:
        dass.score_mask_nm_batched([(W[0], nrm, "cols", "cols", 1.0), (W[1], nrm, "cols", "cols", 1.0),
                                    (bad, torch.ones(24, device=gpu_device), "cols", "cols", 1.0)], 8, 16)
    assert "task 2" in str(e.value)
    torch.cuda.synchronize()
    assert all(torch.all(w == 1) for w in W)


def test_batched_full_size_layers(gpu_device):
    """Three layers of the LLaMA2-7B-shaped config through one batched call, as bench.py launches
    it (Gate/Up share one launch, Down another); every weight of all nine matrices is compared."""
    from paper_2405_01943_amd import synth
    cfg = synth.CONFIGS["llama2_7b"]
    dev = gpu_device
    base = [synth.make_weight(cfg, w, dev, seed=s) for s in range(3) for w in ("wg", "wu", "wd")]
    norms = [synth.make_norms(cfg.d_int, dev, seed=s) for s in range(3)]
    work = [w.clone() for w in base]
    kinds = (("rows", "rows", cfg.alpha_gate_up), ("rows", "rows", cfg.alpha_gate_up), ("cols", "cols", cfg.alpha_down))
    tasks = [(work[3 * s + k], norms[s], kinds[k][0], kinds[k][1], kinds[k][2]) for s in range(3) for k in range(3)]
    dass.score_mask_nm_batched(tasks, 2, 4)
    torch.cuda.synchronize()
    for s in range(3):
        for k in range(3):
            _check(work[3 * s + k], base[3 * s + k], norms[s], kinds[k][:2], kinds[k][2], 2, 4)
