"""GPU parity: dass_mlp_forward (Eq. 2 then Eq. 3, bf16) against the float64 oracle.

Tolerance, derived from the arithmetic.  bf16 keeps 8 significant bits: rounding to nearest has
relative error at most u = 2^-8.  With A = sum_i |y_i Wdown[j, i]| from the oracle:
  - y is rounded to bf16 once: every term of the Eq. 3 sum moves by at most u of itself, the sum
    by at most u A;
  - the f32 evaluation of y and the f32 accumulation of the K = d_int <= 28672 terms: rounding
    errors of 2^-24 relative that add like a random walk, about sqrt(K) 2^-24 A = 1e-5 A = 0.003 u A;
    0.05 u A leaves that a factor of 16 (the worst-case linear bound K 2^-24 A = 0.44 u A is never
    approached: it needs every one of 28672 roundings to go the same way);
  - the output is rounded to bf16 once: at most u of its value.
Hence |gpu - oracle| <= u |oracle| + 1.05 u A.  The first two terms are exact worst cases, so the
bound cannot be much tighter; observed: the worst element at 0.36 of it, the mean below 0.1.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2405_01943_amd as dass
from paper_2405_01943_amd import synth

from gpu_helpers import padded, to_np32

pytestmark = pytest.mark.gpu


def _check(out, ref, ab, what):
    out = np.asarray(out, dtype=np.float64)
    tol = 2.0 ** -8 * (np.abs(ref) + 1.05 * ab) + 1e-30
    err = np.abs(out - ref)
    worst = float(np.max(err / tol))
    assert worst <= 1.0, f"{what}: worst error / tolerance = {worst:.3f}"
    # a systematic error (a dropped K slab, a wrong row) would sit near the bound everywhere;
    # rounding noise averages far below it
    assert float(np.mean(err / tol)) < 0.25, what
    return worst


@pytest.mark.parametrize("act", ["silu", "gelu_tanh", "relu", "gelu_erf"])
@pytest.mark.parametrize("T,d,d_int,pad", [(300, 192, 320, 0), (513, 256, 448, 8), (256, 64, 64, 0), (70, 128, 704, 16)])
def test_forward_small_shapes(gpu_device, act, T, d, d_int, pad):
    g = torch.Generator(device="cpu").manual_seed(T + 7 * d + 13 * d_int)
    X = torch.randn((T, d), generator=g).to(torch.bfloat16).to(gpu_device)
    Wg = (torch.randn((d_int, d), generator=g) * 0.1).to(torch.bfloat16).to(gpu_device)
    Wu = (torch.randn((d_int, d), generator=g) * 0.1).to(torch.bfloat16).to(gpu_device)
    Wd = (torch.randn((d, d_int), generator=g) * 0.1).to(torch.bfloat16).to(gpu_device)
    out = torch.full((T, d), 3.0, dtype=torch.bfloat16, device=gpu_device)
    if pad:
        X, Wd, out = padded(X, pad), padded(Wd, pad), padded(out, pad)
        Wg = padded(Wg, pad)
        Wu = padded(Wu, pad)
    dass.mlp_forward(X, Wg, Wu, Wd, act, out)
    torch.cuda.synchronize()
    ref, ab = oracle.mlp_forward(to_np32(X), to_np32(Wg), to_np32(Wu), to_np32(Wd), act, want_abs=True)
    _check(to_np32(out), ref, ab, f"{act} T={T} d={d} d_int={d_int}")
    if pad:
        assert torch.all(out._base[:, d:] == 7.0)   # nothing written past a row's end


def test_forward_token_chunks_are_independent(gpu_device):
    """Rows of the output depend on their own token only: two halves equal the whole, bit for bit."""
    T, d, d_int = 700, 128, 256
    g = torch.Generator(device="cpu").manual_seed(3)
    X = torch.randn((T, d), generator=g).to(torch.bfloat16).to(gpu_device)
    Wg, Wu = ((torch.randn((d_int, d), generator=g) * 0.1).to(torch.bfloat16).to(gpu_device) for _ in range(2))
    Wd = (torch.randn((d, d_int), generator=g) * 0.1).to(torch.bfloat16).to(gpu_device)
    whole = torch.empty((T, d), dtype=torch.bfloat16, device=gpu_device)
    parts = torch.empty_like(whole)
    dass.mlp_forward(X, Wg, Wu, Wd, "silu", whole)
    dass.mlp_forward(X[:300], Wg, Wu, Wd, "silu", parts[:300])
    dass.mlp_forward(X[300:], Wg, Wu, Wd, "silu", parts[300:])
    torch.cuda.synchronize()
    assert torch.equal(whole.view(torch.int16), parts.view(torch.int16))


def test_forward_full_size_with_pruned_weights(gpu_device):
    """The LLaMA2-7B-shaped MLP with DaSS 2:4 weights on a 32768-token chunk of the calibration
    set, y in a workspace the binding allocates, checked on sampled tokens: all d outputs of the
    first and last token, of both sides of tile boundaries and of seeded random ones."""
    cfg = synth.CONFIGS["llama2_7b"]
    dev = gpu_device
    T, d, d_int = 32768, cfg.d, cfg.d_int
    X = synth.make_x(cfg, 0, T, dev)
    Wg, Wu, Wd = (synth.make_weight(cfg, w, dev) for w in ("wg", "wu", "wd"))
    norms = synth.make_norms(d_int, dev)
    dass.score_mask_nm(Wg, norms, "rows", "rows", 0.5, 2, 4)
    dass.score_mask_nm(Wu, norms, "rows", "rows", 0.5, 2, 4)
    dass.score_mask_nm(Wd, norms, "cols", "cols", 1.0, 2, 4)
    out = torch.empty((T, d), dtype=torch.bfloat16, device=dev)
    dass.mlp_forward(X, Wg, Wu, Wd, cfg.act, out)
    torch.cuda.synchronize()
    rng = np.random.default_rng(0)
    tokens = np.unique(np.concatenate([[0, 1, 255, 256, 257, 1023, 1024, T - 257, T - 256, T - 1],
                                       rng.integers(0, T, size=14)]))
    ref, ab = oracle.mlp_forward(to_np32(X[torch.as_tensor(tokens, device=dev)]), to_np32(Wg), to_np32(Wu),
                                 to_np32(Wd), cfg.act, want_abs=True)
    _check(to_np32(out[torch.as_tensor(tokens, device=dev)]), ref, ab, "7B shape, 2:4 weights")
    assert torch.isfinite(out.float()).all()


def test_forward_at_the_benchmark_token_count(gpu_device):
    """One call over all 262144 calibration tokens of the LLaMA2-7B-shaped MLP with DaSS 2:4 weights,
    as the benchmark times it (y, 5.7 GB, in the caller's workspace), and Eq. 3 again from the
    compressed Down-Proj over the same tokens; sampled tokens: the ends, both sides of tile
    boundaries at the start, the middle and the end of the token range, and seeded random ones."""
    cfg = synth.CONFIGS["llama2_7b"]
    dev = gpu_device
    T, d, d_int = cfg.tokens, cfg.d, cfg.d_int
    assert T == 262144
    X = synth.make_x(cfg, 0, T, dev)
    Wg, Wu, Wd = (synth.make_weight(cfg, w, dev) for w in ("wg", "wu", "wd"))
    norms = synth.make_norms(d_int, dev)
    dass.score_mask_nm(Wg, norms, "rows", "rows", 0.5, 2, 4)
    dass.score_mask_nm(Wu, norms, "rows", "rows", 0.5, 2, 4)
    dass.score_mask_nm(Wd, norms, "cols", "cols", 1.0, 2, 4)
    out = torch.empty((T, d), dtype=torch.bfloat16, device=dev)
    ws = torch.empty(dass.mlp_forward_workspace_bytes(T, d, d_int), dtype=torch.uint8, device=dev)
    dass.mlp_forward(X, Wg, Wu, Wd, cfg.act, out, workspace=ws)
    values = torch.empty((d, d_int // 2), dtype=Wd.dtype, device=dev)
    meta = torch.empty((d, d_int // 8), dtype=torch.uint8, device=dev)
    dass.compress_24(Wd, "cols", values, meta)
    Y = ws.view(torch.bfloat16).view(T, d_int)
    out3 = torch.empty_like(out)
    dass.down_proj_sparse24(Y, values, meta, out3)
    torch.cuda.synchronize()
    rng = np.random.default_rng(1)
    tokens = np.unique(np.concatenate([[0, 255, 256, 1023, 1024, T // 2 - 1, T // 2, T - 1025, T - 1024, T - 257,
                                        T - 256, T - 1], rng.integers(0, T, size=12)]))
    sel = torch.as_tensor(tokens, device=dev)
    ref, ab = oracle.mlp_forward(to_np32(X[sel]), to_np32(Wg), to_np32(Wu), to_np32(Wd), cfg.act, want_abs=True)
    _check(to_np32(out[sel]), ref, ab, "7B shape, 2:4 weights, 262144 tokens")
    ref3, ab3 = oracle.down_sparse24(to_np32(Y[sel]), to_np32(values), meta.cpu().numpy(), want_abs=True)
    err = np.abs(to_np32(out3[sel]).astype(np.float64) - ref3) / (2.0 ** -8 * (np.abs(ref3) + 0.5 * ab3) + 1e-30)
    assert float(err.max()) <= 1.0, f"sparse route at {err.max():.2f} of its tolerance"
    # every token was written: the two routes agree to bf16 rounding everywhere (they round y alike and
    # differ in the order of the f32 sums only)
    step = 4096
    for lo in range(0, T, step):
        a, b = out[lo:lo + step].float(), out3[lo:lo + step].float()
        assert torch.isfinite(a).all() and torch.isfinite(b).all()
        scale = a.abs().mean().item()
        assert scale > 0.0
        assert (a - b).abs().mean().item() <= 0.02 * scale, f"tokens {lo}..{lo + step}: the two routes differ"


@pytest.mark.parametrize("name", ["mistral_7b", "gemma_7b", "llama2_13b", "llama2_70b"])
def test_forward_other_model_shapes(gpu_device, name):
    """The other model shapes (tanh-GELU for the Gemma one; Gate + Up beyond the 256 MB cache for
    Gemma and 70B, which switches the tile order), a ragged token count, sampled tokens."""
    cfg = synth.CONFIGS[name]
    dev = gpu_device
    T, d, d_int = 1024 + 77, cfg.d, cfg.d_int
    X = synth.make_x(cfg, 0, T, dev)
    Wg, Wu, Wd = (synth.make_weight(cfg, w, dev) for w in ("wg", "wu", "wd"))
    out = torch.empty((T, d), dtype=torch.bfloat16, device=dev)
    dass.mlp_forward(X, Wg, Wu, Wd, cfg.act, out)
    # and Eq. 3 again from the compressed 2:4 Down-Proj, on the y the call left in its workspace
    ws = torch.empty(dass.mlp_forward_workspace_bytes(T, d, d_int), dtype=torch.uint8, device=dev)
    norms = synth.make_norms(d_int, dev)
    dass.score_mask_nm(Wd, norms, "cols", "cols", 1.0, 2, 4)
    out2 = torch.empty_like(out)
    dass.mlp_forward(X, Wg, Wu, Wd, cfg.act, out2, workspace=ws)
    values = torch.empty((d, d_int // 2), dtype=Wd.dtype, device=dev)
    meta = torch.empty((d, d_int // 8), dtype=torch.uint8, device=dev)
    dass.compress_24(Wd, "cols", values, meta)
    Y = ws.view(torch.bfloat16).view(T, d_int)
    out3 = torch.empty_like(out)
    dass.down_proj_sparse24(Y, values, meta, out3)
    torch.cuda.synchronize()
    tokens = np.array([0, 255, 256, 1023, 1024, T - 1])
    sel = torch.as_tensor(tokens, device=dev)
    Wd_dense = synth.make_weight(cfg, "wd", dev)
    ref, ab = oracle.mlp_forward(to_np32(X[sel]), to_np32(Wg), to_np32(Wu), to_np32(Wd_dense), cfg.act, want_abs=True)
    _check(to_np32(out[sel]), ref, ab, f"{name}, dense weights")
    ref2, ab2 = oracle.mlp_forward(to_np32(X[sel]), to_np32(Wg), to_np32(Wu), to_np32(Wd), cfg.act, want_abs=True)
    _check(to_np32(out2[sel]), ref2, ab2, f"{name}, 2:4 Down-Proj")
    ref3, ab3 = oracle.down_sparse24(to_np32(Y[sel]), to_np32(values), meta.cpu().numpy(), want_abs=True)
    err = np.abs(to_np32(out3[sel]).astype(np.float64) - ref3) / (2.0 ** -8 * (np.abs(ref3) + 0.5 * ab3) + 1e-30)
    assert float(err.max()) <= 1.0, f"{name}: sparse route at {err.max():.2f} of its tolerance"
