"""GPU: the library's calls are plain stream work (kernel launches only, no allocation, no
synchronisation), so a whole pruning step can be captured into a HIP graph and replayed.  Every
replay is checked like an eager run, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import oracle
import paper_2405_01943_amd as dass

from gpu_helpers import bits_equal, first_mismatch, to_np32

pytestmark = pytest.mark.gpu


def test_pruning_step_replayed_from_a_graph(gpu_device):
    dev = gpu_device
    T, d, d_int, act = 1536, 256, 704, "silu"
    g = torch.Generator(device="cpu").manual_seed(21)
    X = torch.randn((T, d), generator=g).to(torch.bfloat16).to(dev)
    W0 = [(torch.randn(shape, generator=g) * 0.05).to(torch.bfloat16).to(dev)
          for shape in ((d_int, d), (d_int, d), (d, d_int))]
    W = [w.clone() for w in W0]
    sumsq = torch.empty(d_int, device=dev)
    norms = torch.empty(d_int, device=dev)
    in_sumsq = torch.empty(d, device=dev)
    in_norms = torch.empty(d, device=dev)
    ws_in = torch.empty(max(16, dass.input_norms_workspace_bytes(T, d)), dtype=torch.uint8, device=dev)
    ws_nm = torch.empty(max(16, dass.nm_workspace_bytes(d_int, d, "rows"), dass.nm_workspace_bytes(d, d_int, "cols")),
                        dtype=torch.uint8, device=dev)
    vals = torch.empty((d, d_int // 2), dtype=torch.bfloat16, device=dev)
    meta = torch.empty((d, d_int // 8), dtype=torch.uint8, device=dev)
    nxt = torch.empty((T, d), dtype=torch.bfloat16, device=dev)
    ws_f = torch.empty(dass.mlp_forward_workspace_bytes(T, d, d_int), dtype=torch.uint8, device=dev)
    kinds = (("rows", 0.5), ("rows", 0.5), ("cols", 1.0))

    def step():
        for w, w0 in zip(W, W0):
            w.copy_(w0)
        dass.calib_norms(X, W0[0], W0[1], act, sumsq, norms_out=norms)
        dass.input_norms(X, in_sumsq, norms_out=in_norms, workspace=ws_in)
        for w, (axis, alpha) in zip(W, kinds):
            dass.score_mask_nm(w, norms, axis, axis, alpha, 2, 4, workspace=ws_nm)
        dass.compress_24(W[2], "cols", vals, meta)
        dass.mlp_forward(X, W[0], W[1], W[2], act, nxt, workspace=ws_f)

    def check(tag):
        n32 = norms.cpu().numpy()
        want = oracle.norms(oracle.sumsq(to_np32(X), to_np32(W0[0]), to_np32(W0[1]), act))
        assert float(np.max(np.abs(n32 - want) / want)) <= 2e-3, tag
        for w, w0, (axis, alpha) in zip(W, W0, kinds):
            ref, _ = oracle.mask_nm(to_np32(w0), n32, axis, axis, alpha, 2, 4)
            assert bits_equal(w, ref), f"{tag}: {first_mismatch(w, ref)}"
        ov, om, _ = oracle.compress_24(to_np32(W[2]), "cols")
        assert np.array_equal(to_np32(vals).view(np.uint32), ov.view(np.uint32)), tag
        assert np.array_equal(meta.cpu().numpy(), om), tag
        ref, ab = oracle.mlp_forward(to_np32(X), *(to_np32(w) for w in W), act, want_abs=True)
        err = np.abs(to_np32(nxt).astype(np.float64) - ref) / (2.0 ** -8 * (np.abs(ref) + 1.05 * ab) + 1e-30)
        assert float(err.max()) <= 1.0, f"{tag}: block output at {err.max():.2f} of its tolerance"
        return in_norms.clone()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                       # eager, also warms every kernel up before the capture
    side.synchronize()
    eager_in = check("eager")

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for replay in range(3):
        for t in (sumsq, norms, in_sumsq, in_norms):    # eager work between the replays
            t.fill_(-1.0)
        for t in (*W, vals, nxt):
            t.zero_()
        meta.fill_(0xEE)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got_in = check(f"replay {replay}")
        # the pass without atomics gives the same bits every time
        assert torch.equal(got_in.view(torch.int32), eager_in.view(torch.int32))


def test_unstructured_selection_replayed_from_a_graph(gpu_device):
    """The per-line unstructured selection of a large Gate-Proj-shaped and Down-Proj-shaped matrix (the
    passes over 64-column tiles: six launches that hand results to one another through the workspace,
    and the one-launch row-line kernel, each followed by its gated second try) captured and replayed;
    among the matrices one that the passes hand over to the second try (a column of equal scores)."""
    dev = gpu_device
    d, d_int = 1032, 2048
    g = torch.Generator(device="cpu").manual_seed(33)
    Wg0 = (torch.randn((d_int, d), generator=g) * 0.02).to(torch.bfloat16)
    Wd0 = (torch.randn((d, d_int), generator=g) * 0.02).to(torch.bfloat16)
    Wt0 = Wg0.clone()
    Wt0[:, 3] = 0.25                                   # equal scores wherever the norms are equal
    norms = (torch.rand(d_int, generator=g) * 30 + 0.01)
    norms_t = norms.clone()
    norms_t[: d_int // 2] = 4.0
    Wg0, Wd0, Wt0, norms, norms_t = (t.to(dev) for t in (Wg0, Wd0, Wt0, norms, norms_t))
    Wg, Wd, Wt = Wg0.clone(), Wd0.clone(), Wt0.clone()
    ws = [torch.empty(dass.unstructured_workspace_bytes(*w.shape, w.dtype, axis, axis), dtype=torch.uint8, device=dev)
          for w, axis in ((Wg, "rows"), (Wd, "cols"), (Wt, "rows"))]

    def step():
        Wg.copy_(Wg0)
        Wd.copy_(Wd0)
        Wt.copy_(Wt0)
        dass.score_mask_unstructured(Wg, norms, "rows", "rows", 0.5, d_int // 2, workspace=ws[0])
        dass.score_mask_unstructured(Wd, norms, "cols", "cols", 1.0, d_int // 2, workspace=ws[1])
        dass.score_mask_unstructured(Wt, norms_t, "rows", "rows", 1.0, d_int // 2, workspace=ws[2])

    want = [oracle.mask_unstructured(to_np32(w0), n.cpu().numpy(), axis, axis, alpha, d_int // 2)[0]
            for w0, n, axis, alpha in ((Wg0, norms, "rows", 0.5), (Wd0, norms, "cols", 1.0), (Wt0, norms_t, "rows", 1.0))]

    def check(tag):
        for w, ref in zip((Wg, Wd, Wt), want):
            assert bits_equal(w, ref), f"{tag}: {first_mismatch(w, ref)}"

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    side.synchronize()
    check("eager")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for replay in range(3):
        for t in (Wg, Wd, Wt, *ws):                      # eager work between the replays
            t.fill_(0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        check(f"replay {replay}")
