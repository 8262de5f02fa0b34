"""GPU check of dass_score_mask_unstructured_static, the entry point that allocates nothing: its
result must equal, bit for bit, that of dass_score_mask_unstructured given a workspace (which the
other tests compare with the oracle), on two calls in a row, the second on a smaller input, so
that what the first call left in the library's device scratch is seen not to leak."""
import ctypes

import pytest
import torch

import paper_2405_01943_amd as dass
from paper_2405_01943_amd import synth

pytestmark = pytest.mark.gpu


def _pair(rows, cols, dtype, norm_axis, group_axis, alpha, n_prune, device, seed, with_mask):
    g = torch.Generator(device="cpu").manual_seed(seed)
    W0 = (torch.randn((rows, cols), generator=g) * 0.02).to(dtype).to(device)
    norms = synth.make_norms(rows if norm_axis == "rows" else cols, device, seed=seed)
    a, b = W0.clone(), W0.clone()
    ma = torch.zeros(rows * cols // 8, dtype=torch.uint8, device=device) if with_mask else None
    mb = torch.zeros_like(ma) if with_mask else None
    ws = torch.empty(max(16, dass.unstructured_workspace_bytes(rows, cols, dtype, norm_axis, group_axis)),
                     dtype=torch.uint8, device=device)
    dass.score_mask_unstructured(a, norms, norm_axis, group_axis, alpha, n_prune, mask_out=ma, workspace=ws)
    dass.score_mask_unstructured_static(b, norms, norm_axis, group_axis, alpha, n_prune, mask_out=mb)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16 if dtype == torch.bfloat16 else torch.int32),
                       b.view(torch.int16 if dtype == torch.bfloat16 else torch.int32))
    if with_mask:
        assert torch.equal(ma, mb)
    n_lines = cols if group_axis == "rows" else rows
    assert int((b == 0).sum().item()) >= n_prune * n_lines    # it did prune


# alpha = 0.75 has no exact f32 recipe: the factor vector goes through the scratch and the multi-pass
# kernels read it.  alpha = 0.5 / 1 take the register-resident kernel (scratch untouched).
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("alpha", [0.75, 0.5, 1.0])
def test_static_scratch_two_calls_second_smaller(gpu_device, dtype, alpha):
    # Gate/Up form (lines are columns, factor per row), then Down form (lines are rows, factor per column)
    _pair(1536, 520, dtype, "rows", "rows", alpha, 700, gpu_device, seed=1, with_mask=True)
    _pair(264, 72, dtype, "rows", "rows", alpha, 131, gpu_device, seed=2, with_mask=False)
    _pair(300, 4104, dtype, "cols", "cols", alpha, 2052, gpu_device, seed=3, with_mask=False)
    _pair(37, 264, dtype, "cols", "cols", alpha, 100, gpu_device, seed=4, with_mask=True)


def test_static_scratch_long_column_lines_and_limit(gpu_device):
    # column lines longer than the register-resident kernel holds: the static form has no room for the
    # transposed copy and takes the multi-pass kernels; same bits
    _pair(16392, 64, torch.bfloat16, "rows", "rows", 0.5, 8196, gpu_device, seed=5, with_mask=False)
    _pair(512, 64, torch.bfloat16, "rows", "rows", 0.5, 256, gpu_device, seed=6, with_mask=False)
    # beyond the scratch: a clear error, nothing touched
    W = torch.ones((65544, 8), dtype=torch.bfloat16, device=gpu_device)
    norms = torch.ones(65544, device=gpu_device)
    with pytest.raises(dass.DassError) as e:
        dass.score_mask_unstructured_static(W, norms, "rows", "cols", 1.0, 4)
    assert e.value.status_name == "DASS_ERR_WORKSPACE" and "65536" in str(e.value)
    torch.cuda.synchronize()
    assert bool(torch.all(W == 1))
