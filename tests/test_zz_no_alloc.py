"""The entry point that allocates nothing (fdc_linear_static): through the C ABI
against fdc_linear (same kernels, so bit-identical) and against the plain fp64
product, on calls in a row that share the library's static scratch array, the
later ones with smaller inputs than the one before."""
import numpy as np
import pytest

from synth_inputs import draw_normal_bf16
from tests.helpers import rel_err

pytestmark = pytest.mark.gpu


def _case(torch, M, N, K, seed):
    from paper_2602_02864_amd import fdc_linear, fdc_linear_static, fdc_pack_weight
    rng = np.random.default_rng(seed)
    W = draw_normal_bf16(rng, (N, K), 0.02)
    x = rng.standard_normal((M, K)).astype(np.float32)
    wp = fdc_pack_weight(torch.from_numpy(W).cuda().to(torch.bfloat16).contiguous())
    xd = torch.from_numpy(x).cuda()
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    fdc_linear_static(xd, wp, N, out=y)                # nothing is allocated from here ...
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before     # ... to here
    ref = fdc_linear(xd, wp, N)
    torch.cuda.synchronize()
    got = y.cpu().numpy()
    assert np.isfinite(got).all()
    assert np.array_equal(got, ref.cpu().numpy()), (M, N, K)
    assert rel_err(got, x.astype(np.float64) @ W.astype(np.float64).T) < 2e-5


def test_static_scratch_linear_matches_the_workspace_entry_point_on_calls_in_a_row():
    import torch
    # split-K partials fill most of the array, then smaller calls reuse it:
    # streaming kernel with splits, one split, the tiled kernel, one row
    for i, (M, N, K) in enumerate([(16, 3584, 18944), (8, 4608, 3584), (5, 1000, 256), (16, 32000, 896),
                                   (40, 1000, 256), (129, 1152, 896), (1, 16, 32)]):
        _case(torch, M, N, K, 7000 + i)


def test_static_scratch_linear_refuses_what_does_not_fit():
    import torch
    from paper_2602_02864_amd import FdcError, binding as fb, fdc_linear_static
    M, N, K = 256, 37888, 3584
    assert fb.lib().fdc_linear_scratch_bytes(M, N, K) > (8 << 20)
    x = torch.zeros(M, K, device="cuda")
    w = torch.zeros(8, dtype=torch.bfloat16, device="cuda")      # never read: the size check comes first
    y = torch.zeros(M, N, device="cuda")
    with pytest.raises(FdcError) as e:
        fdc_linear_static(x, w, N, out=y)
    assert e.value.code == fb.FDC_ECAP
    # the array still works afterwards
    _case(torch, 3, 48, 64, 7100)
