"""moe_grouped_swiglu_static (the entry point that allocates nothing) against
moe_grouped_swiglu on the same inputs: same kernels, so the outputs must be bit-identical.
Two calls in a row, the second with fewer rows, so that what the first call left in the
library's scratch array cannot leak into the second result."""
import pytest
import torch

import paper_2604_10152_amd as sm

pytestmark = pytest.mark.gpu


def _case(rows_per_expert, d, f, dtype, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    E = len(rows_per_expert)
    n = sum(rows_per_expert)
    offs = torch.tensor([0] + list(torch.tensor(rows_per_expert).cumsum(0)), dtype=torch.int32,
                        device="cuda")
    x = (torch.randn(n, d, generator=g, device="cuda") / d ** 0.5).to(dtype)
    wg = (torch.randn(E, f, d, generator=g, device="cuda") * 0.05).to(dtype)
    wu = (torch.randn(E, f, d, generator=g, device="cuda") * 0.05).to(dtype)
    wd = (torch.randn(E, d, f, generator=g, device="cuda") * 0.05).to(dtype)
    return x, offs, wg, wu, wd


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_static_scratch_matches_workspace_variant(dtype):
    sm.load_library()
    d, f = 256, 512
    # first call: large enough to leave plenty of stale rows in the scratch array
    for rows, seed in (([300, 0, 37, 1, 513, 256, 330, 70], 5), ([9, 40, 0, 17, 3, 0, 0, 64], 6)):
        x, offs, wg, wu, wd = _case(rows, d, f, dtype, seed)
        n = x.shape[0]
        want = torch.full((n, d), float("nan"), dtype=dtype, device="cuda")
        got = torch.full((n, d), float("nan"), dtype=dtype, device="cuda")
        ws = torch.empty(sm.moe_grouped_swiglu_workspace_bytes(n, d, f, len(rows), dtype),
                         dtype=torch.uint8, device="cuda")
        sm.moe_grouped_swiglu(x, offs, wg, wu, wd, want, ws)
        sm.moe_grouped_swiglu_static(x, offs, wg, wu, wd, got)
        torch.cuda.synchronize()
        assert not torch.isnan(want.float()).any()
        assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), (dtype, rows)


def test_static_scratch_rejects_oversize():
    lib = sm.load_library()
    x, offs, wg, wu, wd = _case([4, 4], 64, 64, torch.bfloat16, 1)
    y = torch.empty(8, 64, dtype=torch.bfloat16, device="cuda")
    # n_rows * d_ff * 2 bytes just above the 16 MiB limit: rejected before any launch
    n_big, f_big = 8193, 1024
    st = lib.moe_grouped_swiglu_static(x.data_ptr(), offs.data_ptr(), wg.data_ptr(), wu.data_ptr(),
                                       wd.data_ptr(), n_big, 64, f_big, 2, 1, y.data_ptr(), None)
    assert st == 4
