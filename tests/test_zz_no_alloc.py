"""sfmp_gemm_static: the entry point that allocates nothing (scratch = a static device array of the library).

Its output must equal sfmp_gemm's bit for bit, on two calls in a row of which the second is smaller (the scratch keeps
the first call's contents), on every path that uses scratch memory; sizes beyond the static buffer are refused."""
import numpy as np
import pytest

import sfmp_workloads as W

pytestmark = pytest.mark.gpu


def _both(torch, S, p):
    from gpu_util import device_problem, run_gemm
    dp, cp, rp = device_problem(p)
    want = run_gemm(p, dp, cp, rp)
    X = torch.from_numpy(np.ascontiguousarray(p.X)).to("cuda:0")
    Y = torch.full((p.M, p.N), float("nan"), dtype=torch.float16, device="cuda:0")
    S.sfmp_gemm_static(X, cp, dp.layout, dp.s2, dp.s3, dp.s4, dp.index, dp.scales, dp.zeros, dp.bitmap, rp, Y)
    torch.cuda.synchronize()
    return want, Y.cpu().numpy()


# (K, N, M) pairs: a larger call, then a smaller one through the same scratch memory
@pytest.mark.parametrize("first,second", [
    ((4352, 512, 8), (1024, 384, 6)),      # staged activations of the small-batch kernel
    ((2048, 1024, 200), (1024, 512, 40)),  # matrix-core path: gathered activations, product before the un-permute
    ((4096, 2048, 200), (4096, 256, 40)),  # split K with fp32 partial products, then chunks of 16 rows
    ((1024, 512, 300), (512, 512, 1)),     # a call that needs no scratch after one that does
])
def test_static_scratch_matches_workspace_entry_point(first, second):
    import torch
    import paper_2602_01027_amd as S
    assert torch.cuda.is_available()
    for i, (K, N, M) in enumerate((first, second)):
        p = W.make_problem("static", K, N, M, 8800 + K + N + M, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3}, outliers=True,
                           fast_codes=True)
        assert S.sfmp_gemm_workspace(S.sfmp_pack(p.codes, p.bitmap)[0], M) <= 16 * 2 ** 20
        want, got = _both(torch, S, p)
        assert np.isfinite(got.astype(np.float32)).all()
        assert np.array_equal(want.view(np.uint16), got.view(np.uint16)), (i, K, N, M)


def test_static_scratch_refuses_what_does_not_fit():
    import torch
    import paper_2602_01027_amd as S
    from gpu_util import device_problem
    p = W.make_problem("static.big", 4096, 1024, 2048, 8899, fractions={3: 0.5, 4: 0.5}, fast_codes=True)
    dp, cp, rp = device_problem(p)
    assert S.sfmp_gemm_workspace(dp.layout, p.M) > 16 * 2 ** 20
    X = torch.from_numpy(p.X).to("cuda:0")
    Y = torch.zeros((p.M, p.N), dtype=torch.float16, device="cuda:0")
    with pytest.raises(S.SfmpError) as e:
        S.sfmp_gemm_static(X, cp, dp.layout, dp.s2, dp.s3, dp.s4, dp.index, dp.scales, dp.zeros, dp.bitmap, rp, Y)
    assert e.value.code == -10
    assert "static" in str(e.value)
