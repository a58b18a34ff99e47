"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Integer work (packed bytes, unpacked codes) must match bit for bit; fp16 outputs must be within
a relative Frobenius error of 2e-3 of the float64 oracle (the stated acceptance bound) - over the whole output and
over every tile row of it on its own - and every element within the bound derived from the kernels' arithmetic
(tests/gpu_util.py).  Workspaces are handed over filled with 0xFF bytes.
"""
import dataclasses

import numpy as np
import pytest

from oracle import sfmp_oracle as O
import sfmp_workloads as W

pytestmark = pytest.mark.gpu
TOL = 2e-3


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (no fallback path exists)")
    return torch


def _check(p, Y, rows=None, m_rows=None, elementwise=True):
    """Compare Y (fp16 [M,N]) with the oracle: relative Frobenius error <= 2e-3 overall and per tile row, and the
    derived per-element bound (tests/gpu_util.py).  `rows` = sampled reordered output features, `m_rows` = sampled
    activation rows (both default to everything)."""
    from gpu_util import check_against_oracle
    err = check_against_oracle(p, Y, feature_rows=rows, m_rows=m_rows, elementwise=elementwise)
    if rows is None and m_rows is None and p.N * p.K <= 16 * 2 ** 20:
        # the oracle's own whole-product routine (row un-permutation included) on everything that is small
        ref = O.gemm(p.X, p.col_perm, p.codes, p.scales, p.zeros, p.row_perm)
        assert O.rel_frobenius(Y, ref) <= TOL
    return err


# ---------------------------------------------------------------------------------------------
# unpack: bit-exact
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("case", ["tiny", "all2", "all3", "all4", "ragged"])
def test_unpack_bit_exact(torch_cuda, case):
    import paper_2602_01027_amd as S
    from gpu_util import device_problem
    torch = torch_cuda
    if case == "tiny":
        p = W.make_problem("tiny", 512, 512, 1, 1000)
    elif case == "ragged":
        p = W.make_problem("r", 640, 384, 1, 77)
    else:
        b = int(case[-1])
        p = W.make_problem(case, 384, 256, 1, 80 + b, bitmap=np.full((2, 3), b, dtype=np.int8))
    # codes that exercise every bit of every field: replace by uniform random codes of the tile's width
    rng = np.random.default_rng(5)
    bm = np.repeat(np.repeat(p.bitmap, 128, axis=0), 128, axis=1)
    p = dataclasses.replace(p, codes=(rng.integers(0, 16, size=bm.shape) % (1 << bm)).astype(np.uint8))
    dp, _, _ = device_problem(p)
    out = torch.full((p.N, p.K), 255, dtype=torch.uint8, device="cuda:0")
    S.sfmp_unpack(dp.layout, dp.s2, dp.s3, dp.s4, dp.index, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.array_equal(got, p.codes)
    # and the oracle's own unpack of the library's packed bytes agrees (bytes <-> codes both ways)
    assert np.array_equal(O.unpack(p.N, p.K, dp.s2.cpu().numpy(), dp.s3.cpu().numpy(), dp.s4.cpu().numpy(),
                                   dp.index.cpu().numpy()), p.codes)


# ---------------------------------------------------------------------------------------------
# config 1 and small edge cases
# ---------------------------------------------------------------------------------------------
def test_config1_tiny(torch_cuda):
    from gpu_util import run_gemm
    for label, K, N, M, seed, kw in W.config_cases(1):
        p = W.make_problem(label, K, N, M, seed, **kw)
        _check(p, run_gemm(p))


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8, 15, 16, 17, 63, 64, 65, 130])
def test_edge_M_ragged_shape(torch_cuda, M):
    # N = 640 = 5 tile rows (ragged last workgroup of 4 tile rows), K = 896 = 7 tiles (ragged last K chunk)
    from gpu_util import run_gemm
    p = W.make_problem("edge", 896, 640, M, 4242, fractions=None, outliers=True)
    _check(p, run_gemm(p))


@pytest.mark.parametrize("variant", ["all2", "all3", "all4", "clustered", "no_perm", "col_only", "row_only"])
@pytest.mark.parametrize("M", [1, 7, 48])
def test_bitmap_and_permutation_variants(torch_cuda, variant, M):
    from gpu_util import run_gemm
    K, N = 1024, 512
    kw = dict(fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3})
    if variant.startswith("all"):
        kw["bitmap"] = np.full((N // 128, K // 128), int(variant[-1]), dtype=np.int8)
    elif variant == "clustered":
        kw["bitmap"] = W.clustered_bitmap(N // 128, K // 128, {2: 0.5, 3: 0.25, 4: 0.25})
    elif variant == "no_perm":
        kw.update(use_col_perm=False, use_row_perm=False)
    elif variant == "col_only":
        kw.update(use_row_perm=False)
    elif variant == "row_only":
        kw.update(use_col_perm=False)
    p = W.make_problem(variant, K, N, M, 99, **kw)
    _check(p, run_gemm(p))


@pytest.mark.parametrize("K,N,M", [(66560, 256, 1), (66560, 256, 3), (66560, 256, 16), (128, 66048, 2)])
def test_decode_extreme_aspect(torch_cuda, K, N, M):
    # K = 520 tiles: more than 64 work items per wavefront, and an activation vector too long for the M = 1
    # kernel's LDS; N = 516 tile rows: more than 16 slabs per workgroup with one workgroup per CU
    from gpu_util import run_gemm
    p = W.make_problem("aspect", K, N, M, 777, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3}, fast_codes=True)
    _check(p, run_gemm(p))


@pytest.mark.parametrize("K,M", [(8192, 2), (5504, 2), (8192, 3), (5632, 3), (8192, 4), (4096, 4), (4096, 5)])
def test_small_batch_both_activation_stagings(torch_cuda, K, M):
    # M <= 4: up to 32 KiB of activations (M x K fp16) are staged into LDS by the kernel itself, larger ones by a
    # separate launch into the workspace; both sides of that limit, the limit itself ((8192, 2), (4096, 4)) and an
    # odd number of tile columns
    from gpu_util import run_gemm
    p = W.make_problem("staging", K, 384, M, 5150 + K + M, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3}, outliers=True,
                       fast_codes=True)
    _check(p, run_gemm(p))


@pytest.mark.parametrize("K,N,M", [
    (1024, 28672, 2),   # resident activations, 16 wavefronts, 7 slabs per workgroup in registers (8-wide vectors)
    (4352, 28672, 4),   # 4 rows, activations too large to be resident (34 KiB): staged, 16 wavefronts
    (1024, 28672, 8),   # 8 rows through the rings, 16 wavefronts
    (512, 40960, 3),    # 10 slabs per workgroup: 8 wavefronts, 16-wide vectors, resident
    (4352, 40960, 4),   # the same, staged
    (1024, 40960, 7),   # the same, 8 rows
    (1024, 40960, 12),  # 16 rows (always 8 wavefronts)
])
def test_ring_kernel_configurations(torch_cuda, K, N, M):
    # the compiled forms of the small-batch kernel that the layer shapes above do not reach: wide matrices put more
    # than 4 (more than 8) slabs on a workgroup.  Sampled output features, every tile row hit.
    from gpu_util import run_gemm
    p = W.make_problem("ringcfg", K, N, M, 6200 + N // 128 + M, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3}, fast_codes=True)
    rng = np.random.default_rng(M)
    rows = np.unique(np.concatenate([np.arange(N // 128) * 128 + rng.integers(0, 128, N // 128),
                                     rng.choice(N, size=128, replace=False)]))
    _check(p, run_gemm(p), rows=rows)


def test_batched_small_batch_mixed_staging(torch_cuda):
    # one problem whose activations would fit the in-kernel staging and one whose do not: the batch takes the
    # staged path for both, and gives bit for bit what separate calls (which differ in path) give
    import paper_2602_01027_amd as S
    from gpu_util import device_problem, run_gemm
    torch = torch_cuda
    M = 2
    probs = [W.make_problem("fits", 2048, 384, M, 61, fractions={2: 0.5, 4: 0.5}),
             W.make_problem("too_long", 16384, 256, M, 62, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3}, fast_codes=True)]
    batch, keep = [], []
    for p in probs:
        dp, cp, rp = device_problem(p)
        Y = torch.full((M, p.N), float("nan"), dtype=torch.float16, device="cuda:0")
        batch.append((torch.from_numpy(p.X).to("cuda:0"), cp, dp, rp, Y))
        keep.append((dp, cp, rp))
    ws = torch.empty(S.sfmp_gemm_batched_workspace(batch, M), dtype=torch.uint8, device="cuda:0").fill_(0xFF)
    S.sfmp_gemm_batched(batch, M, ws)
    torch.cuda.synchronize()
    for p, (_, _, _, _, Y), (dp, cp, rp) in zip(probs, batch, keep):
        y = Y.cpu().numpy()
        _check(p, y)
        assert np.array_equal(run_gemm(p, dp, cp, rp).view(np.uint16), y.view(np.uint16))


@pytest.mark.parametrize("K,N,M", [(4096, 512, 17), (4096, 512, 100), (4096, 1024, 128), (4096, 1152, 128),
                                   (4096, 4096, 32), (4096, 4096, 33), (4096, 8192, 64), (4096, 4096, 96), (4096, 4096, 97),
                                   (4096, 6144, 64), (4096, 6144, 65), (4096, 14336, 32), (4096, 14336, 33),
                                   (8192, 8192, 32), (8192, 8192, 40), (14336, 4096, 32), (14336, 4096, 33)])
def test_medium_batch_chunked_and_prefill_sides(torch_cuda, K, N, M):
    # 16 < M <= 128 with K >= 4096: chunks of 16 rows through the batched ring kernel where that measured faster
    # (last chunk of 1 and of 4 rows, the full 8 chunks; with K <= 8192 two chunks on any matrix, four up to 1536 tiles,
    # six up to 1024; two on N <= 4096 with a longer K), the MFMA kernel with a split K beyond; both sides of each limit
    from gpu_util import run_gemm
    p = W.make_problem("medium", K, N, M, 6200 + N + M, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3}, outliers=True,
                       fast_codes=True)
    rows = None if N <= 512 else np.random.default_rng(M).choice(N, 384, replace=False)
    _check(p, run_gemm(p), rows)


@pytest.mark.parametrize("K,N,M,row_perm", [(4096, 16384, 40, False), (4096, 2048, 200, True), (3072, 1024, 300, False)])
def test_short_prompt_split_k(torch_cuda, K, N, M, row_perm):
    # few workgroups otherwise: K cut into 3 to 8 ranges with fp32 partial products and a reduction pass; with and
    # without the row un-permute folded into that pass, ragged M, 64-row blocks
    from gpu_util import run_gemm
    p = W.make_problem("splitk", K, N, M, 7300 + N + M, fractions={2: 0.25, 3: 0.25, 4: 0.5}, outliers=True,
                       fast_codes=True, use_row_perm=row_perm)
    assert (p.row_perm is not None) == row_perm
    rows = np.random.default_rng(M).choice(N, 384, replace=False)
    y1 = run_gemm(p)
    _check(p, y1, rows)
    assert np.array_equal(y1.view(np.uint16), run_gemm(p).view(np.uint16))  # fixed reduction order


def test_workspace_is_reusable_and_result_deterministic(torch_cuda):
    from gpu_util import device_problem, make_workspace, run_gemm
    p = W.make_problem("reuse", 2048, 1024, 4, 31337, fractions={2: 0.5, 3: 0.5}, outliers=True)
    dp, cp, rp = device_problem(p)
    ws = make_workspace(dp.layout, p.M)
    y1 = run_gemm(p, dp, cp, rp, ws)
    y2 = run_gemm(p, dp, cp, rp, ws)
    _check(p, y1)
    assert np.array_equal(y1.view(np.uint16), y2.view(np.uint16))
    # a second, smaller M through the same (larger) workspace
    p1 = W.with_activations(p, 1, outliers=True)
    _check(p1, run_gemm(p1, dp, cp, rp, ws))


def test_gemm_argument_errors(torch_cuda):
    import ctypes as C
    import paper_2602_01027_amd as S
    from gpu_util import device_problem
    torch = torch_cuda
    p = W.make_problem("err", 1024, 256, 4, 3)
    dp, cp, rp = device_problem(p)
    X = torch.from_numpy(p.X).to("cuda:0")
    Y = torch.empty((4, p.N), dtype=torch.float16, device="cuda:0")
    small = torch.zeros(256, dtype=torch.uint8, device="cuda:0")
    need = S.sfmp_gemm_workspace(dp.layout, 4)
    assert need > 256
    with pytest.raises(S.SfmpError) as ei:
        S.sfmp_gemm(X, cp, dp.layout, dp.s2, dp.s3, dp.s4, dp.index, dp.scales, dp.zeros, dp.bitmap, rp, Y, small)
    assert ei.value.code == -5


# ---------------------------------------------------------------------------------------------
# the benchmark configurations at full size
# ---------------------------------------------------------------------------------------------
_CACHE = {}


def _config_problem(cid, si):
    """Weights / bitmap / permutations of shape si of config cid (shared by all its M values)."""
    key = (cid, si)
    if key not in _CACHE:
        _CACHE.clear()  # keep one big layer in host memory at a time
        spec = W.CONFIGS[cid]
        label, K, N = spec.shapes[si]
        p = W.make_problem(label, K, N, 1, 1000 * cid + si, w_std=spec.w_std[si], fractions=spec.fractions,
                           outliers=spec.outliers, use_col_perm=spec.col_perm, use_row_perm=spec.row_perm[si])
        _CACHE[key] = p
    return _CACHE[key]


def _distinct_shapes(cid):
    seen, out = set(), []
    for si, (label, K, N) in enumerate(W.CONFIGS[cid].shapes):
        if (K, N) not in seen:
            seen.add((K, N))
            out.append(si)
    return out


def _prefill_row_subset(M, seed):
    """Activation rows compared on the largest prefill shapes: the first and the last row of every 64-row block
    (the kernels' blocks are 64, 128 or 256 rows) plus 16 random rows.  Every output row touches every weight tile,
    so all N output features of these rows exercise the whole matrix."""
    edges = np.concatenate([np.arange(0, M, 64), np.arange(63, M, 64), [M - 1]])
    extra = np.random.default_rng(seed).choice(M, size=min(16, M), replace=False)
    return np.unique(np.concatenate([edges, extra]))


def _run_config_shape(cid, si):
    """One shape of a benchmark configuration at full size, every M of the configuration.  Every output feature is
    compared (the oracle walks the matrix in blocks of 1024 features); for M = 2048 on matrices above 64 Mi weights
    a documented subset of the activation rows."""
    from gpu_util import device_problem, run_gemm
    spec = W.CONFIGS[cid]
    base = _config_problem(cid, si)
    dp, cp, rp = device_problem(base)
    errs = {}
    for M in spec.Ms:
        p = W.with_activations(base, M, outliers=spec.outliers)
        m_rows = None
        if M > 256 and base.N * base.K > 64 * 2 ** 20:
            m_rows = _prefill_row_subset(M, cid * 100 + si)
        errs[M] = _check(p, run_gemm(p, dp, cp, rp), m_rows=m_rows)
    print(f"config {cid} {base.label} K={base.K} N={base.N} avg_bits={base.avg_bits:.3f} rel_frob={errs}", flush=True)


@pytest.mark.parametrize("si", _distinct_shapes(2))
def test_config2_8b_decode(torch_cuda, si):
    _run_config_shape(2, si)


@pytest.mark.parametrize("si", _distinct_shapes(3))
def test_config3_8b_fractional(torch_cuda, si):
    _run_config_shape(3, si)


@pytest.mark.parametrize("si", _distinct_shapes(4))
def test_config4_70b_decode(torch_cuda, si):
    _run_config_shape(4, si)


@pytest.mark.parametrize("si", _distinct_shapes(5))
def test_config5_prefill(torch_cuda, si):
    _run_config_shape(5, si)


def test_bench_step_replayed_as_graph_matches_oracle(torch_cuda):
    """The step that bench.py times, exactly as it launches it: the seven projections of the 8B decode layer
    (configs[1], fully quantised) in four launches (q|k|v, o, gate|up, down through sfmp_gemv_batched), captured in one
    HIP graph per weight replica and replayed in rotation.  All seven outputs of every replay against the oracle."""
    import bench
    torch = torch_cuda
    problems = bench.build_problems(W, 2)
    layer = bench.Layer(problems, 3)
    graphs = bench.capture_step_graphs(torch, layer, bench.FUSED_GROUPS)
    first = None
    for rnd in range(2):
        for r, g in enumerate(graphs):
            for d in layer.proj:
                d["Y"].fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            ys = [d["Y"].cpu().numpy() for d in layer.proj]
            if first is None:
                first = ys
                for p, y in zip(problems, ys):
                    _check(p, y)
            else:  # the replicas hold the same weights: every replay must repeat the first bit for bit
                for y0, y in zip(first, ys):
                    assert np.array_equal(y0.view(np.uint16), y.view(np.uint16)), (rnd, r)


@pytest.mark.parametrize("M", [4, 16, 40])
def test_small_batch_calls_replayed_as_graph(torch_cuda, M):
    """Small-batch calls under HIP-graph capture: a batched launch of three projections over shared activations (staging
    kernel + ring kernel; at M = 4 the resident form, at M = 16 the activations in registers), one long-K call whose
    activations travel through the ring slots, and at M = 40 the chunked form, all in one graph.  Replayed three times
    with new activations written by eager work between the replays; every replay bit for bit what eager calls give."""
    import dataclasses
    import paper_2602_01027_amd as S
    from gpu_util import device_problem, make_workspace
    torch = torch_cuda
    base = W.make_problem("g0", 1024, 512, M, 8900 + M, fractions={2: 0.5, 3: 0.5}, outliers=True)
    shared = [base] + [dataclasses.replace(W.make_problem(f"g{i}", 1024, n, M, 8910 + i), X=base.X, col_perm=base.col_perm)
                       for i, n in enumerate((256, 384), 1)]
    longk = W.make_problem("gl", 9216, 256, M, 8920)
    Xs = torch.from_numpy(base.X).to("cuda:0")
    Xl = torch.from_numpy(longk.X).to("cuda:0")
    cps = torch.from_numpy(base.col_perm).to("cuda:0")
    batch, keep = [], []
    for p in shared:
        dp, cp, rp = device_problem(p)
        batch.append((Xs, cps, dp, rp, torch.empty((M, p.N), dtype=torch.float16, device="cuda:0")))
        keep.append(dp)
    dl, cpl, rpl = device_problem(longk)
    Yl = torch.empty((M, longk.N), dtype=torch.float16, device="cuda:0")
    wsl = make_workspace(dl.layout, M)
    use_batched = M <= 16
    if use_batched:
        wsb = torch.empty(S.sfmp_gemm_batched_workspace(batch, M), dtype=torch.uint8, device="cuda:0").fill_(0xFF)
    else:
        wss = [make_workspace(b[2].layout, M) for b in batch]

    def launch(stream):
        if use_batched:
            S.sfmp_gemm_batched(batch, M, wsb, stream=stream)
        else:
            for (X, cp, dp, rp, Y), ws in zip(batch, wss):
                S.sfmp_gemm(X, cp, dp.layout, dp.s2, dp.s3, dp.s4, dp.index, dp.scales, dp.zeros, dp.bitmap, rp, Y, ws, stream=stream)
        S.sfmp_gemm(Xl, cpl, dl.layout, dl.s2, dl.s3, dl.s4, dl.index, dl.scales, dl.zeros, dl.bitmap, rpl, Yl, wsl, stream=stream)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        launch(side)
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        launch(torch.cuda.current_stream())
    torch.cuda.synchronize()
    rng = np.random.default_rng(77)
    for rep in range(3):
        # new activations (eager copies), outputs poisoned, workspaces poisoned
        xs = (rng.normal(size=base.X.shape)).astype(np.float16)
        xl = (rng.normal(size=longk.X.shape)).astype(np.float16)
        Xs.copy_(torch.from_numpy(xs)); Xl.copy_(torch.from_numpy(xl))
        for b in batch:
            b[4].fill_(float("nan"))
        Yl.fill_(float("nan"))
        wsl.fill_(0xFF)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = [b[4].cpu().numpy().copy() for b in batch] + [Yl.cpu().numpy().copy()]
        for b in batch:
            b[4].fill_(float("nan"))
        Yl.fill_(float("nan"))
        launch(torch.cuda.current_stream())
        torch.cuda.synchronize()
        eager = [b[4].cpu().numpy() for b in batch] + [Yl.cpu().numpy()]
        for a, e in zip(got, eager):
            assert np.isfinite(a.astype(np.float32)).all()
            assert np.array_equal(a.view(np.uint16), e.view(np.uint16)), rep
        if rep == 0:  # and the values are right
            for p, y, x in zip(shared + [longk], got, [xs, xs, xs, xl]):
                _check(dataclasses.replace(p, X=x), y)


# ---------------------------------------------------------------------------------------------
# several M = 1 problems in one launch
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("shapes", [[(512, 512)], [(896, 640), (512, 1024), (1024, 256)],
                                    [(4096, 4096), (4096, 1024), (4096, 1024)], [(4096, 14336), (4096, 14336)]])
def test_gemv_batched(torch_cuda, shapes):
    import paper_2602_01027_amd as S
    from gpu_util import device_problem
    torch = torch_cuda
    probs, batch = [], []
    for i, (K, N) in enumerate(shapes):
        p = W.make_problem(f"b{i}", K, N, 1, 7000 + 13 * i + K, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3},
                           use_row_perm=(i % 2 == 0), use_col_perm=(i != 1))
        dp, cp, rp = device_problem(p)
        X = torch.from_numpy(p.X).to("cuda:0")
        Y = torch.full((1, N), float("nan"), dtype=torch.float16, device="cuda:0")
        probs.append(p)
        batch.append((X, cp, dp, rp, Y))
    S.sfmp_gemv_batched(batch)
    torch.cuda.synchronize()
    for p, (_, _, _, _, Y) in zip(probs, batch):
        _check(p, Y.cpu().numpy())
    # the batched launch computes exactly what separate launches compute
    from gpu_util import run_gemm
    for p, (_, cp, dp, rp, Y) in zip(probs, batch):
        y_single = run_gemm(p, dp, cp, rp)
        assert np.array_equal(y_single.view(np.uint16), Y.cpu().numpy().view(np.uint16))


@pytest.mark.parametrize("M", [1, 2, 4, 7, 16])
def test_gemm_batched_shared_activations(torch_cuda, M):
    # q|k|v-like: three matrices over the same activations and column permutation (one staged copy), plus a fourth
    # problem with its own activations, K and no column permutation
    import dataclasses
    import paper_2602_01027_amd as S
    from gpu_util import device_problem, run_gemm
    torch = torch_cuda
    base = W.make_problem("s0", 1024, 512, M, 8100, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3}, outliers=True)
    probs = [base]
    for i, N in enumerate((256, 384)):
        q = W.make_problem(f"s{i + 1}", 1024, N, M, 8200 + i, fractions={2: 0.5, 3: 0.5}, use_row_perm=(i == 0))
        probs.append(dataclasses.replace(q, X=base.X, col_perm=base.col_perm))
    probs.append(W.make_problem("own", 896, 640, M, 8300, fractions=None, use_col_perm=False))
    Xd = torch.from_numpy(base.X).to("cuda:0")
    cpd = torch.from_numpy(base.col_perm).to("cuda:0")
    batch, keep = [], []
    for i, p in enumerate(probs):
        dp, cp, rp = device_problem(p)
        X = Xd if i < 3 else torch.from_numpy(p.X).to("cuda:0")
        Y = torch.full((M, p.N), float("nan"), dtype=torch.float16, device="cuda:0")
        batch.append((X, cpd if i < 3 else None, dp, rp, Y))
        keep.append((dp, cp, rp))
    need = S.sfmp_gemm_batched_workspace(batch, M)
    shared = S.sfmp_gemm_batched_workspace(batch[:3], M)
    single = S.sfmp_gemm_batched_workspace(batch[:1], M)
    assert shared == single  # one staged copy for the three problems that share X and col_perm
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0").fill_(0xFF)
    S.sfmp_gemm_batched(batch, M, ws)
    torch.cuda.synchronize()
    for p, (_, _, _, _, Y), (dp, cp, rp) in zip(probs, batch, keep):
        y = Y.cpu().numpy()
        _check(p, y)
        # the batched launch computes exactly what separate launches compute
        assert np.array_equal(run_gemm(p, dp, cp, rp).view(np.uint16), y.view(np.uint16))


@pytest.mark.parametrize("M,group", [(2, 128), (5, 128), (16, 128), (3, 64), (16, 64)])
def test_gemm_batched_five_slabs_per_workgroup_short_K(torch_cuda, M, group):
    # two problems of 640 slabs on 128 workgroups each: five slabs per workgroup, with K = 2560 (20 tile columns:
    # wavefronts 0-3 have two, the others one) and K = 1024 (8 tile columns: half of the wavefronts have none); the
    # form of the small-batch kernel that keeps the activations in registers and every wavefront's sums in LDS
    import paper_2602_01027_amd as S
    from gpu_util import device_problem, run_gemm
    torch = torch_cuda
    probs = [W.make_problem("a", 2560, 10240, M, 8400, fractions={2: 0.5, 3: 0.5}, outliers=True, group=group),
             W.make_problem("b", 1024, 10240, M, 8401, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3}, group=group)]
    batch, keep = [], []
    for p in probs:
        dp, cp, rp = device_problem(p)
        X = torch.from_numpy(p.X).to("cuda:0")
        Y = torch.full((M, p.N), float("nan"), dtype=torch.float16, device="cuda:0")
        batch.append((X, cp, dp, rp, Y))
        keep.append((dp, cp, rp))
    ws = torch.empty(S.sfmp_gemm_batched_workspace(batch, M), dtype=torch.uint8, device="cuda:0").fill_(0xFF)
    S.sfmp_gemm_batched(batch, M, ws)
    torch.cuda.synchronize()
    for p, (_, _, _, _, Y), (dp, cp, rp) in zip(probs, batch, keep):
        y = Y.cpu().numpy()
        _check(p, y)
        assert np.array_equal(run_gemm(p, dp, cp, rp).view(np.uint16), y.view(np.uint16))


@pytest.mark.parametrize("K,N,M,group", [(5120, 1024, 6, 128), (8192, 2048, 16, 128), (8192, 1024, 9, 128), (6144, 1024, 3, 64),
                                         (8192, 1024, 16, 64), (8192, 1280, 16, 256)])
def test_small_batch_three_and_four_tile_columns_per_wavefront(torch_cuda, K, N, M, group):
    # 4096 < K <= 8192: the activations of a wavefront's three or four tile columns are held in registers (K = 5120:
    # wavefronts 0-7 have three tile columns, the others two; K = 6144 at group length 64: no resident form at M = 3)
    from gpu_util import run_gemm
    p = W.make_problem("ra4", K, N, M, 8600 + M + K // 128, fractions={2: 0.4, 3: 0.3, 4: 0.3}, outliers=True, group=group)
    _check(p, run_gemm(p))


@pytest.mark.parametrize("K,N,M,group", [(9216, 512, 5, 128), (14336, 1024, 16, 128), (14336, 4096, 16, 128), (28672, 1024, 8, 64),
                                         (16512, 384, 7, 128), (14336, 1024, 40, 128), (28672, 8192, 8, 256)])
def test_small_batch_long_K(torch_cuda, K, N, M, group):
    # K > 8192 at 5 <= M <= 16 (and chunks of 16 rows: M = 40): more tile columns per wavefront than fit in registers,
    # the activations travel through the ring slots; repeated calls give the same bits
    from gpu_util import device_problem, run_gemm
    p = W.make_problem("longk", K, N, M, 8700 + M + K // 128, fractions={2: 0.3, 3: 0.4, 4: 0.3}, outliers=True, group=group,
                       fast_codes=N * K > (1 << 27))
    dp, cp, rp = device_problem(p)
    Y = run_gemm(p, dp, cp, rp)
    if N * K > (1 << 27):
        _check(p, Y, m_rows=[0, M - 1])
    else:
        _check(p, Y)
    for _ in range(3):
        assert np.array_equal(run_gemm(p, dp, cp, rp).view(np.uint16), Y.view(np.uint16))


@pytest.mark.parametrize("K,N,M", [(1024, 40960, 3), (1024, 40960, 8), (4224, 36864, 8), (4224, 36864, 16)])
def test_small_batch_more_than_2048_slabs(torch_cuda, K, N, M):
    # more than 8 slabs per workgroup on 256 workgroups: the launch takes 512 workgroups (two per CU in turn, 5 slabs
    # each) and keeps 16 wavefronts; K = 1024 with the activations resident in LDS (M = 3) or in registers, K = 4224
    # (33 tile columns) with the activations travelling through the ring slots
    from gpu_util import run_gemm
    p = W.make_problem("wide", K, N, M, 8500 + M + K, fractions={2: 0.5, 3: 0.25, 4: 0.25})
    _check(p, run_gemm(p))


# ---------------------------------------------------------------------------------------------
# group lengths 256 / 512, bf16 parameters, (m_b, n_b) bit-allocation blocks
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("M", [1, 5, 16, 48, 200])
@pytest.mark.parametrize("group,scale_format,block", [(64, "fp16", (1, 1)), (64, "bf16", (4, 1)), (128, "bf16", (4, 1)),
                                                      (256, "fp16", (2, 2)), (256, "bf16", (4, 2)), (512, "bf16", (4, 4))])
def test_group_length_and_parameter_format(torch_cuda, group, scale_format, block, M):
    # K = 1536: 12 tile columns = 24 groups of 64 (two per tile) or 6 / 3 groups of 256 / 512; N = 1024: two
    # (512 x n_b) block rows.  M = 200: the matrix-core kernel with 128-row blocks
    from gpu_util import run_gemm
    p = W.make_problem("fmt", 1536, 1024, M, 606 + group, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3}, outliers=True,
                       group=group, scale_format=scale_format, block=block)
    assert p.scales.shape == (1536 // group, 1024)
    _check(p, run_gemm(p))


@pytest.mark.parametrize("M", [1, 8, 64])
def test_small_magnitude_weights_bf16_parameters(torch_cuda, M):
    # weights of standard deviation 1e-5 with bf16 scales and zeros: the scales (about 3e-6) lie below fp16's normal
    # range.  The decode kernels (M <= 16) widen the parameters to fp32 and meet the usual bounds.  The matrix-core path
    # (M = 64 here) converts them to fp16 and rounds the dequantised weight to fp16, which the header documents as
    # costing up to 2^-25 absolute per parameter and per weight below 2^-14: a code of at most 15 times the scale's
    # error, the zero's error and the weight's rounding give 17 * 2^-25 per weight on top of the usual bound.
    from gpu_util import run_gemm, elementwise_tolerance, FLOOR16
    p = W.make_problem("tinyw", 1024, 512, M, 4711, w_std=1e-5, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3},
                       scale_format="bf16")
    assert float(np.abs(p.scales).max()) < 2.0 ** -14
    Y = run_gemm(p)
    if M <= 16:
        _check(p, Y)
        return
    ref = O.gemm(p.X, p.col_perm, p.codes, p.scales, p.zeros, p.row_perm)
    w_hat = O.dequant(p.codes, p.scales, p.zeros)
    Xabs = np.abs(O.permute_activation(p.X, p.col_perm))
    A = Xabs @ np.abs(w_hat).T
    B = Xabs @ O.dequant(p.codes, np.abs(p.scales), np.abs(p.zeros)).T
    X1 = Xabs.sum(axis=1)[:, None]
    inv = np.empty_like(p.row_perm)
    inv[p.row_perm] = np.arange(p.N, dtype=np.int32)
    tol = elementwise_tolerance(M, p.K, ref[:, p.row_perm], A, B, X1) + 17 * FLOOR16 * X1
    assert np.all(np.abs(Y.astype(np.float64)[:, p.row_perm] - ref[:, p.row_perm]) <= tol)
    assert O.rel_frobenius(Y, ref) <= 2e-2  # degraded, as documented, but not garbage


@pytest.mark.parametrize("M", [1, 3, 12])
def test_batched_launch_group_64(torch_cuda, M):
    # group length 64 through the batched launches (GEMV, ring kernel); a batch that mixes it with another group
    # length is refused (one launch runs one group-length class)
    import paper_2602_01027_amd as S
    from gpu_util import device_problem, run_gemm
    torch = torch_cuda
    probs, batch, keep = [], [], []
    for i, (fmt, N) in enumerate([("fp16", 384), ("bf16", 256)]):
        p = W.make_problem(f"g64.{i}", 1024, N, M, 950 + i, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3}, group=64,
                           scale_format=fmt, outliers=True)
        dp, cp, rp = device_problem(p)
        Y = torch.full((M, p.N), float("nan"), dtype=torch.float16, device="cuda:0")
        probs.append(p)
        batch.append((torch.from_numpy(p.X).to("cuda:0"), cp, dp, rp, Y))
        keep.append((dp, cp, rp))
    ws = torch.empty(S.sfmp_gemm_batched_workspace(batch, M), dtype=torch.uint8, device="cuda:0").fill_(0xFF)
    S.sfmp_gemm_batched(batch, M, ws)
    torch.cuda.synchronize()
    for p, (_, _, _, _, Y), (dp, cp, rp) in zip(probs, batch, keep):
        y = Y.cpu().numpy()
        _check(p, y)
        assert np.array_equal(run_gemm(p, dp, cp, rp).view(np.uint16), y.view(np.uint16))
    other = W.make_problem("g128", 1024, 256, M, 960, fractions={2: 0.5, 4: 0.5})
    dpo, cpo, rpo = device_problem(other)
    Yo = torch.zeros((M, other.N), dtype=torch.float16, device="cuda:0")
    mixed = batch[:1] + [(torch.from_numpy(other.X).to("cuda:0"), cpo, dpo, rpo, Yo)]
    with pytest.raises(S.SfmpError) as e:
        S.sfmp_gemm_batched(mixed, M, ws)
    assert e.value.code == -2


def test_batched_launch_with_mixed_parameter_formats(torch_cuda):
    import paper_2602_01027_amd as S
    from gpu_util import device_problem
    torch = torch_cuda
    probs, batch = [], []
    for i, (group, fmt) in enumerate([(128, "fp16"), (256, "bf16"), (512, "fp16")]):
        p = W.make_problem(f"m{i}", 1024, 256 + 128 * i, 3, 900 + i, fractions={2: 0.5, 4: 0.5}, group=group,
                           scale_format=fmt, block=(1, group // 128))
        dp, cp, rp = device_problem(p)
        X = torch.from_numpy(p.X).to("cuda:0")
        Y = torch.full((3, p.N), float("nan"), dtype=torch.float16, device="cuda:0")
        probs.append(p)
        batch.append((X, cp, dp, rp, Y))
    ws = torch.empty(S.sfmp_gemm_batched_workspace(batch, 3), dtype=torch.uint8, device="cuda:0").fill_(0xFF)
    S.sfmp_gemm_batched(batch, 3, ws)
    torch.cuda.synchronize()
    for p, (_, _, _, _, Y) in zip(probs, batch):
        _check(p, Y.cpu().numpy())


@pytest.mark.parametrize("M", [1, 8, 40])
def test_allocated_bitmap_from_salience(torch_cuda, M):
    # the bitmap the offline side produces (sorted salience, Algorithm 1, (512, 128) blocks): wide tiles clustered
    from gpu_util import run_gemm
    lay = W.allocation.allocated_layout(2048, 1536, 2.75, np.random.default_rng(12), block=(4, 1))
    p = W.make_problem("alloc", 1536, 2048, M, 515, bitmap=lay["bitmap"], outliers=True)
    assert set(np.unique(p.bitmap).tolist()) == {2, 3, 4}
    _check(p, run_gemm(p))



# ---------------------------------------------------------------------------------------------
# permutation folding: the first product stays in reordered row order, the second gathers from it
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("M", [1, 4, 48])
def test_folded_permutations_two_matrix_chain(torch_cuda, M):
    import paper_2602_01027_amd as S
    from gpu_util import device_problem, run_gemm
    torch = torch_cuda
    p1 = W.make_problem("up", 512, 1024, M, 9100, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3}, outliers=True)
    p2 = W.make_problem("down", 1024, 384, M, 9200, fractions={2: 0.5, 3: 0.5})
    assert p1.row_perm is not None and p2.col_perm is not None
    dp1, cp1, rp1 = device_problem(p1)
    dp2, cp2, rp2 = device_problem(p2)
    relu = lambda y: np.maximum(y, np.float16(0))
    # plain: un-permute the first product, gather for the second
    Y1 = run_gemm(p1, dp1, cp1, rp1)
    _check(p1, Y1)
    X2 = relu(Y1)
    Y2 = run_gemm(p2, dp2, cp2, rp2, X=X2)
    _check(dataclasses.replace(p2, X=X2), Y2)
    # folded: no un-permute, one folded gather
    Y1t = run_gemm(p1, dp1, cp1, None)
    assert np.array_equal(Y1t.view(np.uint16), Y1[:, p1.row_perm].view(np.uint16))
    folded = S.sfmp_fold_perms(p1.row_perm, p2.col_perm)
    assert np.array_equal(folded, O.fold_perms(p1.row_perm, p2.col_perm))
    Y2f = run_gemm(p2, dp2, torch.from_numpy(folded).to("cuda:0"), rp2, X=relu(Y1t))
    assert np.array_equal(Y2f.view(np.uint16), Y2.view(np.uint16))


# ---------------------------------------------------------------------------------------------
# seeded random small shapes across the corners of the path selection
# ---------------------------------------------------------------------------------------------
def test_random_small_shapes(torch_cuda):
    # tile-row and tile-column counts around the limits of the decode forms (1, 16/17, 32/33, 64/65 tile columns per
    # 16 wavefronts; 8/9, 17, 33, 40 tile rows), every M class, all group lengths and both parameter formats, with and
    # without permutations and activation outliers; whole outputs against the oracle, and repeatable
    from gpu_util import device_problem, run_gemm
    rng = np.random.default_rng(2)
    done = 0
    for c in range(110):
        ntr = int(rng.choice([1, 2, 3, 5, 8, 9, 17, 33, 40]))
        ntc = int(rng.choice([1, 2, 7, 8, 15, 16, 17, 31, 32, 33, 48, 63, 64, 65, 72]))
        M = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 40]))
        group = int(rng.choice([64, 128, 128, 256])) if ntc % 2 == 0 else int(rng.choice([64, 128]))
        fmt = str(rng.choice(["fp16", "bf16"]))
        outliers, use_cp, use_rp = bool(rng.integers(2)), bool(rng.integers(4)), bool(rng.integers(4))
        N, K = 128 * ntr, 128 * ntc
        if N * K > 24 * 2 ** 20:
            continue
        p = W.make_problem(f"rnd{c}", K, N, M, 90000 + c, fractions={2: 0.3, 3: 0.4, 4: 0.3}, outliers=outliers,
                           use_col_perm=use_cp, use_row_perm=use_rp, group=group, scale_format=fmt)
        dp, cp, rp = device_problem(p)
        Y = run_gemm(p, dp, cp, rp)
        try:
            _check(p, Y)
        except AssertionError as ex:
            raise AssertionError(f"case {c}: N={N} K={K} M={M} group={group} {fmt}: {ex}") from None
        assert np.array_equal(run_gemm(p, dp, cp, rp).view(np.uint16), Y.view(np.uint16)), (c, N, K, M)
        done += 1
    assert done >= 80


def test_random_batches(torch_cuda):
    # seeded random batches through sfmp_gemv_batched / sfmp_gemm_batched: one to eight problems of unrelated shapes
    # (or sharing K and the activations, as q, k and v do), every M class of the decode path, mixed parameter formats
    # and group lengths (64 for all problems or for none: one launch runs one class); a launch picks ONE form of the
    # kernel for the whole batch, by its largest K and its largest share of slabs per workgroup.  Every output against
    # the oracle, and a second call (workspace refilled with other bytes) gives the same bits.
    import paper_2602_01027_amd as S
    from gpu_util import device_problem
    torch = torch_cuda
    rng = np.random.default_rng(5)
    done = 0
    for c in range(36):
        count = int(rng.integers(1, 9))
        M = int(rng.choice([1, 1, 2, 3, 4, 5, 8, 9, 16]))
        g64 = bool(rng.integers(4) == 0)
        K0 = 128 * int(rng.choice([1, 4, 8, 16, 20, 32, 33, 64, 72, 112]))
        share = bool(rng.integers(2))
        probs = []
        for i in range(count):
            K = K0 if (share or rng.integers(2)) else 128 * int(rng.choice([2, 8, 32, 40]))
            N = 128 * int(rng.choice([1, 2, 3, 8, 9, 17, 32, 80]))
            if N * K > 16 * 2 ** 20:
                N = 128 * 8
            group = 64 if g64 else int(rng.choice([128, 128, 256])) if (K // 128) % 2 == 0 else 128
            probs.append(W.make_problem(f"rb{c}.{i}", K, N, M, 95000 + 16 * c + i, fractions={2: 0.3, 3: 0.4, 4: 0.3},
                                        outliers=bool(rng.integers(2)), use_col_perm=bool(rng.integers(4)),
                                        use_row_perm=bool(rng.integers(4)), group=group,
                                        scale_format=str(rng.choice(["fp16", "bf16"]))))
        batch, shared = [], {}
        for p in probs:
            dp, cp, rp = device_problem(p)
            if share and p.K in shared:  # the same activations through this problem's own column permutation
                X = shared[p.K]
                p.X[...] = X.cpu().numpy()
            else:
                X = shared[p.K] = torch.from_numpy(p.X).to("cuda:0")
            batch.append((X, cp, dp, rp, torch.full((M, p.N), float("nan"), dtype=torch.float16, device="cuda:0")))
        ws = None if M == 1 else torch.empty(S.sfmp_gemm_batched_workspace(batch, M), dtype=torch.uint8, device="cuda:0")
        outs = []
        for fill in (0xFF, 0x7F):
            for b in batch:
                b[4].fill_(float("nan"))
            if M == 1:
                S.sfmp_gemv_batched(batch)
            else:
                ws.fill_(fill)
                S.sfmp_gemm_batched(batch, M, ws)
            torch.cuda.synchronize()
            outs.append([b[4].cpu().numpy().copy() for b in batch])
        for p, y0, y1 in zip(probs, outs[0], outs[1]):
            try:
                _check(p, y0)
            except AssertionError as ex:
                raise AssertionError(f"case {c}: M={M} {[(q.N, q.K, q.group) for q in probs]}: {p.label}: {ex}") from None
            assert np.array_equal(y0.view(np.uint16), y1.view(np.uint16)), (c, p.label)
        done += 1
    assert done == 36


# ---------------------------------------------------------------------------------------------
# what the error bound of the decode kernels assumes about the matrix instruction, pinned on the hardware
# ---------------------------------------------------------------------------------------------
def test_mfma_alignment_model(torch_cuda):
    """v_mfma_f32_16x16x32_f16 with an fp16-denormal operand (the decode kernels' codes, q * 2^(p-24)).  The products are
    aligned by NOMINAL exponents (2^-14 for the denormal, whatever its leading bit) and 24 bits are kept below the
    largest: within the 8 products of a lane the cut is exactly at 2^(E - 38), E = the lane's largest activation
    exponent, and the bits below are cut off, not rounded; a lone product of another lane comes through at fp32
    precision.  In general a product loses less than 2^(E - 38), E over the 32 activations of the instruction, and only
    if its own exponent is at most E - 4: tests/gpu_util.py::mfma_alignment_loss turns that into a term of the
    per-element bound of the decode kernels, and this test pins it on the hardware."""
    from paper_2602_01027_amd import probe
    torch = torch_cuda
    rows_a, rows_b, expect = [], [], []
    for pos in (0, 2, 6):
        for slot in (1, 7, 8, 31):           # 1, 7: same lane as element 0; 8, 31: other lanes
            for E in range(0, 16):
                a = np.zeros(32); b = np.zeros(32)
                a[0], b[0] = 2.0 ** E, 2.0 ** (pos - 24)
                a[slot], b[slot] = 1025.0 / 1024.0, 3.0 * 2.0 ** (pos - 24)   # 3075 units of 2^(pos-34)
                rows_a.append(a); rows_b.append(b)
                big = 2.0 ** (E + pos - 24)
                if slot < 8:
                    cut = max(E - 4 - pos, 0)  # bits of the small product below 2^(E-38), in its units of 2^(pos-34)
                    kept = (3075 >> cut) << cut
                    expect.append(big + kept * 2.0 ** (pos - 34))  # fits in fp32 exactly
                else:
                    expect.append(float(np.float32(big + 3075 * 2.0 ** (pos - 34))))  # fp32 of the exact sum
    A = torch.from_numpy(np.array(rows_a, dtype=np.float16)).to("cuda:0")
    B = torch.from_numpy(np.array(rows_b, dtype=np.float16)).to("cuda:0")
    assert np.array_equal(B.cpu().numpy().astype(np.float64), np.array(rows_b))  # the denormals survive the upload
    got = probe.mfma_dot(A, B).cpu().numpy().astype(np.float64)
    assert np.array_equal(got, np.array(expect)), np.nonzero(got != np.array(expect))[0][:8]

    # random operands shaped like the kernels' (2-bit codes at position 0; with and without an outlier column; all
    # four lanes, and one lane alone): the error stays within the bound, and it is far above fp32 rounding
    rng = np.random.default_rng(11)
    n = 4096
    for outlier, one_lane in ((True, False), (False, False), (True, True)):
        a = rng.normal(size=(n, 32))
        if outlier:
            a[:, 5] *= 20.0
        if one_lane:
            a[:, 8:] = 0.0
        a = a.astype(np.float16).astype(np.float64)
        b = rng.integers(0, 4, size=(n, 32)).astype(np.float64) * 2.0 ** -24
        got = probe.mfma_dot(torch.from_numpy(a.astype(np.float16)).to("cuda:0"),
                             torch.from_numpy(b.astype(np.float16)).to("cuda:0")).cpu().numpy().astype(np.float64)
        prod = a * b
        exact = prod.sum(axis=1)
        _, e = np.frexp(np.abs(a))
        e = np.maximum(e - 1, -14)
        E = np.where(a != 0, e, -100).max(axis=1)
        lossy = ((prod != 0) & (e <= E[:, None] - 4)).sum(axis=1)
        bound = lossy * np.ldexp(1.0, E - 38) + 2.0 ** -23 * np.abs(exact)
        err = np.abs(got - exact)
        assert np.all(err <= bound), float((err / np.maximum(bound, 1e-300)).max())
        i = int(np.argmax(err))
        assert err[i] > 50 * 2.0 ** -24 * np.abs(prod[i]).sum()  # not an fp32-accurate sum of exact products


# ---------------------------------------------------------------------------------------------
# one-bit lookup-table GEMV on the bit-plane format (the paper's own kernel scheme), M = 1
# ---------------------------------------------------------------------------------------------
def _run_lut(torch, p, table_format="fp32"):
    import paper_2602_01027_amd as S
    dev = "cuda:0"
    planes, tile_off = S.sfmp_lut_pack(p.codes, p.bitmap)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    ws = torch.zeros(S.sfmp_lut_gemv_workspace(p.N, p.K), dtype=torch.uint8, device=dev)
    Y = torch.full((p.N,), float("nan"), dtype=torch.float16, device=dev)
    cp = d(p.col_perm) if p.col_perm is not None else None
    rp = d(p.row_perm) if p.row_perm is not None else None
    S.sfmp_lut_gemv(d(p.X[0]), cp, p.N, p.K, d(planes), d(tile_off.view(np.int32)), d(p.scales), d(p.zeros), rp, Y, ws,
                    table_format=table_format)
    torch.cuda.synchronize()
    return Y.cpu().numpy()[None, :]


@pytest.mark.parametrize("K,N,fractions,perms", [
    (128, 128, {2: 1.0}, True), (512, 384, None, True), (1152, 640, None, False), (4096, 1024, {2: 0.5, 4: 0.5}, True),
    (1024, 4096, {3: 1.0}, True)])
def test_lut_gemv_against_oracles(torch_cuda, K, N, fractions, perms):
    from oracle import sfmp_lut_oracle as LO
    p = W.make_problem("lut", K, N, 1, 4100 + K + N, fractions=fractions, use_col_perm=perms, use_row_perm=perms)
    Y = _run_lut(torch_cuda, p)
    _check(p, Y, elementwise=False)  # against the plain definition (the table scheme has its own arithmetic)
    if K * N <= 512 * 384:  # and against the table algorithm itself, where that finishes in seconds
        planes, tile_off = LO.lut_pack(p.codes, p.bitmap)
        ref = LO.lut_gemv(p.X[0], p.col_perm, N, K, planes, tile_off, p.scales, p.zeros, p.row_perm)
        assert O.rel_frobenius(Y, ref[None, :]) <= TOL


@pytest.mark.parametrize("K,N,fractions,perms", [
    (128, 128, {4: 1.0}, True), (512, 384, None, True), (1152, 640, None, False), (4096, 1024, {2: 0.5, 4: 0.5}, True)])
def test_lut_gemv_fp16_tables_against_oracles(torch_cuda, K, N, fractions, perms):
    # 2-byte table entries (Appendix F): against the plain definition at the stated bound, and, where the table
    # algorithm of the oracle finishes in seconds, against that algorithm with its entries rounded to fp16 the same
    # way: what is left then is the order of the fp32 sums and the final rounding
    from oracle import sfmp_lut_oracle as LO
    p = W.make_problem("lut16", K, N, 1, 4300 + K + N, fractions=fractions, use_col_perm=perms, use_row_perm=perms)
    Y = _run_lut(torch_cuda, p, "fp16")
    _check(p, Y, elementwise=False)
    if K * N <= 1152 * 640:
        planes, tile_off = LO.lut_pack(p.codes, p.bitmap)
        ref16 = LO.lut_gemv(p.X[0], p.col_perm, N, K, planes, tile_off, p.scales, p.zeros, p.row_perm, table_dtype=np.float16)
        ref = LO.lut_gemv(p.X[0], p.col_perm, N, K, planes, tile_off, p.scales, p.zeros, p.row_perm)
        e16 = O.rel_frobenius(Y, ref16[None, :])
        assert e16 <= 4e-4, e16  # fp16 rounding of the result alone is 2^-11 / sqrt(3) = 2.8e-4 in this norm
        # and the kernel is closer to the oracle that rounds its entries than the two oracles are to each other
        # once the entries' rounding shows (K > 128: more than one tile column of looked-up values per output)
        if K > 128:
            assert np.linalg.norm(Y[0] - ref16) <= np.linalg.norm(Y[0] - ref) * 1.05


def test_lut_gemv_rejects_unknown_table_format(torch_cuda):
    import paper_2602_01027_amd as S
    p = W.make_problem("lutfmt", 128, 128, 1, 4399)
    with pytest.raises(S.SfmpError) as e:
        _run_lut(torch_cuda, p, 7)
    assert e.value.code == -8


def test_lut_gemv_full_size_sampled_and_repeatable(torch_cuda):
    # the gate projection of the 8B layer at full size: sampled rows against the oracle, two runs bit-identical,
    # and agreement with the MFMA path of the library on the same matrix
    from gpu_util import run_gemm
    p = W.make_problem("lut.gate", 4096, 14336, 1, 4242)
    Y1 = _run_lut(torch_cuda, p)
    Y2 = _run_lut(torch_cuda, p)
    assert np.array_equal(Y1.view(np.uint16), Y2.view(np.uint16))
    rows = np.random.default_rng(5).choice(p.N, size=96, replace=False)
    _check(p, Y1, rows=np.sort(rows), elementwise=False)
    assert O.rel_frobenius(Y1, run_gemm(p).astype(np.float64)) <= 2 * TOL


def test_lut_gemv_workspace_reuse(torch_cuda):
    # one workspace, with arbitrary contents, used by several products of different shapes one after the other
    import paper_2602_01027_amd as S
    torch = torch_cuda
    probs = [W.make_problem("lut.ws", K, N, 1, 4300 + i) for i, (K, N) in enumerate([(512, 640), (256, 1024), (512, 640)])]
    nbytes = max(S.sfmp_lut_gemv_workspace(p.N, p.K) for p in probs)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    ws.fill_(0xAB)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    outs = []
    for rep in range(2):
        for p in probs:
            planes, tile_off = S.sfmp_lut_pack(p.codes, p.bitmap)
            Y = torch.full((p.N,), float("nan"), dtype=torch.float16, device="cuda:0")
            S.sfmp_lut_gemv(d(p.X[0]), d(p.col_perm), p.N, p.K, d(planes), d(tile_off.view(np.int32)), d(p.scales),
                            d(p.zeros), d(p.row_perm), Y, ws)
            torch.cuda.synchronize()
            outs.append(Y.cpu().numpy()[None, :])
            _check(p, outs[-1], elementwise=False)
    for i in range(3):
        assert np.array_equal(outs[i].view(np.uint16), outs[i + 3].view(np.uint16))


def test_lut_gemv_argument_errors(torch_cuda):
    import paper_2602_01027_amd as S
    torch = torch_cuda
    p = W.make_problem("lut.err", 256, 256, 1, 77)
    planes, tile_off = S.sfmp_lut_pack(p.codes, p.bitmap)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    Y = torch.zeros(p.N, dtype=torch.float16, device="cuda:0")
    small = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(S.SfmpError) as e:
        S.sfmp_lut_gemv(d(p.X[0]), None, p.N, p.K, d(planes), d(tile_off.view(np.int32)), d(p.scales), d(p.zeros), None, Y, small)
    assert e.value.code == -5
