"""Host side of the C ABI (no GPU): exported symbols, packer bytes vs the oracle, error codes."""
import ctypes as C
import os
import re

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import paper_2602_01027_amd as S
from oracle import sfmp_oracle as O
import sfmp_workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "sfmp.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(sfmp_[a-z_0-9]+)\s*\(", header))
    assert declared == set(S.binding.EXPORTS), declared ^ set(S.binding.EXPORTS)
    lib = S.load_library()
    for name in declared:
        assert getattr(lib, name) is not None


def test_layout_struct_matches_header_size():
    # 8 int32 + 4 int64 + 2 int32 = 72 bytes, no padding
    assert C.sizeof(S.SfmpLayout) == 72


@settings(max_examples=10, deadline=None)
@given(st.integers(0, 2 ** 31 - 1), st.integers(1, 3), st.integers(1, 4))
def test_packer_bytes_equal_oracle(seed, ntr, ntc):
    rng = np.random.default_rng(seed)
    bitmap = rng.integers(2, 5, size=(ntr, ntc)).astype(np.int8)
    bm = np.repeat(np.repeat(bitmap, 128, axis=0), 128, axis=1)
    codes = (rng.integers(0, 16, size=bm.shape) % (1 << bm)).astype(np.uint8)
    L, s2, s3, s4, index = S.sfmp_pack(codes, bitmap)
    ref = O.pack(codes, bitmap)
    assert np.array_equal(s2, ref["s2"]) and np.array_equal(s3, ref["s3"]) and np.array_equal(s4, ref["s4"])
    assert np.array_equal(index, ref["index"])
    assert (L.N, L.K, L.tile, L.group) == (ntr * 128, ntc * 128, 128, 128)
    assert (L.count2, L.count3, L.count4) == tuple(int((bitmap == b).sum()) for b in (2, 3, 4))
    assert (L.bytes_s2, L.bytes_s3, L.bytes_s4) == (s2.size, s3.size, s4.size)
    assert L.index_words == O.index_words(ntr, ntc) and L.bytes_index == 4 * L.index_words


def test_packer_on_tiny_config_and_single_width_bitmaps():
    p = W.make_problem("tiny", 512, 512, 1, 1000)
    L, s2, s3, s4, index = S.sfmp_pack(p.codes, p.bitmap)
    ref = O.pack(p.codes, p.bitmap)
    assert np.array_equal(np.concatenate([s2, s3, s4]), np.concatenate([ref["s2"], ref["s3"], ref["s4"]]))
    for b in (2, 3, 4):
        bitmap = np.full((2, 2), b, dtype=np.int8)
        q = W.make_problem("u", 256, 256, 1, 5 + b, bitmap=bitmap)
        L, s2, s3, s4, index = S.sfmp_pack(q.codes, bitmap)
        ref = O.pack(q.codes, bitmap)
        assert np.array_equal(index, ref["index"])
        for a, name in ((s2, "s2"), (s3, "s3"), (s4, "s4")):
            assert np.array_equal(a, ref[name])
        assert [L.count2, L.count3, L.count4][b - 2] == 4


def test_error_codes():
    lib = S.load_library()
    L = S.SfmpLayout()
    bm = np.full((1, 1), 3, dtype=np.int8)
    ptr = bm.ctypes.data_as(C.c_void_p)
    assert lib.sfmp_pack_query(None, 128, 128, C.byref(L)) == -1  # NULL
    assert lib.sfmp_pack_query(ptr, 100, 128, C.byref(L)) == -2  # SHAPE
    assert lib.sfmp_pack_query(ptr, 128, 0, C.byref(L)) == -2
    bad = np.full((1, 1), 5, dtype=np.int8)
    assert lib.sfmp_pack_query(bad.ctypes.data_as(C.c_void_p), 128, 128, C.byref(L)) == -3  # BITWIDTH
    bad[0, 0] = 1
    assert lib.sfmp_pack_query(bad.ctypes.data_as(C.c_void_p), 128, 128, C.byref(L)) == -3
    # code out of range: nothing written
    codes = np.zeros((128, 128), dtype=np.uint8)
    codes[77, 3] = 8
    with pytest.raises(S.SfmpError) as ei:
        S.sfmp_pack(codes, bm)
    assert ei.value.code == -4
    # workspace query argument checks
    L = S.sfmp_pack_query(bm, 128, 128)
    n = C.c_int64(0)
    assert lib.sfmp_gemm_workspace(C.byref(L), 0, C.byref(n)) == -2
    assert lib.sfmp_gemm_workspace(None, 1, C.byref(n)) == -1
    broken = S.SfmpLayout.from_buffer_copy(L)
    broken.count3 = 7
    assert lib.sfmp_gemm_workspace(C.byref(broken), 1, C.byref(n)) == -8  # LAYOUT
    assert S.sfmp_gemm_workspace(L, 1) >= 256 and S.sfmp_gemm_workspace(L, 1) % 256 == 0
    # gemm refuses NULL buffers before touching any device
    assert lib.sfmp_gemm(None, 1, None, C.byref(L), None, None, None, None, None, None, None, None, None, None, 0,
                         None) == -1
    # alignment is checked before any device work as well (the pointers are never dereferenced on the host)
    ok = [C.c_void_p(0x7f0000001000 + 0x10000 * i) for i in range(8)]

    def gemm_with(X=ok[0], cp=ok[1], scales=ok[2], Y=ok[3], M=1):
        return lib.sfmp_gemm(X, M, cp, C.byref(L), None, ok[4], None, ok[5], scales, ok[6], None, None, Y, ok[7], 1 << 20,
                             None)
    assert gemm_with(X=C.c_void_p(0x7f0000001008)) == -9  # ALIGN: X needs 16 bytes
    assert gemm_with(cp=C.c_void_p(0x7f0000011004)) == -9
    assert gemm_with(scales=C.c_void_p(0x7f0000021002)) == -9
    assert gemm_with(Y=C.c_void_p(0x7f0000031001)) == -9      # Y: 2 bytes at M <= 16 ...
    assert gemm_with(Y=C.c_void_p(0x7f0000031002), M=17) == -9  # ... 16 bytes beyond
    for code in range(-10, 1):
        assert S.sfmp_strerror(code)
    assert "unknown" in S.sfmp_strerror(-99)


def test_check_perm():
    assert S.sfmp_check_perm(np.array([2, 0, 1], dtype=np.int32)) == 0
    assert S.sfmp_check_perm(np.array([2, 0, 2], dtype=np.int32)) == -7
    assert S.sfmp_check_perm(np.array([0, 3, 1], dtype=np.int32)) == -7
    assert S.sfmp_check_perm(np.array([0, -1, 1], dtype=np.int32)) == -7


def test_layout_set_quant_accepts_the_documented_formats_only():
    bitmap = np.full((1, 4), 3, dtype=np.int8)  # N = 128, K = 512
    L = S.sfmp_pack_query(bitmap, 128, 512)
    assert (L.group, L.scale_format) == (128, 0)
    for group in (64, 128, 256, 512):
        for fmt, code in (("fp16", 0), ("bf16", 1)):
            S.sfmp_layout_set_quant(L, group, fmt)
            assert (L.group, L.scale_format) == (group, code)
    S.sfmp_layout_set_quant(L, 128, "fp16")
    lib = S.load_library()
    for group, fmt in ((32, 0), (1024, 0), (384, 0), (128, 2), (256, -1)):
        assert lib.sfmp_layout_set_quant(C.byref(L), group, fmt) == -8
        assert (L.group, L.scale_format) == (128, 0)  # a rejected call leaves the layout alone
    # K must be a multiple of the group
    L3 = S.sfmp_pack_query(np.full((1, 3), 2, dtype=np.int8), 128, 384)
    assert lib.sfmp_layout_set_quant(C.byref(L3), 256, 0) == -8
    assert lib.sfmp_layout_set_quant(None, 128, 0) == -1


def test_fold_perms_matches_oracle_and_its_defining_property():
    # NEXT: permutation folding.  The C ABI result equals the oracle's (written as a search), and both satisfy
    # the property that defines them: gathering from the reordered product with the folded permutation fetches
    # what the plain gather fetches from the un-permuted one.
    import paper_2602_01027_amd as S
    from oracle import sfmp_oracle as O
    rng = np.random.default_rng(5)
    for n in (1, 7, 128, 1000):
        r = rng.permutation(n).astype(np.int32)
        c = rng.permutation(n).astype(np.int32)
        f = S.sfmp_fold_perms(r, c)
        assert np.array_equal(f, O.fold_perms(r, c))
        Y = rng.standard_normal((3, n))
        Yt = Y[:, r]                      # the product left in reordered row order
        assert np.array_equal(Yt[:, f], Y[:, c])
        f_id = S.sfmp_fold_perms(r, None)
        assert np.array_equal(f_id, O.fold_perms(r, None))
        assert np.array_equal(Yt[:, f_id], Y)  # identity next permutation: the fold is the inverse
    assert S.sfmp_check_perm(f) == 0
    with pytest.raises(S.SfmpError):
        S.sfmp_fold_perms(np.array([0, 0, 1], dtype=np.int32), None)
    with pytest.raises(S.SfmpError):
        S.sfmp_fold_perms(np.array([0, 2, 1], dtype=np.int32), np.array([0, 3, 1], dtype=np.int32))


def _plan_mirror(N, K, M):
    """The documented path selection of sfmp_gemm, restated: which kernels a call takes and the workspace it needs."""
    ntr, ntc = N // 128, K // 128
    up256 = lambda v: (v + 255) // 256 * 256
    if M <= 16:
        if M == 1 and K <= 32768 - 1:  # the GEMV kernel holds the activation vector in LDS: no workspace
            return "gemv", None
        mb = 4 if M <= 4 else 8 if M <= 8 else 16
        # a wavefront with at most four tile columns keeps the activations in registers (staged as 16 rows), unless
        # the kernel stages M <= 4 rows into LDS by itself (at most 32 KiB of them)
        grid = min(8 * ntr, 256)
        for rounds in (2, 3, 4):  # up to four workgroups per CU in turn, to get down to 8 slabs per workgroup
            if -(-8 * ntr // grid) > 8 and -(-8 * ntr // (256 * rounds)) <= 8:
                grid = 256 * rounds
        if -(-8 * ntr // grid) > 16:
            grid = (-(-8 * ntr // 16) + 7) // 8 * 8
        max_slabs = -(-8 * ntr // grid)
        nw = 16 if max_slabs <= 8 else 8
        resident = mb == 4 and M * K * 2 <= 32 * 1024 and K // 8 <= 4 * nw * 64
        # (that form keeps each wavefront's finished sums in LDS, 1 KiB per slab, beside two ring slots of 1280 bytes)
        if not resident and ntc <= 4 * nw and nw * (max_slabs * 1024 + 2 * 1280) <= 160 * 1024:
            mb = 16
        return "ring", up256(ntc * mb * 256)
    chunks = (M + 15) // 16
    if ntr <= 8:
        chunked = chunks <= 8
    elif ntc <= 64:  # K <= 8192: the chunks keep their activations in registers
        tiles = ntr * ntc
        chunked = chunks <= 2 or (chunks <= 4 and tiles <= 1536) or (chunks <= 6 and tiles <= 1024)
    else:
        chunked = chunks <= 2 and ntr <= 32
    if M <= 128 and ntc >= 32 and chunked:
        return "chunked", chunks * up256(ntc * 16 * 256)
    bm = 64 if ((M + 127) // 128) * ntr <= 128 else 128
    blocks = ((M + bm - 1) // bm) * ntr
    ks = 1
    if blocks <= 256:
        ks = max(1, min(512 // blocks, ntc // 8, 8))
        if ks < 3 and ntc < 64:
            ks = 1
    xperm = up256(((M + 127) // 128) * 128 * K * 2)
    ytmp = up256(ks * M * N * 4 if ks > 1 else M * N * 2)
    return f"mfma bm={bm} ksplit={ks}", xperm + ytmp


@pytest.mark.parametrize("N,K,M", [(4096, 4096, 4), (4096, 4096, 3), (14336, 4096, 5), (32768, 4096, 2), (57344, 4096, 8), (57344, 8192, 8), (4096, 8192, 3), (4096, 14336, 16), (1024, 4096, 128), (1152, 4096, 128),
                                    (4096, 4096, 32), (4096, 4096, 33), (4096, 4096, 96), (4096, 4096, 97), (6144, 4096, 64), (14336, 4096, 32),
                                    (14336, 4096, 33), (8192, 8192, 32), (8192, 8192, 48), (28672, 8192, 32), (4096, 14336, 32), (4096, 14336, 256), (14336, 4096, 48),
                                    (14336, 4096, 256), (4096, 4096, 2048), (28672, 8192, 2048), (4096, 2048, 100),
                                    (8192, 28672, 512)])
def test_workspace_query_follows_the_documented_path_selection(N, K, M):
    bitmap = np.full((N // 128, K // 128), 3, dtype=np.int8)
    L = S.sfmp_pack_query(bitmap, N, K)
    name, expected = _plan_mirror(N, K, M)
    got = S.sfmp_gemm_workspace(L, M)
    if expected is not None:
        assert got == max(256, expected), (name, got, expected)
    else:
        assert got == 256, (name, got)


# ---- bit-plane format of the lookup-table GEMV: the library's packer against the oracle's, byte for byte ----------
@pytest.mark.parametrize("seed,N,K,fractions", [(21, 128, 128, {4: 1.0}), (22, 256, 384, None), (23, 384, 256, {2: 0.6, 3: 0.4})])
def test_lut_pack_bytes_match_oracle(seed, N, K, fractions):
    from oracle import sfmp_lut_oracle as LO
    p = W.make_problem("lutpack", K, N, 1, seed, fractions=fractions)
    planes, tile_off = S.sfmp_lut_pack(p.codes, p.bitmap)
    ref_planes, ref_off = LO.lut_pack(p.codes, p.bitmap)
    assert np.array_equal(tile_off, ref_off)
    assert np.array_equal(planes, ref_planes)
    assert np.array_equal(LO.lut_unpack(N, K, planes, tile_off), p.codes)


def test_lut_pack_errors():
    codes = np.zeros((128, 128), dtype=np.uint8)
    with pytest.raises(S.SfmpError) as e:
        S.sfmp_lut_pack(codes, np.array([[5]], dtype=np.int8))
    assert e.value.code == -3
    codes[3, 7] = 4
    with pytest.raises(S.SfmpError) as e:
        S.sfmp_lut_pack(codes, np.array([[2]], dtype=np.int8))
    assert e.value.code == -4
    with pytest.raises(S.SfmpError) as e:
        S.sfmp_lut_pack(np.zeros((100, 128), dtype=np.uint8), np.array([[2]], dtype=np.int8))
    assert e.value.code == -2
    assert S.sfmp_lut_gemv_workspace(4096, 4096) % 256 == 0


def test_float_reciprocal_item_index_is_exact():
    """The decode kernels find the slab index of an item as floor((e + 0.5) * rcp(c)) in fp32 instead of an integer
    division (e < 1024 items, c <= 64 tile columns per wavefront).  Exact even if the hardware reciprocal is off by
    two units in the last place in either direction."""
    e = np.arange(1024)
    g = e.astype(np.float32) + np.float32(0.5)
    for c in range(1, 65):
        r = np.float32(1) / np.float32(c)
        lo = np.nextafter(np.nextafter(r, np.float32(0)), np.float32(0))
        hi = np.nextafter(np.nextafter(r, np.float32(2)), np.float32(2))
        for rr in (lo, r, hi):
            j = (g * np.float32(rr)).astype(np.uint32)
            assert np.array_equal(j, e // c), c
