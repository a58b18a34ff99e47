"""The host code of the library (packer, bit-plane packer, validators, permutation folding: csrc/sfmp_host.cpp) built
with g++ under -fsanitize=address,undefined and driven by tests/host_sanitizer_driver.cpp on exact-size heap buffers.
A sanitizer report aborts the driver; what it writes is compared with the oracle byte for byte."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import sfmp_oracle as O
from oracle import sfmp_lut_oracle as LO

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOST_SRC = os.path.join(ROOT, "paper_2602_01027_amd", "csrc", "sfmp_host.cpp")
DRIVER_SRC = os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("g++ not available")
    exe = str(tmp_path_factory.mktemp("san") / "host_sanitizer_driver")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan", HOST_SRC, DRIVER_SRC, "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    return exe


@pytest.mark.parametrize("seed,ntr,ntc", [(1, 1, 1), (2, 2, 3), (3, 3, 2), (4, 1, 5)])
def test_host_code_under_sanitizers_matches_oracle(driver, tmp_path, seed, ntr, ntc):
    rng = np.random.default_rng(seed)
    N, K = 128 * ntr, 128 * ntc
    bitmap = rng.integers(2, 5, size=(ntr, ntc)).astype(np.int8)
    if seed == 4:
        bitmap[:] = 3  # two empty streams (NULL stream pointers)
    bm = np.repeat(np.repeat(bitmap, 128, axis=0), 128, axis=1)
    codes = (rng.integers(0, 16, size=bm.shape) % (1 << bm)).astype(np.uint8)
    n = 37 * seed
    row_perm, col_perm = rng.permutation(n).astype(np.int32), rng.permutation(n).astype(np.int32)
    case, out = tmp_path / "case.bin", tmp_path / "out.bin"
    with open(case, "wb") as f:
        f.write(np.array([N, K, n], dtype=np.int32).tobytes())
        f.write(bitmap.tobytes())
        f.write(codes.tobytes())
        f.write(row_perm.tobytes())
        f.write(col_perm.tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([driver, str(case), str(out)], capture_output=True, text=True, env=env)
    assert r.returncode == 0, r.stdout + r.stderr
    raw = open(out, "rb").read()
    sizes = np.frombuffer(raw[:48], dtype=np.int64)
    pos = 48

    def take(count, dtype):
        nonlocal pos
        a = np.frombuffer(raw[pos:pos + count * np.dtype(dtype).itemsize], dtype=dtype)
        pos += a.nbytes
        return a

    s2, s3, s4 = take(sizes[0], np.uint8), take(sizes[1], np.uint8), take(sizes[2], np.uint8)
    index = take(sizes[3], np.int32)
    planes, tile_off = take(sizes[4], np.uint8), take(sizes[5], np.uint32)
    folded = take(n, np.int32)
    errs = take(10, np.int32)
    assert pos == len(raw)
    ref = O.pack(codes, bitmap)
    assert np.array_equal(s2, ref["s2"]) and np.array_equal(s3, ref["s3"]) and np.array_equal(s4, ref["s4"])
    assert np.array_equal(index, ref["index"])
    ref_planes, ref_off = LO.lut_pack(codes, bitmap)
    assert np.array_equal(planes, ref_planes) and np.array_equal(tile_off, ref_off)
    assert np.array_equal(folded, O.fold_perms(row_perm, col_perm))
    # CODE_RANGE x2, BITWIDTH, SHAPE, PERM x4 (out of range, through fold, negative, duplicate), LAYOUT, then OK
    assert errs.tolist() == [-4, -4, -3, -2, -7, -7, -7, -7, -8, 0]
