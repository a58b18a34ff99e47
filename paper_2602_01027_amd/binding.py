"""ctypes binding of libsfmp.so.  Host buffers are numpy arrays, device buffers are torch tensors
(torch only owns device memory and streams here).  No fallback: a missing library raises."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class SfmpError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"sfmp error {code}: {text}")
        self.code = code


class SfmpLayout(C.Structure):
    _fields_ = [
        ("N", C.c_int32), ("K", C.c_int32), ("tile", C.c_int32), ("group", C.c_int32),
        ("count2", C.c_int32), ("count3", C.c_int32), ("count4", C.c_int32), ("index_words", C.c_int32),
        ("bytes_s2", C.c_int64), ("bytes_s3", C.c_int64), ("bytes_s4", C.c_int64), ("bytes_index", C.c_int64),
        ("scale_format", C.c_int32), ("reserved", C.c_int32),
    ]


class SfmpGemvProblem(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("X", "col_perm", "layout", "s2", "s3", "s4", "index", "scales", "zeros",
                                          "bitmap", "row_perm", "Y")]


EXPORTS = ("sfmp_strerror", "sfmp_pack_query", "sfmp_layout_set_quant", "sfmp_pack", "sfmp_unpack", "sfmp_gemm_workspace",
           "sfmp_workspace_init", "sfmp_gemm", "sfmp_gemm_static", "sfmp_gemv_batched", "sfmp_gemm_batched_workspace",
           "sfmp_gemm_batched", "sfmp_check_perm", "sfmp_fold_perms", "sfmp_lut_pack_query",
           "sfmp_lut_pack", "sfmp_lut_gemv_workspace", "sfmp_lut_gemv")


def lib_path() -> str:
    return os.path.join(_HERE, "libsfmp.so")


def load_library():
    """Loads the in-tree libsfmp.so; raises if it has not been built (there is no other path)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: build it with `python -m paper_2602_01027_amd.build` "
                                "(or __graft_entry__.build()); there is no CPU fallback")
    lib = C.CDLL(path)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    LP = C.POINTER(SfmpLayout)
    lib.sfmp_strerror.restype = C.c_char_p
    lib.sfmp_strerror.argtypes = [C.c_int]
    lib.sfmp_pack_query.argtypes = [vp, i32, i32, LP]
    lib.sfmp_pack.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp, LP]
    lib.sfmp_unpack.argtypes = [LP, vp, vp, vp, vp, vp, vp]
    lib.sfmp_gemm_workspace.argtypes = [LP, i32, C.POINTER(i64)]
    lib.sfmp_workspace_init.argtypes = [vp, i64, vp]
    lib.sfmp_gemm.argtypes = [vp, i32, vp, LP, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, vp]
    lib.sfmp_gemm_static.argtypes = [vp, i32, vp, LP, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.sfmp_gemv_batched.argtypes = [vp, i32, vp]
    lib.sfmp_check_perm.argtypes = [vp, i32]
    lib.sfmp_lut_pack_query.argtypes = [vp, i32, i32, C.POINTER(i64), C.POINTER(i64)]
    lib.sfmp_lut_pack.argtypes = [vp, vp, i32, i32, vp, vp]
    lib.sfmp_lut_gemv_workspace.argtypes = [i32, i32, C.POINTER(i64)]
    lib.sfmp_lut_gemv.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, i32, vp, i64, vp]
    lib.sfmp_fold_perms.argtypes = [vp, vp, i32, vp]
    for name in EXPORTS:
        if name != "sfmp_strerror":
            getattr(lib, name).restype = C.c_int
    _LIB = lib
    return lib


def sfmp_strerror(code: int) -> str:
    return load_library().sfmp_strerror(int(code)).decode()


def _check(code: int) -> None:
    if code != 0:
        raise SfmpError(code, sfmp_strerror(code))


def _host_ptr(a: Optional[np.ndarray]):
    if a is None or a.size == 0:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.c_void_p)


def _dev_ptr(t):
    if t is None:
        return None
    if t.numel() == 0:
        return None
    assert t.is_cuda and t.is_contiguous()
    return C.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def sfmp_pack_query(bitmap: np.ndarray, N: int, K: int) -> SfmpLayout:
    L = SfmpLayout()
    bm = np.ascontiguousarray(bitmap, dtype=np.int8)
    _check(load_library().sfmp_pack_query(_host_ptr(bm), N, K, C.byref(L)))
    return L


def sfmp_pack(codes: np.ndarray, bitmap: np.ndarray):
    """Host packer.  Returns (layout, s2, s3, s4, index) with numpy uint8 / int32 host arrays."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    bm = np.ascontiguousarray(bitmap, dtype=np.int8)
    N, K = codes.shape
    L = sfmp_pack_query(bm, N, K)
    s2 = np.empty(L.bytes_s2, dtype=np.uint8)
    s3 = np.empty(L.bytes_s3, dtype=np.uint8)
    s4 = np.empty(L.bytes_s4, dtype=np.uint8)
    index = np.empty(L.index_words, dtype=np.int32)
    out = SfmpLayout()
    _check(load_library().sfmp_pack(_host_ptr(codes), _host_ptr(bm), N, K, _host_ptr(s2), _host_ptr(s3),
                                    _host_ptr(s4), _host_ptr(index), C.byref(out)))
    return out, s2, s3, s4, index


def sfmp_check_perm(perm: np.ndarray) -> int:
    p = np.ascontiguousarray(perm, dtype=np.int32)
    return int(load_library().sfmp_check_perm(_host_ptr(p), int(p.size)))


def sfmp_fold_perms(row_perm_prev: np.ndarray, col_perm_next: Optional[np.ndarray]) -> np.ndarray:
    """folded[j] = inverse(row_perm_prev)[col_perm_next[j]] (col_perm_next None = identity), int32."""
    r = np.ascontiguousarray(row_perm_prev, dtype=np.int32)
    c = None if col_perm_next is None else np.ascontiguousarray(col_perm_next, dtype=np.int32)
    out = np.empty(r.size, dtype=np.int32)
    _check(load_library().sfmp_fold_perms(_host_ptr(r), None if c is None else _host_ptr(c), int(r.size),
                                          _host_ptr(out)))
    return out


@dataclass
class DevicePacked:
    """Device-resident packed matrix (torch tensors own the memory)."""
    layout: SfmpLayout
    s2: object
    s3: object
    s4: object
    index: object
    scales: object
    zeros: object
    bitmap: object


def upload_packed(layout, s2, s3, s4, index, scales, zeros, bitmap, device="cuda:0") -> DevicePacked:
    import torch

    def up(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(device)

    def bits(a):
        """The 16 stored bits of each parameter: fp16 arrays as they are, float32 arrays (bf16 values) by their top
        half; handed to torch as float16 storage, which the library reads as raw 16-bit words."""
        a = np.ascontiguousarray(a)
        if a.dtype == np.float32:
            a = (a.view(np.uint32) >> 16).astype(np.uint16)
        return a.view(np.float16)

    return DevicePacked(layout, up(s2), up(s3), up(s4), up(index), up(bits(scales)), up(bits(zeros)),
                        up(bitmap.astype(np.int8)))


def sfmp_layout_set_quant(layout: SfmpLayout, group: int = 128, scale_format: str = "fp16") -> SfmpLayout:
    """Sets the group length (128 / 256 / 512) and the storage type ("fp16" / "bf16") of scales and zeros."""
    _check(load_library().sfmp_layout_set_quant(C.byref(layout), int(group), {"fp16": 0, "bf16": 1}[scale_format]))
    return layout


def sfmp_unpack(layout: SfmpLayout, s2, s3, s4, index, codes_out, stream=None) -> None:
    _check(load_library().sfmp_unpack(C.byref(layout), _dev_ptr(s2), _dev_ptr(s3), _dev_ptr(s4), _dev_ptr(index),
                                      _dev_ptr(codes_out), _stream_ptr(stream)))


def sfmp_gemm_workspace(layout: SfmpLayout, M: int) -> int:
    n = C.c_int64(0)
    _check(load_library().sfmp_gemm_workspace(C.byref(layout), int(M), C.byref(n)))
    return int(n.value)


def sfmp_workspace_init(workspace, stream=None) -> None:
    nbytes = workspace.numel() * workspace.element_size()
    _check(load_library().sfmp_workspace_init(_dev_ptr(workspace), nbytes, _stream_ptr(stream)))


def sfmp_gemm(X, col_perm, layout: SfmpLayout, s2, s3, s4, index, scales, zeros, bitmap, row_perm, Y, workspace,
              stream=None) -> None:
    M = int(X.shape[0])
    nbytes = workspace.numel() * workspace.element_size()
    _check(load_library().sfmp_gemm(_dev_ptr(X), M, _dev_ptr(col_perm), C.byref(layout), _dev_ptr(s2), _dev_ptr(s3),
                                    _dev_ptr(s4), _dev_ptr(index), _dev_ptr(scales), _dev_ptr(zeros),
                                    _dev_ptr(bitmap), _dev_ptr(row_perm), _dev_ptr(Y), _dev_ptr(workspace), nbytes,
                                    _stream_ptr(stream)))


def sfmp_gemm_static(X, col_perm, layout: SfmpLayout, s2, s3, s4, index, scales, zeros, bitmap, row_perm, Y,
                     stream=None) -> None:
    """sfmp_gemm on the library's own static scratch memory (no workspace argument, no allocation)."""
    M = int(X.shape[0])
    _check(load_library().sfmp_gemm_static(_dev_ptr(X), M, _dev_ptr(col_perm), C.byref(layout), _dev_ptr(s2),
                                           _dev_ptr(s3), _dev_ptr(s4), _dev_ptr(index), _dev_ptr(scales),
                                           _dev_ptr(zeros), _dev_ptr(bitmap), _dev_ptr(row_perm), _dev_ptr(Y),
                                           _stream_ptr(stream)))


def make_gemv_batch(problems):
    """Marshal a list of (X, col_perm, DevicePacked, row_perm, Y) into a ctypes array for sfmp_gemv_batched.

    Returns (array, keepalive); keep `keepalive` referenced for as long as the array is used."""
    arr = (SfmpGemvProblem * len(problems))()
    keep = []
    for i, (X, cp, dp, rp, Y) in enumerate(problems):
        def ptr(t):
            return t.data_ptr() if t is not None and t.numel() else None
        arr[i].X, arr[i].col_perm = ptr(X), ptr(cp)
        arr[i].layout = C.addressof(dp.layout)
        arr[i].s2, arr[i].s3, arr[i].s4, arr[i].index = ptr(dp.s2), ptr(dp.s3), ptr(dp.s4), ptr(dp.index)
        arr[i].scales, arr[i].zeros, arr[i].bitmap = ptr(dp.scales), ptr(dp.zeros), ptr(dp.bitmap)
        arr[i].row_perm, arr[i].Y = ptr(rp), ptr(Y)
        keep.append((X, cp, dp, rp, Y))
    return arr, keep


def sfmp_gemv_batched(problems, stream=None) -> None:
    """problems: list of (X [1,K] fp16, col_perm or None, DevicePacked, row_perm or None, Y [1,N] fp16)."""
    arr, _keep = make_gemv_batch(problems)
    _check(load_library().sfmp_gemv_batched(C.cast(arr, C.c_void_p), len(problems), _stream_ptr(stream)))


def sfmp_gemm_batched_workspace(problems, M: int) -> int:
    """Workspace bytes for sfmp_gemm_batched on these problems (tuples as for sfmp_gemv_batched, X [M,K], Y [M,N])."""
    arr, _keep = make_gemv_batch(problems)
    out = C.c_int64(0)
    _check(load_library().sfmp_gemm_batched_workspace(C.cast(arr, C.c_void_p), len(problems), C.c_int32(M),
                                                      C.byref(out)))
    return int(out.value)


def sfmp_gemm_batched(problems, M: int, workspace, stream=None) -> None:
    """Up to 8 independent products with a common M <= 16 in one launch (plus one staging launch for M >= 2)."""
    arr, _keep = make_gemv_batch(problems)
    _check(load_library().sfmp_gemm_batched(C.cast(arr, C.c_void_p), len(problems), C.c_int32(M),
                                            C.c_void_p(workspace.data_ptr()), C.c_int64(workspace.numel()),
                                            _stream_ptr(stream)))


def sfmp_lut_pack(codes: np.ndarray, bitmap: np.ndarray):
    """codes [N, K] uint8, bitmap [N/128, K/128] int8 (host) -> (planes uint8 [bytes], tile_off uint32 [ntiles + 1])."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    bitmap = np.ascontiguousarray(bitmap, dtype=np.int8)
    N, K = codes.shape
    nbytes, words = C.c_int64(0), C.c_int64(0)
    lib = load_library()
    _check(lib.sfmp_lut_pack_query(_host_ptr(bitmap), N, K, C.byref(nbytes), C.byref(words)))
    planes = np.zeros(int(nbytes.value), dtype=np.uint8)
    tile_off = np.zeros(int(words.value), dtype=np.uint32)
    _check(lib.sfmp_lut_pack(_host_ptr(codes), _host_ptr(bitmap), N, K, _host_ptr(planes), _host_ptr(tile_off)))
    return planes, tile_off


def sfmp_lut_gemv_workspace(N: int, K: int) -> int:
    out = C.c_int64(0)
    _check(load_library().sfmp_lut_gemv_workspace(int(N), int(K), C.byref(out)))
    return int(out.value)


LUT_TABLE_FORMATS = {"fp32": 0, "fp16": 1}


def sfmp_lut_gemv(X, col_perm, N: int, K: int, planes, tile_off, scales, zeros, row_perm, Y, workspace,
                  stream=None, table_format="fp32") -> None:
    """Device tensors throughout (see include/sfmp.h): X fp16 [K], Y fp16 [N]; table_format "fp32", "fp16" or the
    header's integer."""
    nbytes = workspace.numel() * workspace.element_size()
    fmt = LUT_TABLE_FORMATS[table_format] if isinstance(table_format, str) else int(table_format)
    _check(load_library().sfmp_lut_gemv(_dev_ptr(X), _dev_ptr(col_perm), int(N), int(K), _dev_ptr(planes),
                                        _dev_ptr(tile_off), _dev_ptr(scales), _dev_ptr(zeros), _dev_ptr(row_perm),
                                        _dev_ptr(Y), fmt, _dev_ptr(workspace), nbytes, _stream_ptr(stream)))
