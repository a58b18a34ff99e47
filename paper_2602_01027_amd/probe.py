"""Binding of libsfmp_probe.so, the benchmark's streaming-read probe (csrc/sfmp_probe.h).  Not part of the product
library; only bench.py uses it."""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


def lib_path() -> str:
    return os.path.join(_HERE, "libsfmp_probe.so")


def load_library():
    global _LIB
    if _LIB is None:
        if not os.path.exists(lib_path()):
            raise FileNotFoundError(f"{lib_path()} is missing: build it with `python -m paper_2602_01027_amd.build`")
        lib = C.CDLL(lib_path())
        lib.sfmp_probe_stream_read.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        lib.sfmp_probe_stream_read.restype = C.c_int
        lib.sfmp_probe_mfma_dot.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        lib.sfmp_probe_mfma_dot.restype = C.c_int
        _LIB = lib
    return _LIB


def stream_read(src, out, stream=None) -> None:
    """Reads the device tensor `src` (a multiple of 16 bytes) once; `out` = device tensor of at least 2048 bytes."""
    import torch
    nbytes = src.numel() * src.element_size()
    assert out.numel() * out.element_size() >= 2048
    s = stream if stream is not None else torch.cuda.current_stream()
    rc = load_library().sfmp_probe_stream_read(C.c_void_p(src.data_ptr()), nbytes, C.c_void_p(out.data_ptr()),
                                               C.c_void_p(s.cuda_stream))
    if rc != 0:
        raise RuntimeError(f"sfmp_probe_stream_read failed with {rc}")


def mfma_dot(a, b, stream=None):
    """out [n] fp32 (device) = element (0, 0) of one v_mfma_f32_16x16x32_f16 per row of the device tensors a, b (fp16
    [n, 32]): A row 0 = a[t], B column 0 = b[t], everything else zero."""
    import torch
    assert a.dtype == torch.float16 and b.dtype == torch.float16 and a.shape == b.shape and a.shape[1] == 32
    assert a.is_contiguous() and b.is_contiguous()
    out = torch.empty(a.shape[0], dtype=torch.float32, device=a.device)
    s = stream if stream is not None else torch.cuda.current_stream()
    rc = load_library().sfmp_probe_mfma_dot(C.c_void_p(a.data_ptr()), C.c_void_p(b.data_ptr()), int(a.shape[0]),
                                            C.c_void_p(out.data_ptr()), C.c_void_p(s.cuda_stream))
    if rc != 0:
        raise RuntimeError(f"sfmp_probe_mfma_dot failed with {rc}")
    return out
