"""MI355X-native SFMP mixed-precision GEMM/GEMV: thin Python binding over the C ABI (libsfmp.so).

Argument marshalling only; every step of the path runs in the HIP kernels of the library.
The names mirror include/sfmp.h.
"""
from .binding import (  # noqa: F401
    SfmpError,
    SfmpLayout,
    DevicePacked,
    lib_path,
    load_library,
    sfmp_strerror,
    sfmp_pack_query,
    sfmp_layout_set_quant,
    sfmp_pack,
    sfmp_unpack,
    sfmp_gemm_workspace,
    sfmp_workspace_init,
    sfmp_gemm,
    sfmp_gemm_static,
    sfmp_gemv_batched,
    sfmp_gemm_batched,
    sfmp_gemm_batched_workspace,
    make_gemv_batch,
    sfmp_check_perm,
    sfmp_fold_perms,
    sfmp_lut_pack,
    sfmp_lut_gemv_workspace,
    sfmp_lut_gemv,
    upload_packed,
)
