"""MI355X-native half-precision GEMM: thin Python binding over the C ABI in include/hgemm.h.

All arithmetic runs in the HIP kernels of ``libhgemm.so``; this package only marshals
arguments.  There is no CPU fallback: if the library is missing, import of
``paper_2512_02551_amd.binding`` users fails loudly.
"""
from .binding import (  # noqa: F401
    HgemmError, Layouts, Plan, candidates, hgemm, lib_path, load, padded, plan, plan_choice, predict_us, spec_help,
    status_string, tile_of_workgroup, tiles, calibrate_mfma, calibrate_hbm_read, EXPORTS, run_static,
    STATIC_SCRATCH_BYTES, ERR_WORKSPACE,
)
