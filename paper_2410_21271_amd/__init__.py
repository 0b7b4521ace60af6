"""MI355X (gfx950) library for the EoRA compensated compressed linear layer
y = x.What^T + (x.A^T).B^T  (arXiv 2410.21271, Sec. 3 forward equation; Alg. 1 step 7).

This package is only the thin ctypes binding of libeora.so: argument marshalling, no arithmetic.
Every step of the layer runs in the HIP kernels under csrc/.  Importing the binding fails loudly
when the shared library has not been built (python paper_2410_21271_amd/build.py).
"""
from .binding import (  # noqa: F401
    EoraError, lib, lib_path, status_string,
    qweight_bytes, qzeros_bytes, scales_bytes, sp24_values_bytes, sp24_indices_bytes, workspace_bytes, workspace_bytes_group,
    workspace_init, workspace_error, debug_set_spin_limit, debug_set_resident_min_blocks, debug_set_factors_route, debug_last_launch, debug_probe, new_workspace,
    pack_q, pack_factor_f16, pack_factor_q4, pack_factor_q3, pack_sp24,
    linear_q, linear_q_static, linear_q_group, linear_sp24, unpack_q, dequant_q, expand_sp24,
    sp24q4_tiles_bytes, sp24q4_meta_bytes, pack_sp24q4, linear_sp24q4, expand_sp24q4,
    factors_workspace_bytes, factors, linear_q_multi, factors_store_f16, factors_store_q, linear_sp24_group,
)
