"""CPU oracle package (test infrastructure only; see pq_oracle.py)."""

from .pq_oracle import (  # noqa: F401
    QMAX, QMIN, build_c, calibrate_absmax, calibrate_mse, calibrate_mse_zp, epilogue, gemm_i64, group_even_odd, hadamard,
    linear, linear_bits, linear_dynamic, linear_zp, minmax_params, pack, quantize, quantize_bits, quantize_dynamic, quantize_groups_dynamic, quantize_heads, quantize_zp, rmsnorm, silu_mul, rotate, threads,
    ungroup_even_odd, unpack, weight_rtn,
)
