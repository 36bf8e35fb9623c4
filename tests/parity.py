"""Shared helpers for the GPU parity tests (error metric and tolerances)."""
import numpy as np

# Tolerances on  max|gpu - oracle| / max|oracle|  per tenant output tensor: fp32 tenants accumulate in
# fp32 on the GPU against fp64 in the oracle; bf16 tenants store every graph tensor in bfloat16 on both
# sides and differ by accumulation order plus the one-ulp (2^-8) rounding flips it causes.
TOL = {"f32": 1e-4, "bf16": 2e-2}


def rel_err(gpu, ref):
    ref = ref.astype(np.float64)
    return float(np.abs(gpu.astype(np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))
