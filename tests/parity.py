"""Shared helpers for the GPU parity tests (error metric and tolerances)."""
import numpy as np

# Tolerances on  max|gpu - oracle| / max|oracle|  per tenant output tensor: fp32 tenants accumulate in
# fp32 on the GPU against fp64 in the oracle; bf16 tenants store every graph tensor in bfloat16 on both
# sides and differ by accumulation order plus the one-ulp (2^-8) rounding flips it causes.
TOL = {"f32": 1e-4, "bf16": 2e-2}


def rel_err(gpu, ref):
    ref = ref.astype(np.float64)
    return float(np.abs(gpu.astype(np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


# One operator evaluated by the oracle on the very inputs the GPU operator read ("teacher forced"): the two results
# differ by accumulation order only (fp32 on the GPU, fp64 in the oracle), i.e. far below one bfloat16 unit in the last
# place, so after bfloat16 storage an element is either identical or one unit off (2^-8 .. 2^-7 of its magnitude).
# Normalised by the tensor's largest magnitude that is at most 2^-7.  fp32 tenants keep the end-to-end tolerance.
TOL_ONE_OP = {"f32": 1e-4, "bf16": 2.0 ** -7 * 1.001}
