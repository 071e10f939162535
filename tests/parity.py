"""Helpers shared by the GPU parity tests (no test cases here)."""
import numpy as np

# Spec tolerance for floating-point outputs (bf16 in, fp32 accumulate).
REL_TOL = 2e-2


def rel_err(got, ref):
    """max_i |g_i - r_i| / max(|r_i|, rms(r)): elements smaller than the tensor's RMS are
    judged on absolute error relative to the RMS."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    rms = float(np.sqrt(np.mean(ref * ref)))
    if rms == 0.0:
        return float(np.max(np.abs(got - ref)))
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rms)))
