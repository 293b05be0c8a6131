"""Error metrics and gates for comparing the HIP path with the oracle.

bf16 KV: max-abs <= 1e-2 and relative L2 <= 5e-3, the latter taken per sequence (worst one
gates).  fp8 KV: max-abs <= 5e-2 against the oracle run on the dequantised values."""
import numpy as np

from paper_2605_06068_amd import workloads as W

BF16_MAX_ABS = 1e-2
BF16_REL_L2 = 5e-3
FP8_MAX_ABS = 5e-2


def errors(got: np.ndarray, want: np.ndarray):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape
    max_abs = float(np.max(np.abs(got - want))) if got.size else 0.0
    rel = 0.0
    for b in range(got.shape[0]):
        den = np.linalg.norm(want[b])
        num = np.linalg.norm(got[b] - want[b])
        if den > 0:
            rel = max(rel, float(num / den))
        else:
            assert num == 0
    return max_abs, rel


def assert_parity(got, want, kv_dtype, what=""):
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    max_abs, rel = errors(got, want)
    if kv_dtype == W.KV_BF16:
        assert max_abs <= BF16_MAX_ABS and rel <= BF16_REL_L2, f"{what}: max_abs={max_abs:.3e} rel_l2={rel:.3e}"
    else:
        assert max_abs <= FP8_MAX_ABS, f"{what}: max_abs={max_abs:.3e} rel_l2={rel:.3e}"
    return max_abs, rel
