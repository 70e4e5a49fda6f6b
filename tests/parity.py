"""Comparison rules for GPU results against the float64 checker.

fp32 inputs: max abs error 1e-5 on outputs and LSE.
bf16 / fp8 inputs: per (row, head) max|gpu-ref| <= 2e-3 * max|ref|, elementwise
|gpu-ref| <= 2e-3*|ref| + 2e-3*rms(ref) (GPU output taken in fp32, before any cast), and LSE within 1e-4 abs.
"""
import numpy as np

FP32_ABS = 1e-5
LOWP_REL = 2e-3
LSE_ABS = 1e-4
MERGE_VS_UNSHARDED_ABS = 1e-5


def check_output(desc, got_o, got_lse, ref_o, ref_lse, what=""):
    got_o = np.asarray(got_o, np.float64)
    got_lse = np.asarray(got_lse, np.float64)
    assert got_o.shape == ref_o.shape and got_lse.shape == ref_lse.shape, what
    assert not np.isnan(got_o).any(), f"{what}: NaN in output"
    err = np.abs(got_o - ref_o)
    if desc.kv_dtype == "f32":
        assert err.max(initial=0) <= FP32_ABS, f"{what}: max abs {err.max():.3e}"
        lse_tol = FP32_ABS
    else:
        ref_max = np.abs(ref_o).max(axis=-1, keepdims=True)
        rms = np.sqrt((ref_o ** 2).mean(axis=-1, keepdims=True))
        worst = (err.max(axis=-1, keepdims=True) / np.maximum(ref_max, 1e-30)).max(initial=0)
        assert np.all(err.max(axis=-1, keepdims=True) <= LOWP_REL * ref_max + 1e-30), \
            f"{what}: row max rel {worst:.3e}"
        assert np.all(err <= LOWP_REL * np.abs(ref_o) + LOWP_REL * rms + 1e-30), f"{what}: elementwise bound"
        lse_tol = LSE_ABS
    fin = np.isfinite(ref_lse)
    assert np.array_equal(np.isneginf(got_lse), np.isneginf(ref_lse)), f"{what}: -inf pattern of LSE"
    if fin.any():
        e = np.abs(got_lse[fin] - ref_lse[fin]).max()
        assert e <= lse_tol, f"{what}: LSE abs {e:.3e}"
    return float(err.max(initial=0))
