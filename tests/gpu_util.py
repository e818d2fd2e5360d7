"""Helpers for the GPU parity tests: torch is used for device memory only."""
import numpy as np
import torch

LOGIT_RTOL = 2e-2      # max |delta| <= 2e-2 * max(1, |ref|)   (tolerance of the benchmark definition)
BIT_GUARD = 1e-2       # hard bits must agree wherever |oracle logit| > 1e-2


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def empty(shape, dtype):
    return torch.empty(shape, dtype=dtype, device="cuda")


def check_logits(gpu_logits, ref_logits, gpu_bits=None, what=""):
    g = np.asarray(gpu_logits, dtype=np.float64)
    r = np.asarray(ref_logits, dtype=np.float64)
    assert np.isfinite(g).all(), f"{what}: non-finite logits"
    err = np.abs(g - r) / np.maximum(1.0, np.abs(r))
    worst = float(err.max())
    print(f"[parity] {what}: max scaled logit error {worst:.3e} (limit {LOGIT_RTOL})")
    assert worst <= LOGIT_RTOL, f"{what}: logit error {worst}"
    if gpu_bits is not None:
        gb = np.asarray(gpu_bits)
        assert np.array_equal(gb, (g > 0).astype(np.uint8)), f"{what}: bits are not (logit > 0)"
        sure = np.abs(r) > BIT_GUARD
        assert np.array_equal(gb[sure], (r[sure] > 0).astype(np.uint8)), f"{what}: hard bits differ"
    return worst
