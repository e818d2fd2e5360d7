"""Helpers for the GPU parity tests: torch is used for device memory only."""
import numpy as np
import torch

LOGIT_RTOL = 2e-2      # max |delta| <= 2e-2 * max(1, |ref|)   (tolerance of the benchmark definition)
BIT_GUARD = 1e-2       # hard bits must agree wherever |oracle logit| > 1e-2
FLAT_RTOL = LOGIT_RTOL  # flat (one-colour) images are held to the same bound; reported apart when it differs


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def empty(shape, dtype):
    return torch.empty(shape, dtype=dtype, device="cuda")


def check_logits(gpu_logits, ref_logits, gpu_bits=None, what="", flat=None):
    """flat: optional bool mask of images that are flat (one colour): held to FLAT_RTOL, reported apart."""
    g = np.asarray(gpu_logits, dtype=np.float64)
    r = np.asarray(ref_logits, dtype=np.float64)
    assert np.isfinite(g).all(), f"{what}: non-finite logits"
    if flat is not None and np.any(flat) and FLAT_RTOL != LOGIT_RTOL:
        flat = np.asarray(flat, dtype=bool)
        ef = np.abs(g[flat] - r[flat]) / np.maximum(1.0, np.abs(r[flat]))
        print(f"[parity] {what}: {int(flat.sum())} flat images, max scaled logit error {float(ef.max()):.3e} (limit {FLAT_RTOL})")
        assert float(ef.max()) <= FLAT_RTOL, f"{what}: logit error {float(ef.max())} on flat images"
        if gpu_bits is not None:
            assert np.array_equal(np.asarray(gpu_bits)[flat], (g[flat] > 0).astype(np.uint8))
        if not np.any(~flat):
            return float(ef.max())
        g, r = g[~flat], r[~flat]
        gpu_bits = None if gpu_bits is None else np.asarray(gpu_bits)[~flat]
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
