"""Pins for the pre-processing oracle (oracle/preprocess.py).

Paper anchors: Table 1 (resize to x, centre crop x, to tensor) and Appendix A "Kernel Fusion for
Preprocessing" (one pass from the raw buffer).  Compared with: cases whose answer is known in closed form
(identity size, constant image, exact 2:1 reduction), pixels worked out by hand, and a library's bilinear
interpolation evaluated in float64.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import preprocess as pp


def test_identity_size_is_a_centre_crop():
    rng = np.random.default_rng(1)
    raw = rng.integers(0, 256, size=(2, 16, 24, 3), dtype=np.uint8)      # shorter side 16 = x
    out = pp.preprocess(raw, 16)
    assert pp.resized_shape(16, 24, 16) == (16, 24)
    assert np.array_equal(out, raw[:, :, 4:20, :].transpose(0, 3, 1, 2))
    raw_t = np.ascontiguousarray(raw.transpose(0, 2, 1, 3))              # portrait: rows are cropped
    assert np.array_equal(pp.preprocess(raw_t, 16), raw_t[:, 4:20, :, :].transpose(0, 3, 1, 2))


def test_constant_image_stays_constant():
    raw = np.full((1, 37, 53, 3), 0, dtype=np.uint8)
    raw[..., 0], raw[..., 1], raw[..., 2] = 7, 200, 255
    out = pp.preprocess(raw, 24)
    assert (out[0, 0] == 7).all() and (out[0, 1] == 200).all() and (out[0, 2] == 255).all()


def test_exact_two_to_one_reduction_is_the_rounded_block_mean():
    rng = np.random.default_rng(2)
    raw = rng.integers(0, 256, size=(1, 32, 32, 3), dtype=np.uint8)
    out = pp.preprocess(raw, 16)
    blocks = raw[0].astype(np.int64).reshape(16, 2, 16, 2, 3).sum(axis=(1, 3))     # sums of 2 x 2 blocks
    want = ((blocks + 2) // 4).transpose(2, 0, 1)                                    # mean, rounded half up
    assert np.array_equal(out[0], want)


def test_taps_by_hand():
    # 4 -> 8 (enlarging by two): destination 0 sits at source -0.25 -> clamped to 0; destination 1 at 0.25;
    # destination 2 at 0.75; destination 7 at 3.25 -> clamped to the last sample
    assert pp.source_taps(0, 4, 8) == (0, 1, 2048, 0)
    assert pp.source_taps(1, 4, 8) == (0, 1, 1536, 512)
    assert pp.source_taps(2, 4, 8) == (0, 1, 512, 1536)
    assert pp.source_taps(7, 4, 8) == (3, 3, 2048, 0)
    # 3 -> 2: destination 0 at 0.25, destination 1 at 1.75
    assert pp.source_taps(0, 3, 2) == (0, 1, 1536, 512)
    assert pp.source_taps(1, 3, 2) == (1, 2, 512, 1536)
    # one row [0, 100, 200] stretched over three rows -> 3 x 3 image reduced to 2 x 2:
    raw = np.zeros((1, 3, 3, 3), dtype=np.uint8)
    raw[0, :, :, 0] = [[0, 100, 200]] * 3
    out = pp.preprocess(raw, 2)
    assert out[0, 0].tolist() == [[25, 175], [25, 175]]          # 0.75*0 + 0.25*100, 0.25*100 + 0.75*200


@pytest.mark.parametrize("H,W,x", [(48, 64, 32), (50, 37, 24), (20, 31, 28), (96, 96, 40), (33, 70, 33)])
def test_against_library_bilinear_in_float64(H, W, x):
    rng = np.random.default_rng(H + W + x)
    raw = rng.integers(0, 256, size=(2, H, W, 3), dtype=np.uint8)
    out = pp.preprocess(raw, x).astype(np.float64)
    Hr, Wr = pp.resized_shape(H, W, x)
    t = torch.from_numpy(raw).permute(0, 3, 1, 2).double()
    ref = F.interpolate(t, size=(Hr, Wr), mode="bilinear", align_corners=False, antialias=False)
    cy, cx = (Hr - x) // 2, (Wr - x) // 2
    ref = ref[:, :, cy:cy + x, cx:cx + x].numpy()
    d = np.abs(out - ref)
    assert d.max() <= 0.5 + 255 * 2.0 / 2048 + 1e-9          # rounding + two quantised weights
    assert np.abs(out - np.floor(ref + 0.5)).max() <= 1       # at most one grey level from the float result
    assert (out == np.floor(ref + 0.5)).mean() > 0.95


def test_a_tile_is_a_window_of_the_full_result_and_origins_are_clamped():
    rng = np.random.default_rng(3)
    raw = rng.integers(0, 256, size=(3, 40, 56, 3), dtype=np.uint8)
    full = pp.preprocess(raw, 32)
    off = np.array([[0, 0], [5, 9], [100, -4]], dtype=np.int32)
    tiles = pp.preprocess(raw, 32, off, 12)
    assert np.array_equal(tiles[0], full[0, :, 0:12, 0:12])
    assert np.array_equal(tiles[1], full[1, :, 5:17, 9:21])
    assert np.array_equal(tiles[2], full[2, :, 20:32, 0:12])    # clamped to [0, 32 - 12]
