"""Pins for the tile-selection oracle (oracle/tileselect.py).

Paper anchor: Listing 1 (Section 6), `select_patch`: windows of the tile size at half-tile stride, variance
per window and channel, summed over channels, the largest wins.  Compared with: a window computed by hand,
numpy's unbiased variance, the listing's own expression run by torch on the normalised image, and inputs
whose answer is known by construction.
"""
import numpy as np
import pytest
import torch

from oracle import tileselect

MEAN = np.array([0.485, 0.456, 0.406])
STD = np.array([0.229, 0.224, 0.225])
W_NORM = 1.0 / STD ** 2


def test_one_window_by_hand():
    # window [[0,255],[0,255]]: S1 = 510, S2 = 130050, n = 4: n S2 - S1^2 = 520200 - 260100 = 260100
    # (= n (n-1) var with var = 4 * 127.5^2 / 3 = 21675); second channel constant -> 0; third [[1,2],[3,4]]:
    # S1 = 10, S2 = 30 -> 120 - 100 = 20 (var = 5/3, 12 * 5/3 = 20)
    img = np.zeros((1, 3, 2, 2), dtype=np.uint8)
    img[0, 0] = [[0, 255], [0, 255]]
    img[0, 1] = 77
    img[0, 2] = [[1, 2], [3, 4]]
    s = tileselect.window_scores(img, 2, 1, [1.0, 1.0, 1.0])
    assert s.shape == (1, 1) and s[0, 0] == 260100 + 0 + 20
    s = tileselect.window_scores(img, 2, 1, [0.5, 3.0, 2.0])
    assert s[0, 0] == 130050 + 40


@pytest.mark.parametrize("H,W,win,stride", [(16, 16, 8, 4), (24, 40, 8, 4), (64, 64, 32, 16), (20, 31, 6, 5)])
def test_scores_are_scaled_unbiased_variances(H, W, win, stride):
    rng = np.random.default_rng(H * W + win)
    img = rng.integers(0, 256, size=(3, 3, H, W), dtype=np.uint8)
    s = tileselect.window_scores(img, win, stride, W_NORM)
    nH, nW = (H - win) // stride + 1, (W - win) // stride + 1
    n = win * win
    for i in range(3):
        for wy in range(nH):
            for wx in range(nW):
                ref = 0.0
                for c in range(3):
                    blk = img[i, c, wy * stride:wy * stride + win, wx * stride:wx * stride + win].astype(np.float64)
                    ref += np.var(blk, ddof=1) * W_NORM[c]
                assert s[i, wy * nW + wx] == pytest.approx(ref * n * (n - 1), rel=1e-12)


def test_against_the_listing_expression_on_the_normalised_image():
    rng = np.random.default_rng(5)
    img = rng.integers(0, 256, size=(4, 3, 96, 128), dtype=np.uint8)
    win, stride = 64, 32
    x = (torch.from_numpy(img).double() / 255.0 - torch.tensor(MEAN).view(1, 3, 1, 1)) / torch.tensor(STD).view(1, 3, 1, 1)
    p = x.unfold(2, win, stride).unfold(3, win, stride)
    listing = p.var((-1, -2)).sum(1)                          # [N, nH, nW]
    off, s = tileselect.select_tiles_variance(img, win, stride, W_NORM)
    n = win * win
    assert np.allclose(s.reshape(listing.shape), listing.numpy() * (255.0 ** 2 * n * (n - 1)), rtol=1e-10)
    flat = listing.reshape(4, -1)
    nW = listing.shape[2]
    for i in range(4):
        top2 = torch.topk(flat[i], 2).values
        if float(top2[0] - top2[1]) > 1e-9 * float(top2[0]):   # a clear winner: same window
            j = int(flat[i].argmax())
            assert tuple(off[i]) == (j // nW * stride, j % nW * stride)


def test_constant_image_takes_the_first_window():
    img = np.full((2, 3, 32, 48), 200, dtype=np.uint8)
    off, s = tileselect.select_tiles_variance(img, 16, 8, W_NORM)
    assert (s == 0).all() and (off == 0).all()


def test_planted_window_is_found_and_ties_go_to_the_first():
    rng = np.random.default_rng(9)
    img = np.full((3, 3, 64, 64), 128, dtype=np.uint8)
    noise = rng.integers(0, 256, size=(3, 16, 16), dtype=np.uint8)
    img[0, :, 32:48, 16:32] = noise                            # exactly window (wy, wx) = (4, 2) at stride 8
    img[1, :, 8:24, 40:56] = noise
    img[2, :, 8:24, 0:16] = noise                              # two identical windows: the first one wins
    img[2, :, 40:56, 32:48] = noise
    off, s = tileselect.select_tiles_variance(img, 16, 8, W_NORM)
    assert off.tolist() == [[32, 16], [8, 40], [8, 0]]
    assert s[2, 1 * 7 + 0] == s[2, 5 * 7 + 4]


def test_channel_weights_decide():
    img = np.full((1, 3, 8, 16), 10, dtype=np.uint8)
    img[0, 0, :, 0:8] = np.arange(64, dtype=np.uint8).reshape(8, 8)         # variance in channel 0, left window
    img[0, 2, :, 8:16] = (2 * np.arange(64)).astype(np.uint8).reshape(8, 8)  # 4x the variance in channel 2, right
    off, _ = tileselect.select_tiles_variance(img, 8, 8, [1.0, 1.0, 1.0])
    assert off.tolist() == [[0, 8]]
    off, _ = tileselect.select_tiles_variance(img, 8, 8, [5.0, 1.0, 1.0])
    assert off.tolist() == [[0, 0]]
