"""Oracle for variance-based tile selection.  TEST INFRASTRUCTURE ONLY (same rules as oracle/__init__.py).

What it follows: Listing 1 (Section 6), the user-defined tiling strategy `select_patch`: the image is cut
into windows of the tile size at half-tile stride (64 and 32 in the listing), every window gets the
variance of its pixels, per channel, summed over the channels, and the window with the largest value is
the tile that goes to the extractor.

Readings where the listing is loose or silent:
  * the listing takes the argmax along one axis of the window grid only; the reading here is the argmax
    over ALL windows, the first one in row-major order on ties;
  * the variance is the unbiased one (the default of the tensor library the listing is written in);
  * the listing's input is the pre-processed (normalised) image: channel c is scaled by 1/std_c, so its
    variance counts with weight 1/std_c^2 (the mean shift and the common factor 1/255 do not matter).

Exact form.  For a window with n = win*win pixels, S1 = sum x, S2 = sum x^2 over the raw u8 values,
    n (n-1) var = n S2 - S1^2          (an integer, below 2^53 for win <= 512)
and the score of a window is
    score = ((V_0 * w_0) + V_1 * w_1) + V_2 * w_2,   V_c = float64(n S2_c - S1_c^2),   w_c given (float64),
evaluated in IEEE float64 in exactly this order without fused multiply-add, so that two implementations
agree bit for bit.  It equals 255^2 n (n-1) times the listing's sum of variances when w_c = 1/std_c^2.

Pins (tests/test_oracle_tileselect.py): a window worked out by hand, numpy's var(ddof=1), the listing's
own expression evaluated by torch on the normalised image, constant images, planted high-variance windows,
the tie rule.
"""
from __future__ import annotations

import numpy as np


def window_scores(images, win: int, stride: int, chan_weight) -> np.ndarray:
    """images u8 [N,C,H,W] -> scores f64 [N, nH*nW], windows in row-major order."""
    images = np.asarray(images, dtype=np.uint8)
    N, C, H, W = images.shape
    w = np.asarray(chan_weight, dtype=np.float64)
    assert w.shape == (C,)
    assert 0 < win <= min(H, W) and stride > 0 and win <= 512
    nH, nW = (H - win) // stride + 1, (W - win) // stride + 1
    n = win * win
    scores = np.zeros((N, nH * nW), dtype=np.float64)
    for i in range(N):
        for wy in range(nH):
            for wx in range(nW):
                acc = np.float64(0.0)
                for c in range(C):
                    blk = images[i, c, wy * stride:wy * stride + win, wx * stride:wx * stride + win].astype(np.int64)
                    s1, s2 = int(blk.sum()), int((blk * blk).sum())
                    v = n * s2 - s1 * s1                      # exact (python integer)
                    term = np.float64(v) * w[c]               # one rounding
                    acc = term if c == 0 else acc + term      # one rounding per addition
                scores[i, wy * nW + wx] = acc
    return scores


def select_tiles_variance(images, win: int, stride: int, chan_weight):
    """-> (off_yx i32 [N,2], scores f64 [N, nH*nW]): origin of the first window with the largest score."""
    scores = window_scores(images, win, stride, chan_weight)
    N, _, H, W = np.asarray(images).shape
    nW = (W - win) // stride + 1
    off = np.zeros((N, 2), dtype=np.int32)
    for i in range(N):
        best = 0
        for j in range(1, scores.shape[1]):
            if scores[i, j] > scores[i, best]:                # strict: the first maximum wins
                best = j
        off[i] = (best // nW * stride, best % nW * stride)
    return off, scores
