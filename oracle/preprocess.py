"""Oracle for the fused pre-processing step.  TEST INFRASTRUCTURE ONLY (same rules as oracle/__init__.py).

What it follows: Table 1 (pre-process stage: resize to x, centre crop x, to tensor, normalise) and Appendix A
"Kernel Fusion for Preprocessing" (raw image -> resize -> centre crop -> normalise consumed from the raw
buffer in one pass, "a unified affine mapping"), followed by the tile crop of Section 4.3.  Normalisation
is not done here: the detection path applies it inside the first convolution, so this step ends at the
u8 tensor a tile is cut from.

Readings (the paper names the operations, not their arithmetic):
  * raw image: u8, height x width x 3 interleaved (what an image decoder hands over);
  * resize: the shorter side becomes x, the longer one floor(x * long / short) (at least x); bilinear with
    pixel centres at half-integers and no anti-aliasing filter: the source coordinate of destination row Y
    is (Y + 1/2) * H_in / H_r - 1/2, clamped to [0, H_in - 1];
  * centre crop: rows [(H_r - x) // 2, ... + x) and the same for columns;
  * to tensor: planar channel order, one plane per colour;
  * fixed-point interpolation, so that every implementation gets the same bytes: the fractional part of a
    source coordinate is rounded to 11 bits (w1 = round(frac * 2048), w0 = 2048 - w1), the four products
    pixel * wy * wx are added exactly, and the sum is rounded half up: (sum + 2^21) >> 22;
  * a tile (origin inside the cropped x by x image, clamped as in the tile crop) restricts the rows and
    columns that are produced; nothing else of the image is computed.

Everything is integer arithmetic.  Pins (tests/test_oracle_preprocess.py): identity size (a plain centre
crop), constant images, exact 2:1 reduction (2 x 2 means, rounded half up), a library's bilinear
interpolation in float64 (agreement within one grey level, the fixed-point weights being the only
difference), hand-computed pixels, and that a tile equals the same window of the full result.
"""
from __future__ import annotations

import numpy as np

COEF_BITS = 11
ONE = 1 << COEF_BITS


def resized_shape(H_in: int, W_in: int, x: int):
    if H_in <= W_in:
        return x, max(x, x * W_in // H_in)
    return max(x, x * H_in // W_in), x


def source_taps(dst: int, n_in: int, n_res: int):
    """Destination index in the resized axis -> (i0, i1, w0, w1): taps and 11-bit weights."""
    num = (2 * dst + 1) * n_in - n_res          # numerator of the source coordinate over 2 * n_res
    den = 2 * n_res
    if num < 0:
        num = 0
    i0, a = num // den, num % den
    if i0 >= n_in - 1:
        i0, a = n_in - 1, 0
    i1 = min(i0 + 1, n_in - 1)
    w1 = (a * ONE + n_res) // den               # round(frac * 2048)
    return i0, i1, ONE - w1, w1


def preprocess(raw, x: int, off_yx=None, tile: int = 0) -> np.ndarray:
    """raw u8 [N,H_in,W_in,3] -> u8 [N,3,T,T], T = tile or x (tile = 0: the whole cropped image)."""
    raw = np.asarray(raw, dtype=np.uint8)
    N, H_in, W_in, ch = raw.shape
    assert ch == 3
    Hr, Wr = resized_shape(H_in, W_in, x)
    cy, cx = (Hr - x) // 2, (Wr - x) // 2
    T = tile if tile else x
    out = np.zeros((N, 3, T, T), dtype=np.uint8)
    for n in range(N):
        oy = ox = 0
        if tile and off_yx is not None:
            oy = min(max(int(off_yx[n][0]), 0), x - tile)
            ox = min(max(int(off_yx[n][1]), 0), x - tile)
        ytaps = [source_taps(cy + oy + t, H_in, Hr) for t in range(T)]
        xtaps = [source_taps(cx + ox + t, W_in, Wr) for t in range(T)]
        img = raw[n].astype(np.int64)
        for ty, (y0, y1, wy0, wy1) in enumerate(ytaps):
            for tx, (x0, x1, wx0, wx1) in enumerate(xtaps):
                for c in range(3):
                    s = (img[y0, x0, c] * wy0 * wx0 + img[y0, x1, c] * wy0 * wx1 +
                         img[y1, x0, c] * wy1 * wx0 + img[y1, x1, c] * wy1 * wx1)
                    out[n, c, ty, tx] = (int(s) + (1 << (2 * COEF_BITS - 1))) >> (2 * COEF_BITS)
    return out
