"""Seeded synthetic inputs for the batched watermark-detection path.

This module only draws random numbers and shapes them: images, tile offsets,
network weights, Reed-Solomon messages and error patterns.  It holds none of
the method's arithmetic (no field arithmetic, no encoding, no convolution), so
the CPU oracle and the HIP path can both be fed from it without sharing code.

Every stream is a Philox counter-based generator keyed by
(BASE_SEED, config index, purpose tag, block index): any image can be
regenerated on its own without generating the ones before it.

The shapes follow the detection set-up of the paper (Section 4.3 and the
experimental set-up of Section 7: 256x256 RGB images, one l x l tile per image,
a 48-bit message by default) as fixed by the five benchmark configurations.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np

BASE_SEED = 250902447

# purpose tags
_T_IMAGE, _T_OFFSET, _T_WEIGHT, _T_RS, _T_FIELD = 1, 2, 3, 4, 5

MEAN = (0.485, 0.456, 0.406)
STD = (0.229, 0.224, 0.225)


@dataclass(frozen=True)
class Config:
    """One benchmark configuration (shapes only)."""
    index: int
    name: str
    n_images: int
    H: int
    W: int
    tile: int
    n_blocks: int
    channels: int
    n_bits: int
    m: int            # bits per RS symbol
    prim_poly: int
    n: int            # RS codeword symbols
    k: int            # RS message symbols
    fcr: int = 1
    n_codewords: int = 0   # size of the separate random-codeword set
    chunk: int = 0         # streaming chunk size (images), 0 = not streamed

    @property
    def t(self) -> int:
        return (self.n - self.k) // 2

    def flops_per_image(self) -> int:
        """Algorithmic conv FLOPs per image: 2*9*C_in*C_out*l^2 per layer."""
        l2 = self.tile * self.tile
        c = self.channels
        first = 2 * 9 * 3 * c * l2
        mid = (self.n_blocks - 1) * 2 * 9 * c * c * l2
        last = 2 * 9 * c * self.n_bits * l2
        return first + mid + last


CONFIGS: Dict[str, Config] = {
    "C1": Config(0, "C1", 16, 256, 256, 32, 4, 32, 60, 4, 0x13, 15, 11, 1, 1024),
    "C2": Config(1, "C2", 4096, 256, 256, 64, 8, 64, 48, 4, 0x13, 12, 8),
    "C3": Config(2, "C3", 4096, 256, 256, 256, 8, 64, 48, 4, 0x13, 12, 8),
    "C4": Config(3, "C4", 16384, 512, 512, 128, 8, 64, 96, 8, 0x11D, 12, 8, 1, 1 << 20),
    "C5": Config(4, "C5", 1 << 20, 256, 256, 64, 8, 64, 48, 4, 0x13, 12, 8, 1, 0, 8192),
}


def _rng(cfg_index: int, tag: int, block: int = 0) -> np.random.Generator:
    ss = np.random.SeedSequence([BASE_SEED, cfg_index, tag, block])
    return np.random.Generator(np.random.Philox(ss))


def images(cfg: Config, start: int, count: int, out: np.ndarray | None = None, threads: int = 1) -> np.ndarray:
    """uint8 [count,3,H,W], uniform 0..255; image i depends only on (cfg.index, i).  threads > 1 fills disjoint
    runs of images from that many host threads (same bytes: every image has its own generator)."""
    per = 3 * cfg.H * cfg.W
    if out is None:
        out = np.empty((count, 3, cfg.H, cfg.W), dtype=np.uint8)
    flat = out.reshape(count, per)

    def fill(lo: int, hi: int) -> None:
        for j in range(lo, hi):
            g = _rng(cfg.index, _T_IMAGE, start + j)
            flat[j] = np.frombuffer(g.bytes(per), dtype=np.uint8)

    if threads <= 1 or count < 2 * threads:
        fill(0, count)
    else:
        from concurrent.futures import ThreadPoolExecutor
        step = (count + threads - 1) // threads
        with ThreadPoolExecutor(threads) as pool:
            list(pool.map(lambda t: fill(t * step, min(count, (t + 1) * step)), range(threads)))
    return out


def field_images(cfg: Config, start: int, count: int) -> np.ndarray:
    """uint8 [count,3,H,W] images that differ from one another in the large: per image and channel a random
    level, a random linear ramp across the image, and uniform noise of a random amplitude (0 = a smooth image),
    clipped to 0..255.  Unlike i.i.d. noise, whose pooled features are the same for every image, these give
    every image its own soft bits; image i depends only on (cfg.index, i).  About a twelfth of the images are
    flat instead (field_is_flat): black, white, or one level per channel."""
    out = np.empty((count, 3, cfg.H, cfg.W), dtype=np.uint8)
    yy, xx = np.meshgrid(np.arange(cfg.H, dtype=np.float64), np.arange(cfg.W, dtype=np.float64), indexing="ij")
    for j in range(count):
        g = _rng(cfg.index, _T_FIELD, start + j)
        flat = int(g.integers(0, 12)) == 0
        level = g.uniform(0.0, 255.0, size=3)
        ramp = g.uniform(-160.0, 160.0, size=(3, 2))        # grey levels across the whole height / width
        amp = g.choice([0.0, 8.0, 48.0, 128.0])
        noise = g.uniform(-1.0, 1.0, size=(3, cfg.H, cfg.W))
        for c in range(3):
            v = level[c] + ramp[c, 0] * (yy / cfg.H - 0.5) + ramp[c, 1] * (xx / cfg.W - 0.5) + amp * noise[c]
            if flat:
                v = np.full_like(v, (0.0, 255.0, level[c])[(start + j) % 3])
            out[j, c] = np.clip(np.rint(v), 0, 255).astype(np.uint8)
    return out


def field_is_flat(cfg: Config, start: int, count: int) -> np.ndarray:
    """bool [count]: which images of field_images(cfg, start, count) are flat."""
    return np.array([int(_rng(cfg.index, _T_FIELD, start + j).integers(0, 12)) == 0 for j in range(count)], dtype=bool)


def offsets(cfg: Config, start: int, count: int, policy: str = "random") -> np.ndarray:
    """int32 [count,2] tile origins (y,x).

    random      : any complete tile, uniform in [0,H-l] x [0,W-l]
    random_grid : a uniformly chosen cell of the size-aligned l x l grid
    fixed       : the top-left corner
    (the three tiling strategies of Table 1 of the paper).  Offsets for image i
    depend only on (cfg.index, policy, i // 4096).
    """
    out = np.zeros((count, 2), dtype=np.int32)
    if policy == "fixed" or cfg.tile >= cfg.H and cfg.tile >= cfg.W:
        return out
    blk = 4096
    ptag = {"random": 0, "random_grid": 1}[policy]
    i = start
    while i < start + count:
        b = i // blk
        g = _rng(cfg.index, _T_OFFSET, 2 * b + ptag)
        if policy == "random":
            ys = g.integers(0, cfg.H - cfg.tile + 1, size=blk, dtype=np.int32)
            xs = g.integers(0, cfg.W - cfg.tile + 1, size=blk, dtype=np.int32)
        else:
            ys = g.integers(0, cfg.H // cfg.tile, size=blk, dtype=np.int32) * cfg.tile
            xs = g.integers(0, cfg.W // cfg.tile, size=blk, dtype=np.int32) * cfg.tile
        lo = i - b * blk
        hi = min(blk, start + count - b * blk)
        out[i - start:i - start + hi - lo, 0] = ys[lo:hi]
        out[i - start:i - start + hi - lo, 1] = xs[lo:hi]
        i += hi - lo
    return out


def extractor_weights(in_ch: int, n_blocks: int, channels: int, n_bits: int,
                      seed_index: int = 0) -> Dict[str, np.ndarray]:
    """Random-init weights of the conv bit-extractor, all fp32.

    conv_w : concatenated OIHW: [C,in_ch,3,3], (n_blocks-1) x [C,C,3,3], [n_bits,C,3,3];
             He-normal, std = sqrt(2 / (9*C_in))
    scale  : [n_blocks*C] ~ N(1, 0.1)   (folded batch-norm scale)
    bias   : [n_blocks*C] ~ N(0, 0.1)   (folded batch-norm bias)
    lin_w  : [n_bits, n_bits] row-major (out, in), std = sqrt(2 / n_bits)
    lin_b  : [n_bits] zeros
    """
    g = _rng(seed_index, _T_WEIGHT, 0)
    c = channels
    parts = []
    cin = in_ch
    for _ in range(n_blocks):
        parts.append(g.normal(0.0, np.sqrt(2.0 / (9 * cin)), size=(c, cin, 3, 3)))
        cin = c
    parts.append(g.normal(0.0, np.sqrt(2.0 / (9 * c)), size=(n_bits, c, 3, 3)))
    conv_w = np.concatenate([p.reshape(-1) for p in parts]).astype(np.float32)
    scale = g.normal(1.0, 0.1, size=n_blocks * c).astype(np.float32)
    bias = g.normal(0.0, 0.1, size=n_blocks * c).astype(np.float32)
    lin_w = g.normal(0.0, np.sqrt(2.0 / n_bits), size=(n_bits, n_bits)).astype(np.float32)
    lin_b = np.zeros(n_bits, dtype=np.float32)
    return {"in_ch": in_ch, "n_blocks": n_blocks, "channels": c, "n_bits": n_bits,
            "conv_w": conv_w, "scale": scale, "bias": bias, "lin_w": lin_w, "lin_b": lin_b,
            "mean": np.array(MEAN, dtype=np.float32), "std": np.array(STD, dtype=np.float32)}


def config_weights(cfg: Config) -> Dict[str, np.ndarray]:
    return extractor_weights(3, cfg.n_blocks, cfg.channels, cfg.n_bits, seed_index=cfg.index)


def rs_cases(cfg_index: int, count: int, n: int, k: int, m: int, max_err: int = 3,
             block: int = 0) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Random messages and symbol-error patterns for a Reed-Solomon test set.

    Returns (msgs u8 [count,k], err u8 [count,n], nerr i32 [count]).  `err` is the
    additive (XOR) error word: `nerr[i]` uniform in 0..max_err, that many distinct
    positions uniform in 0..n-1, each with a uniform non-zero symbol value; zero
    elsewhere.  Encoding the messages is the caller's business.
    """
    g = _rng(cfg_index, _T_RS, block)
    q = 1 << m
    msgs = g.integers(0, q, size=(count, k), dtype=np.uint8)
    nerr = g.integers(0, max_err + 1, size=count, dtype=np.int32)
    # distinct positions: rank of uniform keys
    keys = g.random(size=(count, n))
    order = np.argsort(keys, axis=1)                 # random permutation per row
    vals = g.integers(1, q, size=(count, n), dtype=np.uint8)
    err = np.zeros((count, n), dtype=np.uint8)
    rank = np.empty_like(order)
    rows = np.arange(count)[:, None]
    rank[rows, order] = np.arange(n)[None, :]
    mask = rank < nerr[:, None]
    err[mask] = vals[mask]
    return msgs, err, nerr


def random_words(cfg_index: int, count: int, n: int, m: int, block: int = 1000) -> np.ndarray:
    """Uniformly random received words u8 [count,n] (symbols < 2^m)."""
    g = _rng(cfg_index, _T_RS, block)
    return g.integers(0, 1 << m, size=(count, n), dtype=np.uint8)


def key_cases(cfg_index: int, count: int, k: int, m: int, block: int = 2000) -> Tuple[np.ndarray, np.ndarray]:
    """A secret key and recovered messages to hold against it.

    Returns (key u8 [k], msgs u8 [count,k]).  A third of the messages are the key with 0..k*m/4 randomly
    chosen bits flipped (a watermarked image after decoding), the rest are uniform (an image that carries
    no watermark); message 0 is the key itself.
    """
    g = _rng(cfg_index, _T_RS, block)
    q = 1 << m
    key = g.integers(0, q, size=k, dtype=np.uint8)
    msgs = g.integers(0, q, size=(count, k), dtype=np.uint8)
    marked = g.random(size=count) < 1.0 / 3.0
    if count:
        marked[0] = True
    nflip = g.integers(0, k * m // 4 + 1, size=count)
    if count:
        nflip[0] = 0
    order = np.argsort(g.random(size=(count, k * m)), axis=1)
    for i in np.nonzero(marked)[0]:
        w = key.copy()
        for b in order[i, :nflip[i]]:
            w[b // m] ^= np.uint8(1 << (b % m))
        msgs[i] = w
    return key, msgs
