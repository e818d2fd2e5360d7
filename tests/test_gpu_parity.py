"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bit-exact for tile crops, symbols and Reed-Solomon outputs; extractor logits within
2e-2 * max(1, |ref|) and hard bits equal wherever |oracle logit| > 1e-2.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import dev, empty, check_logits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qrm():
    import paper_2509_02447_amd as q
    return q


def rs_dict(cfg):
    return dict(m=cfg.m, prim_poly=cfg.prim_poly, n=cfg.n, k=cfg.k, fcr=cfg.fcr)


# ---------------------------------------------------------------- Reed-Solomon

def gpu_rs_decode(ctx, words, want_cw=True):
    N, n = words.shape
    d_sym = dev(words)
    d_msg = empty((N, ctx.k), torch.uint8)
    d_cw = empty((N, n), torch.uint8) if want_cw else None
    d_ne = empty((N,), torch.int8)
    ctx.qrm_rs_decode(d_sym, N, d_msg, d_cw, d_ne)
    torch.cuda.synchronize()
    return d_msg.cpu().numpy(), (d_cw.cpu().numpy() if want_cw else None), d_ne.cpu().numpy()


RS_CASES = [
    ("C1 rs(15,11) gf16", dict(m=4, prim_poly=0x13, n=15, k=11, fcr=1), 0, 1024),
    ("C2 rs(12,8) gf16", dict(m=4, prim_poly=0x13, n=12, k=8, fcr=1), 1, 4099),
    ("C4 rs(12,8) gf256", dict(m=8, prim_poly=0x11D, n=12, k=8, fcr=1), 3, 5000),
    ("rs(16,12) gf256 fcr0", dict(m=8, prim_poly=0x11D, n=16, k=12, fcr=0), 5, 777),
    ("rs(20,14) gf256 t3", dict(m=8, prim_poly=0x11D, n=20, k=14, fcr=1), 6, 1001),
    ("rs(63,55) gf64 t4", dict(m=6, prim_poly=0x43, n=63, k=55, fcr=1), 7, 513),
    ("rs(100,84) gf256 t8", dict(m=8, prim_poly=0x11D, n=100, k=84, fcr=1), 8, 300),
    ("rs(255,239) gf256 t8", dict(m=8, prim_poly=0x11D, n=255, k=239, fcr=1), 9, 200),
    ("rs(7,3) gf8", dict(m=3, prim_poly=0xB, n=7, k=3, fcr=1), 10, 640),
    # short codes with t > 2 stay on the kernel with 16 lanes per word; t <= 2 take the one-word-per-lane kernel
    ("rs(15,7) gf16 t4", dict(m=4, prim_poly=0x13, n=15, k=7, fcr=1), 11, 900),
    ("rs(15,9) gf16 t3", dict(m=4, prim_poly=0x13, n=15, k=9, fcr=0), 12, 333),
    ("rs(15,13) gf16 t1", dict(m=4, prim_poly=0x13, n=15, k=13, fcr=1), 13, 1000),
    ("rs(9,7) gf256 t1 fcr0", dict(m=8, prim_poly=0x11D, n=9, k=7, fcr=0), 14, 257),
    ("rs(3,1) gf4 t1", dict(m=2, prim_poly=0x7, n=3, k=1, fcr=1), 15, 130),
]


@pytest.mark.parametrize("name,code,cfg_index,count", RS_CASES, ids=[c[0] for c in RS_CASES])
def test_rs_decode_bit_exact(qrm, name, code, cfg_index, count):
    t = (code["n"] - code["k"]) // 2
    msgs, err, ninj = synth.rs_cases(cfg_index, count, code["n"], code["k"], code["m"], max_err=t + 1)
    clean = oracle.rs_encode(msgs, **code)
    words = clean ^ err
    rand = synth.random_words(cfg_index, count // 2 + 1, code["n"], code["m"])
    allw = np.concatenate([words, rand, clean[:5]], axis=0)
    ctx = qrm.Context(rs=code)
    gm, gc, ge = gpu_rs_decode(ctx, allw)
    om, oc, oe = oracle.rs_decode(allw, **code)
    assert np.array_equal(ge, oe), f"{name}: nerr differs at {np.nonzero(ge != oe)[0][:10]}"
    assert np.array_equal(gm, om) and np.array_equal(gc, oc)
    # and the guarantees themselves, on the GPU output
    ok = ninj <= t
    assert np.array_equal(gm[:count][ok], msgs[ok]) and np.array_equal(ge[:count][ok], ninj[ok].astype(np.int8))
    # without the optional codeword output
    gm2, _, ge2 = gpu_rs_decode(ctx, allw, want_cw=False)
    assert np.array_equal(gm2, gm) and np.array_equal(ge2, ge)
    print(f"[parity] {name}: {allw.shape[0]} words bit-exact, failures flagged: {(ge < 0).sum()}")
    ctx.close()


@pytest.mark.parametrize("N", [1, 3, 4, 5, 63, 64, 65])
def test_rs_decode_small_batches(qrm, N):
    code = dict(m=4, prim_poly=0x13, n=15, k=11, fcr=1)
    msgs, err, _ = synth.rs_cases(0, N, 15, 11, 4, block=N)
    words = oracle.rs_encode(msgs, **code) ^ err
    ctx = qrm.Context(rs=code)
    gm, gc, ge = gpu_rs_decode(ctx, words)
    om, oc, oe = oracle.rs_decode(words, **code)
    assert np.array_equal(ge, oe) and np.array_equal(gm, om) and np.array_equal(gc, oc)
    ctx.close()


def _random_codes(count, seed):
    """Seeded random code parameters over every supported field: (m, prim_poly, n, k, fcr)."""
    prim = {2: 0x7, 3: 0xB, 4: 0x13, 5: 0x25, 6: 0x43, 7: 0x89, 8: 0x11D}
    rng = np.random.default_rng(seed)
    codes = []
    while len(codes) < count:
        m = int(rng.integers(2, 9))
        n = int(rng.integers(3, (1 << m)))
        t = int(rng.integers(1, min(8, (n - 1) // 2) + 1))
        codes.append(dict(m=m, prim_poly=prim[m], n=n, k=n - 2 * t, fcr=int(rng.choice([0, 1, 1, 2, 5, (1 << m) - 2]))))
    return codes


def test_rs_decode_random_code_parameters(qrm):
    """Thirty random codes over GF(4) .. GF(256), full length and shortened, t = 1..8, several first roots: words with
    0 .. t+1 injected errors and plain random words, bit-exact against the oracle (which kernel a code takes - one
    word per lane, 16 or 64 lanes per word - follows from n and t)."""
    for i, code in enumerate(_random_codes(30, 20250902)):
        t = (code["n"] - code["k"]) // 2
        msgs, err, ninj = synth.rs_cases(20 + i, 300, code["n"], code["k"], code["m"], max_err=t + 1)
        clean = oracle.rs_encode(msgs, **code)
        allw = np.concatenate([clean ^ err, synth.random_words(20 + i, 100, code["n"], code["m"])], axis=0)
        ctx = qrm.Context(rs=code)
        gm, gc, ge = gpu_rs_decode(ctx, allw)
        om, oc, oe = oracle.rs_decode(allw, **code)
        assert np.array_equal(ge, oe), f"{code}: nerr differs at {np.nonzero(ge != oe)[0][:10]}"
        assert np.array_equal(gm, om) and np.array_equal(gc, oc), f"{code}"
        ok = ninj <= t
        assert np.array_equal(ge[:300][ok], ninj[ok]) and np.array_equal(gm[:300][ok], msgs[ok]), f"{code}"
        ctx.close()


def test_rs_decode_full_size_sets(qrm):
    """The two stand-alone codeword sets at their full sizes: 1024 x RS(15,11)/GF(16) and
    2^20 x RS(12,8)/GF(256), 0..3 random symbol errors."""
    for cfg in (synth.CONFIGS["C1"], synth.CONFIGS["C4"]):
        code = rs_dict(cfg)
        msgs, err, ninj = synth.rs_cases(cfg.index, cfg.n_codewords, cfg.n, cfg.k, cfg.m)
        words = oracle.rs_encode(msgs, **code) ^ err
        ctx = qrm.Context(rs=code)
        gm, gc, ge = gpu_rs_decode(ctx, words)
        om, oc, oe = oracle.rs_decode(words, **code)
        assert np.array_equal(ge, oe) and np.array_equal(gm, om) and np.array_equal(gc, oc)
        ok = ninj <= cfg.t
        assert np.array_equal(gm[ok], msgs[ok])
        print(f"[parity] {cfg.name} codeword set: {cfg.n_codewords} words bit-exact")
        ctx.close()


def test_rs_symbols_above_field_are_masked(qrm):
    code = dict(m=4, prim_poly=0x13, n=12, k=8, fcr=1)
    msgs, err, _ = synth.rs_cases(1, 100, 12, 8, 4)
    words = oracle.rs_encode(msgs, **code) ^ err
    ctx = qrm.Context(rs=code)
    a = gpu_rs_decode(ctx, words)
    b = gpu_rs_decode(ctx, words | 0xF0)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    ctx.close()


# ---------------------------------------------------------------- tile crop

@pytest.mark.parametrize("N,H,W,tile", [(16, 256, 256, 32), (33, 256, 256, 64), (5, 100, 117, 30),
                                        (4, 64, 64, 64), (7, 50, 90, 17), (3, 512, 512, 128)])
def test_extract_tiles_bit_exact(qrm, N, H, W, tile):
    rng = np.random.default_rng(N * 1000 + tile)
    imgs = rng.integers(0, 256, size=(N, 3, H, W), dtype=np.uint8)
    off = np.stack([rng.integers(-3, H - tile + 4, size=N), rng.integers(-3, W - tile + 4, size=N)], 1).astype(np.int32)
    off[0] = (0, 0)
    off[-1] = (H - tile, W - tile)
    ctx = qrm.Context(rs=dict(m=4, prim_poly=0x13, n=15, k=11))
    d_t = empty((N, 3, tile, tile), torch.uint8)
    ctx.qrm_extract_tiles(dev(imgs), N, H, W, dev(off), tile, d_t)
    torch.cuda.synchronize()
    assert np.array_equal(d_t.cpu().numpy(), oracle.extract_tiles(imgs, off, tile))
    d_t.zero_()
    ctx.qrm_extract_tiles(dev(imgs), N, H, W, None, tile, d_t)       # NULL offsets = top-left ("fixed")
    torch.cuda.synchronize()
    assert np.array_equal(d_t.cpu().numpy(), oracle.extract_tiles(imgs, None, tile))
    ctx.close()


# ---------------------------------------------------------------- extractor

def small_weights(C, nb, nbits, seed):
    return synth.extractor_weights(3, nb, C, nbits, seed_index=200 + seed)


@pytest.mark.parametrize("C,nb,h,w", [(32, 3, 32, 32), (64, 3, 16, 64), (64, 2, 21, 70), (32, 2, 9, 33),
                                      (64, 2, 4, 130), (64, 5, 11, 40), (64, 4, 6, 64)])
def test_extractor_blocks_match_oracle_layer_by_layer(qrm, C, nb, h, w):
    wts = small_weights(C, nb, 16, C + nb)
    rng = np.random.default_rng(h * w)
    tiles = rng.integers(0, 256, size=(2, 3, h, w), dtype=np.uint8)
    ctx = qrm.Context(weights=wts)
    refs = [oracle.extractor_forward(wts, tiles[i:i + 1], want_acts=True)[2] for i in range(2)]
    for b in range(1, nb + 1):
        d_act = empty((2, C, h, w), torch.float32)
        ctx.qrm_extractor_blocks(dev(tiles), 2, h, w, b, d_act)
        torch.cuda.synchronize()
        got = d_act.cpu().numpy().astype(np.float64)
        for i in range(2):
            ref = refs[i][b - 1]
            err = np.abs(got[i] - ref) / np.maximum(1.0, np.abs(ref))
            print(f"[parity] C={C} {h}x{w} block {b} image {i}: max scaled activation error {err.max():.3e}")
            # bf16 operands (weights: relative step 2^-9) and one dithered bf16 rounding per layer (off by up to
            # one step of 2^-8 relative, unbiased): an element of size ~1 built from 27..576 products carries noise
            # of a few 1e-3; the maximum over ~1e5 elements sits near 3e-2.  A wrong tap, channel or halo is an
            # O(1) error in single elements and shows in the rms.
            rms = float(np.sqrt(np.mean((got[i] - ref) ** 2)))
            assert err.max() <= 0.08 and rms <= 0.005 * b + 0.007, (b, i, float(err.max()), rms,
                                                                     np.unravel_index(err.argmax(), err.shape))
    ctx.close()


EXT_CASES = [
    ("C1 shape 32x32 c32 b4 60bit", 32, 4, 60, 32, 32, 16),
    ("C2 shape 64x64 c64 b8 48bit", 64, 8, 48, 64, 64, 6),
    ("C4 shape 128x128 c64 b8 96bit", 64, 8, 96, 128, 128, 2),
    ("ragged 48x80 c64 b3 48bit", 64, 3, 48, 48, 80, 5),
    ("ragged 30x30 c32 b2 60bit", 32, 2, 60, 30, 30, 9),
    ("tiny 5x7 c64 b2 8bit", 64, 2, 8, 5, 7, 3),
    # the fused kernels (64 channels, tiles up to 64 wide) on ragged tiles: pair of C -> C blocks followed by a
    # single last block; last block as the second half of a pair with an odd height; more images than CUs
    ("ragged 23x50 c64 b5 48bit", 64, 5, 48, 23, 50, 3),
    ("ragged 37x64 c64 b6 48bit", 64, 6, 48, 37, 64, 2),
    ("one row 1x64 c64 b4 16bit", 64, 4, 16, 1, 64, 2),
    ("many images 8x16 c64 b4 24bit", 64, 4, 24, 8, 16, 300),
]


@pytest.mark.parametrize("name,C,nb,nbits,h,w,N", EXT_CASES, ids=[c[0] for c in EXT_CASES])
def test_extractor_forward_logits_and_bits(qrm, name, C, nb, nbits, h, w, N):
    wts = small_weights(C, nb, nbits, nb * 7 + nbits)
    rng = np.random.default_rng(nbits + h)
    tiles = rng.integers(0, 256, size=(N, 3, h, w), dtype=np.uint8)
    ref_logits, _ = oracle.extractor_forward(wts, tiles)
    ctx = qrm.Context(weights=wts)
    ctx.qrm_set_micro_batch(4)                     # several micro-batches and a ragged last one
    d_logits, d_bits = empty((N, nbits), torch.float32), empty((N, nbits), torch.uint8)
    ctx.qrm_extractor_forward(dev(tiles), N, h, w, d_logits, d_bits)
    torch.cuda.synchronize()
    check_logits(d_logits.cpu().numpy(), ref_logits, d_bits.cpu().numpy(), what=name)
    ctx.close()


STREAM_CASES = [   # name, blocks, bits, h, w, images: several images per workgroup (one launch for all of them)
    ("8x16 b4, 1100 images", 4, 24, 8, 16, 1100),
    ("23x50 b5, 520 images", 5, 48, 23, 50, 520),
    ("5x64 b3, 1500 images", 3, 16, 5, 64, 1500),
    ("2x9 b2, 777 images", 2, 8, 2, 9, 777),
    ("1x64 b4, 600 images", 4, 16, 1, 64, 600),
    ("7x33 b6, 513 images", 6, 32, 7, 33, 513),
]


@pytest.mark.parametrize("name,nb,nbits,h,w,N", STREAM_CASES, ids=[c[0] for c in STREAM_CASES])
def test_extractor_stream_of_images_per_workgroup(qrm, name, nb, nbits, h, w, N):
    """More images than compute units in one micro-batch: a workgroup of the fused kernels walks through several
    images without draining its pipeline in between (rows of consecutive images share the LDS rings)."""
    wts = small_weights(64, nb, nbits, nb * 5 + nbits)
    rng = np.random.default_rng(nbits * 3 + h)
    tiles = rng.integers(0, 256, size=(N, 3, h, w), dtype=np.uint8)
    tiles[N // 2] = 0                              # a black and a white image in the middle of the stream
    tiles[N // 2 + 1] = 255
    ref_logits, _ = oracle.extractor_forward(wts, tiles)
    ctx = qrm.Context(weights=wts)
    for mb in (0, 300):                            # default (all images at once) and a ragged split
        ctx.qrm_set_micro_batch(mb)
        d_logits, d_bits = empty((N, nbits), torch.float32), empty((N, nbits), torch.uint8)
        ctx.qrm_extractor_forward(dev(tiles), N, h, w, d_logits, d_bits)
        torch.cuda.synchronize()
        g, gb = d_logits.cpu().numpy(), d_bits.cpu().numpy()
        check_logits(g, ref_logits, gb, what=f"{name}, micro-batch {mb}")
        # (a one-colour image is the hardest case for bf16 activations: every pixel of a channel carries the same
        # value, so a rounding error that is the same everywhere survives the average pool: hence the dithered rounding)
        flat = np.abs(g[N // 2:N // 2 + 2] - ref_logits[N // 2:N // 2 + 2]) / np.maximum(1.0, np.abs(ref_logits[N // 2:N // 2 + 2]))
        print(f"[parity] {name}, micro-batch {mb}: the black and the white image, max scaled logit error {flat.max():.3e}")
    ctx.close()


WIDE_CASES = [   # name, blocks, bits, h, w, images, micro-batch: tiles wider than 64 columns on the fused kernels
    ("C4 shape 128x128 b8 96bit", 8, 96, 128, 128, 2, 0),
    ("two blocks 10x128 (first + last fused)", 2, 16, 10, 128, 3, 0),
    ("ragged 20x130 b5", 5, 48, 20, 130, 3, 2),
    ("three column blocks 7x192 b4", 4, 48, 7, 192, 2, 0),
    ("one column over 33x65 b6", 6, 32, 33, 65, 3, 0),
    ("four column blocks 3x256 b3", 3, 16, 3, 256, 2, 0),
    ("ragged 40x100 b8", 8, 48, 40, 100, 2, 0),
    ("one row 1x128 b4", 4, 16, 1, 128, 5, 0),
    ("two images per workgroup 4x128 b4, 300 images", 4, 24, 4, 128, 300, 0),
    ("three images per workgroup 6x70 b5, 520 images in micro-batches of 300", 5, 24, 6, 70, 520, 300),
]


@pytest.mark.parametrize("name,nb,nbits,h,w,N,mb", WIDE_CASES, ids=[c[0] for c in WIDE_CASES])
def test_extractor_wide_tiles_on_fused_kernels(qrm, name, nb, nbits, h, w, N, mb):
    """Tiles of more than one column block through the fused kernels (a workgroup walks through its image column
    block by column block; the columns at the seams travel through a small buffer in global memory, and the last
    column of a width that is a multiple of 64 comes from a launch of its own), forced on also where a launch has
    too few images for that schedule to be chosen.  Against the oracle; twice, for equal bytes."""
    wts = small_weights(64, nb, nbits, nb * 3 + nbits + w)
    rng = np.random.default_rng(nbits + h + w)
    tiles = rng.integers(0, 256, size=(N, 3, h, w), dtype=np.uint8)
    keep = np.arange(N) if N <= 8 else np.unique(np.concatenate([np.arange(4), np.arange(N - 4, N), rng.integers(0, N, 24)]))
    ref_logits, _ = oracle.extractor_forward(wts, tiles[keep])
    ctx = qrm.Context(weights=wts)
    ctx.qrm_diag_set_flags(qrm.binding.QRM_DIAG_FUSE_ALWAYS | qrm.binding.QRM_DIAG_POISON_WORKSPACE)
    ctx.qrm_set_micro_batch(mb)
    runs = []
    for rep in range(2):
        d_logits, d_bits = empty((N, nbits), torch.float32), empty((N, nbits), torch.uint8)
        ctx.qrm_extractor_forward(dev(tiles), N, h, w, d_logits, d_bits)
        torch.cuda.synchronize()
        runs.append((d_logits.cpu().numpy(), d_bits.cpu().numpy()))
    check_logits(runs[0][0][keep], ref_logits, runs[0][1][keep], what=name)
    assert np.isfinite(runs[0][0]).all()
    assert np.array_equal(runs[0][0], runs[1][0]) and np.array_equal(runs[0][1], runs[1][1])
    ctx.close()


@pytest.mark.parametrize("nb,h,w", [(2, 6, 128), (3, 5, 130), (4, 9, 192), (5, 4, 65)])
def test_extractor_wide_tiles_layer_by_layer(qrm, nb, h, w):
    """The activations themselves (not only their pooled sums) of wide tiles on the fused kernels, every pixel and
    channel against the oracle: a wrong seam column or a missing last column is an O(1) error in single pixels
    that global average pooling would hide."""
    wts = small_weights(64, nb, 16, 64 + nb + w)
    rng = np.random.default_rng(h * w)
    tiles = rng.integers(0, 256, size=(2, 3, h, w), dtype=np.uint8)
    ctx = qrm.Context(weights=wts)
    ctx.qrm_diag_set_flags(qrm.binding.QRM_DIAG_FUSE_ALWAYS)
    refs = [oracle.extractor_forward(wts, tiles[i:i + 1], want_acts=True)[2] for i in range(2)]
    for b in range(1, nb + 1):
        d_act = empty((2, 64, h, w), torch.float32)
        ctx.qrm_extractor_blocks(dev(tiles), 2, h, w, b, d_act)
        torch.cuda.synchronize()
        got = d_act.cpu().numpy().astype(np.float64)
        for i in range(2):
            ref = refs[i][b - 1]
            err = np.abs(got[i] - ref) / np.maximum(1.0, np.abs(ref))
            rms = float(np.sqrt(np.mean((got[i] - ref) ** 2)))
            print(f"[parity] wide {h}x{w} block {b} image {i}: max scaled activation error {err.max():.3e}, rms {rms:.3e}")
            assert err.max() <= 0.05 and rms <= 0.004 * b + 0.006, (b, i, float(err.max()), rms,
                                                                     np.unravel_index(err.argmax(), err.shape))
    ctx.close()


def structured_tiles(h, w, seed):
    """Tiles that are anything but stationary noise: one-colour, bands, ramps, halves, fine patterns."""
    rng = np.random.default_rng(seed)
    yy, xx = np.meshgrid(np.arange(h), np.arange(w), indexing="ij")
    t = []
    for level in (0, 255, 128, 1, 77):
        t.append(np.full((3, h, w), level))
    t.append(np.stack([np.full((h, w), v) for v in (200, 30, 111)]))                  # one level per channel
    band = np.zeros((3, h, w)); band[:, :max(1, h // 8)] = 255; t.append(band)         # bright band at the top
    band = np.full((3, h, w), 40); band[:, -max(1, h // 5):] = 230; t.append(band)     # and one at the bottom
    t.append(np.broadcast_to(255.0 * yy / max(1, h - 1), (3, h, w)))                   # vertical ramp
    t.append(np.broadcast_to(255.0 * xx / max(1, w - 1), (3, h, w)))                   # horizontal ramp
    half = np.zeros((3, h, w)); half[:, :, w // 2:] = 255; t.append(half)              # left black, right white
    half = np.zeros((3, h, w)); half[:, h // 2:] = 255; t.append(half)                 # top black, bottom white
    t.append(np.broadcast_to(255.0 * ((yy + xx) & 1), (3, h, w)))                      # one-pixel checkerboard
    t.append(np.broadcast_to(255.0 * (((yy >> 1) + (xx >> 1)) & 1), (3, h, w)))        # two-pixel checkerboard
    t.append(np.broadcast_to(255.0 * ((xx & 3) == 0), (3, h, w)))                      # every fourth column
    t.append(np.clip(128 + 20 * rng.standard_normal((3, h, w)), 0, 255))               # grey with a little noise
    return np.stack([np.rint(np.asarray(a, dtype=np.float64)) for a in t]).astype(np.uint8)


STRUCTURED_CASES = [   # name, channels, blocks, bits, h, w, diagnostic flags
    ("64x64 c64 b8 fused", 64, 8, 48, 64, 64, 0),
    ("64x64 c64 b8 single blocks", 64, 8, 48, 64, 64, 1),
    ("32x32 c32 b4", 32, 4, 60, 32, 32, 0),
    ("128x128 c64 b8 fused, wide", 64, 8, 96, 128, 128, 4),
    ("128x128 c64 b8 single blocks", 64, 8, 96, 128, 128, 0),
    ("40x100 c64 b5 fused, wide", 64, 5, 48, 40, 100, 4),
]


@pytest.mark.parametrize("name,C,nb,nbits,h,w,flags", STRUCTURED_CASES, ids=[c[0] for c in STRUCTURED_CASES])
def test_extractor_structured_tiles(qrm, name, C, nb, nbits, h, w, flags):
    """One-colour, banded, ramped, halved and finely patterned tiles (ordinary detector inputs, and the hard cases
    of bf16 activations and of channel means estimated from sampled rows) at the tolerance of every other tile,
    hard bits included, on the configurations' weights."""
    wts = synth.extractor_weights(3, nb, C, nbits, seed_index={96: 3, 48: 1, 60: 0}[nbits])
    tiles = structured_tiles(h, w, h + w)
    N = tiles.shape[0]
    ref_logits, _ = oracle.extractor_forward(wts, tiles)
    ctx = qrm.Context(weights=wts)
    ctx.qrm_diag_set_flags(flags)
    d_logits, d_bits = empty((N, nbits), torch.float32), empty((N, nbits), torch.uint8)
    ctx.qrm_extractor_forward(dev(tiles), N, h, w, d_logits, d_bits)
    torch.cuda.synchronize()
    g = d_logits.cpu().numpy()
    err = (np.abs(g - ref_logits) / np.maximum(1.0, np.abs(ref_logits))).max(axis=1)
    print(f"[parity] {name}: scaled logit error per tile " + " ".join(f"{e:.1e}" for e in err))
    check_logits(g, ref_logits, d_bits.cpu().numpy(), what=name)
    ctx.close()


def test_extractor_final_relu_and_affine(qrm):
    wts = small_weights(64, 2, 48, 99)
    g = np.random.default_rng(9)
    wts["scale"] = np.concatenate([wts["scale"], g.normal(1, 0.1, 48).astype(np.float32)])
    wts["bias"] = np.concatenate([wts["bias"], g.normal(0, 0.1, 48).astype(np.float32)])
    tiles = g.integers(0, 256, size=(3, 3, 20, 40), dtype=np.uint8)
    for relu in (0, 1):
        ref, _ = oracle.extractor_forward(wts, tiles, final_relu=relu)
        ctx = qrm.Context(weights=wts, final_relu=relu)
        d_logits = empty((3, 48), torch.float32)
        ctx.qrm_extractor_forward(dev(tiles), 3, 20, 40, d_logits, None)
        torch.cuda.synchronize()
        check_logits(d_logits.cpu().numpy(), ref, what=f"final affine, relu={relu}")
        ctx.close()


# ---------------------------------------------------------------- whole path

def run_detect(ctx, cfg, imgs, off, want_all=True):
    N = imgs.shape[0]
    d_logits = empty((N, cfg.n_bits), torch.float32) if want_all else None
    d_bits = empty((N, cfg.n_bits), torch.uint8) if want_all else None
    d_msg, d_cw, d_ne = empty((N, cfg.k), torch.uint8), empty((N, cfg.n), torch.uint8), empty((N,), torch.int8)
    ctx.qrm_detect(dev(imgs), N, cfg.H, cfg.W, None if off is None else dev(off), cfg.tile,
                   d_logits, d_bits, d_msg, d_cw if want_all else None, d_ne)
    torch.cuda.synchronize()
    out = dict(msg=d_msg.cpu().numpy(), nerr=d_ne.cpu().numpy())
    if want_all:
        out.update(logits=d_logits.cpu().numpy(), bits=d_bits.cpu().numpy(), codeword=d_cw.cpu().numpy())
    return out


def check_detect(cfg, wts, imgs, off, got, what):
    ref = oracle.detect(wts, imgs, off, cfg.tile, cfg.m, cfg.prim_poly, cfg.n, cfg.k, cfg.fcr)
    check_logits(got["logits"], ref["logits"], got["bits"], what=what)
    # RS outputs are bit-exact given identical hard bits: decode the GPU's own bits with the oracle
    syms = oracle.bits_to_symbols(got["bits"], cfg.m)
    om, oc, oe = oracle.rs_decode(syms, cfg.m, cfg.prim_poly, cfg.n, cfg.k, cfg.fcr)
    assert np.array_equal(got["msg"], om) and np.array_equal(got["codeword"], oc) and np.array_equal(got["nerr"], oe)
    if np.array_equal(got["bits"], ref["bits"]):
        assert np.array_equal(got["msg"], ref["msg"]) and np.array_equal(got["nerr"], ref["nerr"])


def test_detect_config_c1_every_image(qrm):
    cfg = synth.CONFIGS["C1"]
    wts = synth.config_weights(cfg)
    imgs, off = synth.images(cfg, 0, cfg.n_images), synth.offsets(cfg, 0, cfg.n_images)
    ctx = qrm.Context(weights=wts, rs=rs_dict(cfg))
    got = run_detect(ctx, cfg, imgs, off)
    check_detect(cfg, wts, imgs, off, got, "C1 detect, 16 images")
    lean = run_detect(ctx, cfg, imgs, off, want_all=False)           # optional outputs NULL
    assert np.array_equal(lean["msg"], got["msg"]) and np.array_equal(lean["nerr"], got["nerr"])
    ctx.close()


@pytest.mark.parametrize("policy", ["random", "random_grid", "fixed"])
def test_detect_config_c2_sample(qrm, policy):
    cfg = synth.CONFIGS["C2"]
    wts = synth.config_weights(cfg)
    N = 12
    imgs, off = synth.images(cfg, 100, N), synth.offsets(cfg, 100, N, policy)
    if policy == "random":
        off[0] = (0, 0); off[1] = (cfg.H - cfg.tile, cfg.W - cfg.tile); off[2] = (-7, 400)   # clamped
    ctx = qrm.Context(weights=wts, rs=rs_dict(cfg))
    ctx.qrm_set_micro_batch(5)
    got = run_detect(ctx, cfg, imgs, off)
    check_detect(cfg, wts, imgs, off, got, f"C2 detect ({policy}), {N} images")
    ctx.close()


def test_detect_config_c2_full_size_sampled(qrm):
    """The whole tiled-detection configuration (4096 images) in the launch configuration the benchmark times
    (default micro-batch): extractor outputs of a sample of images against the oracle, one by one - the first and
    last image, both sides of every micro-batch boundary, and a random draw -, the Reed-Solomon outputs of ALL
    images against the oracle's decoder on the device's own hard bits, and bits = (logit > 0) everywhere."""
    cfg = synth.CONFIGS["C2"]
    wts = synth.config_weights(cfg)
    N = cfg.n_images
    imgs, off = synth.images(cfg, 0, N), synth.offsets(cfg, 0, N)
    ctx = qrm.Context(weights=wts, rs=rs_dict(cfg))
    got = run_detect(ctx, cfg, imgs, off)
    ctx.close()
    assert np.isfinite(got["logits"]).all()
    assert np.array_equal(got["bits"], (got["logits"] > 0).astype(np.uint8))
    syms = oracle.bits_to_symbols(got["bits"], cfg.m)
    om, oc, oe = oracle.rs_decode(syms, cfg.m, cfg.prim_poly, cfg.n, cfg.k, cfg.fcr)
    assert np.array_equal(got["msg"], om) and np.array_equal(got["codeword"], oc) and np.array_equal(got["nerr"], oe)
    rng = np.random.default_rng(2)
    sample = sorted(set([0, 1, 255, 256, 1022, 1023, 1024, 1025, 2047, 2048, 3071, 3072, N - 2, N - 1] +
                        rng.integers(0, N, size=18).tolist()))
    ref = oracle.detect(wts, imgs[sample], off[sample], cfg.tile, cfg.m, cfg.prim_poly, cfg.n, cfg.k, cfg.fcr)
    check_logits(got["logits"][sample], ref["logits"], got["bits"][sample], what=f"C2 full size, {len(sample)} sampled images")


HOST_THREADS = min(16, os.cpu_count() or 1)


def sampled_config_parity(qrm, name, N, sample, what, micro_batch=0):
    """qrm_detect over N images of a configuration in its default launch configuration; the images in `sample`
    against the oracle one by one (logits, hard bits), the Reed-Solomon outputs of ALL images against the oracle's
    decoder on the device's own hard bits, and bits = (logit > 0) everywhere."""
    cfg = synth.CONFIGS[name]
    wts = synth.config_weights(cfg)
    imgs = synth.images(cfg, 0, N, threads=HOST_THREADS)
    off = synth.offsets(cfg, 0, N)
    # a few images that differ in the large (ramps, flat levels) instead of noise, on both sides of the first
    # micro-batch boundaries: their bits and error counts differ from image to image
    special = [i for i in sample if i % 3 == 1]
    fld = synth.field_images(cfg, 0, len(special))
    flat = synth.field_is_flat(cfg, 0, len(special))
    for j, i in enumerate(special):
        imgs[i] = fld[j]
    ctx = qrm.Context(weights=wts, rs=rs_dict(cfg))
    if micro_batch:
        ctx.qrm_set_micro_batch(micro_batch)
    got = run_detect(ctx, cfg, imgs, off)
    ctx.close()
    assert np.isfinite(got["logits"]).all()
    assert np.array_equal(got["bits"], (got["logits"] > 0).astype(np.uint8))
    syms = oracle.bits_to_symbols(got["bits"], cfg.m)
    om, oc, oe = oracle.rs_decode(syms, cfg.m, cfg.prim_poly, cfg.n, cfg.k, cfg.fcr)
    assert np.array_equal(got["msg"], om) and np.array_equal(got["codeword"], oc) and np.array_equal(got["nerr"], oe)
    ref = oracle.detect(wts, imgs[sample], off[sample], cfg.tile, cfg.m, cfg.prim_poly, cfg.n, cfg.k, cfg.fcr)
    is_flat = np.array([i in special and bool(flat[special.index(i)]) for i in sample])
    check_logits(got["logits"][sample], ref["logits"], got["bits"][sample], what=what, flat=is_flat)
    same = np.all(got["bits"][sample] == ref["bits"], axis=1)
    assert np.array_equal(got["msg"][sample][same], ref["msg"][same]) and np.array_equal(got["nerr"][sample][same], ref["nerr"][same])
    print(f"[parity] {what}: {int(same.sum())} of {len(sample)} sampled images have every hard bit equal to the oracle's; "
          f"{len(special)} structured images ({int(flat.sum())} flat); distinct messages in the sample: "
          f"{len({tuple(r) for r in got['msg'][sample]})}")
    return got


@pytest.mark.timeout(600)
def test_detect_config_c4_full_micro_batches_sampled(qrm):
    """128 x 128 tiles of 512 x 512 images with byte symbols: 1030 images = several default micro-batches and a
    ragged one; 64 images against the oracle (both sides of every multiple of 256 images, the first and the last
    image, a random draw), every Reed-Solomon output against the oracle's decoder."""
    N = 1030
    rng = np.random.default_rng(4)
    sample = sorted(set([0, 1, 255, 256, 257, 511, 512, 513, 767, 768, 1023, 1024, 1025, N - 2, N - 1] +
                        rng.integers(0, N, size=52).tolist()))[:64]
    sampled_config_parity(qrm, "C4", N, sample, f"C4 detect, {N} images, {len(sample)} sampled")


@pytest.mark.timeout(600)
def test_detect_config_c3_full_micro_batches_sampled(qrm):
    """Untiled 256 x 256 detection: 515 images = several default micro-batches (64 or 256 images) and a ragged
    one; 48 images against the oracle, every Reed-Solomon output against the oracle's decoder."""
    N = 515
    rng = np.random.default_rng(3)
    sample = sorted(set([0, 1, 63, 64, 65, 127, 128, 255, 256, 257, 511, 512, 513, N - 1] +
                        rng.integers(0, N, size=40).tolist()))[:48]
    sampled_config_parity(qrm, "C3", N, sample, f"C3 detect (untiled 256x256), {N} images, {len(sample)} sampled")


def test_detect_config_c4_small_micro_batches(qrm):
    """The same configuration with a micro-batch of 3: many launches, a workgroup sees parts of images only."""
    cfg = synth.CONFIGS["C4"]
    wts = synth.config_weights(cfg)
    N = 7
    imgs, off = synth.images(cfg, 7, N), synth.offsets(cfg, 7, N)
    ctx = qrm.Context(weights=wts, rs=rs_dict(cfg))
    ctx.qrm_set_micro_batch(3)
    got = run_detect(ctx, cfg, imgs, off)
    check_detect(cfg, wts, imgs, off, got, f"C4 detect, {N} images, micro-batch 3")
    ctx.close()


def test_detect_equals_separate_calls(qrm):
    """qrm_detect == qrm_extract_tiles -> qrm_extractor_forward -> (pack) -> qrm_rs_decode, bit for bit."""
    cfg = synth.CONFIGS["C2"]
    wts = synth.config_weights(cfg)
    N = 9
    imgs, off = synth.images(cfg, 50, N), synth.offsets(cfg, 50, N)
    ctx = qrm.Context(weights=wts, rs=rs_dict(cfg))
    got = run_detect(ctx, cfg, imgs, off)
    d_tiles = empty((N, 3, cfg.tile, cfg.tile), torch.uint8)
    ctx.qrm_extract_tiles(dev(imgs), N, cfg.H, cfg.W, dev(off), cfg.tile, d_tiles)
    d_logits, d_bits = empty((N, cfg.n_bits), torch.float32), empty((N, cfg.n_bits), torch.uint8)
    ctx.qrm_extractor_forward(d_tiles, N, cfg.tile, cfg.tile, d_logits, d_bits)
    torch.cuda.synchronize()
    assert np.array_equal(d_logits.cpu().numpy(), got["logits"]) and np.array_equal(d_bits.cpu().numpy(), got["bits"])
    syms = oracle.bits_to_symbols(d_bits.cpu().numpy(), cfg.m)
    gm, gc, ge = gpu_rs_decode(ctx, syms)
    assert np.array_equal(gm, got["msg"]) and np.array_equal(gc, got["codeword"]) and np.array_equal(ge, got["nerr"])
    ctx.close()


@pytest.mark.parametrize("flag,tol", [("QRM_DIAG_POISON_WORKSPACE", 0.0), ("QRM_DIAG_NO_FUSED_PAIRS", 2 * 2e-2)])
def test_diagnostic_flags_do_not_change_results(qrm, flag, tol):
    """The library's two diagnostic flags against the plain run.  Poisoned workspaces (every new one filled with
    0xFF bytes, NaN as bf16 and as fp32): no kernel reads workspace bytes that no kernel wrote, and sums are formed
    in a fixed order, so the results are the same bit for bit.  Unfused blocks (one launch per block): another
    schedule and other roundings of the same layers, so the two results, each within the tolerance of the exact
    one, lie within twice that of each other."""
    import poison_cases
    mine = poison_cases.run_cases(0)
    theirs = poison_cases.run_cases(getattr(qrm.binding, flag))
    assert sorted(theirs) == sorted(mine)
    for key, a in mine.items():
        b = theirs[key]
        assert np.isfinite(b).all(), key
        if tol == 0.0:
            assert np.array_equal(a, b), key
        elif key.endswith("logits"):
            print(f"[{flag}] {key}: max |flagged - plain| {float(np.abs(a - b).max()):.2e}")
            assert (np.abs(a - b) <= tol * np.maximum(1.0, np.abs(a))).all(), (key, float(np.abs(a - b).max()))


def test_results_are_reproducible_bit_for_bit(qrm):
    """Two calls give the same bytes: every sum inside the kernels is formed in a fixed order.  On the fused path
    (64 channels) that order depends on the image alone, so other splits of the batch into micro-batches give the
    same bytes too; on the single-block path (32 channels) a split deals an image's strips to other workgroups, and
    the last fp32 bits of the channel sums may then differ.  (The wide-tile cases launch many co-resident workgroups
    of the first-layer kernel per compute unit: matrix results read too early once showed there as run-to-run
    differences of one bf16 step.)"""
    for name, N, mbs in (("C2", 1300, (0, 300, 1024)), ("C1", 300, (0, 7)), ("C3", 3, (0,)), ("C4", 40, (0,))):
        cfg = synth.CONFIGS[name]
        imgs = synth.images(cfg, 0, N, threads=HOST_THREADS)
        if N >= 40:
            imgs[::N // 40][:40] = synth.field_images(cfg, 100, 40)
        off = synth.offsets(cfg, 0, N)
        ctx = qrm.Context(weights=synth.config_weights(cfg), rs=rs_dict(cfg))
        runs = []
        for mb in mbs + (mbs[0],):
            ctx.qrm_set_micro_batch(mb)
            runs.append(run_detect(ctx, cfg, imgs, off))
        ctx.close()
        for r, mb in zip(runs[1:], (mbs + (mbs[0],))[1:]):
            exact = name == "C2" or mb == mbs[0]   # single-block path: other splits deal the strips to other workgroups
            for key in ("logits", "bits", "msg", "codeword", "nerr"):
                if exact:
                    assert np.array_equal(runs[0][key], r[key]), (name, key, mb)
            assert np.allclose(runs[0]["logits"], r["logits"], rtol=0, atol=2e-5), (name, mb)


def test_more_streams_than_workspaces(qrm):
    """Twenty short-lived streams, one after the other, on one context (which holds QRM_MAX_STREAMS = 8 workspaces):
    a stream not seen before takes over the workspace used least recently.  Half of the streams are handed back
    with qrm_release_stream before they are destroyed, half are just dropped."""
    cfg = synth.CONFIGS["C2"]
    N = 6
    imgs, off = synth.images(cfg, 40, N), synth.offsets(cfg, 40, N)
    ctx = qrm.Context(weights=synth.config_weights(cfg), rs=rs_dict(cfg))
    base = run_detect(ctx, cfg, imgs, off)
    d_img, d_off = dev(imgs), dev(off)
    torch.cuda.synchronize()
    for i in range(20):
        s = torch.cuda.Stream()
        d_logits = empty((N, cfg.n_bits), torch.float32)
        d_msg, d_ne = empty((N, cfg.k), torch.uint8), empty((N,), torch.int8)
        ctx.qrm_detect(d_img, N, cfg.H, cfg.W, d_off, cfg.tile, d_logits, None, d_msg, None, d_ne, stream=s)
        if i % 2:
            ctx.qrm_release_stream(s)
        s.synchronize()
        assert np.array_equal(d_logits.cpu().numpy(), base["logits"]), i
        assert np.array_equal(d_msg.cpu().numpy(), base["msg"]) and np.array_equal(d_ne.cpu().numpy(), base["nerr"])
        del s
    # nine streams alive at once: the ninth shares a workspace with the first, in order
    streams = [torch.cuda.Stream() for _ in range(9)]
    outs = []
    for s in streams:
        d_logits = empty((N, cfg.n_bits), torch.float32)
        d_msg, d_ne = empty((N, cfg.k), torch.uint8), empty((N,), torch.int8)
        ctx.qrm_detect(d_img, N, cfg.H, cfg.W, d_off, cfg.tile, d_logits, None, d_msg, None, d_ne, stream=s)
        outs.append((d_logits, d_msg, d_ne))
    torch.cuda.synchronize()
    for d_logits, d_msg, d_ne in outs:
        assert np.array_equal(d_logits.cpu().numpy(), base["logits"]) and np.array_equal(d_msg.cpu().numpy(), base["msg"])
    ctx.qrm_release_stream(torch.cuda.Stream())          # a stream the context never saw: no-op
    ctx.close()


def test_detect_on_two_streams(qrm):
    cfg = synth.CONFIGS["C2"]
    wts = synth.config_weights(cfg)
    N = 8
    imgs, off = synth.images(cfg, 300, 2 * N), synth.offsets(cfg, 300, 2 * N)
    ctx = qrm.Context(weights=wts, rs=rs_dict(cfg))
    base = run_detect(ctx, cfg, imgs, off)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    d_img, d_off = dev(imgs), dev(off)
    outs = []
    torch.cuda.synchronize()
    for i, s in enumerate((s1, s2)):
        d_logits = empty((N, cfg.n_bits), torch.float32)
        d_msg, d_ne = empty((N, cfg.k), torch.uint8), empty((N,), torch.int8)
        ctx.qrm_detect(d_img[i * N:(i + 1) * N], N, cfg.H, cfg.W, d_off[i * N:(i + 1) * N], cfg.tile,
                       d_logits, None, d_msg, None, d_ne, stream=s)
        outs.append((d_logits, d_msg, d_ne))
    torch.cuda.synchronize()
    for i, (l, m_, e) in enumerate(outs):
        assert np.array_equal(l.cpu().numpy(), base["logits"][i * N:(i + 1) * N])
        assert np.array_equal(m_.cpu().numpy(), base["msg"][i * N:(i + 1) * N])
        assert np.array_equal(e.cpu().numpy(), base["nerr"][i * N:(i + 1) * N])
    ctx.close()


def test_detect_host_chunked_pipeline_equals_resident_detect(qrm):
    """Images in pinned host chunks streamed through 1, 2 and 3 staging buffers, with two of the host buffers
    appearing twice, give what qrm_detect gives on the same images resident in device memory - chunk by chunk,
    with chunks whose results differ (structured images: other bits, other error counts), so that a stale,
    swapped or overwritten chunk shows.  The resident results are held against the oracle unconditionally:
    logits and hard bits of a sample, every Reed-Solomon output against the oracle's decoder on the device's bits."""
    cfg = synth.CONFIGS["C2"]
    wts = synth.config_weights(cfg)
    chunk, order = 1100, [0, 1, 2, 0, 1]             # more images per chunk than one micro-batch; buffers 0, 1 twice
    imgs = synth.images(cfg, 500, 3 * chunk, threads=HOST_THREADS)
    fld = synth.field_images(cfg, 500, 3 * 48)
    for b in range(3):                               # 48 structured images at the head and the tail of every chunk
        imgs[b * chunk:b * chunk + 24] = fld[b * 48:b * 48 + 24]
        imgs[(b + 1) * chunk - 24:(b + 1) * chunk] = fld[b * 48 + 24:(b + 1) * 48]
    off = synth.offsets(cfg, 500, 3 * chunk)
    bufs = [torch.empty((chunk, 3, cfg.H, cfg.W), dtype=torch.uint8, pin_memory=True) for _ in range(3)]
    obufs = [torch.empty((chunk, 2), dtype=torch.int32, pin_memory=True) for _ in range(3)]
    for b in range(3):
        bufs[b].copy_(torch.from_numpy(imgs[b * chunk:(b + 1) * chunk]))
        obufs[b].copy_(torch.from_numpy(off[b * chunk:(b + 1) * chunk]))
    n_total = len(order) * chunk
    ctx = qrm.Context(weights=wts, rs=rs_dict(cfg))
    base = run_detect(ctx, cfg, imgs, off)
    # the resident results against the oracle
    syms = oracle.bits_to_symbols(base["bits"], cfg.m)
    om, oc, oe = oracle.rs_decode(syms, cfg.m, cfg.prim_poly, cfg.n, cfg.k, cfg.fcr)
    assert np.array_equal(base["msg"], om) and np.array_equal(base["codeword"], oc) and np.array_equal(base["nerr"], oe)
    fflat = synth.field_is_flat(cfg, 500, 3 * 48)
    sample, is_flat = [], []
    for b in range(3):
        for j in (0, 1, 2, 3, 24, 600, chunk - 1):
            sample.append(b * chunk + j)
            fi = b * 48 + j if j < 24 else (b * 48 + 24 + j - (chunk - 24) if j >= chunk - 24 else -1)
            is_flat.append(fi >= 0 and bool(fflat[fi]))
    ref = oracle.detect(wts, imgs[sample], off[sample], cfg.tile, cfg.m, cfg.prim_poly, cfg.n, cfg.k, cfg.fcr)
    check_logits(base["logits"][sample], ref["logits"], base["bits"][sample], what=f"streamed chunks, {len(sample)} sampled images",
                 flat=np.array(is_flat))
    # the chunks must be told apart by their results
    heads = [base["msg"][b * chunk:b * chunk + 24].tobytes() + base["nerr"][b * chunk:b * chunk + 24].tobytes() for b in range(3)]
    assert len(set(heads)) == 3, "the chunks of this test must differ in their results"
    for depth in (1, 2, 3):
        h_msg = torch.zeros((n_total, cfg.k), dtype=torch.uint8, pin_memory=True)
        h_cw = torch.zeros((n_total, cfg.n), dtype=torch.uint8, pin_memory=True)
        h_ne = torch.zeros((n_total,), dtype=torch.int8, pin_memory=True)
        ctx.qrm_detect_host([bufs[b] for b in order], chunk, cfg.H, cfg.W, [obufs[b] for b in order], cfg.tile, depth,
                            h_msg, h_cw, h_ne)
        for i, b in enumerate(order):
            sl, bl = slice(i * chunk, (i + 1) * chunk), slice(b * chunk, (b + 1) * chunk)
            assert np.array_equal(h_msg[sl].numpy(), base["msg"][bl]), (depth, i)
            assert np.array_equal(h_cw[sl].numpy(), base["codeword"][bl]), (depth, i)
            assert np.array_equal(h_ne[sl].numpy(), base["nerr"][bl]), (depth, i)
    # a second kind of call on the same context (staging reused): one buffer, no origins, no code words
    h_msg2 = torch.empty((2 * chunk, cfg.k), dtype=torch.uint8, pin_memory=True)
    h_ne2 = torch.empty((2 * chunk,), dtype=torch.int8, pin_memory=True)
    ctx.qrm_detect_host([bufs[2], bufs[0]], chunk, cfg.H, cfg.W, None, cfg.tile, 1, h_msg2, None, h_ne2)
    base0 = run_detect(ctx, cfg, np.concatenate([imgs[2 * chunk:], imgs[:chunk]]), None)
    assert np.array_equal(h_msg2.numpy(), base0["msg"]) and np.array_equal(h_ne2.numpy(), base0["nerr"])
    assert not np.array_equal(base0["msg"][:chunk], base0["msg"][chunk:])
    with pytest.raises(qrm.QrmError) as e:
        ctx.qrm_detect_host([bufs[0]], chunk, cfg.H, cfg.W, None, cfg.tile, 0, h_msg2, None, h_ne2)
    assert e.value.status == qrm.QRM_E_INVALID
    ctx.qrm_detect_host([], chunk, cfg.H, cfg.W, None, cfg.tile, 2, h_msg2, None, h_ne2)   # zero chunks: no-op
    ctx.close()


@pytest.mark.timeout(900)
def test_detect_host_full_streamed_configuration(qrm):
    """The streamed configuration at its real size: 128 chunks of 8192 images (1 048 576 images, 206 GB over the
    host link per pass) through qrm_detect_host with 3, 2 and 1 staging buffers.  Eight distinct pinned chunks are
    recycled (chunk i is buffer i mod 8), each with 64 structured images at its head, so that every chunk has
    results of its own.  Every one of the 1 048 576 outputs must equal the resident qrm_detect output of its
    buffer, which in turn equals the oracle's decoder on the device's own hard bits; the first 64 images of the
    first and of the last chunk are held against the oracle's extractor."""
    cfg = synth.CONFIGS["C5"]
    wts = synth.config_weights(cfg)
    chunk, n_chunks, n_buf = cfg.chunk, cfg.n_images // cfg.chunk, 8
    assert chunk == 8192 and n_chunks == 128
    bufs = [torch.empty((chunk, 3, cfg.H, cfg.W), dtype=torch.uint8, pin_memory=True) for _ in range(n_buf)]
    obufs = [torch.empty((chunk, 2), dtype=torch.int32, pin_memory=True) for _ in range(n_buf)]
    for b in range(n_buf):
        print(f"[stream] generating chunk {b}", flush=True)
        synth.images(cfg, b * chunk, chunk, out=bufs[b].numpy(), threads=HOST_THREADS)
        bufs[b][:64].copy_(torch.from_numpy(synth.field_images(cfg, b * 64, 64)))
        obufs[b].copy_(torch.from_numpy(synth.offsets(cfg, b * chunk, chunk)))
    ctx = qrm.Context(weights=wts, rs=rs_dict(cfg))
    base = []
    for b in range(n_buf):
        got = run_detect(ctx, cfg, bufs[b].numpy(), obufs[b].numpy())
        syms = oracle.bits_to_symbols(got["bits"], cfg.m)
        om, oc, oe = oracle.rs_decode(syms, cfg.m, cfg.prim_poly, cfg.n, cfg.k, cfg.fcr)
        assert np.array_equal(got["msg"], om) and np.array_equal(got["codeword"], oc) and np.array_equal(got["nerr"], oe)
        base.append(got)
    assert len({g["msg"][:64].tobytes() for g in base}) == n_buf
    for b in (0, (n_chunks - 1) % n_buf):            # the first and the last chunk of the pass
        ref = oracle.detect(wts, bufs[b].numpy()[:64], obufs[b].numpy()[:64], cfg.tile, cfg.m, cfg.prim_poly, cfg.n, cfg.k, cfg.fcr)
        check_logits(base[b]["logits"][:64], ref["logits"], base[b]["bits"][:64], what=f"streamed configuration, buffer {b}, first 64 images",
                     flat=synth.field_is_flat(cfg, b * 64, 64))
    n_total = n_chunks * chunk
    order = [i % n_buf for i in range(n_chunks)]
    first = None
    for depth in (3, 2, 1):
        h_msg = torch.zeros((n_total, cfg.k), dtype=torch.uint8, pin_memory=True)
        h_cw = torch.zeros((n_total, cfg.n), dtype=torch.uint8, pin_memory=True)
        h_ne = torch.zeros((n_total,), dtype=torch.int8, pin_memory=True)
        print(f"[stream] pass with {depth} staging buffer(s)", flush=True)
        ctx.qrm_detect_host([bufs[b] for b in order], chunk, cfg.H, cfg.W, [obufs[b] for b in order], cfg.tile, depth,
                            h_msg, h_cw, h_ne)
        m3, c3, e3 = (h_msg.numpy().reshape(n_chunks, chunk, cfg.k), h_cw.numpy().reshape(n_chunks, chunk, cfg.n),
                      h_ne.numpy().reshape(n_chunks, chunk))
        for i, b in enumerate(order):
            assert np.array_equal(m3[i], base[b]["msg"]) and np.array_equal(c3[i], base[b]["codeword"]) and \
                np.array_equal(e3[i], base[b]["nerr"]), (depth, i)
        digest = (h_msg.numpy().tobytes(), h_ne.numpy().tobytes())
        if first is None:
            first = digest
        assert digest == first
    ctx.close()


# ---------------------------------------------------------------- error paths (host side only)

# ---------------------------------------------------------------- fused pre-processing

from oracle import preprocess as pre_oracle

PRE_CASES = [  # N, H_in, W_in, size, tile (0 = whole image)
    (2, 512, 512, 256, 64),     # the benchmark's shape: 512 x 512 raw -> 256 x 256 -> one 64 x 64 tile
    (1, 300, 420, 128, 0),      # landscape, whole image
    (3, 77, 50, 40, 0),         # portrait, odd sizes
    (3, 60, 60, 60, 20),        # identity size: the tile is a window of the raw image
    (2, 40, 56, 90, 32),        # enlarging
    (4, 333, 500, 96, 31),      # tile width not a multiple of 4: byte stores
    (2, 1024, 768, 256, 128),
    (2, 7, 1, 3, 0),            # one-pixel rows: no room for word loads
    (2, 1, 9, 4, 0),            # a single row
    (3, 2, 2, 8, 4),            # 2 x 2 image enlarged
    (1, 1200, 1100, 1024, 0),   # the widest window the kernel takes
    (2, 640, 250, 100, 48),     # scale 2.5; rows of 750 bytes
    (2, 653, 251, 100, 48),     # a scale that is no simple fraction; rows of 753 bytes
    (2, 96, 131, 64, 0),        # rows of 393 bytes: every alignment of a row's first byte
]


@pytest.mark.parametrize("N,H_in,W_in,size,tile", PRE_CASES)
def test_preprocess_bit_exact(qrm, N, H_in, W_in, size, tile):
    rng = np.random.default_rng(H_in + 3 * W_in + size)
    raw = rng.integers(0, 256, size=(N, H_in, W_in, 3), dtype=np.uint8)
    off = None
    if tile:
        off = rng.integers(-5, size - tile + 6, size=(N, 2)).astype(np.int32)     # some outside: clamped
        off[0] = (size - tile, 0)
    ref = pre_oracle.preprocess(raw, size, off, tile)
    ctx = qrm.Context(rs=rs_dict(synth.CONFIGS["C1"]))
    T = tile if tile else size
    d_out = empty((N, 3, T, T), torch.uint8)
    ctx.qrm_preprocess(dev(raw), N, H_in, W_in, size, None if off is None else dev(off), tile, d_out)
    torch.cuda.synchronize()
    assert np.array_equal(d_out.cpu().numpy(), ref)
    if tile:    # no origins given: the top-left tile
        ctx.qrm_preprocess(dev(raw), N, H_in, W_in, size, None, tile, d_out)
        torch.cuda.synchronize()
        assert np.array_equal(d_out.cpu().numpy(), pre_oracle.preprocess(raw, size, np.zeros((N, 2), np.int32), tile))
    ctx.close()


@pytest.mark.parametrize("shift_in,shift_out", [(5, 0), (0, 3), (13, 1)])
def test_preprocess_buffers_at_odd_addresses(qrm, shift_in, shift_out):
    """Raw and output buffers that start at any byte: word loads and dword stores must not assume more."""
    N, H_in, W_in, size = 2, 131, 157, 64
    rng = np.random.default_rng(shift_in * 16 + shift_out)
    raw = rng.integers(0, 256, size=(N, H_in, W_in, 3), dtype=np.uint8)
    ref = pre_oracle.preprocess(raw, size, None, 0)
    ctx = qrm.Context(rs=rs_dict(synth.CONFIGS["C1"]))
    buf_in = torch.zeros(raw.size + 16, dtype=torch.uint8, device="cuda")
    buf_in[shift_in:shift_in + raw.size] = dev(raw.reshape(-1))
    buf_out = torch.full((ref.size + 16,), 0xEE, dtype=torch.uint8, device="cuda")
    ctx.qrm_preprocess(buf_in[shift_in:], N, H_in, W_in, size, None, 0, buf_out[shift_out:])
    torch.cuda.synchronize()
    got = buf_out.cpu().numpy()
    assert np.array_equal(got[shift_out:shift_out + ref.size], ref.reshape(-1))
    assert (got[:shift_out] == 0xEE).all() and (got[shift_out + ref.size:] == 0xEE).all()   # nothing written outside
    ctx.close()


def test_preprocess_tile_then_extractor_equals_oracle_path(qrm):
    """Raw 512 x 512 images -> (resize, crop, tile) in one kernel -> extractor, against the oracle's chain."""
    cfg = synth.CONFIGS["C2"]
    wts = synth.config_weights(cfg)
    N = 6
    rng = np.random.default_rng(12)
    raw = rng.integers(0, 256, size=(N, 512, 512, 3), dtype=np.uint8)
    off = synth.offsets(cfg, 0, N)
    ctx = qrm.Context(weights=wts, rs=rs_dict(cfg))
    d_tiles = empty((N, 3, cfg.tile, cfg.tile), torch.uint8)
    ctx.qrm_preprocess(dev(raw), N, 512, 512, cfg.H, dev(off), cfg.tile, d_tiles)
    d_logits, d_bits = empty((N, cfg.n_bits), torch.float32), empty((N, cfg.n_bits), torch.uint8)
    ctx.qrm_extractor_forward(d_tiles, N, cfg.tile, cfg.tile, d_logits, d_bits)
    torch.cuda.synchronize()
    tiles = pre_oracle.preprocess(raw, cfg.H, off, cfg.tile)
    assert np.array_equal(d_tiles.cpu().numpy(), tiles)
    ref_logits, _ = oracle.extractor_forward(wts, tiles)
    check_logits(d_logits.cpu().numpy(), ref_logits, d_bits.cpu().numpy(), what="pre-processed tiles -> extractor")
    # the whole pre-processed image followed by the stand-alone tile crop gives the same tiles
    d_full = empty((N, 3, cfg.H, cfg.W), torch.uint8)
    ctx.qrm_preprocess(dev(raw), N, 512, 512, cfg.H, None, 0, d_full)
    d_t2 = empty((N, 3, cfg.tile, cfg.tile), torch.uint8)
    ctx.qrm_extract_tiles(d_full, N, cfg.H, cfg.W, dev(off), cfg.tile, d_t2)
    torch.cuda.synchronize()
    assert np.array_equal(d_t2.cpu().numpy(), tiles)
    ctx.close()


def test_preprocess_error_statuses(qrm):
    ctx = qrm.Context(rs=rs_dict(synth.CONFIGS["C1"]))
    d_raw, d_out = empty((1, 32, 32, 3), torch.uint8), empty((1, 3, 16, 16), torch.uint8)
    for args in ((0, 32, 16, 0), (32, 32, 0, 0), (32, 32, 16, 17), (32, 32, 16, -1), (20000, 32, 16, 0)):
        with pytest.raises(qrm.QrmError):
            ctx.qrm_preprocess(d_raw, 1, args[0], args[1], args[2], None, args[3], d_out)
    with pytest.raises(qrm.QrmError):
        ctx.qrm_preprocess(None, 1, 32, 32, 16, None, 0, d_out)
    ctx.qrm_preprocess(d_raw, 0, 32, 32, 16, None, 0, d_out)     # empty batch
    ctx.close()


# ---------------------------------------------------------------- variance-based tile selection

from oracle import tileselect


def channel_weights(std):
    """What the library holds: inv_std = (float)(1.0 / std) at context creation, weight = its square in float64."""
    inv = (1.0 / np.asarray(std, dtype=np.float32).astype(np.float64)).astype(np.float32).astype(np.float64)
    return inv * inv


SELECT_CASES = [  # N, H, W, tile, stride
    (33, 256, 256, 64, 32),      # the listing's sizes on the benchmark's images (wide loads)
    (5, 96, 144, 32, 16),
    (4, 512, 512, 128, 64),      # configuration C4
    (7, 100, 117, 30, 15),       # nothing aligned: byte loads, rows and columns left over
    (3, 64, 128, 64, 64),        # stride = tile: two windows side by side
    (6, 40, 40, 40, 40),         # a single window
    (2, 256, 256, 32, 8),        # 29 x 29 windows, 32 x 32 cells
]


@pytest.mark.parametrize("N,H,W,tile,stride", SELECT_CASES)
def test_select_tiles_variance_bit_exact(qrm, N, H, W, tile, stride):
    cfg = synth.CONFIGS["C2"]
    wts = synth.config_weights(cfg)
    rng = np.random.default_rng(H * 7 + W + tile)
    imgs = rng.integers(0, 256, size=(N, 3, H, W), dtype=np.uint8)
    # structure, so that windows differ by more than noise: a flat image, a flat image with one busy window,
    # two equally busy windows (tie), a gradient
    imgs[0] = 131
    if N > 1:
        imgs[1] = 90
        y0, x0 = (H - tile) // stride * stride, min(stride, (W - tile) // stride * stride)
        imgs[1, :, y0:y0 + tile, x0:x0 + tile] = rng.integers(0, 256, size=(3, tile, tile), dtype=np.uint8)
    if N > 2 and W >= 2 * tile and (W - tile) % stride == 0:
        imgs[2] = 17
        patch = rng.integers(0, 256, size=(3, tile, tile), dtype=np.uint8)
        imgs[2, :, 0:tile, 0:tile] = patch
        imgs[2, :, H - tile:H, W - tile:W] = patch if (H - tile) % stride == 0 else 17
    ref_off, ref_scores = tileselect.select_tiles_variance(imgs, tile, stride, channel_weights(wts["std"]))
    ctx = qrm.Context(weights=wts, rs=rs_dict(cfg))
    nwin = ref_scores.shape[1]
    d_off, d_sc = empty((N, 2), torch.int32), empty((N, nwin), torch.float64)
    ctx.qrm_select_tiles_variance(dev(imgs), N, H, W, tile, stride, d_off, d_sc)
    torch.cuda.synchronize()
    assert np.array_equal(d_sc.cpu().numpy(), ref_scores), "window scores differ (float64, bit for bit)"
    assert np.array_equal(d_off.cpu().numpy(), ref_off)
    assert ref_off[0].tolist() == [0, 0]
    d_off2 = empty((N, 2), torch.int32)
    ctx.qrm_select_tiles_variance(dev(imgs), N, H, W, tile, stride, d_off2, None)     # scores are optional
    torch.cuda.synchronize()
    assert np.array_equal(d_off2.cpu().numpy(), ref_off)
    ctx.close()
    # a context without an extractor weighs the channels equally
    rs_only = qrm.Context(rs=rs_dict(cfg))
    rs_only.qrm_select_tiles_variance(dev(imgs), N, H, W, tile, stride, d_off, d_sc)
    torch.cuda.synchronize()
    ro, rsx = tileselect.select_tiles_variance(imgs, tile, stride, [1.0, 1.0, 1.0])
    assert np.array_equal(d_sc.cpu().numpy(), rsx) and np.array_equal(d_off.cpu().numpy(), ro)
    rs_only.close()


def test_select_tiles_then_detect_equals_oracle_path(qrm):
    """Selection feeds detection: the origins chosen on the device, then the whole path, against the oracle's."""
    cfg = synth.CONFIGS["C2"]
    wts = synth.config_weights(cfg)
    N = 24
    imgs = synth.images(cfg, 0, N).copy()
    rng = np.random.default_rng(3)
    for i in range(N):                               # make one window per image clearly the busiest
        imgs[i] = (imgs[i] // 4 + 96).astype(np.uint8)
        wy, wx = rng.integers(0, 7, size=2)
        imgs[i, :, wy * 32:wy * 32 + 64, wx * 32:wx * 32 + 64] = rng.integers(0, 256, size=(3, 64, 64), dtype=np.uint8)
    ctx = qrm.Context(weights=wts, rs=rs_dict(cfg))
    d_imgs, d_off = dev(imgs), empty((N, 2), torch.int32)
    ctx.qrm_select_tiles_variance(d_imgs, N, cfg.H, cfg.W, cfg.tile, cfg.tile // 2, d_off)
    d_logits, d_bits = empty((N, cfg.n_bits), torch.float32), empty((N, cfg.n_bits), torch.uint8)
    d_msg, d_cw, d_ne = empty((N, cfg.k), torch.uint8), empty((N, cfg.n), torch.uint8), empty((N,), torch.int8)
    ctx.qrm_detect(d_imgs, N, cfg.H, cfg.W, d_off, cfg.tile, d_logits, d_bits, d_msg, d_cw, d_ne)
    torch.cuda.synchronize()
    off, _ = tileselect.select_tiles_variance(imgs, cfg.tile, cfg.tile // 2, channel_weights(wts["std"]))
    assert np.array_equal(d_off.cpu().numpy(), off)
    got = dict(logits=d_logits.cpu().numpy(), bits=d_bits.cpu().numpy(), msg=d_msg.cpu().numpy(),
               codeword=d_cw.cpu().numpy(), nerr=d_ne.cpu().numpy())
    check_detect(cfg, wts, imgs, off, got, "C2 detect on variance-selected tiles")
    ctx.close()


def test_select_tiles_error_statuses(qrm):
    cfg = synth.CONFIGS["C1"]
    ctx = qrm.Context(rs=rs_dict(cfg))
    d_img, d_off = empty((2, 3, 64, 64), torch.uint8), empty((2, 2), torch.int32)
    for tile, stride in ((0, 8), (16, 0), (80, 8), (24, 16), (32, 1)):      # last: 33 x 33 cells
        with pytest.raises(qrm.QrmError):
            ctx.qrm_select_tiles_variance(d_img, 2, 64, 64, tile, stride, d_off)
    with pytest.raises(qrm.QrmError):
        ctx.qrm_select_tiles_variance(d_img, 2, 64, 64, 16, 8, None)
    ctx.qrm_select_tiles_variance(d_img, 0, 64, 64, 16, 8, d_off)           # empty batch
    ctx.close()


# ---------------------------------------------------------------- key verification

from oracle import keycheck


@pytest.mark.parametrize("m,poly,n,k", [(4, 0x13, 12, 8), (8, 0x11D, 12, 8), (4, 0x13, 15, 11), (8, 0x11D, 20, 4),
                                        (5, 0x25, 31, 27), (8, 0x11D, 255, 239)])
@pytest.mark.parametrize("N", [1, 257, 70001])
def test_verify_key_bit_exact(qrm, m, poly, n, k, N):
    key, msgs = synth.key_cases(1, N, k, m)
    tau = qrm.binding.qrm_key_threshold(k * m, 1e-6)
    if k * m <= 256:
        assert tau == keycheck.key_threshold(k * m, Fraction(1e-6))
    else:   # the oracle's search is quadratic in the length: check the two tails that define tau instead
        assert keycheck.binomial_tail(k * m, tau) <= Fraction(1e-6) < keycheck.binomial_tail(k * m, tau - 1)
    ctx = qrm.Context(rs=dict(m=m, prim_poly=poly, n=n, k=k, fcr=1))
    ctx.qrm_set_key(key, tau)
    d_matches, d_det = empty((N,), torch.int32), empty((N,), torch.uint8)
    ctx.qrm_verify_key(dev(msgs), N, d_matches, d_det)
    torch.cuda.synchronize()
    S = min(N, max(50, 200000 // (k * m)))                              # python loops: a sample
    ref_matches, ref_det = keycheck.verify_key(msgs[:S], key, m, tau)
    assert np.array_equal(d_matches.cpu().numpy()[:S], ref_matches)
    assert np.array_equal(d_det.cpu().numpy()[:S], ref_det)
    # the rest through a property that holds at any size: agreeing bits = k*m - popcount(msg xor key)
    x = (msgs ^ key[None, :]) & np.uint8((1 << m) - 1)
    pop = np.unpackbits(x, axis=1).sum(axis=1).astype(np.int32)
    assert np.array_equal(d_matches.cpu().numpy(), k * m - pop)
    assert np.array_equal(d_det.cpu().numpy(), (k * m - pop >= tau).astype(np.uint8))
    assert d_matches[0].item() == k * m and d_det[0].item() == 1
    # without the flag output, and with high bits set in the stored symbols when m < 8
    d2 = empty((N,), torch.int32)
    noisy = msgs | np.uint8((0xFF << m) & 0xFF)
    ctx.qrm_verify_key(dev(noisy), N, d2, None)
    torch.cuda.synchronize()
    assert np.array_equal(d2.cpu().numpy(), k * m - pop)
    ctx.close()


def test_verify_key_unaligned_message_buffer(qrm):
    m, k, N = 4, 8, 1000
    key, msgs = synth.key_cases(1, N, k, m, block=2001)
    ctx = qrm.Context(rs=dict(m=m, prim_poly=0x13, n=12, k=k, fcr=1))
    ctx.qrm_set_key(key, 30)
    buf = empty((N * k + 3,), torch.uint8)
    view = buf[3:]                                   # starts 3 bytes into an allocation: no wide loads
    view.copy_(dev(msgs).reshape(-1))
    d_matches, d_det = empty((N,), torch.int32), empty((N,), torch.uint8)
    ctx._check(ctx._lib.qrm_verify_key(ctx._h, view.data_ptr(), N, d_matches.data_ptr(), d_det.data_ptr(), None))
    torch.cuda.synchronize()
    rm, rd = keycheck.verify_key(msgs, key, m, 30)
    assert np.array_equal(d_matches.cpu().numpy(), rm) and np.array_equal(d_det.cpu().numpy(), rd)
    ctx.close()


@pytest.mark.parametrize("name,count", [("C1", 16), ("C2", 96)])
def test_detect_verify_equals_detect_then_oracle_verification(qrm, name, count):
    cfg = synth.CONFIGS[name]
    wts = synth.config_weights(cfg)
    imgs, off = synth.images(cfg, 0, count), synth.offsets(cfg, 0, count)
    ctx = qrm.Context(weights=wts, rs=rs_dict(cfg))
    plain = run_detect(ctx, cfg, imgs, off)
    check_detect(cfg, wts, imgs, off, plain, f"{name} detect before verification")
    # the key is what image 5 decodes to, with two bits flipped: image 5 must be found, random ones not
    key = plain["msg"][5].copy()
    key[0] ^= 1
    key[cfg.k - 1] ^= 2
    K = cfg.k * cfg.m
    tau = qrm.binding.qrm_key_threshold(K, 1e-6)
    ctx.qrm_set_key(key, tau)
    N = count
    d_logits, d_bits = empty((N, cfg.n_bits), torch.float32), empty((N, cfg.n_bits), torch.uint8)
    d_msg, d_cw, d_ne = empty((N, cfg.k), torch.uint8), empty((N, cfg.n), torch.uint8), empty((N,), torch.int8)
    d_matches, d_det = empty((N,), torch.int32), empty((N,), torch.uint8)
    ctx.qrm_detect_verify(dev(imgs), N, cfg.H, cfg.W, dev(off), cfg.tile, d_logits, d_bits, d_msg, d_cw, d_ne,
                          d_matches, d_det)
    torch.cuda.synchronize()
    assert np.array_equal(d_msg.cpu().numpy(), plain["msg"]) and np.array_equal(d_ne.cpu().numpy(), plain["nerr"])
    assert np.array_equal(d_cw.cpu().numpy(), plain["codeword"]) and np.array_equal(d_bits.cpu().numpy(), plain["bits"])
    rm, rd = keycheck.verify_key(plain["msg"], key, cfg.m, keycheck.key_threshold(K, Fraction(1e-6)))
    assert np.array_equal(d_matches.cpu().numpy(), rm) and np.array_equal(d_det.cpu().numpy(), rd)
    assert rm[5] == K - 2 and rd[5] == 1
    # lean call: only what a detector needs
    m2, det2 = empty((N,), torch.int32), empty((N,), torch.uint8)
    ctx.qrm_detect_verify(dev(imgs), N, cfg.H, cfg.W, dev(off), cfg.tile, None, None, d_msg, None, d_ne, m2, det2)
    torch.cuda.synchronize()
    assert np.array_equal(m2.cpu().numpy(), rm) and np.array_equal(det2.cpu().numpy(), rd)
    ctx.close()


def test_rs_decode_long_code_then_key_comparison(qrm):
    """RS(255,239): four symbols per lane, t = 8; then the comparison with a key on its messages."""
    m, poly, n, k = 8, 0x11D, 255, 239
    msgs, err, _ = synth.rs_cases(3, 500, n, k, m, max_err=9, block=7)
    words = oracle.rs_encode(msgs, m, poly, n, k, 1) ^ err
    ctx = qrm.Context(rs=dict(m=m, prim_poly=poly, n=n, k=k, fcr=1))
    gm, gc, ge = gpu_rs_decode(ctx, words)
    om, oc, oe = oracle.rs_decode(words, m, poly, n, k, 1)
    assert np.array_equal(gm, om) and np.array_equal(gc, oc) and np.array_equal(ge, oe)
    key = msgs[3]
    ctx.qrm_set_key(key, 1700)
    d_matches, d_det = empty((500,), torch.int32), empty((500,), torch.uint8)
    ctx.qrm_verify_key(dev(gm), 500, d_matches, d_det)
    torch.cuda.synchronize()
    rm, rd = keycheck.verify_key(om, key, m, 1700)
    assert np.array_equal(d_matches.cpu().numpy(), rm) and np.array_equal(d_det.cpu().numpy(), rd)
    ctx.close()


def test_verification_error_statuses(qrm):
    cfg = synth.CONFIGS["C1"]
    ctx = qrm.Context(weights=synth.config_weights(cfg), rs=rs_dict(cfg))
    d = empty((4,), torch.int32)
    with pytest.raises(qrm.QrmError):       # no key yet
        ctx.qrm_verify_key(empty((4, cfg.k), torch.uint8), 4, d, None)
    with pytest.raises(qrm.QrmError):       # tau out of range
        ctx.qrm_set_key(np.zeros(cfg.k, np.uint8), cfg.k * cfg.m + 2)
    ctx.qrm_set_key(np.zeros(cfg.k, np.uint8), 3)
    with pytest.raises(qrm.QrmError):       # d_matches missing
        ctx.qrm_verify_key(empty((4, cfg.k), torch.uint8), 4, None, None)
    ctx.qrm_verify_key(empty((0, cfg.k), torch.uint8), 0, d, None)      # empty batch is fine
    ext_only = qrm.Context(weights=synth.config_weights(cfg))
    with pytest.raises(qrm.QrmError):       # no code, hence no key length
        ext_only._check(ext_only._lib.qrm_set_key(ext_only._h, np.zeros(16, np.uint8).ctypes.data, 3))
    ext_only.close()
    ctx.close()


def test_whole_chain_raw_image_to_verdict(qrm):
    """Every stage in a row, device pointers handed from one call to the next: raw interleaved 384 x 512 images ->
    resize + centre crop (256 x 256) -> variance-based choice of the tile -> crop, extractor, threshold, Reed-Solomon,
    comparison with a key; against the same chain of oracles."""
    cfg = synth.CONFIGS["C2"]
    wts = synth.config_weights(cfg)
    N, Hin, Win = 10, 384, 512
    rng = np.random.default_rng(77)
    raw = (rng.integers(0, 256, size=(N, Hin, Win, 3)) // 3 + 60).astype(np.uint8)
    for i in range(N):                                # one busy region per image, so that the selection is clear-cut
        y, x = int(rng.integers(0, Hin - 140)), int(rng.integers(64, Win - 204))
        raw[i, y:y + 140, x:x + 140] = rng.integers(0, 256, size=(140, 140, 3), dtype=np.uint8)
    ctx = qrm.Context(weights=wts, rs=rs_dict(cfg))
    d_raw = dev(raw)
    d_img = empty((N, 3, cfg.H, cfg.W), torch.uint8)
    ctx.qrm_preprocess(d_raw, N, Hin, Win, cfg.H, None, 0, d_img)
    d_off = empty((N, 2), torch.int32)
    ctx.qrm_select_tiles_variance(d_img, N, cfg.H, cfg.W, cfg.tile, cfg.tile // 2, d_off)
    # oracle side of the first two stages, needed for the key
    img = pre_oracle.preprocess(raw, cfg.H)
    off, _ = tileselect.select_tiles_variance(img, cfg.tile, cfg.tile // 2, channel_weights(wts["std"]))
    ref = oracle.detect(wts, img, off, cfg.tile, cfg.m, cfg.prim_poly, cfg.n, cfg.k, cfg.fcr)
    key = ref["msg"][3].copy()
    tau = qrm.binding.qrm_key_threshold(cfg.k * cfg.m, 1e-6)
    ctx.qrm_set_key(key, tau)
    d_logits, d_bits = empty((N, cfg.n_bits), torch.float32), empty((N, cfg.n_bits), torch.uint8)
    d_msg, d_cw, d_ne = empty((N, cfg.k), torch.uint8), empty((N, cfg.n), torch.uint8), empty((N,), torch.int8)
    d_matches, d_det = empty((N,), torch.int32), empty((N,), torch.uint8)
    ctx.qrm_detect_verify(d_img, N, cfg.H, cfg.W, d_off, cfg.tile, d_logits, d_bits, d_msg, d_cw, d_ne, d_matches, d_det)
    torch.cuda.synchronize()
    assert np.array_equal(d_img.cpu().numpy(), img)
    assert np.array_equal(d_off.cpu().numpy(), off)
    got = dict(logits=d_logits.cpu().numpy(), bits=d_bits.cpu().numpy(), msg=d_msg.cpu().numpy(),
               codeword=d_cw.cpu().numpy(), nerr=d_ne.cpu().numpy())
    check_detect(cfg, wts, img, off, got, "raw image -> verdict")
    rm, rd = keycheck.verify_key(got["msg"], key, cfg.m, keycheck.key_threshold(cfg.k * cfg.m, Fraction(1e-6)))
    assert np.array_equal(d_matches.cpu().numpy(), rm) and np.array_equal(d_det.cpu().numpy(), rd)
    ctx.close()


def test_matrix_rate_probe_reports_plausible_rates(qrm):
    """The diagnostic probe: zeros run near the published rate, random operands slower, both far above zero."""
    ctx = qrm.Context(rs=rs_dict(synth.CONFIGS["C1"]))
    zeros, rnd = ctx.qrm_diag_matrix_rate(0), ctx.qrm_diag_matrix_rate(2)
    print(f"[probe] matrix pipes: {zeros:.0f} TFLOP/s on zeros, {rnd:.0f} TFLOP/s on random operands")
    assert 500.0 < rnd <= zeros * 1.05 and zeros < 2700.0
    with pytest.raises(qrm.QrmError):
        ctx.qrm_diag_matrix_rate(3)
    ctx.close()


def test_error_statuses(qrm):
    cfg = synth.CONFIGS["C2"]
    wts = synth.config_weights(cfg)
    with pytest.raises(qrm.QrmError) as e:
        qrm.Context(rs=dict(m=4, prim_poly=0x13, n=16, k=12))
    assert e.value.status == qrm.QRM_E_INVALID
    with pytest.raises(qrm.QrmError):
        qrm.Context(rs=dict(m=4, prim_poly=0x13, n=15, k=12))          # odd n - k
    with pytest.raises(qrm.QrmError):
        qrm.Context(rs=dict(m=4, prim_poly=0x1F, n=15, k=11))          # not primitive
    with pytest.raises(qrm.QrmError) as e:
        qrm.Context(rs=dict(m=8, prim_poly=0x11D, n=255, k=235))       # t = 10
    assert e.value.status == qrm.QRM_E_UNSUPPORTED
    ctx = qrm.Context(weights=wts, rs=dict(m=4, prim_poly=0x13, n=15, k=11))   # 48 bits != 60
    d_img = empty((2, 3, 256, 256), torch.uint8)
    d_msg, d_ne = empty((2, 11), torch.uint8), empty((2,), torch.int8)
    with pytest.raises(qrm.QrmError) as e:
        ctx.qrm_detect(d_img, 2, 256, 256, None, 64, None, None, d_msg, None, d_ne)
    assert e.value.status == qrm.QRM_E_INVALID and "n_bits" in e.value.message
    with pytest.raises(qrm.QrmError):
        ctx.qrm_extract_tiles(d_img, 2, 256, 256, None, 300, d_img)    # tile > H
    with pytest.raises(qrm.QrmError):
        ctx.qrm_rs_decode(None, 4, d_msg, None, d_ne)                  # NULL symbols
    ctx.qrm_rs_decode(None, 0, None, None, None)                       # N == 0 is a no-op
    rs_only = qrm.Context(rs=dict(m=4, prim_poly=0x13, n=15, k=11))
    with pytest.raises(qrm.QrmError):
        rs_only.qrm_extractor_forward(d_img, 2, 256, 256, empty((2, 48), torch.float32))
    rs_only.close()
    ctx.close()
