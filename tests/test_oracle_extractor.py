"""Pins for the tile-crop / extractor / threshold / bit-packing half of the CPU oracle.

The oracle's convolution stack is compared with: a pure-Python direct sum written here,
torch's fp64 conv2d (an independent library routine), delta-kernel identities (output =
shifted input, zero outside the tile), closed forms for constant inputs, and the
normalisation formula evaluated by hand.

Paper anchors: Section 4.3 (one l x l tile of the 256 x 256 image is passed to the
extractor), Table 1 (toTensor + normalize; random / random grid / fixed tiles), Section 4.1
(hard bit = sign of the soft output), Appendix B Algorithm "RS_Encode" step 1 (bits are
grouped into m-bit symbols).
"""
import numpy as np
import pytest
import torch

import oracle
import synth


def tiny_weights(in_ch, nb, C, nbits, seed=0):
    w = synth.extractor_weights(in_ch, nb, C, nbits, seed_index=100 + seed)
    return w


def split_conv(w):
    in_ch, nb, C, nbits = w["in_ch"], w["n_blocks"], w["channels"], w["n_bits"]
    out, off, cin = [], 0, in_ch
    for _ in range(nb):
        sz = C * cin * 9
        out.append(w["conv_w"][off:off + sz].reshape(C, cin, 3, 3)); off += sz; cin = C
    out.append(w["conv_w"][off:].reshape(nbits, C, 3, 3))
    return out


def python_forward(w, tile):
    """Direct sums in pure Python (independent of the oracle's C)."""
    in_ch, nb, C, nbits = w["in_ch"], w["n_blocks"], w["channels"], w["n_bits"]
    _, h, wd = tile.shape
    a = [[[(float(tile[c, i, j]) / 255.0 - float(w["mean"][c])) / float(w["std"][c])
           for j in range(wd)] for i in range(h)] for c in range(in_ch)]
    convs = split_conv(w)

    def conv(a, wt, scale, bias, relu):
        co, ci = wt.shape[0], wt.shape[1]
        out = [[[0.0] * wd for _ in range(h)] for _ in range(co)]
        for o in range(co):
            for i in range(h):
                for j in range(wd):
                    s = 0.0
                    for c in range(ci):
                        for di in range(3):
                            for dj in range(3):
                                ii, jj = i + di - 1, j + dj - 1
                                if 0 <= ii < h and 0 <= jj < wd:
                                    s += float(wt[o, c, di, dj]) * a[c][ii][jj]
                    if scale is not None:
                        s = s * float(scale[o]) + float(bias[o])
                    out[o][i][j] = max(s, 0.0) if relu else s
        return out
    for b in range(nb):
        a = conv(a, convs[b], w["scale"][b * C:(b + 1) * C], w["bias"][b * C:(b + 1) * C], True)
    f = conv(a, convs[nb], None, None, False)
    pooled = [sum(sum(row) for row in f[o]) / (h * wd) for o in range(nbits)]
    return [float(w["lin_b"][o]) + sum(float(w["lin_w"][o, i]) * pooled[i] for i in range(nbits))
            for o in range(nbits)]


def torch_forward(w, tiles):
    in_ch, nb, C, nbits = w["in_ch"], w["n_blocks"], w["channels"], w["n_bits"]
    x = torch.from_numpy(tiles.astype(np.float64)) / 255.0
    mean = torch.tensor(w["mean"][:in_ch].astype(np.float64)).view(1, -1, 1, 1)
    std = torch.tensor(w["std"][:in_ch].astype(np.float64)).view(1, -1, 1, 1)
    x = (x - mean) / std
    convs = split_conv(w)
    acts = []
    for b in range(nb):
        x = torch.nn.functional.conv2d(x, torch.from_numpy(convs[b].astype(np.float64)), padding=1)
        s = torch.from_numpy(w["scale"][b * C:(b + 1) * C].astype(np.float64)).view(1, -1, 1, 1)
        t = torch.from_numpy(w["bias"][b * C:(b + 1) * C].astype(np.float64)).view(1, -1, 1, 1)
        x = torch.relu(x * s + t)
        acts.append(x)
    x = torch.nn.functional.conv2d(x, torch.from_numpy(convs[nb].astype(np.float64)), padding=1)
    p = x.mean(dim=(2, 3))
    z = p @ torch.from_numpy(w["lin_w"].astype(np.float64)).T + torch.from_numpy(w["lin_b"].astype(np.float64))
    return z.numpy(), [a.numpy() for a in acts], p.numpy()


def test_matches_pure_python_direct_sum():
    w = tiny_weights(3, 2, 2, 4)
    rng = np.random.default_rng(0)
    tile = rng.integers(0, 256, size=(1, 3, 5, 6), dtype=np.uint8)     # non-square on purpose
    logits, bits = oracle.extractor_forward(w, tile)
    ref = python_forward(w, tile[0])
    assert np.allclose(logits[0], ref, rtol=1e-12, atol=1e-12)
    assert np.array_equal(bits[0], (np.array(ref) > 0).astype(np.uint8))


@pytest.mark.parametrize("in_ch,nb,C,nbits,h,wd", [(3, 2, 4, 8, 7, 9), (3, 4, 8, 12, 16, 16), (1, 1, 3, 4, 3, 3)])
def test_matches_torch_conv2d_fp64(in_ch, nb, C, nbits, h, wd):
    w = tiny_weights(in_ch, nb, C, nbits, seed=1)
    rng = np.random.default_rng(1)
    tiles = rng.integers(0, 256, size=(3, in_ch, h, wd), dtype=np.uint8)
    logits, bits, pooled = oracle.extractor_forward(w, tiles, want_pooled=True)
    ref, _, pref = torch_forward(w, tiles)
    assert np.allclose(logits, ref, rtol=1e-11, atol=1e-11)
    assert np.allclose(pooled, pref, rtol=1e-11, atol=1e-11)
    _, _, acts = oracle.extractor_forward(w, tiles[:1], want_acts=True)
    _, aref, _ = torch_forward(w, tiles[:1])
    for b in range(nb):
        assert np.allclose(acts[b], aref[b][0], rtol=1e-11, atol=1e-11)


def delta_net(di, dj, bias=10.0):
    """One block, 3 -> 3 channels, kernel = a single 1 at tap (di,dj) on the diagonal."""
    conv1 = np.zeros((3, 3, 3, 3), np.float32)
    for c in range(3):
        conv1[c, c, di, dj] = 1.0
    final = np.zeros((3, 3, 3, 3), np.float32)
    for c in range(3):
        final[c, c, 1, 1] = 1.0
    return {"in_ch": 3, "n_blocks": 1, "channels": 3, "n_bits": 3,
            "conv_w": np.concatenate([conv1.ravel(), final.ravel()]),
            "scale": np.ones(3, np.float32), "bias": np.full(3, bias, np.float32),
            "lin_w": np.eye(3, dtype=np.float32), "lin_b": np.zeros(3, np.float32),
            "mean": np.array(synth.MEAN, np.float32), "std": np.array(synth.STD, np.float32)}


def test_normalisation_closed_form():
    w = delta_net(1, 1)
    tile = np.zeros((1, 3, 4, 4), np.uint8)
    tile[0, 0], tile[0, 1], tile[0, 2] = 0, 128, 255
    _, _, acts = oracle.extractor_forward(w, tile, want_acts=True)
    for c, v in enumerate((0, 128, 255)):
        mean, std = np.float64(np.float32(synth.MEAN[c])), np.float64(np.float32(synth.STD[c]))
        assert np.allclose(acts[0][c], (v / 255.0 - mean) / std + 10.0, rtol=0, atol=1e-12)
    # by-hand value for the first channel at 0: -0.485/0.229
    assert abs(acts[0][0][0, 0] - 10.0 - (-0.485 / 0.229)) < 1e-6


@pytest.mark.parametrize("di,dj", [(0, 0), (0, 2), (2, 0), (2, 2), (1, 0), (0, 1)])
def test_delta_kernel_shifts_and_zero_pads(di, dj):
    """out[i][j] = in[i+di-1][j+dj-1] (cross-correlation), zero outside the tile, in normalised space."""
    w = delta_net(di, dj)
    rng = np.random.default_rng(2)
    tile = rng.integers(0, 256, size=(1, 3, 6, 5), dtype=np.uint8)
    _, _, acts = oracle.extractor_forward(w, tile, want_acts=True)
    for c in range(3):
        mean, std = np.float64(np.float32(synth.MEAN[c])), np.float64(np.float32(synth.STD[c]))
        norm = (tile[0, c].astype(np.float64) / 255.0 - mean) / std
        exp = np.zeros((6, 5))
        for i in range(6):
            for j in range(5):
                ii, jj = i + di - 1, j + dj - 1
                exp[i, j] = norm[ii, jj] if (0 <= ii < 6 and 0 <= jj < 5) else 0.0
        assert np.allclose(acts[0][c] - 10.0, exp, atol=1e-12)


def test_constant_input_all_ones_kernel_pool_closed_form():
    """Final conv + average pool on a constant map: each unit of input contributes
    ((l-2)^2*9 + 4(l-2)*6 + 4*4) / l^2 through a 3x3 all-ones kernel with zero padding."""
    l = 8
    w = delta_net(1, 1, bias=0.0)
    w["mean"] = np.zeros(3, np.float32); w["std"] = np.ones(3, np.float32)
    final = np.zeros((3, 3, 3, 3), np.float32)
    final[0, 0] = 1.0; final[1, 1] = 1.0; final[2, 0] = 1.0; final[2, 2] = 1.0
    w["conv_w"] = np.concatenate([w["conv_w"][:81], final.ravel()])
    tile = np.full((1, 3, l, l), 255, np.uint8)                  # normalised value exactly 1
    _, _, pooled = oracle.extractor_forward(w, tile, want_pooled=True)
    unit = ((l - 2) ** 2 * 9 + 4 * (l - 2) * 6 + 4 * 4) / l ** 2
    assert np.allclose(pooled[0], [unit, unit, 2 * unit], atol=1e-12)


def test_relu_and_affine_order():
    # block = relu(scale * conv + bias): with scale -1 and bias 0.5 a positive conv output is clipped
    w = delta_net(1, 1, bias=0.5)
    w["scale"] = np.array([-1.0, 1.0, 2.0], np.float32)
    w["mean"] = np.zeros(3, np.float32); w["std"] = np.ones(3, np.float32)
    tile = np.full((1, 3, 3, 3), 255, np.uint8)
    _, _, acts = oracle.extractor_forward(w, tile, want_acts=True)
    assert np.allclose(acts[0][0], 0.0) and np.allclose(acts[0][1], 1.5) and np.allclose(acts[0][2], 2.5)


def test_threshold_at_zero_and_linear_bias():
    w = delta_net(1, 1)
    w["lin_w"] = np.zeros((3, 3), np.float32)
    w["lin_b"] = np.array([0.0, 1e-30, -1e-30], np.float32)
    tile = np.zeros((2, 3, 3, 3), np.uint8)
    logits, bits = oracle.extractor_forward(w, tile)
    assert np.array_equal(bits, [[0, 1, 0], [0, 1, 0]])          # logit == 0 -> bit 0
    assert logits[0, 1] > 0 > logits[0, 2]


def test_final_relu_switch():
    w = tiny_weights(3, 1, 2, 4, seed=3)
    tile = np.random.default_rng(3).integers(0, 256, size=(1, 3, 4, 4), dtype=np.uint8)
    _, _, p0 = oracle.extractor_forward(w, tile, final_relu=0, want_pooled=True)
    _, _, p1 = oracle.extractor_forward(w, tile, final_relu=1, want_pooled=True)
    assert np.all(p1 >= p0 - 1e-15) and np.any(p1 > p0 + 1e-9)


def test_bits_to_symbols_msb_first():
    bits = np.array([[1, 0, 0, 0, 0, 0, 0, 1, 1, 0, 1, 0]], np.uint8)
    assert oracle.bits_to_symbols(bits, 4).tolist() == [[8, 1, 10]]
    bits8 = np.array([[1, 0, 0, 0, 0, 0, 0, 1, 0, 1, 1, 1, 1, 1, 1, 1]], np.uint8)
    assert oracle.bits_to_symbols(bits8, 8).tolist() == [[129, 127]]


def test_extract_tiles_matches_slicing_and_clamps():
    rng = np.random.default_rng(4)
    imgs = rng.integers(0, 256, size=(5, 3, 20, 24), dtype=np.uint8)
    off = np.array([[0, 0], [12, 16], [3, 7], [-5, 30], [100, -1]], np.int32)
    t = oracle.extract_tiles(imgs, off, 8)
    cl = [(0, 0), (12, 16), (3, 7), (0, 16), (12, 0)]
    for i, (y, x) in enumerate(cl):
        assert np.array_equal(t[i], imgs[i, :, y:y + 8, x:x + 8])
    assert np.array_equal(oracle.extract_tiles(imgs, None, 20)[:, :, :, :], imgs[:, :, :20, :20])
    with pytest.raises(ValueError):
        oracle.extract_tiles(imgs, off, 21)


def test_detect_composes_the_stages():
    cfg = synth.CONFIGS["C1"]
    w = synth.extractor_weights(3, 1, 4, 60, seed_index=50)
    imgs = synth.images(cfg, 0, 2)
    off = synth.offsets(cfg, 0, 2)
    r = oracle.detect(w, imgs, off, 8, cfg.m, cfg.prim_poly, cfg.n, cfg.k)
    assert r["tiles"].shape == (2, 3, 8, 8) and r["logits"].shape == (2, 60)
    assert np.array_equal(r["bits"], (r["logits"] > 0).astype(np.uint8))
    assert np.array_equal(r["symbols"], oracle.bits_to_symbols(r["bits"], 4))
    m2, c2, e2 = oracle.rs_decode(r["symbols"], cfg.m, cfg.prim_poly, cfg.n, cfg.k)
    assert np.array_equal(m2, r["msg"]) and np.array_equal(e2, r["nerr"])
