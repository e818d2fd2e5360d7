"""ctypes front-end of the CPU oracle (oracle/qrm_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It never touches the HIP library, and the HIP binding never imports it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qrm_oracle.c")
_LIB = os.path.join(_HERE, "libqrm_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over images only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
    return _lib


def _p(a: Optional[np.ndarray], ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _u8(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint8)


def _f32(a) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def num_threads() -> int:
    return int(lib().orc_num_threads())


# ------------------------------------------------------------------ field / RS

def gf_tables(m: int, prim_poly: int):
    q = 1 << m
    e = np.zeros(q - 1, dtype=np.int32)
    l = np.zeros(q, dtype=np.int32)
    rc = lib().orc_gf_tables(m, C.c_uint(prim_poly), _p(e, C.c_int32), _p(l, C.c_int32))
    if rc:
        raise ValueError(f"orc_gf_tables rc={rc}")
    return e, l


def gf_mul(m: int, prim_poly: int, a: int, b: int) -> int:
    return int(lib().orc_gf_mul(m, C.c_uint(prim_poly), int(a), int(b)))


def rs_generator(m: int, prim_poly: int, n: int, k: int, fcr: int = 1) -> np.ndarray:
    g = np.zeros(n - k + 1, dtype=np.int32)
    rc = lib().orc_rs_generator(m, C.c_uint(prim_poly), n, k, fcr, _p(g, C.c_int32))
    if rc:
        raise ValueError(f"orc_rs_generator rc={rc}")
    return g


def rs_encode(msgs, m: int, prim_poly: int, n: int, k: int, fcr: int = 1) -> np.ndarray:
    msgs = _u8(msgs).reshape(-1, k)
    cws = np.zeros((msgs.shape[0], n), dtype=np.uint8)
    rc = lib().orc_rs_encode(m, C.c_uint(prim_poly), n, k, fcr, _p(msgs, C.c_uint8),
                             C.c_int64(msgs.shape[0]), _p(cws, C.c_uint8))
    if rc:
        raise ValueError(f"orc_rs_encode rc={rc}")
    return cws


def rs_syndromes(syms, m: int, prim_poly: int, n: int, k: int, fcr: int = 1) -> np.ndarray:
    syms = _u8(syms).reshape(-1, n)
    S = np.zeros((syms.shape[0], n - k), dtype=np.uint8)
    rc = lib().orc_rs_syndromes(m, C.c_uint(prim_poly), n, k, fcr, _p(syms, C.c_uint8),
                                C.c_int64(syms.shape[0]), _p(S, C.c_uint8))
    if rc:
        raise ValueError(f"orc_rs_syndromes rc={rc}")
    return S


def rs_decode(syms, m: int, prim_poly: int, n: int, k: int, fcr: int = 1):
    """-> (msg u8 [N,k], codeword u8 [N,n], nerr i8 [N]); nerr = -1 marks a failure."""
    syms = _u8(syms).reshape(-1, n)
    N = syms.shape[0]
    msgs = np.zeros((N, k), dtype=np.uint8)
    cws = np.zeros((N, n), dtype=np.uint8)
    nerr = np.zeros(N, dtype=np.int8)
    rc = lib().orc_rs_decode(m, C.c_uint(prim_poly), n, k, fcr, _p(syms, C.c_uint8), C.c_int64(N),
                             _p(msgs, C.c_uint8), _p(cws, C.c_uint8), _p(nerr, C.c_int8))
    if rc:
        raise ValueError(f"orc_rs_decode rc={rc}")
    return msgs, cws, nerr


# ------------------------------------------------------------------ tiles / extractor

def extract_tiles(images, off_yx, tile: int) -> np.ndarray:
    images = _u8(images)
    N, ch, H, W = images.shape
    assert ch == 3
    off = None if off_yx is None else np.ascontiguousarray(off_yx, dtype=np.int32).reshape(N, 2)
    tiles = np.zeros((N, 3, tile, tile), dtype=np.uint8)
    rc = lib().orc_extract_tiles(_p(images, C.c_uint8), C.c_int64(N), H, W, _p(off, C.c_int32),
                                 tile, _p(tiles, C.c_uint8))
    if rc:
        raise ValueError(f"orc_extract_tiles rc={rc}")
    return tiles


def extractor_forward(wts: Dict, tiles, final_relu: int = 0, want_acts: bool = False,
                      want_pooled: bool = False):
    """tiles u8 [N,in_ch,h,w] -> (logits f64 [N,n_bits], bits u8 [N,n_bits][, acts][, pooled])."""
    tiles = _u8(tiles)
    N, ch, h, w = tiles.shape
    in_ch, nb, Cc, nbits = (int(wts[k]) for k in ("in_ch", "n_blocks", "channels", "n_bits"))
    assert ch == in_ch
    conv_w = _f32(wts["conv_w"])
    expect = Cc * in_ch * 9 + (nb - 1) * Cc * Cc * 9 + nbits * Cc * 9
    assert conv_w.size == expect, (conv_w.size, expect)
    scale, bias = _f32(wts.get("scale")), _f32(wts.get("bias"))
    has_final = int(scale is not None and scale.size == nb * Cc + nbits)
    lin_w, lin_b = _f32(wts["lin_w"]), _f32(wts.get("lin_b"))
    mean, std = _f32(wts["mean"]), _f32(wts["std"])
    logits = np.zeros((N, nbits), dtype=np.float64)
    bits = np.zeros((N, nbits), dtype=np.uint8)
    acts = np.zeros((nb, Cc, h, w), dtype=np.float64) if want_acts else None
    pooled = np.zeros((N, nbits), dtype=np.float64) if want_pooled else None
    if want_acts:
        assert N == 1
    f = lib().orc_extractor_forward
    rc = f(in_ch, nb, Cc, nbits, int(final_relu), has_final,
           _p(conv_w, C.c_float), _p(scale, C.c_float), _p(bias, C.c_float),
           _p(lin_w, C.c_float), _p(lin_b, C.c_float), _p(mean, C.c_float), _p(std, C.c_float),
           _p(tiles, C.c_uint8), C.c_int64(N), h, w,
           _p(logits, C.c_double), _p(bits, C.c_uint8), _p(acts, C.c_double), _p(pooled, C.c_double))
    if rc:
        raise ValueError(f"orc_extractor_forward rc={rc}")
    out = [logits, bits]
    if want_acts:
        out.append(acts)
    if want_pooled:
        out.append(pooled)
    return tuple(out)


def bits_to_symbols(bits, m: int) -> np.ndarray:
    bits = _u8(bits)
    N, nbits = bits.shape
    syms = np.zeros((N, nbits // m), dtype=np.uint8)
    rc = lib().orc_bits_to_symbols(_p(bits, C.c_uint8), C.c_int64(N), nbits, m, _p(syms, C.c_uint8))
    if rc:
        raise ValueError(f"orc_bits_to_symbols rc={rc}")
    return syms


def detect(wts: Dict, images, off_yx, tile: int, m: int, prim_poly: int, n: int, k: int, fcr: int = 1):
    """The whole path for a batch: crop -> extractor -> threshold -> symbols -> RS decode.

    -> dict(tiles, logits, bits, symbols, msg, codeword, nerr)
    """
    tiles = extract_tiles(images, off_yx, tile)
    logits, bits = extractor_forward(wts, tiles)
    syms = bits_to_symbols(bits, m)
    assert syms.shape[1] == n
    msg, cw, nerr = rs_decode(syms, m, prim_poly, n, k, fcr)
    return {"tiles": tiles, "logits": logits, "bits": bits, "symbols": syms,
            "msg": msg, "codeword": cw, "nerr": nerr}
