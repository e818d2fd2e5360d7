"""ctypes binding of libqrm.so: same names as the C ABI (include/qrm.h), argument marshalling only.

Tensors are torch CUDA(ROCm) tensors used purely as device memory; streams are torch streams.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

QRM_OK, QRM_E_INVALID, QRM_E_UNSUPPORTED, QRM_E_NOMEM, QRM_E_DEVICE = 0, 1, 2, 3, 4

_HERE = os.path.dirname(os.path.abspath(__file__))
# QRM_LIBRARY selects another build of the same library (same ABI), e.g. one with different tuning constants
_LIB_PATH = os.environ.get("QRM_LIBRARY") or os.path.join(_HERE, "libqrm.so")
_lib = None


class QrmError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"qrm status {status}: {message}")
        self.status = status
        self.message = message


class _ExtDesc(C.Structure):
    _fields_ = [("in_ch", C.c_int32), ("n_blocks", C.c_int32), ("channels", C.c_int32), ("n_bits", C.c_int32),
                ("conv_w", C.POINTER(C.c_float)), ("scale", C.POINTER(C.c_float)), ("bias", C.POINTER(C.c_float)),
                ("final_affine", C.c_int32), ("final_relu", C.c_int32),
                ("lin_w", C.POINTER(C.c_float)), ("lin_b", C.POINTER(C.c_float)),
                ("mean", C.c_float * 3), ("std", C.c_float * 3)]


class _RsDesc(C.Structure):
    _fields_ = [("m", C.c_int32), ("prim_poly", C.c_uint32), ("n", C.c_int32), ("k", C.c_int32), ("fcr", C.c_int32)]


EXPORTS = ["qrm_create", "qrm_destroy", "qrm_last_error", "qrm_set_micro_batch", "qrm_workspace_bytes",
           "qrm_extract_tiles", "qrm_preprocess", "qrm_select_tiles_variance", "qrm_extractor_forward", "qrm_extractor_blocks", "qrm_rs_decode", "qrm_detect",
           "qrm_detect_host", "qrm_plan_streams", "qrm_key_threshold", "qrm_set_key", "qrm_verify_key", "qrm_detect_verify",
           "qrm_profile_enable", "qrm_profile_read", "qrm_profile_read_chunks", "qrm_release_stream", "qrm_detect_static", "qrm_version"]
DIAG_EXPORTS = ["qrm_diag_set_flags", "qrm_diag_matrix_rate"]      # include/qrm_diag.h: bench and test tooling

QRM_MAX_STREAMS = 8   # include/qrm.h
QRM_DIAG_NO_FUSED_PAIRS, QRM_DIAG_POISON_WORKSPACE, QRM_DIAG_FUSE_ALWAYS = 1, 2, 4
(QRM_PROFILE_PAIR_FIRST, QRM_PROFILE_PAIR_MID, QRM_PROFILE_PAIR_LAST, QRM_PROFILE_BLOCK_FIRST, QRM_PROFILE_BLOCK_MID,
 QRM_PROFILE_BLOCK_LAST, QRM_PROFILE_HEAD, QRM_PROFILE_RS_DECODE, QRM_PROFILE_KINDS) = range(9)
PROFILE_KIND_NAMES = ["pair_first", "pair_mid", "pair_last", "block_first", "block_mid", "block_last", "head", "rs_decode"]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libqrm.so; building is the job of build.py / __graft_entry__.build(), not of the import."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -m paper_2509_02447_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.qrm_create.argtypes = [C.POINTER(_ExtDesc), C.POINTER(_RsDesc), C.c_int, C.POINTER(vp)]
    lib.qrm_create.restype = C.c_int
    lib.qrm_destroy.argtypes = [vp]
    lib.qrm_destroy.restype = None
    lib.qrm_last_error.argtypes = [vp]
    lib.qrm_last_error.restype = C.c_char_p
    lib.qrm_set_micro_batch.argtypes = [vp, i32]
    lib.qrm_set_micro_batch.restype = C.c_int
    lib.qrm_workspace_bytes.argtypes = [vp, i64, i32, i32]
    lib.qrm_workspace_bytes.restype = C.c_size_t
    lib.qrm_extract_tiles.argtypes = [vp, vp, i64, i32, i32, vp, i32, vp, vp]
    lib.qrm_extract_tiles.restype = C.c_int
    lib.qrm_preprocess.argtypes = [vp, vp, i64, i32, i32, i32, vp, i32, vp, vp]
    lib.qrm_preprocess.restype = C.c_int
    lib.qrm_select_tiles_variance.argtypes = [vp, vp, i64, i32, i32, i32, i32, vp, vp, vp]
    lib.qrm_select_tiles_variance.restype = C.c_int
    lib.qrm_extractor_forward.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp]
    lib.qrm_extractor_forward.restype = C.c_int
    lib.qrm_extractor_blocks.argtypes = [vp, vp, i64, i32, i32, i32, vp, vp]
    lib.qrm_extractor_blocks.restype = C.c_int
    lib.qrm_rs_decode.argtypes = [vp, vp, i64, vp, vp, vp, vp]
    lib.qrm_rs_decode.restype = C.c_int
    lib.qrm_detect.argtypes = [vp, vp, i64, i32, i32, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.qrm_detect.restype = C.c_int
    lib.qrm_detect_static.argtypes = [vp, vp, i64, i32, i32, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.qrm_detect_static.restype = C.c_int
    lib.qrm_detect_host.argtypes = [vp, C.POINTER(vp), i32, i32, i32, i32, C.POINTER(vp), i32, i32, vp, vp, vp]
    lib.qrm_detect_host.restype = C.c_int
    lib.qrm_key_threshold.argtypes = [i32, C.c_double]
    lib.qrm_key_threshold.restype = C.c_int32
    lib.qrm_plan_streams.argtypes = [i32, C.POINTER(C.c_double), C.POINTER(C.c_double), i64, i64, i32, C.c_double,
                                     C.c_double, i32, C.POINTER(i32), C.POINTER(i64), C.POINTER(C.c_double),
                                     C.POINTER(i32)]
    lib.qrm_plan_streams.restype = C.c_int
    lib.qrm_set_key.argtypes = [vp, vp, i32]
    lib.qrm_set_key.restype = C.c_int
    lib.qrm_verify_key.argtypes = [vp, vp, i64, vp, vp, vp]
    lib.qrm_verify_key.restype = C.c_int
    lib.qrm_detect_verify.argtypes = [vp, vp, i64, i32, i32, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.qrm_detect_verify.restype = C.c_int
    lib.qrm_profile_enable.argtypes = [vp, i32]
    lib.qrm_profile_enable.restype = C.c_int
    lib.qrm_profile_read.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_double)]
    lib.qrm_profile_read.restype = C.c_int
    lib.qrm_profile_read_chunks.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(i32)]
    lib.qrm_profile_read_chunks.restype = C.c_int
    lib.qrm_release_stream.argtypes = [vp, vp]
    lib.qrm_release_stream.restype = C.c_int
    lib.qrm_diag_set_flags.argtypes = [vp, i32]
    lib.qrm_diag_set_flags.restype = C.c_int
    lib.qrm_diag_matrix_rate.argtypes = [vp, i32, C.POINTER(C.c_double)]
    lib.qrm_diag_matrix_rate.restype = C.c_int
    lib.qrm_version.argtypes = []
    lib.qrm_version.restype = C.c_char_p
    _lib = lib
    return lib


def version() -> str:
    return load_library().qrm_version().decode()


def qrm_key_threshold(n_bits: int, fpr: float) -> int:
    return int(load_library().qrm_key_threshold(int(n_bits), float(fpr)))


def qrm_plan_streams(t, u, B: int, b0: int, P: int, M_cap: float, eps: float, tau: int):
    """-> (status, s list, m list, J, accepted): streams and micro-batch per stage (host-only)."""
    K = len(t)
    ta, ua = (C.c_double * K)(*[float(x) for x in t]), (C.c_double * K)(*[float(x) for x in u])
    s, m = (C.c_int32 * K)(), (C.c_int64 * K)()
    J, acc = C.c_double(0.0), C.c_int32(0)
    st = load_library().qrm_plan_streams(K, ta, ua, int(B), int(b0), int(P), float(M_cap), float(eps), int(tau), s, m,
                                         C.byref(J), C.byref(acc))
    return int(st), list(s), list(m), float(J.value), int(acc.value)


def _fptr(a: Optional[np.ndarray]):
    if a is None:
        return None
    return a.ctypes.data_as(C.POINTER(C.c_float))


def _dptr(t) -> Optional[int]:
    """Device pointer of a torch tensor (or None)."""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous and on the GPU"
    return t.data_ptr()


def _hptr(t) -> Optional[int]:
    """Host pointer of a CPU torch tensor or a numpy array (or None)."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        assert t.flags["C_CONTIGUOUS"], "host arrays must be contiguous"
        return t.ctypes.data
    assert not t.is_cuda and t.is_contiguous(), "host tensors must be contiguous and on the CPU"
    return t.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


class Context:
    """Owns one qrm_ctx.  `weights` is the dict produced by synth.extractor_weights (host fp32 arrays),
    `rs` a dict(m=, prim_poly=, n=, k=, fcr=).  Either may be None."""

    def __init__(self, weights: Optional[dict] = None, rs: Optional[dict] = None, device: int = 0,
                 final_relu: int = 0):
        self._lib = load_library()
        self._h = C.c_void_p()
        ext_p, rs_p = None, None
        keep = []
        if weights is not None:
            d = _ExtDesc()
            d.in_ch, d.n_blocks = int(weights["in_ch"]), int(weights["n_blocks"])
            d.channels, d.n_bits = int(weights["channels"]), int(weights["n_bits"])
            nb, Cc, nbits = d.n_blocks, d.channels, d.n_bits
            arr = {}
            for key in ("conv_w", "scale", "bias", "lin_w", "lin_b"):
                v = weights.get(key)
                arr[key] = None if v is None else np.ascontiguousarray(v, dtype=np.float32)
                keep.append(arr[key])
            expect = Cc * d.in_ch * 9 + (nb - 1) * Cc * Cc * 9 + nbits * Cc * 9
            if arr["conv_w"] is None or arr["conv_w"].size != expect:
                raise ValueError("conv_w has the wrong number of elements")
            d.conv_w, d.scale, d.bias = _fptr(arr["conv_w"]), _fptr(arr["scale"]), _fptr(arr["bias"])
            d.final_affine = int(arr["scale"] is not None and arr["scale"].size == nb * Cc + nbits)
            d.final_relu = int(final_relu)
            d.lin_w, d.lin_b = _fptr(arr["lin_w"]), _fptr(arr["lin_b"])
            for i in range(3):
                d.mean[i] = float(weights["mean"][i])
                d.std[i] = float(weights["std"][i])
            ext_p = C.byref(d)
            self.n_bits, self.channels, self.n_blocks = nbits, Cc, nb
        if rs is not None:
            r = _RsDesc(int(rs["m"]), int(rs["prim_poly"]), int(rs["n"]), int(rs["k"]), int(rs.get("fcr", 1)))
            rs_p = C.byref(r)
            self.n, self.k, self.m = int(rs["n"]), int(rs["k"]), int(rs["m"])
        st = self._lib.qrm_create(ext_p, rs_p, int(device), C.byref(self._h))
        if st != QRM_OK:
            raise QrmError(st, self._lib.qrm_last_error(None).decode())

    # -- plumbing
    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            self._lib.qrm_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != QRM_OK:
            raise QrmError(st, self._lib.qrm_last_error(self._h).decode())

    def last_error(self) -> str:
        return self._lib.qrm_last_error(self._h).decode()

    # -- the C ABI, one method per entry point
    def qrm_set_micro_batch(self, images: int):
        self._check(self._lib.qrm_set_micro_batch(self._h, int(images)))

    def qrm_profile_enable(self, on: bool):
        self._check(self._lib.qrm_profile_enable(self._h, int(bool(on))))

    def qrm_profile_read(self, kind: int):
        """-> (milliseconds, launches, algorithmic FLOPs) of the timed launches of one kind since enable."""
        ms, n, fl = C.c_double(), C.c_int64(), C.c_double()
        self._check(self._lib.qrm_profile_read(self._h, int(kind), C.byref(ms), C.byref(n), C.byref(fl)))
        return ms.value, n.value, fl.value

    def qrm_profile_read_chunks(self, max_chunks: int):
        """-> float64 array [chunks, 5]: upload start / end, kernels start / end, download end (ms) of the last
        qrm_detect_host call made with profiling on."""
        buf = np.zeros((max(1, int(max_chunks)), 5), dtype=np.float64)
        n = C.c_int32()
        self._check(self._lib.qrm_profile_read_chunks(self._h, int(max_chunks), buf.ctypes.data_as(C.POINTER(C.c_double)),
                                                      C.byref(n)))
        return buf[:min(int(n.value), int(max_chunks))]

    def qrm_release_stream(self, stream=None):
        self._check(self._lib.qrm_release_stream(self._h, _stream_handle(stream)))

    def qrm_diag_set_flags(self, flags: int):
        self._check(self._lib.qrm_diag_set_flags(self._h, int(flags)))

    def qrm_diag_matrix_rate(self, data: int) -> float:
        """-> TFLOP/s the matrix pipes sustain on zeros (0), a constant (1) or random operands (2)."""
        v = C.c_double()
        self._check(self._lib.qrm_diag_matrix_rate(self._h, int(data), C.byref(v)))
        return v.value

    def qrm_workspace_bytes(self, N: int, tile_h: int, tile_w: int) -> int:
        return int(self._lib.qrm_workspace_bytes(self._h, int(N), int(tile_h), int(tile_w)))

    def qrm_extract_tiles(self, d_images, N, H, W, d_off_yx, tile, d_tiles, stream=None):
        self._check(self._lib.qrm_extract_tiles(self._h, _dptr(d_images), int(N), int(H), int(W), _dptr(d_off_yx),
                                                int(tile), _dptr(d_tiles), _stream_handle(stream)))

    def qrm_preprocess(self, d_raw, N, H_in, W_in, size, d_off_yx, tile, d_out, stream=None):
        self._check(self._lib.qrm_preprocess(self._h, _dptr(d_raw), int(N), int(H_in), int(W_in), int(size),
                                             _dptr(d_off_yx), int(tile), _dptr(d_out), _stream_handle(stream)))

    def qrm_select_tiles_variance(self, d_images, N, H, W, tile, stride, d_off_yx, d_scores=None, stream=None):
        self._check(self._lib.qrm_select_tiles_variance(self._h, _dptr(d_images), int(N), int(H), int(W), int(tile),
                                                        int(stride), _dptr(d_off_yx), _dptr(d_scores),
                                                        _stream_handle(stream)))

    def qrm_extractor_forward(self, d_tiles, N, h, w, d_logits, d_bits=None, stream=None):
        self._check(self._lib.qrm_extractor_forward(self._h, _dptr(d_tiles), int(N), int(h), int(w), _dptr(d_logits),
                                                    _dptr(d_bits), _stream_handle(stream)))

    def qrm_extractor_blocks(self, d_tiles, N, h, w, n_run, d_act, stream=None):
        self._check(self._lib.qrm_extractor_blocks(self._h, _dptr(d_tiles), int(N), int(h), int(w), int(n_run),
                                                   _dptr(d_act), _stream_handle(stream)))

    def qrm_rs_decode(self, d_symbols, N, d_msg, d_codeword, d_nerr, stream=None):
        self._check(self._lib.qrm_rs_decode(self._h, _dptr(d_symbols), int(N), _dptr(d_msg), _dptr(d_codeword),
                                            _dptr(d_nerr), _stream_handle(stream)))

    def qrm_detect(self, d_images, N, H, W, d_off_yx, tile, d_logits, d_bits, d_msg, d_codeword, d_nerr,
                   stream=None):
        self._check(self._lib.qrm_detect(self._h, _dptr(d_images), int(N), int(H), int(W), _dptr(d_off_yx),
                                         int(tile), _dptr(d_logits), _dptr(d_bits), _dptr(d_msg), _dptr(d_codeword),
                                         _dptr(d_nerr), _stream_handle(stream)))

    def qrm_detect_static(self, d_images, N, H, W, d_off_yx, tile, d_logits, d_bits, d_msg, d_codeword, d_nerr,
                          stream=None):
        self._check(self._lib.qrm_detect_static(self._h, _dptr(d_images), int(N), int(H), int(W), _dptr(d_off_yx),
                                                int(tile), _dptr(d_logits), _dptr(d_bits), _dptr(d_msg),
                                                _dptr(d_codeword), _dptr(d_nerr), _stream_handle(stream)))

    def qrm_detect_host(self, h_chunks, chunk_images, H, W, h_off_chunks, tile, depth, h_msg, h_codeword, h_nerr):
        """h_chunks / h_off_chunks: sequences of host buffers (pinned CPU tensors or numpy arrays), one per chunk."""
        n = len(h_chunks)
        chunks = (C.c_void_p * max(1, n))(*[_hptr(t) for t in h_chunks])
        offs = None
        if h_off_chunks is not None:
            assert len(h_off_chunks) == n
            offs = (C.c_void_p * max(1, n))(*[_hptr(t) for t in h_off_chunks])
        self._check(self._lib.qrm_detect_host(self._h, chunks, int(n), int(chunk_images), int(H), int(W), offs, int(tile),
                                              int(depth), _hptr(h_msg), _hptr(h_codeword), _hptr(h_nerr)))

    def qrm_set_key(self, h_key, tau: int):
        key = np.ascontiguousarray(h_key, dtype=np.uint8).reshape(-1)
        assert key.size == self.k, "the key has k symbols"
        self._check(self._lib.qrm_set_key(self._h, key.ctypes.data, int(tau)))

    def qrm_verify_key(self, d_msg, N, d_matches, d_detected=None, stream=None):
        self._check(self._lib.qrm_verify_key(self._h, _dptr(d_msg), int(N), _dptr(d_matches), _dptr(d_detected),
                                             _stream_handle(stream)))

    def qrm_detect_verify(self, d_images, N, H, W, d_off_yx, tile, d_logits, d_bits, d_msg, d_codeword, d_nerr,
                          d_matches, d_detected=None, stream=None):
        self._check(self._lib.qrm_detect_verify(self._h, _dptr(d_images), int(N), int(H), int(W), _dptr(d_off_yx),
                                                int(tile), _dptr(d_logits), _dptr(d_bits), _dptr(d_msg),
                                                _dptr(d_codeword), _dptr(d_nerr), _dptr(d_matches), _dptr(d_detected),
                                                _stream_handle(stream)))
