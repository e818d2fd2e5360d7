"""MI355X-native batched watermark detection (QRMark hot path): thin binding over libqrm.so.

The package only marshals arguments: every step of the path (tile crop, extractor, thresholding,
Reed-Solomon decoding) runs in the hand-written HIP kernels behind the C ABI declared in
include/qrm.h.  There is no CPU fallback: if the library is missing or fails to load, import of
`paper_2509_02447_amd.binding` raises.
"""
from .binding import (QrmError, Context, lib_path, load_library, version,  # noqa: F401
                      QRM_OK, QRM_E_INVALID, QRM_E_UNSUPPORTED, QRM_E_NOMEM, QRM_E_DEVICE,
                      QRM_MAX_STREAMS, qrm_plan_streams, qrm_key_threshold)
