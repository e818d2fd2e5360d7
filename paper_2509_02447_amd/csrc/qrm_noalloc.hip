// qrm_detect_static: the detection path of qrm_detect for callers that cannot allocate device memory (code
// under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  The workspace that
// qrm_detect takes from the context's pool (activation buffers of a micro-batch, channel statistics, packed
// symbols) is a file-scope device array here, of a fixed size; nothing in this file calls hipMalloc / hipFree,
// creates an event or a stream, or calls a library routine that does.
#include "qrm_ctx.h"

using namespace qrm;

namespace {

// The workspace itself.  Each device the library runs on holds its own copy, at its own address, until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) uint8_t scratch[QRM_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
uint8_t *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, looked up once
hipError_t g_scratch_err[kMaxDevices];
bool g_scratch_known[kMaxDevices];

__global__ void clear_zero_block_kernel(u32x4 *p) // the kZeroBytes the convolutions read their padding from
{
    if (threadIdx.x < kZeroBytes / 16) p[threadIdx.x] = (u32x4){0u, 0u, 0u, 0u};
}

} // namespace

namespace qrm {

// Called by qrm_create with `device` current: looks the array's address on that device up (once per device).
hipError_t static_scratch_init(int device)
{
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_scratch_known[device]) {
        void *p = nullptr;
        g_scratch_err[device] = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        g_scratch_ptr[device] = (uint8_t *)p;
        g_scratch_known[device] = true;
    }
    return g_scratch_err[device];
}

} // namespace qrm

extern "C" qrm_status qrm_detect_static(qrm_ctx *c, const uint8_t *d_images, int64_t N, int32_t H, int32_t W,
                                        const int32_t *d_off_yx, int32_t tile, float *d_logits, uint8_t *d_bits,
                                        uint8_t *d_msg, uint8_t *d_codeword, int8_t *d_nerr, void *stream)
{
    if (!c) return QRM_E_INVALID;
    qrm_status st = check_detect_args(c, d_images, N, H, W, tile, d_msg, d_nerr, false, nullptr);
    if (st != QRM_OK) return st;
    if (N == 0) return QRM_OK;
    if (c->device < 0 || c->device >= kMaxDevices || !g_scratch_known[c->device] || g_scratch_err[c->device] != hipSuccess ||
        !g_scratch_ptr[c->device])
        return fail(c, QRM_E_DEVICE, "the static workspace's address is not known on this device (hipGetSymbolAddress failed at qrm_create)");
    hipError_t e = hipSetDevice(c->device);
    if (e != hipSuccess) return hip_fail(c, e, "hipSetDevice");
    uint8_t *ws = g_scratch_ptr[c->device]; // the device address: never the array's name
    hipStream_t s = (hipStream_t)stream;

    // the largest micro-batch whose workspace fits the array
    const size_t per_img = (size_t)tile * tile * c->C * 2;
    WsLayout L{};
    bool fits = false;
    for (size_t mb = (QRM_STATIC_SCRATCH_BYTES / 2) / per_img; mb >= 1; mb = mb > 8 ? mb - mb / 8 : mb - 1) {
        L = ws_layout(c, N, tile, tile, true, mb * per_img);
        if (L.mb >= 1 && L.total <= QRM_STATIC_SCRATCH_BYTES) { fits = true; break; }
    }
    if (!fits) {
        char buf[200];
        snprintf(buf, sizeof buf, "N = %lld images of %d x %d tiles need more than the %u MiB of the static workspace",
                 (long long)N, tile, tile, (unsigned)(QRM_STATIC_SCRATCH_BYTES >> 20));
        return fail(c, QRM_E_UNSUPPORTED, buf);
    }
    // The array keeps what the previous call left.  Every kernel of the path writes what it later reads,
    // except the block of zeros at the start, which is cleared here (by a kernel: a memset node must not
    // end up in a captured graph).
    hipLaunchKernelGGL(clear_zero_block_kernel, dim3(1), dim3(64), 0, s, (u32x4 *)ws);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(c, e, "clear_zero_block launch");
    uint8_t *d_sym = ws + symbols_offset(L);
    TileSrc src{d_images, d_off_yx, H, W, {c->mean[0], c->mean[1], c->mean[2]},
                {c->inv_std[0], c->inv_std[1], c->inv_std[2]}};
    st = run_extractor(c, ws, L, src, N, tile, tile, -1, d_logits, d_bits, d_sym, c->rs.m, nullptr, false, s);
    if (st != QRM_OK) return st;
    e = launch_rs_decode(c->rs, d_sym, N, d_msg, d_codeword, d_nerr, KeyArgs{}, s);
    if (e != hipSuccess) return hip_fail(c, e, "rs_decode launch");
    return QRM_OK;
}
