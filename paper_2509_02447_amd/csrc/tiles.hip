// Stand-alone tile crop for gfx950 (Section 4.3 / Table 1 "Tile" of the paper): copies the tile x tile
// window at a per-image origin out of each of the three u8 planes.  HBM-bound byte shuffling: one
// block per (image, plane); when everything is 4-byte friendly each lane assembles one aligned output
// dword from two aligned input dwords (funnel shift by the source misalignment), otherwise bytes.
#include "qrm_internal.h"

namespace qrm {

namespace {

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

template <bool WORDS>
__global__ __launch_bounds__(256) void extract_tiles_kernel(const uint8_t *__restrict__ img, int H, int W,
                                                            const int32_t *__restrict__ off, int tile,
                                                            uint8_t *__restrict__ out)
{
    const int64_t plane = blockIdx.x; // n*3 + c
    const int64_t n = plane / 3;
    int oy = 0, ox = 0;
    if (off) {
        oy = clampi(off[2 * n], 0, H - tile);
        ox = clampi(off[2 * n + 1], 0, W - tile);
    }
    const uint8_t *src = img + plane * (int64_t)H * W + (int64_t)oy * W + ox;
    uint8_t *dst = out + plane * (int64_t)tile * tile;
    if (WORDS) {
        const int wpr = tile >> 2; // dwords per output row
        const int total = wpr * tile;
        for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {
            const int row = idx / wpr, col = (idx - row * wpr) << 2;
            const uint8_t *s = src + (int64_t)row * W + col;
            const uintptr_t a = (uintptr_t)s;
            const uint32_t *aligned = (const uint32_t *)(a & ~(uintptr_t)3);
            const unsigned sh = (unsigned)(a & 3u);
            uint32_t lo = aligned[0];
            uint32_t v = lo;
            if (sh) {
                uint32_t hi = aligned[1];
                v = __builtin_amdgcn_alignbyte(hi, lo, sh);
            }
            *(uint32_t *)(dst + (int64_t)row * tile + col) = v;
        }
    } else {
        const int total = tile * tile;
        for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {
            const int row = idx / tile, col = idx - row * tile;
            dst[idx] = src[(int64_t)row * W + col];
        }
    }
}

} // namespace

hipError_t launch_extract_tiles(const uint8_t *img, int64_t N, int H, int W, const int32_t *off, int tile,
                                uint8_t *out, hipStream_t s)
{
    if (N <= 0) return hipSuccess;
    // dword path: output rows are whole dwords, the output is dword aligned, and every aligned input
    // dword that overlaps the image buffer lies inside it (base aligned, total size a multiple of 4)
    const bool words = (tile % 4 == 0) && (((uintptr_t)out & 3u) == 0) && (((uintptr_t)img & 3u) == 0) &&
                       (((int64_t)N * 3 * H * W) % 4 == 0);
    const int64_t planes = N * 3;
    // grid.x is limited to 2^31-1; batches beyond that are split
    const int64_t kMaxGrid = 3LL << 28; // whole images per launch
    for (int64_t p0 = 0; p0 < planes; p0 += kMaxGrid) {
        const int64_t cnt = planes - p0 < kMaxGrid ? planes - p0 : kMaxGrid;
        const uint8_t *img0 = img + p0 * (int64_t)H * W;
        const int32_t *off0 = off ? off + 2 * (p0 / 3) : nullptr;
        uint8_t *out0 = out + p0 * (int64_t)tile * tile;
        if (words)
            hipLaunchKernelGGL(extract_tiles_kernel<true>, dim3((unsigned)cnt), dim3(256), 0, s, img0, H, W, off0,
                               tile, out0);
        else
            hipLaunchKernelGGL(extract_tiles_kernel<false>, dim3((unsigned)cnt), dim3(256), 0, s, img0, H, W, off0,
                               tile, out0);
    }
    return hipGetLastError();
}

} // namespace qrm
