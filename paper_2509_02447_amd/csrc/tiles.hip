// Stand-alone tile crop for gfx950 (Section 4.3 / Table 1 "Tile" of the paper): copies the tile x tile
// window at a per-image origin out of each of the three u8 planes.  HBM-bound byte shuffling: one
// block per (image, plane); when everything is 4-byte friendly each lane assembles one aligned output
// dword from two aligned input dwords (funnel shift by the source misalignment), otherwise bytes.
// Also here: variance-based tile selection (further down).
#include <algorithm>
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

// ------------------------------------------------------------------------------------------------
// Variance-based tile selection (Listing 1 of the paper, `select_patch`): windows of win x win pixels at
// a stride that divides win; score of a window = sum over channels of w_c * (n S2_c - S1_c^2), i.e. the
// channel's unbiased variance up to the common factor n (n-1); the first window with the largest score
// is the tile.  HBM-bound: every pixel that lies in some window is read exactly once.
//
// One workgroup per image.  The image is cut into cells of stride x stride pixels; a window is a square of
// (win / stride)^2 cells.  Phase 1: every lane walks down a run of rows of one 16-byte (or 1-byte) column
// chunk, sums x (v_sad_u8) and x^2 (v_dot4_u32_u8) in registers and adds them to the cell's 32-bit sums in
// LDS when it crosses into the next cell row.  Phase 2: one lane per window adds up its cells (64 bit),
// forms the exact integers n S2 - S1^2, and the score in float64 in a fixed order with no fused
// multiply-add; a workgroup reduction picks the first maximum.
// ------------------------------------------------------------------------------------------------
constexpr int kMaxCells = 1024; // cells per channel a workgroup can hold

struct SelectArgs {
    int H, W, win, stride;
    int nH, nW;     // windows
    int nCy, nCx;   // cells that lie in some window
    double w[3];    // channel weights
};

template <int VEC>
__global__ __launch_bounds__(256) void tile_variance_kernel(const uint8_t *__restrict__ img, SelectArgs a,
                                                            int32_t *__restrict__ off_yx, double *__restrict__ scores)
{
    __shared__ uint32_t s_sum[3][kMaxCells], s_sq[3][kMaxCells];
    __shared__ double s_best[256];
    __shared__ int s_idx[256];
    const int tid = threadIdx.x;
    const int64_t n = blockIdx.x;
    const int cells = a.nCy * a.nCx;
    for (int i = tid; i < 3 * kMaxCells; i += 256) {
        (&s_sum[0][0])[i] = 0u;
        (&s_sq[0][0])[i] = 0u;
    }
    __syncthreads();

    // ---- phase 1: cell sums
    const int Hc = a.nCy * a.stride, Wc = a.nCx * a.stride; // the part of the image that windows cover
    const int ncx = Wc / VEC;                                // column chunks per row
    const int TX = ncx < 256 ? ncx : 256;
    const int n_rg = 256 / TX;                               // row groups
    const int R = (Hc + n_rg - 1) / n_rg;                    // rows per group
    const int rg = tid / TX;
    const uint8_t *base = img + n * 3 * (int64_t)a.H * a.W;
    if (rg < n_rg) {
        const int r0 = rg * R, r1 = min(Hc, r0 + R);
        for (int c = 0; c < 3; ++c) {
            const uint8_t *plane = base + (int64_t)c * a.H * a.W;
            for (int cx = tid - rg * TX; cx < ncx; cx += TX) {
                const int cellx = cx * VEC / a.stride;
                const uint8_t *col = plane + cx * VEC;
                for (int seg = r0; seg < r1;) { // the run's rows, one cell row at a time
                    const int cy = seg / a.stride;
                    const int seg_end = min(r1, (cy + 1) * a.stride);
                    uint32_t s1 = 0, s2 = 0;
#pragma unroll 4
                    for (int r = seg; r < seg_end; ++r) { // independent loads: several in flight per lane
                        const uint8_t *p = col + (int64_t)r * a.W;
                        if (VEC == 16) {
                            const uint4 v = *(const uint4 *)p;
                            s1 = __builtin_amdgcn_sad_u8(v.x, 0u, s1);
                            s1 = __builtin_amdgcn_sad_u8(v.y, 0u, s1);
                            s1 = __builtin_amdgcn_sad_u8(v.z, 0u, s1);
                            s1 = __builtin_amdgcn_sad_u8(v.w, 0u, s1);
                            s2 = __builtin_amdgcn_udot4(v.x, v.x, s2, false);
                            s2 = __builtin_amdgcn_udot4(v.y, v.y, s2, false);
                            s2 = __builtin_amdgcn_udot4(v.z, v.z, s2, false);
                            s2 = __builtin_amdgcn_udot4(v.w, v.w, s2, false);
                        } else {
                            const uint32_t x = *p;
                            s1 += x;
                            s2 += x * x;
                        }
                    }
                    atomicAdd(&s_sum[c][cy * a.nCx + cellx], s1);
                    atomicAdd(&s_sq[c][cy * a.nCx + cellx], s2);
                    seg = seg_end;
                }
            }
        }
    }
    __syncthreads();
    (void)cells;

    // ---- phase 2: window scores, first maximum
    const int k = a.win / a.stride;
    const double npix = (double)a.win * (double)a.win; // exact
    double best = -1.0;                               // scores are >= 0
    int best_idx = 0x7fffffff;
    for (int wi = tid; wi < a.nH * a.nW; wi += 256) {
        const int wy = wi / a.nW, wx = wi - wy * a.nW;
        double score = 0.0;
        for (int c = 0; c < 3; ++c) {
#pragma clang fp contract(off) // each product and each sum is rounded on its own: no fused multiply-add
            unsigned long long S1 = 0, S2 = 0;
            for (int dy = 0; dy < k; ++dy)
                for (int dx = 0; dx < k; ++dx) {
                    S1 += s_sum[c][(wy + dy) * a.nCx + wx + dx];
                    S2 += s_sq[c][(wy + dy) * a.nCx + wx + dx];
                }
            const unsigned long long v = (unsigned long long)(a.win * a.win) * S2 - S1 * S1; // exact, < 2^53
            const double term = (double)v * a.w[c];
            score = c == 0 ? term : score + term;
        }
        (void)npix;
        if (scores) scores[n * (int64_t)(a.nH * a.nW) + wi] = score;
        if (score > best) { // ascending wi: the first maximum stays
            best = score;
            best_idx = wi;
        }
    }
    s_best[tid] = best;
    s_idx[tid] = best_idx;
    __syncthreads();
    for (int half = 128; half >= 1; half >>= 1) {
        if (tid < half) {
            const double o = s_best[tid + half];
            const int oi = s_idx[tid + half];
            if (o > s_best[tid] || (o == s_best[tid] && oi < s_idx[tid])) {
                s_best[tid] = o;
                s_idx[tid] = oi;
            }
        }
        __syncthreads();
    }
    if (tid == 0) {
        const int wi = s_idx[0];
        off_yx[2 * n] = wi / a.nW * a.stride;
        off_yx[2 * n + 1] = wi % a.nW * a.stride;
    }
}

// ------------------------------------------------------------------------------------------------
// Fused pre-processing (Table 1 of the paper: resize to x, centre crop x, to tensor; Appendix A: one pass
// from the raw buffer): raw u8 images, height x width x 3 interleaved, -> planar u8 [3][T][T], where the
// T x T window is either the whole centre crop (T = x) or one tile of it at a per-image origin: only the
// source pixels under that window are touched.  Bilinear, pixel centres at half-integers, fixed point:
// the fraction of a source coordinate is rounded to 11 bits, the four products are exact integers, the
// sum is rounded half up (>> 22).  Integer arithmetic only: the bytes do not depend on the hardware.
//
// One workgroup per (image, strip of rows).  The column taps of the window are computed once into LDS
// (two integer divisions per column), a lane then produces four neighbouring pixels of a row for the
// three colours and writes one dword per plane.
// ------------------------------------------------------------------------------------------------
constexpr int kCoefBits = 11;
constexpr int kMaxTile = 1024; // columns of a window

struct PreArgs {
    int H_in, W_in, x, T;  // raw size, size after resize + crop, window
    int Hr, Wr, cy, cx;    // resized size, origin of the centre crop in it
    int rows_per_block;
};

__device__ __forceinline__ void source_taps(int dst, int n_in, int n_res, int &i0, int &i1, int &w1)
{
    int num = (2 * dst + 1) * n_in - n_res; // numerator of the source coordinate over 2 * n_res
    const int den = 2 * n_res;
    num = num < 0 ? 0 : num;
    i0 = num / den;
    int a = num - i0 * den;
    if (i0 >= n_in - 1) {
        i0 = n_in - 1;
        a = 0;
    }
    i1 = min(i0 + 1, n_in - 1);
    w1 = (a * (1 << kCoefBits) + n_res) / den; // round(fraction * 2048)
}

typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));

// One colour of one window pixel from the dwords that hold its four taps (p00 p01 above p10 p11).  sel picks the
// colour's byte out of the left tap (low half) and the right tap (high half), wx = wx0 | wx1 << 16.  The horizontal
// pass is a two-term dot product of 16-bit fields (< 2^19), the vertical pass two 24-bit products (< 2^30): all
// full-rate instructions, and the same integers as the plain formula.
__device__ __forceinline__ uint32_t bilinear_byte(uint32_t p00, uint32_t p01, uint32_t p10, uint32_t p11, uint32_t sel,
                                                  uint32_t wx, uint32_t wy0, uint32_t wy1)
{
    const uint32_t t = __builtin_amdgcn_perm(p01, p00, sel), b = __builtin_amdgcn_perm(p11, p10, sel);
    const uint32_t top = __builtin_amdgcn_udot2(__builtin_bit_cast(ushort2_t, t), __builtin_bit_cast(ushort2_t, wx), 0u, false);
    const uint32_t bot = __builtin_amdgcn_udot2(__builtin_bit_cast(ushort2_t, b), __builtin_bit_cast(ushort2_t, wx), 0u, false);
    const uint32_t sum = __umul24(top, wy0) + (__umul24(bot, wy1) + (1u << (2 * kCoefBits - 1)));
    return sum >> (2 * kCoefBits);
}
constexpr uint32_t kSelect = 0x0c040c00u; // byte 0 of the second operand -> bits 0..7, byte 0 of the first -> 16..23

// Walks the (row, pixel group) pairs of a strip, 256 at a time, without a division per step.
struct StripWalk {
    int row, grp, d_row, d_grp, groups;
    __device__ StripWalk(int tid, int groups_) : groups(groups_)
    {
        row = tid / groups;
        grp = tid - row * groups;
        d_row = 256 / groups;
        d_grp = 256 - d_row * groups;
    }
    __device__ void next()
    {
        row += d_row;
        grp += d_grp;
        if (grp >= groups) {
            grp -= groups;
            ++row;
        }
    }
};

template <int VEC, bool WORDS>
__global__ __launch_bounds__(256) void preprocess_kernel(const uint8_t *__restrict__ raw, PreArgs a,
                                                         const int32_t *__restrict__ off, uint8_t *__restrict__ out)
{
    __shared__ int s_x0[kMaxTile], s_x1[kMaxTile], s_y0[kMaxTile], s_y1[kMaxTile];
    __shared__ uint32_t s_wx[kMaxTile], s_sel[kMaxTile];
    __shared__ uint16_t s_wy[kMaxTile];
    const int tid = threadIdx.x;
    const int64_t n = blockIdx.x;
    int oy = 0, ox = 0;
    if (off && a.T < a.x) {
        oy = clampi(off[2 * n], 0, a.x - a.T);
        ox = clampi(off[2 * n + 1], 0, a.x - a.T);
    }
    const int r_begin = blockIdx.y * a.rows_per_block, r_end = min(a.T, r_begin + a.rows_per_block);
    for (int t = tid; t < a.T; t += 256) {
        int i0, i1, w1;
        source_taps(a.cx + ox + t, a.W_in, a.Wr, i0, i1, w1);
        // A pixel's three bytes are fetched with ONE (unaligned) dword load: bytes 3i-1 .. 3i+2 for i > 0 (the colours
        // are its upper three bytes), bytes 0 .. 3 for i = 0; both stay inside the row (rows have at least two pixels
        // on this path; one-pixel rows are read byte by byte).  The byte selector carries the "skip one".
        s_x0[t] = WORDS ? (i0 > 0 ? 3 * i0 - 1 : 0) : i0 * 3;
        s_x1[t] = WORDS ? (i1 > 0 ? 3 * i1 - 1 : 0) : i1 * 3;
        s_sel[t] = kSelect + (WORDS && i0 > 0 ? 1u : 0u) + (WORDS && i1 > 0 ? 0x10000u : 0u);
        s_wx[t] = (uint32_t)((1 << kCoefBits) - w1) | (uint32_t)w1 << 16;
    }
    for (int t = tid; t < r_end - r_begin; t += 256) {
        int y0, y1, wy1;
        source_taps(a.cy + oy + r_begin + t, a.H_in, a.Hr, y0, y1, wy1);
        s_y0[t] = y0;
        s_y1[t] = y1;
        s_wy[t] = (uint16_t)wy1;
    }
    __syncthreads();
    const uint8_t *img = raw + n * (int64_t)a.H_in * a.W_in * 3;
    uint8_t *dst = out + n * 3 * (int64_t)a.T * a.T;
    const int64_t plane = (int64_t)a.T * a.T;
    for (StripWalk w(tid, a.T / VEC); w.row < r_end - r_begin; w.next()) {
        const int ty = r_begin + w.row, tx = w.grp * VEC;
        const uint32_t wy1 = s_wy[w.row], wy0 = (1u << kCoefBits) - wy1;
        const uint8_t *row0 = img + (int64_t)s_y0[w.row] * a.W_in * 3, *row1 = img + (int64_t)s_y1[w.row] * a.W_in * 3;
        uint32_t pk[3] = {0u, 0u, 0u};
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            const int b0 = s_x0[tx + v], b1 = s_x1[tx + v];
            const uint32_t wx = s_wx[tx + v], sel = s_sel[tx + v];
            uint32_t p00, p01, p10, p11; // the three colours of the four taps, one per byte
            if (WORDS) {
                __builtin_memcpy(&p00, row0 + b0, 4);
                __builtin_memcpy(&p01, row0 + b1, 4);
                __builtin_memcpy(&p10, row1 + b0, 4);
                __builtin_memcpy(&p11, row1 + b1, 4);
            } else {
                p00 = row0[b0] | row0[b0 + 1] << 8 | row0[b0 + 2] << 16;
                p01 = row0[b1] | row0[b1 + 1] << 8 | row0[b1 + 2] << 16;
                p10 = row1[b0] | row1[b0 + 1] << 8 | row1[b0 + 2] << 16;
                p11 = row1[b1] | row1[b1 + 1] << 8 | row1[b1 + 2] << 16;
            }
#pragma unroll
            for (int c = 0; c < 3; ++c)
                pk[c] |= bilinear_byte(p00, p01, p10, p11, sel + c * 0x10001u, wx, wy0, wy1) << (8 * v);
        }
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            uint8_t *p = dst + c * plane + (int64_t)ty * a.T + tx;
            if (VEC == 4) *(uint32_t *)p = pk[c];
            else *p = (uint8_t)pk[c];
        }
    }
}

} // namespace

void preprocess_resized_shape(int H_in, int W_in, int x, int *Hr, int *Wr)
{
    if (H_in <= W_in) {
        *Hr = x;
        *Wr = (int)std::max<int64_t>(x, (int64_t)x * W_in / H_in);
    } else {
        *Hr = (int)std::max<int64_t>(x, (int64_t)x * H_in / W_in);
        *Wr = x;
    }
}

bool preprocess_supported(int H_in, int W_in, int x, int T)
{
    if (H_in <= 0 || W_in <= 0 || x <= 0 || T <= 0 || T > x || T > kMaxTile) return false;
    if (H_in > 16384 || W_in > 16384) return false;
    int Hr, Wr;
    preprocess_resized_shape(H_in, W_in, x, &Hr, &Wr);
    // (2 * dst + 1) * n_in and fraction * 2048 must stay below 2^31
    return Hr <= 16384 && Wr <= 16384 && (int64_t)(2 * (int64_t)std::max(Hr, Wr) + 1) * std::max(H_in, W_in) < (1LL << 31) &&
           (int64_t)2 * std::max(Hr, Wr) * 2048 < (1LL << 31);
}

hipError_t launch_preprocess(const uint8_t *raw, int64_t N, int H_in, int W_in, int x, const int32_t *off, int T,
                             uint8_t *out, hipStream_t s)
{
    if (N <= 0) return hipSuccess;
    PreArgs a{};
    a.H_in = H_in; a.W_in = W_in; a.x = x; a.T = T;
    preprocess_resized_shape(H_in, W_in, x, &a.Hr, &a.Wr);
    a.cy = (a.Hr - x) / 2;
    a.cx = (a.Wr - x) / 2;
    const bool vec = T % 4 == 0 && ((uintptr_t)out & 3u) == 0;
    const int64_t kMaxGrid = 1LL << 30;
    // enough workgroups for the chip when there are few images, few column-tap computations otherwise
    int strips = (int)std::min<int64_t>((T + 7) / 8, std::max<int64_t>(1, 2048 / N));
    a.rows_per_block = (T + strips - 1) / strips;
    strips = (T + a.rows_per_block - 1) / a.rows_per_block;
    for (int64_t n0 = 0; n0 < N; n0 += kMaxGrid) {
        const int64_t cnt = N - n0 < kMaxGrid ? N - n0 : kMaxGrid;
        const uint8_t *raw0 = raw + n0 * (int64_t)H_in * W_in * 3;
        const int32_t *off0 = off ? off + 2 * n0 : nullptr;
        uint8_t *out0 = out + n0 * 3 * (int64_t)T * T;
        const dim3 grid((unsigned)cnt, (unsigned)strips);
        const bool words = W_in >= 2; // a one-pixel row has no room for a dword
        if (vec && words) hipLaunchKernelGGL((preprocess_kernel<4, true>), grid, dim3(256), 0, s, raw0, a, off0, out0);
        else if (vec) hipLaunchKernelGGL((preprocess_kernel<4, false>), grid, dim3(256), 0, s, raw0, a, off0, out0);
        else if (words) hipLaunchKernelGGL((preprocess_kernel<1, true>), grid, dim3(256), 0, s, raw0, a, off0, out0);
        else hipLaunchKernelGGL((preprocess_kernel<1, false>), grid, dim3(256), 0, s, raw0, a, off0, out0);
    }
    return hipGetLastError();
}

bool select_tiles_supported(int H, int W, int win, int stride)
{
    if (win <= 0 || stride <= 0 || win > H || win > W || win % stride != 0 || win > 512 || stride > 256) return false;
    const int nH = (H - win) / stride + 1, nW = (W - win) / stride + 1, k = win / stride;
    return (int64_t)(nH - 1 + k) * (nW - 1 + k) <= kMaxCells;
}

hipError_t launch_select_tiles_variance(const uint8_t *img, int64_t N, int H, int W, int win, int stride,
                                        const double w[3], int32_t *off_yx, double *scores, hipStream_t s)
{
    if (N <= 0) return hipSuccess;
    SelectArgs a{};
    a.H = H; a.W = W; a.win = win; a.stride = stride;
    a.nH = (H - win) / stride + 1;
    a.nW = (W - win) / stride + 1;
    const int k = win / stride;
    a.nCy = a.nH - 1 + k;
    a.nCx = a.nW - 1 + k;
    for (int c = 0; c < 3; ++c) a.w[c] = w[c];
    // 16-byte loads: chunks must not straddle cells and every row of every image must start 16-byte aligned
    const bool wide = stride % 16 == 0 && W % 16 == 0 && ((uintptr_t)img & 15u) == 0;
    const int64_t kMaxGrid = 1LL << 30;
    for (int64_t n0 = 0; n0 < N; n0 += kMaxGrid) {
        const int64_t cnt = N - n0 < kMaxGrid ? N - n0 : kMaxGrid;
        const uint8_t *img0 = img + n0 * 3 * (int64_t)H * W;
        double *sc0 = scores ? scores + n0 * (int64_t)(a.nH * a.nW) : nullptr;
        if (wide)
            hipLaunchKernelGGL(tile_variance_kernel<16>, dim3((unsigned)cnt), dim3(256), 0, s, img0, a, off_yx + 2 * n0, sc0);
        else
            hipLaunchKernelGGL(tile_variance_kernel<1>, dim3((unsigned)cnt), dim3(256), 0, s, img0, a, off_yx + 2 * n0, sc0);
    }
    return hipGetLastError();
}

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
