// Convolutional bit-extractor H_D (Section 4.1 / 4.3 of the paper) for gfx950.
//
// Every 3x3 convolution is an implicit GEMM on the bf16 matrix cores:
//     D[cout][pixel] += W[cout][k] * X[k][pixel],   k = (tap, cin)
// with v_mfma_f32_32x32x16_bf16: A = a 32(cout) x 16(k) weight fragment, B = a 16(k) x 32(pixel)
// activation fragment, D = 32 x 32 fp32 accumulators.  Activations travel between layers as bf16 NHWC,
// so the 8 consecutive channels a lane feeds to the matrix core are one 16-byte load.
//
//  * Weights are stationary in registers: a wavefront owns 32 output channels and keeps all
//    9 * C/16 of their A fragments (144 VGPRs at C = 64) for the lifetime of a persistent workgroup.
//    The folded batch-norm scale is multiplied into the weights at context creation; bias and ReLU are
//    applied to the accumulators before the single bf16 rounding per layer.
//  * A workgroup (4 wavefronts) stages a strip of (4+2) x (64+2) pixels, halo included, in LDS (pixel
//    stride padded by 16 bytes so that the 16-byte fragment reads are bank-conflict free), zero filling
//    whatever lies outside the tile.  Each fragment read from LDS is used by up to three matrix
//    instructions (the three vertical taps that touch that input row).
//  * Rows of the weight fragments are permuted so that a lane ends up with 16 consecutive output
//    channels of one pixel: the epilogue writes two 16-byte stores per lane.
//  * The first layer reads the u8 image directly (tile crop + normalisation fused: zero padding is
//    applied in the normalised domain and never looks outside the tile), K = 27 padded to 32.
//  * The last layer (C -> n_bits, no ReLU) never writes its output: it is summed over pixels in the
//    accumulators (global average pool), reduced across lanes once per image, and handed to a small
//    kernel that applies the linear layer, thresholds and packs m-bit symbols.
#include "qrm_internal.h"

namespace qrm {

namespace {

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// XCD-aware block order: hardware deals consecutive workgroups round-robin to the 8 XCDs; give each XCD
// a contiguous range of work so that neighbouring strips (which share halo rows) meet in one L2.
__device__ __forceinline__ int xcd_virtual_block(int b, int nblocks)
{
    if (nblocks % 8) return b;
    return (b % 8) * (nblocks / 8) + b / 8;
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x2 __attribute__((ext_vector_type(2)));

// two fp32 -> packed bf16 (round to nearest even) with ReLU applied on the packed pair: a negative bf16
// has its sign bit set, i.e. is negative as a 16-bit integer, so max(.,0) on the halves clamps it.
__device__ __forceinline__ uint32_t pack_bf16_relu(float a, float b, bool relu)
{
    bf16x2 p = {(bf16_t)a, (bf16_t)b};
    s16x2 q = __builtin_bit_cast(s16x2, p);
    if (relu) q = __builtin_elementwise_max(q, (s16x2){0, 0});
    return __builtin_bit_cast(uint32_t, q);
}

// lane (px, half) holds 16 consecutive channels [half*16, half*16+16) of the 32-channel block
__device__ __forceinline__ void store_tile_bf16(bf16_t *dst, const f32x16 &acc, bool relu)
{
    u32x4 lo, hi;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        lo[v] = pack_bf16_relu(acc[2 * v], acc[2 * v + 1], relu);
        hi[v] = pack_bf16_relu(acc[8 + 2 * v], acc[8 + 2 * v + 1], relu);
    }
    *(u32x4 *)dst = lo;
    *(u32x4 *)(dst + 8) = hi;
}

// ------------------------------------------------------------------------------------------------
// conv3x3 C -> C on bf16 NHWC activations.  One strip = kRows x kTileW output pixels.
// ------------------------------------------------------------------------------------------------
template <int C>
struct MidCfg {
    static constexpr int KC = C / 16;                 // 16-channel k chunks per tap
    static constexpr int NCB = C / 32;                // 32-wide output channel blocks
    static constexpr int PS = C * 2 + 16;             // LDS bytes per pixel: C bf16 + one 16-byte pad slot
    static constexpr int SPP = PS / 16;               // 16-byte slots per pixel
    static constexpr int ROW_SLOTS = kHaloW * SPP;    // slots of one staged row (halo columns included)
    static constexpr int PIECES = (ROW_SLOTS + 63) / 64; // wavefront-wide direct-to-LDS loads per row
    static constexpr int ROWB = PIECES * 1024;        // LDS bytes per staged row
    static constexpr int LDS_BYTES = (kRows + 2) * ROWB;
    static constexpr int QPW = (PIECES + 3) / 4;      // pieces of a row one wavefront is responsible for
};

typedef const __attribute__((address_space(1))) void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

// Asynchronous staging of one strip (kRows + 2 rows, halo included) into LDS with direct-to-LDS loads.
// A staged row is cut into PIECES pieces of 64 slots of 16 bytes; one wavefront-wide load fills one
// piece (1 KiB of LDS at row*ROWB + piece*1024), lane l supplying slot piece*64 + l = (column, 8-channel
// chunk).  Wavefront w always handles pieces w, w+4, ..., so the per-lane column decoding is done once
// per strip, not once per load.  Pad slots and pixels outside the tile read from the block of zeros
// that opens the workspace (offset 0 from `ws`): that is the zero padding of the convolution.  All
// sources are addressed as ws + 32-bit byte offset.  The caller waits with s_waitcnt vmcnt(0) and a
// barrier before reading the strip.
template <int C>
__device__ __forceinline__ void issue_strip_loads(uint8_t *lds, const uint8_t *ws, uint32_t img_off, int h, int w,
                                                  int y0, int x0, int wave, int lane)
{
    typedef MidCfg<C> K;
    uint32_t coff[K::QPW]; // byte offset of this lane's slot inside an image row, or ~0u for "zeros"
#pragma unroll
    for (int qi = 0; qi < K::QPW; ++qi) {
        const int slot = (wave + 4 * qi) * 64 + lane;
        const int col = slot / K::SPP, cpos = slot - col * K::SPP;
        const int gx = x0 - 1 + col;
        const bool ok = cpos < C / 8 && col < kHaloW && gx >= 0 && gx < w;
        coff[qi] = ok ? (uint32_t)((gx * C + cpos * 8) * 2) : ~0u;
    }
#pragma unroll
    for (int r = 0; r < kRows + 2; ++r) {
        const int gy = y0 - 1 + r;                                  // same for the whole workgroup
        const bool rowok = gy >= 0 && gy < h;
        const uint32_t rowoff = img_off + (uint32_t)(gy * w * C * 2);
#pragma unroll
        for (int qi = 0; qi < K::QPW; ++qi) {
            const int q = wave + 4 * qi;                            // same for the whole wavefront
            if (q < K::PIECES) {
                const uint32_t off = (rowok && coff[qi] != ~0u) ? rowoff + coff[qi] : 0u;
                __builtin_amdgcn_global_load_lds((gptr_t)(ws + off), (lptr_t)(lds + r * K::ROWB + q * 1024), 16, 0, 0);
            }
        }
    }
}

// Accumulates RW output rows of one 32-pixel x 32-channel block from the staged strip.  Fragments are
// read one (input row, horizontal tap) group ahead of the matrix instructions that consume them; each
// fragment feeds the up to three vertical taps that touch its input row.
// POOL: all rows are summed into acc[0] / acc[1] (global average pool of the last layer); rows at or
// beyond `rows_valid` are skipped (RAGGED: the last strip of a tile whose height is not a multiple of kRows).
template <int C, int RW, bool POOL, bool RAGGED = false>
__device__ __forceinline__ void strip_mma(const uint8_t *lbase, const bf16x8 (&Wr)[9][C / 16], f32x16 *acc,
                                          int rows_valid)
{
    typedef MidCfg<C> K;
    constexpr int NG = (RW + 2) * 3;
    bf16x8 f[2][K::KC];
#pragma unroll
    for (int kc = 0; kc < K::KC; ++kc) f[0][kc] = *(const bf16x8 *)(lbase + kc * 32);
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const int r = g / 3, dx = g % 3;
        if (g + 1 < NG) {
            const int r2 = (g + 1) / 3, dx2 = (g + 1) % 3;
#pragma unroll
            for (int kc = 0; kc < K::KC; ++kc)
                f[(g + 1) & 1][kc] = *(const bf16x8 *)(lbase + r2 * K::ROWB + dx2 * K::PS + kc * 32);
        }
#pragma unroll
        for (int kc = 0; kc < K::KC; ++kc) {
#pragma unroll
            for (int dy = 0; dy < 3; ++dy) {
                const int orow = r - dy;
                if (orow >= 0 && orow < RW) {
                    if (POOL) {
                        if (!RAGGED || orow < rows_valid)
                            acc[orow & 1] = mfma32(Wr[dy * 3 + dx][kc], f[g & 1][kc], acc[orow & 1]);
                    } else {
                        acc[orow] = mfma32(Wr[dy * 3 + dx][kc], f[g & 1][kc], acc[orow]);
                    }
                }
            }
        }
    }
}

template <int C>
__device__ __forceinline__ void load_weight_frags(bf16x8 (&Wr)[9][C / 16], const bf16_t *wfrag, int blk, int lane)
{
    typedef MidCfg<C> K;
    const bf16x8 *wp = (const bf16x8 *)wfrag + (int64_t)blk * 9 * K::KC * 64 + lane;
#pragma unroll
    for (int tap = 0; tap < 9; ++tap)
#pragma unroll
        for (int kc = 0; kc < K::KC; ++kc) Wr[tap][kc] = wp[(tap * K::KC + kc) * 64];
}

// C -> C (+bias, ReLU), bf16 NHWC in / out.  Two workgroups per CU: while one waits for its strip to
// land in LDS the other keeps the matrix cores busy.
template <int C>
__global__ __launch_bounds__(256, 2) void conv_mid_kernel(const uint8_t *__restrict__ ws, uint32_t in_off,
                                                          ConvGeom g, const bf16_t *__restrict__ wfrag,
                                                          const float *__restrict__ bias, bf16_t *__restrict__ out)
{
    typedef MidCfg<C> K;
    constexpr int RG = 2 / K::NCB;     // row groups among the 4 wavefronts
    constexpr int RW = kRows / RG;     // output rows per wavefront
    __shared__ __attribute__((aligned(1024))) uint8_t lds[K::LDS_BYTES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int px = lane & 31, half = lane >> 5;
    const int cb = wave % K::NCB;
    const int xb = (wave / K::NCB) & 1;
    const int rg = wave / (K::NCB * 2);

    bf16x8 Wr[9][K::KC];
    load_weight_frags<C>(Wr, wfrag, cb, lane);
    const float4 *bp = (const float4 *)(bias + cb * 32 + half * 16);

    const int total = g.n_img * g.strips * g.colblks;
    const int nb = gridDim.x;
    const int vb = xcd_virtual_block(blockIdx.x, nb);
    const int per = (total + nb - 1) / nb;
    const int t_begin = vb * per;
    const int t_end = min(total, t_begin + per);
    const uint8_t *lbase = lds + (rg * RW) * K::ROWB + (xb * 32 + px) * K::PS + half * 16;

    auto decode = [&](int t, int &n, int &y0, int &x0) {
        const int colblk = t % g.colblks;
        const int strip = (t / g.colblks) % g.strips;
        n = t / (g.colblks * g.strips);
        y0 = strip * kRows;
        x0 = colblk * kTileW;
    };

    if (t_begin < t_end) {
        int n, y0, x0;
        decode(t_begin, n, y0, x0);
        issue_strip_loads<C>(lds, ws, in_off + (uint32_t)n * (uint32_t)(g.h * g.w * C * 2), g.h, g.w, y0, x0, wave,
                             lane);
    }
    for (int t = t_begin; t < t_end; ++t) {
        int n, y0, x0;
        decode(t, n, y0, x0);

        // accumulators start from the bias (16 consecutive channels per lane)
        f32x16 acc[RW];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 bq = bp[q];
#pragma unroll
            for (int r = 0; r < RW; ++r) {
                acc[r][4 * q] = bq.x; acc[r][4 * q + 1] = bq.y; acc[r][4 * q + 2] = bq.z; acc[r][4 * q + 3] = bq.w;
            }
        }

        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads(); // the strip has landed for every wavefront
        strip_mma<C, RW, false>(lbase, Wr, acc, RW);
        __syncthreads(); // everyone is done reading: the buffer may be refilled
        if (t + 1 < t_end) {
            int n2, y2, x2;
            decode(t + 1, n2, y2, x2);
            issue_strip_loads<C>(lds, ws, in_off + (uint32_t)n2 * (uint32_t)(g.h * g.w * C * 2), g.h, g.w, y2, x2,
                                 wave, lane);
        }

        const int x = x0 + xb * 32 + px;
        const int64_t img_base = (int64_t)n * g.h * g.w;
#pragma unroll
        for (int r = 0; r < RW; ++r) {
            const int y = y0 + rg * RW + r;
            if (y < g.h && x < g.w)
                store_tile_bf16(out + (img_base + (int64_t)y * g.w + x) * C + cb * 32 + half * 16, acc[r], true);
        }
    }
}

// Final conv C -> 64 output channels per grid.y slice, summed over the pixels of one (image, column
// block).  partial[n][colblk*2 + xb][slice*64 + cb*32 + half*16 + v]
template <int C, bool RELU>
__global__ __launch_bounds__(256, 2) void conv_final_kernel(const uint8_t *__restrict__ ws, uint32_t in_off,
                                                            ConvGeom g, int nbp,
                                                            const bf16_t *__restrict__ wfrag,
                                                            const float *__restrict__ bias,
                                                            float *__restrict__ partial)
{
    typedef MidCfg<C> K;
    constexpr int RW = kRows;
    __shared__ __attribute__((aligned(1024))) uint8_t lds[K::LDS_BYTES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int px = lane & 31, half = lane >> 5;
    const int cb = wave & 1, xb = wave >> 1;
    const int slice = blockIdx.y;
    const int cout0 = slice * 64 + cb * 32; // first output channel of this wavefront

    bf16x8 Wr[9][K::KC];
    load_weight_frags<C>(Wr, wfrag, cout0 / 32, lane);
    float bias16[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) bias16[v] = (RELU && bias) ? bias[cout0 + half * 16 + v] : 0.f;

    const int total = g.n_img * g.colblks;
    const int nb = gridDim.x;
    const int vb = xcd_virtual_block(blockIdx.x, nb);
    const int per = (total + nb - 1) / nb;
    const int t_begin = vb * per;
    const int t_end = min(total, t_begin + per);
    const uint8_t *lbase = lds + (xb * 32 + px) * K::PS + half * 16;
    const uint32_t img_bytes = (uint32_t)(g.h * g.w * C * 2);

    for (int t = t_begin; t < t_end; ++t) {
        const int colblk = t % g.colblks;
        const int n = t / g.colblks;
        const int x0 = colblk * kTileW;
        const int x = x0 + xb * 32 + px;

        f32x16 sum[2];
#pragma unroll
        for (int v = 0; v < 16; ++v) { sum[0][v] = 0.f; sum[1][v] = 0.f; }

        __syncthreads();
        issue_strip_loads<C>(lds, ws, in_off + (uint32_t)n * img_bytes, g.h, g.w, 0, x0, wave, lane);
        for (int strip = 0; strip < g.strips; ++strip) {
            const int y0 = strip * kRows;
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (!RELU) {
                if (g.h - y0 >= RW) strip_mma<C, RW, true, false>(lbase, Wr, sum, RW);
                else strip_mma<C, RW, true, true>(lbase, Wr, sum, g.h - y0);
                __syncthreads();
                if (strip + 1 < g.strips)
                    issue_strip_loads<C>(lds, ws, in_off + (uint32_t)n * img_bytes, g.h, g.w, y0 + kRows, x0, wave,
                                         lane);
            } else {
                f32x16 acc[RW];
#pragma unroll
                for (int r = 0; r < RW; ++r)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[r][v] = bias16[v];
                strip_mma<C, RW, false>(lbase, Wr, acc, RW);
                __syncthreads();
                if (strip + 1 < g.strips)
                    issue_strip_loads<C>(lds, ws, in_off + (uint32_t)n * img_bytes, g.h, g.w, y0 + kRows, x0, wave,
                                         lane);
#pragma unroll
                for (int r = 0; r < RW; ++r)
                    if (y0 + r < g.h)
#pragma unroll
                        for (int v = 0; v < 16; ++v) sum[0][v] += fmaxf(acc[r][v], 0.f);
            }
        }

        // mask columns beyond the tile, reduce over the 32 pixel lanes of each half
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            float s = (x < g.w) ? (sum[0][v] + sum[1][v]) : 0.f;
#pragma unroll
            for (int off = 16; off >= 1; off >>= 1) s += __shfl_xor(s, off, 32);
            sum[0][v] = s;
        }
        if (px == 0) {
            float *dst = partial + ((int64_t)n * (g.colblks * 2) + colblk * 2 + xb) * nbp + cout0 + half * 16;
#pragma unroll
            for (int v = 0; v < 16; ++v) dst[v] = sum[0][v];
        }
    }
}

// ------------------------------------------------------------------------------------------------
// First layer: u8 planes -> crop -> normalise -> conv3x3 (3 -> C) + bias + ReLU -> bf16 NHWC.
// One wavefront per (image, row, 32-column block); K = 27 (tap-major, channel-minor) padded to 32.
// ------------------------------------------------------------------------------------------------
template <int C>
__global__ __launch_bounds__(256) void conv_first_kernel(TileSrc src, ConvGeom g, const bf16_t *__restrict__ wfrag,
                                                         const float *__restrict__ bias, bf16_t *__restrict__ out)
{
    constexpr int NCB = C / 32;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int px = lane & 31, half = lane >> 5;

    bf16x8 Wr[NCB][2];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int kc = 0; kc < 2; ++kc) Wr[cb][kc] = ((const bf16x8 *)wfrag)[(cb * 2 + kc) * 64 + lane];

    // per-lane description of its 16 k indices: k = kc*16 + half*8 + e  ->  (tap, channel)
    int koff[16];      // byte offset relative to the centre pixel of plane 0
    int kdy[16], kdx[16];
    float ka[16], kb[16]; // normalised = byte * ka + kb
    const int plane = src.H * src.W;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int kk = (i >> 3) * 16 + half * 8 + (i & 7);
        const bool kvalid = kk < 27;
        const int tap = kvalid ? kk / 3 : 0, c = kvalid ? kk % 3 : 0;
        kdy[i] = kvalid ? tap / 3 - 1 : 1 << 20; // an invalid k never passes the bounds test
        kdx[i] = tap % 3 - 1;
        koff[i] = c * plane + (tap / 3 - 1) * src.W + (tap % 3 - 1);
        const float istd = c == 0 ? src.inv_std[0] : (c == 1 ? src.inv_std[1] : src.inv_std[2]);
        const float mean = c == 0 ? src.mean[0] : (c == 1 ? src.mean[1] : src.mean[2]);
        ka[i] = istd * (1.0f / 255.0f);
        kb[i] = -mean * istd;
    }

    const int cblk32 = (g.w + 31) / 32;
    const int64_t total = (int64_t)g.n_img * g.h * cblk32;
    const int64_t wstride = (int64_t)gridDim.x * 4;
    for (int64_t item = (int64_t)blockIdx.x * 4 + wave; item < total; item += wstride) {
        const int xc = (int)(item % cblk32);
        const int y = (int)((item / cblk32) % g.h);
        const int64_t n = item / ((int64_t)cblk32 * g.h);
        int oy = 0, ox = 0;
        if (src.off) {
            oy = clampi(src.off[2 * n], 0, src.H - g.h);
            ox = clampi(src.off[2 * n + 1], 0, src.W - g.w);
        }
        const int x = xc * 32 + px;
        const uint8_t *centre = src.img + n * 3 * (int64_t)plane + (int64_t)(oy + y) * src.W + ox + x;

        bf16x8 bfrag[2];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int ty = y + kdy[i], tx = x + kdx[i];
            float val = 0.f;
            if (ty >= 0 && ty < g.h && tx >= 0 && tx < g.w) val = fmaf((float)centre[koff[i]], ka[i], kb[i]);
            bfrag[i >> 3][i & 7] = (bf16_t)val;
        }
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            f32x16 acc;
            {
                const float4 *bp = (const float4 *)(bias + cb * 32 + half * 16);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 bq = bp[q];
                    acc[4 * q] = bq.x; acc[4 * q + 1] = bq.y; acc[4 * q + 2] = bq.z; acc[4 * q + 3] = bq.w;
                }
            }
            acc = mfma32(Wr[cb][0], bfrag[0], acc);
            acc = mfma32(Wr[cb][1], bfrag[1], acc);
            if (x < g.w)
                store_tile_bf16(out + ((n * g.h + y) * (int64_t)g.w + x) * C + cb * 32 + half * 16, acc, true);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// pooled -> linear -> logits -> bits -> symbols.  One block of 128 threads per image.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(128) void linear_pack_kernel(const float *__restrict__ partial, int n_part, int nbp,
                                                          int n_bits, float inv_hw, const float *__restrict__ fbias,
                                                          const float *__restrict__ lin_w,
                                                          const float *__restrict__ lin_b, float *__restrict__ logits,
                                                          uint8_t *__restrict__ bits, uint8_t *__restrict__ symbols,
                                                          int m)
{
    __shared__ float pooled[128];
    __shared__ uint8_t sbit[128];
    const int64_t n = blockIdx.x;
    const int o = threadIdx.x;
    if (o < n_bits) {
        float s = 0.f;
        for (int p = 0; p < n_part; ++p) s += partial[(n * n_part + p) * nbp + o];
        pooled[o] = s * inv_hw + (fbias ? fbias[o] : 0.f);
    }
    __syncthreads();
    if (o < n_bits) {
        float z = lin_b ? lin_b[o] : 0.f;
        for (int i = 0; i < n_bits; ++i) z = fmaf(lin_w[o * n_bits + i], pooled[i], z);
        const uint8_t b = z > 0.f ? 1 : 0;
        if (logits) logits[n * n_bits + o] = z;
        if (bits) bits[n * n_bits + o] = b;
        sbit[o] = b;
    }
    __syncthreads();
    if (symbols && o < n_bits / m) {
        int sym = 0;
        for (int u = 0; u < m; ++u) sym |= (int)sbit[o * m + u] << (m - 1 - u);
        symbols[n * (n_bits / m) + o] = (uint8_t)sym;
    }
}

__global__ __launch_bounds__(256) void nhwc_to_nchw_kernel(const bf16_t *__restrict__ in, int64_t total, int hw, int C,
                                                           float *__restrict__ out)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int c = (int)(i % C);
        const int64_t p = i / C; // n*hw + pixel
        const int64_t n = p / hw;
        const int pix = (int)(p % hw);
        out[(n * C + c) * hw + pix] = (float)in[i];
    }
}

int persistent_blocks(int num_cu, int per_cu, int64_t work)
{
    int64_t b = (int64_t)num_cu * per_cu;
    if (b > work) b = work;
    if (b < 1) b = 1;
    return (int)b;
}

} // namespace

hipError_t launch_conv_first(const TileSrc &src, const ConvGeom &g, int C, const bf16_t *wfrag, const float *bias,
                             bf16_t *out, int num_cu, hipStream_t s)
{
    const int64_t items = (int64_t)g.n_img * g.h * ((g.w + 31) / 32);
    const int blocks = persistent_blocks(num_cu, 8, (items + 3) / 4);
    if (C == 64)
        hipLaunchKernelGGL(conv_first_kernel<64>, dim3(blocks), dim3(256), 0, s, src, g, wfrag, bias, out);
    else
        hipLaunchKernelGGL(conv_first_kernel<32>, dim3(blocks), dim3(256), 0, s, src, g, wfrag, bias, out);
    return hipGetLastError();
}

hipError_t launch_conv_mid(const uint8_t *ws, uint32_t in_off, const ConvGeom &g, int C, const bf16_t *wfrag,
                           const float *bias, bf16_t *out, int num_cu, hipStream_t s)
{
    const int64_t tiles = (int64_t)g.n_img * g.strips * g.colblks;
    const int blocks = persistent_blocks(num_cu, 2, tiles);
    if (C == 64)
        hipLaunchKernelGGL(conv_mid_kernel<64>, dim3(blocks), dim3(256), 0, s, ws, in_off, g, wfrag, bias, out);
    else
        hipLaunchKernelGGL(conv_mid_kernel<32>, dim3(blocks), dim3(256), 0, s, ws, in_off, g, wfrag, bias, out);
    return hipGetLastError();
}

hipError_t launch_conv_final(const uint8_t *ws, uint32_t in_off, const ConvGeom &g, int C, int nbp,
                             const bf16_t *wfrag, const float *bias, int relu, float *partial, int num_cu,
                             hipStream_t s)
{
    const int64_t units = (int64_t)g.n_img * g.colblks;
    const int slices = nbp / 64;
    int blocks = persistent_blocks(num_cu, 2, units);
    dim3 grid(blocks, slices);
    if (C == 64) {
        if (relu) hipLaunchKernelGGL((conv_final_kernel<64, true>), grid, dim3(256), 0, s, ws, in_off, g, nbp, wfrag, bias, partial);
        else hipLaunchKernelGGL((conv_final_kernel<64, false>), grid, dim3(256), 0, s, ws, in_off, g, nbp, wfrag, bias, partial);
    } else {
        if (relu) hipLaunchKernelGGL((conv_final_kernel<32, true>), grid, dim3(256), 0, s, ws, in_off, g, nbp, wfrag, bias, partial);
        else hipLaunchKernelGGL((conv_final_kernel<32, false>), grid, dim3(256), 0, s, ws, in_off, g, nbp, wfrag, bias, partial);
    }
    return hipGetLastError();
}

hipError_t launch_linear_pack(const float *partial, int n_part, int nbp, int64_t n_img, int n_bits, float inv_hw,
                              const float *fbias, const float *lin_w, const float *lin_b, float *logits,
                              uint8_t *bits, uint8_t *symbols, int m, hipStream_t s)
{
    if (n_img <= 0) return hipSuccess;
    hipLaunchKernelGGL(linear_pack_kernel, dim3((unsigned)n_img), dim3(128), 0, s, partial, n_part, nbp, n_bits, inv_hw,
                       fbias, lin_w, lin_b, logits, bits, symbols, m);
    return hipGetLastError();
}

hipError_t launch_nhwc_to_nchw(const bf16_t *in, int64_t n_img, int h, int w, int C, float *out, hipStream_t s)
{
    const int64_t total = n_img * h * w * C;
    if (total <= 0) return hipSuccess;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(nhwc_to_nchw_kernel, dim3((unsigned)blocks), dim3(256), 0, s, in, total, h * w, C, out);
    return hipGetLastError();
}

} // namespace qrm
