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
//    applied to the accumulators on the way out, before the single bf16 rounding per layer.
//  * Workgroups are persistent (one per compute unit, eight wavefronts in two groups of four) and stage
//    rows of pixels in LDS rings with direct-to-LDS loads: a pixel takes C * 2 + 16 bytes, so that the
//    16-byte fragment reads are bank-conflict free, and whatever lies outside the tile is loaded from a
//    block of zeros.  Each fragment read from LDS feeds up to three matrix instructions (the three
//    vertical taps that touch that input row).  conv_mid_kernel computes one block per launch (strips of
//    4 rows x 64 columns, the two groups in opposite phases); conv_pair_kernel computes two consecutive
//    blocks per launch and keeps the activations between them in a second LDS ring.
//  * Rows of the weight fragments are permuted so that a lane ends up with 16 consecutive output
//    channels of one pixel: the epilogue writes two 16-byte stores per lane.
//  * The first layer reads the u8 image directly (tile crop + normalisation fused: zero padding is
//    applied in the normalised domain and never looks outside the tile); K = 9 taps x 4 channels (r, g,
//    b, 0) = 36, padded to 48, with the weights as bf16 high part + bf16 residual.
//  * The last block writes no activations when the final convolution has no ReLU: final conv + global
//    average pool are linear, so nine border-aware channel sums per image are all head_kernel needs to
//    apply the final convolution (fp32 weights), the linear layer, the threshold and the symbol packing.
//    With a final ReLU, conv_final_kernel sums the final convolution's output in its accumulators.
#include <type_traits>
#include <utility>

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

// s_waitcnt immediates (gfx9 layout: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14]).  kWaitVm0
// waits for vmcnt(0) only, OR-ing in n <= 15 gives vmcnt(n); kWaitLgkm0 waits for lgkmcnt(0) only.  The
// builtin, unlike an asm statement, is seen by the compiler's own wait-count bookkeeping, which then does
// not add a full drain of its own later.
constexpr int kWaitVm0 = (7 << 4) | (15 << 8);
constexpr int kWaitLgkm0 = 15 | (3 << 14) | (7 << 4);

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding
// global store of the wavefront (a workgroup-scope fence counts direct-to-LDS loads as LDS writes and
// drains the whole vector-memory queue), which would put the write latency of a strip's output on the
// critical path of the next strip.  Callers wait for their direct-to-LDS loads themselves.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0); // own LDS reads / writes are done
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Passes a per-lane value through an empty asm statement: what is derived from the result is recomputed
// where it is used instead of being hoisted and kept in registers across the matrix loop.
__device__ __forceinline__ int pin_in_loop(int v)
{
    asm volatile("" : "+v"(v));
    return v;
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x2 __attribute__((ext_vector_type(2)));

// Activations are rounded to bf16 once per layer.  Round-to-nearest makes the same error wherever the value
// is the same: on a flat or smooth image every pixel of a channel is off in the same direction, and that part
// of the error survives the global average pool (measured: up to 3.4e-2 of a logit on one-colour images,
// against 2e-3 on noise).  The rounding is therefore dithered by position: a pixel adds a fraction u(x, y) of a
// bf16 step to the value's bits and truncates, u in [0, 1) a fixed pseudo-random function of the pixel's place
// in the tile (an integer hash: an ordered pattern would line up with regular image content such as a
// checkerboard).  Single values are off by up to one step instead of half a step; sums over pixels, which is
// all the method looks at, come out unbiased.  Deterministic: the same pixel always gets the same u.
// One hash per group of rows a wavefront finishes together (the group's first row; the only full 32-bit multiply
// is the column's share, the row's share is the same for the whole wavefront and lives on the scalar unit); the
// other rows of the group take the same fraction shifted by a half or by quarters of a step, which spreads the
// fractions of vertically neighbouring pixels evenly.
__device__ __forceinline__ uint32_t dither16(int x, int y)
{
    uint32_t h = (uint32_t)x * 0x9E3779B1u + (uint32_t)y * 0x85EBCA77u;
    h ^= h >> 15;
    h = __umul24(h, 0x00C1B3C5u); // low 24 bits x 24 bits: the product's upper half depends on all of them
    return h >> 16;
}

// two fp32 -> packed bf16, each truncated after `dither` (< 2^16) has been added to its bits, with ReLU
// applied on the packed pair: a negative bf16 has its sign bit set, i.e. is negative as a 16-bit integer, so
// max(.,0) on the halves clamps it.  (Plain instructions: the compiler puts the wait states a matrix result
// needs in front of its own instructions only, never in front of an asm statement.)
__device__ __forceinline__ uint32_t pack_bf16_relu(float a, float b, uint32_t dither, bool relu)
{
    const uint32_t ua = __builtin_bit_cast(uint32_t, a) + dither, ub = __builtin_bit_cast(uint32_t, b) + dither;
    const uint32_t p = __builtin_amdgcn_perm(ub, ua, 0x07060302u); // the high halves: a's below b's
    s16x2 q = __builtin_bit_cast(s16x2, p);
    if (relu) q = __builtin_elementwise_max(q, (s16x2){0, 0});
    return __builtin_bit_cast(uint32_t, q);
}

// lane (px, half) holds 16 consecutive channels [half*16, half*16+16) of the 32-channel block
__device__ __forceinline__ void store_tile_bf16(bf16_t *dst, const f32x16 &acc, uint32_t dither, bool relu)
{
    u32x4 lo, hi;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        lo[v] = pack_bf16_relu(acc[2 * v], acc[2 * v + 1], dither, relu);
        hi[v] = pack_bf16_relu(acc[8 + 2 * v], acc[8 + 2 * v + 1], dither, relu);
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
typedef uint32_t lrow_t; // LDS byte address
__device__ __forceinline__ lrow_t lds_address(const void *p)
{
    return (lrow_t)(uintptr_t)(const __attribute__((address_space(3))) uint8_t *)p;
}

// Asynchronous staging of the rows of one strip (kRows + 2 rows, halo included) into LDS with
// direct-to-LDS loads.  A staged row is cut into PIECES pieces of 64 slots of 16 bytes; one
// wavefront-wide load fills one piece (1 KiB of LDS at slot*ROWB + piece*1024), lane l supplying slot
// piece*64 + l = (column, 8-channel chunk).  Wavefront w (0..3) of the loading group always handles
// pieces w, w+4, ..., so the per-lane column decoding is done once per strip, not once per load.
// Pixels outside the tile must read as zero (zero padding of the convolution): rows above / below the
// tile, halo columns outside it, and the padding slots of a pixel all load from the block of zeros that
// opens the workspace (`ws`).  A pixel is addressed as the image's base `img` + a 32-bit byte offset.
// Window rows first_row..kRows+1 are loaded; window row r goes to row slot (ring_pos + r) mod nslot.
// The caller waits (s_waitcnt vmcnt) and passes a barrier before anyone reads the rows.
constexpr uint32_t kSlotZero = 0xffffffffu; // lane loads zeros

template <int C>
__device__ __forceinline__ void issue_strip_loads(uint8_t *lds, const uint8_t *ws, const uint8_t *img, int h, int w,
                                                  int y0, int x0, int wave, int lane, int first_row = 0,
                                                  int ring_pos = 0, int nslot = kRows + 2)
{
    typedef MidCfg<C> K;
    uint32_t coff[K::QPW]; // byte offset of this lane's slot inside an image row, or the mark
#pragma unroll
    for (int qi = 0; qi < K::QPW; ++qi) {
        const int slot = (wave + 4 * qi) * 64 + lane;
        const int col = slot / K::SPP, cpos = slot - col * K::SPP;
        const int gx = x0 - 1 + col;
        coff[qi] = (cpos < C / 8 && col < kHaloW && gx >= 0 && gx < w) ? (uint32_t)((gx * C + cpos * 8) * 2) : kSlotZero;
    }
#pragma unroll
    for (int r = 0; r < kRows + 2; ++r) {
        if (r < 2 && r < first_row) continue;                       // already in LDS (or known to be zero there)
        const int gy = y0 - 1 + r;                                  // same for the whole workgroup
        const bool rowok = gy >= 0 && gy < h;
        const uint32_t rowoff = (uint32_t)(gy * w * C * 2);
        const int rslot = (ring_pos + r) % nslot;
#pragma unroll
        for (int qi = 0; qi < K::QPW; ++qi) {
            const int q = wave + 4 * qi;                            // same for the whole wavefront
            if (4 * qi + 3 < K::PIECES || q < K::PIECES) {
                const uint8_t *p = (rowok && coff[qi] != kSlotZero) ? img + (rowoff + coff[qi]) : ws;
                __builtin_amdgcn_global_load_lds((gptr_t)p, (lptr_t)(lds + rslot * K::ROWB + q * 1024), 16, 0, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0); // one row's addresses at a time
    }
}

// body(std::integral_constant<int, 0>) ... body(std::integral_constant<int, N - 1>) in this order: a loop whose
// counter is a compile-time constant inside the body (assembly operands with immediate constraints need one)
template <int... I, typename F>
__device__ __forceinline__ void unrolled_impl(std::integer_sequence<int, I...>, F &&body)
{
    (body(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void unrolled(F &&body)
{
    unrolled_impl(std::make_integer_sequence<int, N>{}, body);
}

// One matrix operand (16 bytes per lane) from LDS address `row` + OFFSET, and the wait that says it has landed
// (at most PENDING later LDS operations of the wavefront outstanding).  Assembly, tied to the register: the
// compiler, not knowing which direct-to-LDS load fills which bytes, would otherwise drain the whole
// vector-memory queue (stores included) before the first read.
template <int OFFSET>
__device__ __forceinline__ void frag_read(bf16x8 &dst, lrow_t row)
{
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(row), "n"(OFFSET));
}
template <int PENDING>
__device__ __forceinline__ void frag_wait(bf16x8 &frag)
{
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(frag) : "n"(PENDING));
}

// Accumulates RW output rows of one 32-pixel x 32-channel block from the staged strip.
//
// The RW + 2 staged rows feed 1, 2, 3, .., 3, 2, 1 vertical taps; rows are paired (p, p + (RW+2)/2) so
// that every pair feeds the same number of matrix instructions.  A "set" is the four fragments
// {two rows of a pair} x {two 16-channel k chunks} of one horizontal tap: 8 (RW = 4) matrix
// instructions.  Each fragment register is refilled for set s+1 right after the matrix instructions of
// set s that read it, and the scheduler is fenced so that it keeps that order: every LDS read has the
// matrix instructions of the three other fragments (6 x 32 cycles at RW = 4) to land.  The reads and
// their waits are written as assembly: the compiler, not knowing which direct-to-LDS load fills which
// bytes, would otherwise drain the whole vector-memory queue (stores included) before the first read.
// `rowp` holds the LDS byte address of each staged row for this lane.
// POOL: all rows are summed into acc[0] / acc[1] (global average pool of the last layer); rows at or
// beyond `rows_valid` are skipped (RAGGED: the last strip of a tile whose height is not a multiple of kRows).
// INIT: the accumulators are not read; the first matrix instruction of every output row starts from zero.
template <int C, int RW, bool POOL, bool RAGGED = false, bool INIT = false>
__device__ __forceinline__ void strip_mma(const lrow_t (&rowp)[RW + 2], const bf16x8 (&Wr)[9][C / 16],
                                          f32x16 *acc, int rows_valid)
{
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    bool started[RW] = {};
    typedef MidCfg<C> K;
    constexpr int NP = (RW + 2) / 2;  // row pairs
    constexpr int KP = K::KC / 2;     // pairs of k chunks
    constexpr int NS = 3 * KP * NP;   // sets
    constexpr int NF = 4;                   // fragment registers = reads in flight (6 or 8 measure the same)
    constexpr int NT = 4 * NS;              // fragments, in the order they are used: set by set
    bf16x8 f[NF];
    constexpr auto set_row = [](int s2, int j) { return (s2 % NP) + (j & 1) * NP; };
    constexpr auto set_kc = [](int s2, int j) { return 2 * ((s2 / NP) % KP) + (j >> 1); };
    constexpr auto set_dx = [](int s2) { return s2 / (NP * KP); };
    unrolled<NF>([&](auto tc) {
        constexpr int t = decltype(tc)::value;
        frag_read<set_dx(t / 4) * K::PS + set_kc(t / 4, t % 4) * 32>(f[t], rowp[set_row(t / 4, t % 4)]);
    });
    __builtin_amdgcn_sched_barrier(0);
    unrolled<NT>([&](auto tc) {
        constexpr int t = decltype(tc)::value;
        constexpr int s2 = t / 4, j = t % 4;
        constexpr int dx = set_dx(s2);
        constexpr int r = set_row(s2, j), kc = set_kc(s2, j);
        bf16x8 &fr = f[t % NF];
        // LDS reads return in order: fragment t has landed once at most the NF - 1 reads issued after it
        // (fewer near the end) are outstanding
        frag_wait<(t + NF <= NT ? NF - 1 : NT - 1 - t)>(fr);
#pragma unroll
        for (int dy = 0; dy < 3; ++dy) {
            const int orow = r - dy;
            if (orow >= 0 && orow < RW) {
                if (POOL) {
                    if (!RAGGED || orow < rows_valid) acc[orow & 1] = mfma32(Wr[dy * 3 + dx][kc], fr, acc[orow & 1]);
                } else if (INIT && !started[orow]) {
                    acc[orow] = mfma32(Wr[dy * 3 + dx][kc], fr, zero);
                    started[orow] = true;
                } else {
                    acc[orow] = mfma32(Wr[dy * 3 + dx][kc], fr, acc[orow]);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (t + NF < NT) { // the register is free again: refill it
            constexpr int u = t + NF;
            frag_read<set_dx(u / 4) * K::PS + set_kc(u / 4, u % 4) * 32>(fr, rowp[set_row(u / 4, u % 4)]);
        }
        __builtin_amdgcn_sched_barrier(0);
    });
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

// ---- per-image channel statistics ---------------------------------------------------------------
// Every layer hands the next one per-image channel sums of its (post-ReLU) output.  They serve two
// purposes:
//  (1) weights are bf16 on the matrix cores; the rounding residual W - bf16(W) acts on the mean
//      activation as a constant per output channel, the only part of the rounding error that global
//      average pooling does not wash out.  The consumer adds sum_c rsum[o][c] * mean[c] to its bias
//      (rsum = residual summed over the 9 taps), with mean estimated from every eighth strip.
//  (2) the last conv (C -> n_bits, no ReLU) followed by the global average pool is linear, so it only
//      needs, per channel of the last block's output, the sums over the whole tile, its first / last
//      row, first / last column and four corners (9 numbers): the last block writes no activations.
// A record is written per (image, workgroup that touched it): rec[q*C + c] sums, rec[NQ*C] = pixel count.
// Accumulation order is fixed, so results do not depend on scheduling.
constexpr int kStatPad = 16;
__host__ __device__ constexpr int stat_rec(int C, int nq) { return nq * C + kStatPad; }

// Sum over the 32 pixel lanes of one half-wavefront with DPP lane permutes (no LDS traffic, no waits).
// After the four butterfly steps every lane holds the sum of its row of 16 lanes; the last step adds the
// sum of row 0 (2) into row 1 (3).  The total is valid in lanes with px >= 16 only: kSumLane reads it.
constexpr int kSumLane = 16;
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_f(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float half_sum(float v)
{
    v += dpp_f<0xB1, 0xf>(v);  // quad_perm [1,0,3,2]
    v += dpp_f<0x4E, 0xf>(v);  // quad_perm [2,3,0,1]
    v += dpp_f<0x141, 0xf>(v); // row_half_mirror
    v += dpp_f<0x140, 0xf>(v); // row_mirror
    v += dpp_f<0x142, 0xa>(v); // row_bcast:15 into rows 1 and 3
    return v;
}

// Sums of 16 values per lane over the 32 pixel lanes of one half-wavefront, handed out one value per lane: a
// butterfly that halves the number of values a lane holds while it doubles the number of lanes summed (rows of
// 16 lanes are paired with v_permlane16_swap, then lanes p and 15-p, p and 7-p within 8, p and p^2, p and p^1 with
// DPP moves), 38 instructions instead of 80 for sixteen separate 32-lane sums.  Lane (pxl) ends up with the sum of
// value number reduce16_index(pxl); lanes p and p^1 hold the same one.
__device__ __forceinline__ int reduce16_index(int pxl) { return ((pxl >> 4) & 1) * 8 + ((pxl >> 3) & 1) * 4 + ((pxl >> 2) & 1) * 2 + ((pxl >> 1) & 1); }
__device__ __forceinline__ float reduce16_over_half(const float (&t)[16], int pxl)
{
    float u[8], w[4], x2[2], lo[8], hi[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { lo[j] = t[j]; hi[j] = t[j + 8]; }
    // v_permlane16_swap_b32 a, b: rows 1 and 3 of a <-> rows 0 and 2 of b.  As assembly: this compiler's builtin
    // hands back the first register for both results.  The instruction must not read a register a vector
    // instruction wrote in the two cycles before it, hence the s_nop in front (the compiler, which keeps such
    // distances for its own instructions, does not look into assembly); the operands are sums the compiler's own
    // instructions formed, so the longer distance behind a matrix instruction has been kept by then.
    asm volatile("s_nop 1\n\t"
                 "v_permlane16_swap_b32 %0, %8\n\tv_permlane16_swap_b32 %1, %9\n\t"
                 "v_permlane16_swap_b32 %2, %10\n\tv_permlane16_swap_b32 %3, %11\n\t"
                 "v_permlane16_swap_b32 %4, %12\n\tv_permlane16_swap_b32 %5, %13\n\t"
                 "v_permlane16_swap_b32 %6, %14\n\tv_permlane16_swap_b32 %7, %15\n\t"
                 "s_nop 1"
                 : "+v"(lo[0]), "+v"(lo[1]), "+v"(lo[2]), "+v"(lo[3]), "+v"(lo[4]), "+v"(lo[5]), "+v"(lo[6]), "+v"(lo[7]),
                   "+v"(hi[0]), "+v"(hi[1]), "+v"(hi[2]), "+v"(hi[3]), "+v"(hi[4]), "+v"(hi[5]), "+v"(hi[6]), "+v"(hi[7]));
#pragma unroll
    for (int j = 0; j < 8; ++j) u[j] = lo[j] + hi[j]; // rows 0, 2: value j over both rows; rows 1, 3: value j + 8
    const bool b3 = (pxl & 8) != 0, b2 = (pxl & 4) != 0, b1 = (pxl & 2) != 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) w[j] = (b3 ? u[j + 4] : u[j]) + dpp_f<0x140, 0xf>(b3 ? u[j] : u[j + 4]);      // row_mirror
#pragma unroll
    for (int j = 0; j < 2; ++j) x2[j] = (b2 ? w[j + 2] : w[j]) + dpp_f<0x141, 0xf>(b2 ? w[j] : w[j + 2]);    // row_half_mirror
    float y = (b1 ? x2[1] : x2[0]) + dpp_f<0x4E, 0xf>(b1 ? x2[0] : x2[1]);                                    // quad_perm [2,3,0,1]
    y += dpp_f<0xB1, 0xf>(y);                                                                                   // quad_perm [1,0,3,2]
    return y;
}

// lanes with `pred` add their 16 values into this wavefront's private LDS accumulators
__device__ __forceinline__ void lds_accumulate(float *slot16, const float (&tv)[16], bool pred)
{
    if (pred) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            f32x4 cur = *(f32x4 *)(slot16 + 4 * q);
            cur[0] += tv[4 * q]; cur[1] += tv[4 * q + 1]; cur[2] += tv[4 * q + 2]; cur[3] += tv[4 * q + 3];
            *(f32x4 *)(slot16 + 4 * q) = cur;
        }
    }
}

// Four values of one lane into the wavefront's accumulators with LDS add instructions that return nothing:
// no round trip to wait for (a read-modify-write costs one per call, a dozen per step in the last block).
// Every accumulator has one writer (one lane of one wavefront), LDS executes a wavefront's instructions in
// order, so the sums are formed in program order as before.
__device__ __forceinline__ void lds_accumulate4(float *slot4, const float (&tv)[4], bool pred)
{
    // (written as assembly: the compiler, not knowing which bytes the direct-to-LDS loads in flight fill, would
    // otherwise wait for all of them in front of every one of these updates)
    if (pred) {
        const lrow_t a = lds_address(slot4);
        asm volatile("ds_add_f32 %0, %1\n\tds_add_f32 %0, %2 offset:4\n\tds_add_f32 %0, %3 offset:8\n\tds_add_f32 %0, %4 offset:12"
                     :
                     : "v"(a), "v"(tv[0]), "v"(tv[1]), "v"(tv[2]), "v"(tv[3])
                     : "memory");
    }
}

// Channel sums of the RW output rows (first row yw, column x) held in `acc`, after bias `si` (this lane's
// 16 channels) and ReLU, added to this wavefront's accumulators `my_stat` ([sum index][32 channels] floats,
// already offset to the lane's 16 channels).  LAST = false: sum index 0 only (the whole strip).  LAST = true:
// the nine border-aware sums of the last block: 0 all, 1 / 2 first / last row, 3 / 4 first / last column,
// 5 .. 8 the corners (top-left, top-right, bottom-left, bottom-right).  Four channels at a time: registers
// are scarce next to weights and accumulators.
template <int RW, bool LAST>
__device__ __forceinline__ void strip_statistics(const f32x16 (&acc)[RW], const float *si, float *my_stat, int x, int yw,
                                                 int h, int w, int px)
{
    const bool colok = (uint32_t)x < (uint32_t)w; // (x = -1: the column left of a wide tile's first block)
    const int rl = h - 1 - yw; // image row h-1 relative to this wavefront's rows
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const f32x4 bq = *(const f32x4 *)(si + 4 * q);
        float tv[4] = {0.f, 0.f, 0.f, 0.f}; // sum over this wavefront's valid rows of relu(output)
#pragma unroll
        for (int r = 0; r < RW; ++r)
            if (yw + r < h) {
#pragma unroll
                for (int e = 0; e < 4; ++e) tv[e] += fmaxf(acc[r][4 * q + e] + bq[e], 0.f);
            }
        if (!colok) {
#pragma unroll
            for (int e = 0; e < 4; ++e) tv[e] = 0.f;
        }
        if (LAST) {
            lds_accumulate4(my_stat + 3 * 32 + 4 * q, tv, x == 0);       // first column
            lds_accumulate4(my_stat + 4 * 32 + 4 * q, tv, x == w - 1);   // last column
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) tv[e] = half_sum(tv[e]);
        lds_accumulate4(my_stat + 4 * q, tv, px == kSumLane);            // whole tile (or its sampled strips)
        if (LAST) {
            if (yw == 0) { // image row 0 is this wavefront's first row
                float rv[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) rv[e] = colok ? fmaxf(acc[0][4 * q + e] + bq[e], 0.f) : 0.f;
                lds_accumulate4(my_stat + 5 * 32 + 4 * q, rv, x == 0);
                lds_accumulate4(my_stat + 6 * 32 + 4 * q, rv, x == w - 1);
#pragma unroll
                for (int e = 0; e < 4; ++e) rv[e] = half_sum(rv[e]);
                lds_accumulate4(my_stat + 1 * 32 + 4 * q, rv, px == kSumLane);
            }
            if (rl >= 0 && rl < RW) {
                float rv[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float a = acc[0][4 * q + e];
#pragma unroll
                    for (int r = 1; r < RW; ++r) a = rl == r ? acc[r][4 * q + e] : a;
                    rv[e] = colok ? fmaxf(a + bq[e], 0.f) : 0.f;
                }
                lds_accumulate4(my_stat + 7 * 32 + 4 * q, rv, x == 0);
                lds_accumulate4(my_stat + 8 * 32 + 4 * q, rv, x == w - 1);
#pragma unroll
                for (int e = 0; e < 4; ++e) rv[e] = half_sum(rv[e]);
                lds_accumulate4(my_stat + 2 * 32 + 4 * q, rv, px == kSumLane);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

struct StatArgs {
    const float *tin;   // records of the input's channel sums [n_img][in_slots][stat_rec(C,1)], or nullptr
    int in_slots;
    const float *rsum;  // [c_in][c_out] residual-weight sums of this layer (fp32), or nullptr
    float *tout;        // records written by this launch [n_img][out_slots][stat_rec(C,NQ)], or nullptr
    int out_slots;
    int per;            // tiles per workgroup: divides, or is a multiple of, the tiles of one image
};

constexpr int MODE_MID = 0;  // write activations, sample channel sums from every eighth strip
constexpr int MODE_LAST = 1; // last block: no activations, the nine border-aware channel sums

constexpr int kMidWaves = 8; // wavefronts of a conv_mid workgroup: two groups of four

template <int C, int MODE>
struct MidRing {
    static constexpr int NQ = MODE == MODE_LAST ? 9 : 1;      // sums per channel in a statistics record
    static constexpr int NSLOT = MODE == MODE_LAST ? 14 : 15; // row slots of the LDS ring (>= 12)
    static constexpr int NSUB = kMidWaves / MidCfg<C>::NCB;   // statistics records a workgroup writes per image
};

// C -> C (+bias, ReLU), bf16 NHWC in / out.  One persistent workgroup of eight wavefronts per CU, two
// wavefronts per SIMD.  The workgroup walks down its run of strips; the two groups of four wavefronts
// take alternate strips and work in opposite phases: in phase p group (p & 1) runs the matrix
// instructions of strip p while the other group adds the bias to, converts and stores strip p-1 and
// issues the direct-to-LDS loads of strip p+2.  One workgroup barrier ends a phase.  The matrix cores thus always have one wavefront per SIMD feeding them while the other
// does the vector / memory work, and every load has a whole phase to land before anyone waits for it.
//
// Staged rows live in a ring of NSLOT row slots.  Rows are loaded in the order the run needs them, so
// ring position = number of rows loaded before: strip i of the run loads nr(i) new rows at positions
// base(i).. and reads the six rows from wstart(i):
//   i = 0                      : 6 rows,             wstart = base
//   strip below the previous   : 4 rows (two rows are shared with the strip above), wstart = base - 2
//   first strip of a new image : 5 rows (the row above the tile is zero - and so is the last row the
//                                previous strip loaded, which lay below its tile), wstart = base - 1
template <int C, int MODE>
__global__ __launch_bounds__(64 * kMidWaves, 1) void conv_mid_kernel(const uint8_t *__restrict__ ws, size_t in_off,
                                                                     ConvGeom g, const bf16_t *__restrict__ wfrag,
                                                                     const float *__restrict__ bias, StatArgs st,
                                                                     bf16_t *__restrict__ out)
{
    typedef MidCfg<C> K;
    typedef MidRing<C, MODE> R;
    constexpr int RG = 2 / K::NCB;     // row groups among the 4 wavefronts of a group
    constexpr int RW = kRows / RG;     // output rows per wavefront
    constexpr int NQ = R::NQ, NSLOT = R::NSLOT;
    constexpr int WIN = kRows + 2;     // staged rows one strip reads
    __shared__ __attribute__((aligned(1024))) uint8_t lds[NSLOT * K::ROWB];
    __shared__ __attribute__((aligned(16))) float s_stat[kMidWaves][NQ][32]; // per wavefront, 32 channels of its block
    // bias + rounding-residual correction per image, indexed by image mod 4: it is written two phases
    // before the image's first strip is multiplied and read until one phase after its last, and an
    // image may be a single strip
    __shared__ __attribute__((aligned(16))) float s_init[4][C];
    __shared__ __attribute__((aligned(16))) float s_mean[kMidWaves][C];
    __shared__ float s_cnt[kMidWaves];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 2, w4 = wave & 3;
    const int px = lane & 31, half = lane >> 5;
    const int cb = w4 % K::NCB;
    const int xb = (w4 / K::NCB) & 1;
    const int rg = w4 / (K::NCB * 2);

    bf16x8 Wr[9][K::KC];
    load_weight_frags<C>(Wr, wfrag, cb, lane);

    const int tpi = g.strips * g.colblks; // tiles per image
    const int total = g.n_img * tpi;
    const int vb = xcd_virtual_block(blockIdx.x, gridDim.x);
    const int t_begin = vb * st.per;
    const int ns = min(total, t_begin + st.per) - t_begin; // strips of this workgroup's run
    if (ns <= 0) return;
    const int out_slot = st.per >= tpi ? 0 : (t_begin % tpi) / st.per;
    const lrow_t lbase = lds_address(lds) + (xb * 32 + px) * K::PS + half * 16;
    const size_t img_bytes = (size_t)g.h * g.w * C * 2;

    // ---- geometry of the strips of the run (tile order: image, column block, strip), kept as counters
    // that are advanced once per phase; all wave-uniform
    struct Geo {
        int i;      // index in the run
        int strip;  // strip within its column of the tile
        int colblk; // column block within the image
        int n;      // image
        int base;   // ring position of its first new row
    };
    auto rows_loaded = [&](const Geo &q) { return q.i == 0 ? WIN : (q.strip == 0 ? WIN - 1 : kRows); };
    auto first_row = [&](const Geo &q) { return WIN - rows_loaded(q); }; // first window row that is loaded
    auto wstart = [&](const Geo &q) { return q.base - first_row(q); };
    auto advance = [&](Geo &q) {
        q.base += rows_loaded(q);
        ++q.i;
        if (++q.strip == g.strips) {
            q.strip = 0;
            if (++q.colblk == g.colblks) {
                q.colblk = 0;
                ++q.n;
            }
        }
    };
    Geo gc{0, t_begin % g.strips, (t_begin / g.strips) % g.colblks, t_begin / tpi, 0}; // strip p
    Geo g1 = gc;                                                                          // strip p + 1
    advance(g1);
    Geo g2 = g1;                                                                          // strip p + 2
    advance(g2);
    Geo gp = gc;                                                                          // strip p - 1 (from phase 1 on)

    auto issue = [&](const Geo &q) {
        issue_strip_loads<C>(lds, ws, ws + in_off + (size_t)q.n * img_bytes, g.h, g.w, q.strip * kRows, q.colblk * kTileW, w4,
                             pin_in_loop(lane), first_row(q), wstart(q), NSLOT);
    };
    // s_init[n & 3][o] = bias[o] + sum_c rsum[c][o] * mean_n[c], by the four wavefronts of one group:
    // each takes C/4 outputs, its lanes split the sum over c in 64 / (C/4) parts
    auto prepare_init = [&](int n) {
        constexpr int OPW = C / 4, PARTS = 64 / OPW, CP = C / PARTS;
        const int lane = pin_in_loop(tid & 63);
        const int o = w4 * OPW + lane % OPW, part = lane / OPW;
        float d = 0.f;
        const float *tin = st.tin, *rsum = st.rsum;
        if (tin && rsum) {
            if (lane < C) {
                float sum = 0.f, cnt = 0.f;
                for (int s2 = 0; s2 < st.in_slots; ++s2) {
                    const float *rec = tin + ((int64_t)n * st.in_slots + s2) * stat_rec(C, 1);
                    sum += rec[lane];
                    cnt += rec[C];
                }
                s_mean[wave][lane] = cnt > 0.f ? sum / cnt : 0.f;
            }
#pragma unroll 4
            for (int k = 0; k < CP; ++k) { // (little unrolling: registers are scarce here)
                const int c = part * CP + k;
                d = fmaf(rsum[c * C + o], s_mean[wave][c], d);
            }
#pragma unroll
            for (int sh = OPW; sh < 64; sh <<= 1) d += __shfl_xor(d, sh);
        }
        if (part == 0) s_init[n & 3][o] = bias[o] + d;
    };
    // this wavefront's statistics of image n -> its record; accumulators cleared
    auto flush = [&](int n) {
        if (st.tout) {
            const int lane = pin_in_loop(tid & 63);
            float *rec = st.tout + (((int64_t)n * st.out_slots + out_slot) * R::NSUB + wave / K::NCB) * stat_rec(C, NQ);
            if (lane < 32) {
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    rec[q * C + cb * 32 + lane] = s_stat[wave][q][lane];
                    s_stat[wave][q][lane] = 0.f;
                }
            }
            if (cb == 0 && lane == 0) {
                rec[NQ * C] = s_cnt[wave];
                s_cnt[wave] = 0.f;
            }
        }
    };
    f32x16 acc[RW];
    const int sample_phase = min(3, g.strips - 1); // strips 3, 11, 19, .. are sampled (the last one of a short tile)
    // bias, ReLU, bf16, stores and statistics of strip i (accumulated by this wavefront)
    auto epilogue = [&](const Geo &q) {
        const int lane = pin_in_loop(tid & 63);
        const int px = lane & 31, half = lane >> 5;
        float *my_stat = &s_stat[wave][0][half * 16];
        const int strip = q.strip, n = q.n, x0 = q.colblk * kTileW;
        const int y0 = strip * kRows;
        const int x = x0 + xb * 32 + px;
        const int yw = y0 + rg * RW; // first output row of this wavefront
        // The sums start from zero: bias + correction of the image (s_init, 16 channels per lane) is added
        // on the way out, never in place - the accumulators stay untouched, so that no second copy of them
        // is ever alive next to the weights.
        const float *si = &s_init[n & 3][cb * 32 + half * 16];
        if (MODE == MODE_MID) {
            // the image's activations (same for the whole workgroup) + element offset of this lane's first row
            bf16_t *out_img = out + (size_t)n * g.h * g.w * C;
            const uint32_t dbase = dither16(x, yw);
            const uint32_t e0 = (uint32_t)((yw * g.w + x) * C + cb * 32 + half * 16);
            const bool full = y0 + kRows <= g.h && x0 + kTileW <= g.w; // same for the whole workgroup
#pragma unroll
            for (int hq = 0; hq < 2; ++hq) { // 8 channels = one 16-byte store per row
                const f32x4 b0 = *(const f32x4 *)(si + 8 * hq), b1 = *(const f32x4 *)(si + 8 * hq + 4);
#pragma unroll
                for (int r = 0; r < RW; ++r) {
                    const uint32_t dth = dbase ^ ((uint32_t)r << 14); // the strip's rows: quarter steps apart
                    u32x4 pk;
                    pk[0] = pack_bf16_relu(acc[r][8 * hq + 0] + b0[0], acc[r][8 * hq + 1] + b0[1], dth, true);
                    pk[1] = pack_bf16_relu(acc[r][8 * hq + 2] + b0[2], acc[r][8 * hq + 3] + b0[3], dth, true);
                    pk[2] = pack_bf16_relu(acc[r][8 * hq + 4] + b1[0], acc[r][8 * hq + 5] + b1[1], dth, true);
                    pk[3] = pack_bf16_relu(acc[r][8 * hq + 6] + b1[2], acc[r][8 * hq + 7] + b1[3], dth, true);
                    bf16_t *dst = out_img + (e0 + (uint32_t)(r * g.w * C) + 8 * hq);
                    if (full) *(u32x4 *)dst = pk;
                    else if (yw + r < g.h && x < g.w) *(u32x4 *)dst = pk;
                    __builtin_amdgcn_sched_barrier(0); // one store at a time keeps the temporaries few
                }
            }
        }
        if (st.tout && (MODE == MODE_LAST || (strip & 7) == sample_phase)) {
            strip_statistics<RW, MODE == MODE_LAST>(acc, si, my_stat, x, yw, g.h, g.w, px);
            if (cb == 0 && lane == 0) {
                const int rows = max(0, min(RW, g.h - yw)), cols = max(0, min(32, g.w - (x0 + xb * 32)));
                s_cnt[wave] += (float)(rows * cols);
            }
        }
    };

    // ---- prologue: statistics cleared, corrections of the first image(s), strips 0 and 1 on their way
    if (lane < 32) {
#pragma unroll
        for (int q = 0; q < NQ; ++q) s_stat[wave][q][lane] = 0.f;
    }
    if (lane == 0) s_cnt[wave] = 0.f;
    if (grp == 0) prepare_init(gc.n);
    else if (ns > 1 && g1.n != gc.n) prepare_init(g1.n);
    if (grp == 1) {
        issue(gc);
        if (ns > 1) issue(g1);
    }
    int issued_upto = min(1, ns - 1);
    __builtin_amdgcn_s_waitcnt(kWaitVm0); // weights, and for the loading group strips 0 and 1, are in
    lds_barrier();

    for (int p = 0; p <= ns; ++p) {
        const bool mma_phase = (p & 1) == grp;
        if (mma_phase) {
            if (p < ns) {
                lrow_t rowp[RW + 2];
                const int start = wstart(gc) + rg * RW;
#pragma unroll
                for (int r = 0; r < RW + 2; ++r) rowp[r] = lbase + (uint32_t)((start + r) % NSLOT) * K::ROWB;
                __builtin_amdgcn_s_setprio(3); // the matrix stream goes first whenever both wavefronts of a SIMD are ready
                strip_mma<C, RW, false, false, true>(rowp, Wr, acc, RW);
                __builtin_amdgcn_s_setprio(0);
            }
        } else {
            if (p >= 1) epilogue(gp);
        }
        // Loads: the group that is not multiplying issues strips p + 1 (only if it did not fit earlier) and
        // p + 2, as far as the ring has room (strip p is being read: everything from wstart(p) on is
        // live; strip p + 1 always fits).  Every wavefront keeps the count.
        bool late = false;
        if (issued_upto == p && p + 1 < ns) {
            if (!mma_phase) {
                issue(g1);
                late = true; // this group reads it in the very next phase
            }
            issued_upto = p + 1;
        }
        if (issued_upto == p + 1 && p + 2 < ns && g2.base + rows_loaded(g2) - wstart(gc) <= NSLOT) {
            if (!mma_phase) issue(g2);
            issued_upto = p + 2;
        }
        if (!mma_phase && p + 2 < ns && g2.n != g1.n) prepare_init(g2.n);
        if (p >= 1 && (p == ns || gc.n != gp.n)) flush(gp.n); // strip p - 1 was the last of its image in this run
        // what this group issued a phase ago (or, late, just now) must have landed before the barrier
        if (mma_phase || late) __builtin_amdgcn_s_waitcnt(kWaitVm0);
        lds_barrier();
        gp = gc;
        gc = g1;
        g1 = g2;
        advance(g2);
    }
}

// ------------------------------------------------------------------------------------------------
// Two consecutive C -> C blocks in one kernel (C = 64).
//
// conv_mid is bound by activation traffic as much as by the matrix cores (288 FLOP per byte against a
// machine balance of ~310).  Here the activations between the two blocks never leave the CU: a
// workgroup walks down one image, group A (wavefronts 0-3, weights of the first block) turns input rows
// into rows of the intermediate activation map, which it writes as bf16 into a second LDS ring, and
// group B (wavefronts 4-7, weights of the second block) turns those into output rows.  Global traffic
// per FLOP halves; both wavefronts of a SIMD carry matrix work, so each fills the other's gaps.
//
// Rows are processed two at a time (the two rings of 8 rows of 66 pixels x 144 bytes fill the LDS).  Step s
// of an image of h rows, S = ceil(h/2):
//   A   : s < S: intermediate rows 2s, 2s+1 from input rows 2s-1 .. 2s+2; behind its matrix instructions it
//         waits for the loads it issued a step ago and issues the direct-to-LDS loads of input rows 2s+5, 2s+6
//         (needed in step s+2); then +bias (+correction), ReLU, bf16 -> intermediate ring (zeros outside the
//         tile);  s == S: rows 2S, 2S+1 = zero padding
//   B   : first the epilogue of the rows it accumulated in step s-1 (stores behind which its matrix
//         instructions then run), then output rows 2j, 2j+1, j = s-2, from intermediate rows 2j-1 .. 2j+2
//   end : one workgroup barrier
// (All loads are group A's: the vector-memory instructions of a compute unit issue in order, and loads issued
// by group B at the end of a step would sit in front of its own stores at the start of the next.)
// Row y of either map lives in ring slot (y + 2) mod 8.
// A workgroup's images follow each other without a gap: see the main loop (virtual rows).
// The second block's weights are rounded so that the rounding residuals of the nine taps of every
// (output, input) channel pair cancel (error feedback over the taps): its input never exists as a whole
// image, so there are no channel means to correct its bias with.
//
// WIDE (tiles wider than 64 columns): the rings stay 66 pixels wide and a workgroup walks through its image
// one column block of 64 after the other, left to right, each block top to bottom ("unit" = (image, column
// block); the units of a workgroup form one stream of row pairs as the images do above).  In block b group A
// computes intermediate columns [64 b, 64 b + 64) from input columns [64 b - 1, 64 b + 65), and group B computes
// output columns [64 b - 1, 64 b + 63): one column to the left, so that everything B needs lies at or left of
// A's newest column.  The two intermediate columns left of A's (64 b - 2, 64 b - 1) were computed in block
// b - 1: A writes its last two columns of every row to a small buffer in global memory (the "seam", 256 bytes a
// row, per workgroup, two of them used alternately), from which they come back into ring pixels 0 and 1 a whole
// column block later (for b = 0 those pixels are zero: the padding).  Nothing is computed twice and no
// matrix tile is partly empty.  What is left over is the tile's last column when the width is a multiple of 64:
// the intermediate columns w-2, w-1 of every row go to a per-image seam buffer and conv_seam_kernel, a small
// launch behind this one, computes output column w-1 from them.
// ------------------------------------------------------------------------------------------------
constexpr int kPairRing = 8;
constexpr int kSeamRowBytes = 2 * 64 * 2; // two pixels of 64 bf16 channels: what one row hands over

struct PairArgs {
    const float *tin;   // records of the input's channel sums [n_img][in_slots][stat_rec(C,1)], or nullptr
    int in_slots;
    const float *rsum;  // [c_in][c_out] residual-weight sums of the first block (fp32), or nullptr
    float *tout;        // records of the output's channel sums [n_img][out_slots][stat_rec(C, 1 or 9)], or nullptr
    int out_slots;      // records per image (the first kPairSub of them are written here)
    int ipw;            // images per workgroup
    uint8_t *seam;      // WIDE: [workgroup][2][2 S rows][2 pixels][C] bf16, columns handed to the next column block
    uint8_t *seam_last; // WIDE, width a multiple of 64: [image][2 S rows][2 pixels][C], intermediate columns w-2, w-1
};
constexpr int kPairSub = 2; // statistics records per image: one per pixel-block pair of wavefronts of group B

// FIRST: the first of the two blocks is the network's first block (3 -> C on the raw u8 tile: crop and
//        normalisation fused, weights as bf16 high part + residual, see conv_first_kernel) instead of a
//        C -> C block; `src` replaces ws / in_off, wfragA holds that block's fragments.
// LASTB: the second block is the network's last block: no activations are written, its records carry the
//        nine border-aware channel sums (see strip_statistics).
// WIDE : tiles of more than one column block (see above); the other instantiations keep the straight-line code
//        of the one-block case.
// zeros: kZeroBytes of zeros (the source of the padding); in: the input activations of the launch.
template <int C, bool FIRST, bool LASTB, bool WIDE>
__global__ __launch_bounds__(512, 1) void conv_pair_kernel(const uint8_t *__restrict__ zeros, const uint8_t *__restrict__ in, TileSrc src,
                                                           ConvGeom g, const bf16_t *__restrict__ wfragA,
                                                           const bf16_t *__restrict__ wfragB,
                                                           const float *__restrict__ biasA,
                                                           const float *__restrict__ biasB, PairArgs st,
                                                           bf16_t *__restrict__ out)
{
    typedef MidCfg<C> K;
    static_assert(K::NCB == 2, "the pair kernel is written for 64 channels");
    constexpr int RW = 2;
    constexpr int NQ = LASTB ? 9 : 1;
    constexpr int ROWB = kHaloW * K::PS;          // staged rows are packed: 66 pixels x 144 bytes
    constexpr int SLOTS = ROWB / 16;              // 16-byte slots per row
    constexpr int PIECES = (SLOTS + 63) / 64;     // wavefront-wide loads per row, the last one partial
    __shared__ __attribute__((aligned(1024))) uint8_t ring_in[FIRST ? 1024 : kPairRing * ROWB];
    __shared__ __attribute__((aligned(16))) uint8_t ring_mid[kPairRing * ROWB];
    __shared__ __attribute__((aligned(16))) uint16_t s_pix[FIRST ? kPairRing : 1][kHaloW][4]; // raw pixels as bf16; channel 3 = 1 inside the tile
    __shared__ __attribute__((aligned(16))) float s_initA[C]; // first block: bias (+ rounding-residual correction of the image)
    __shared__ __attribute__((aligned(16))) float s_biasB[C];
    __shared__ __attribute__((aligned(16))) float s_stat[4][NQ][32];
    __shared__ __attribute__((aligned(16))) float s_mean[4][C];
    __shared__ float s_cnt[4];
    // FIRST: group B hands its fp32 accumulators to group A, which has time to spare, for the epilogue:
    // [buffer = row pair parity][wavefront][row * 4 + channel quad][lane] x 4 floats
    __shared__ __attribute__((aligned(16))) float s_accx[FIRST ? 2 * 4 * 8 * 256 : 4];
    constexpr int kFinishGroup = FIRST ? 0 : 1; // the group that finishes output rows (stores, statistics)
    constexpr int kSkew = WIDE ? 1 : 0;         // group B's columns lie this far left of group A's

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 2, w4 = wave & 3;
    const int px = lane & 31, half = lane >> 5;
    const int cb = w4 & 1, xb = w4 >> 1;

    // C -> C weights (group B; group A unless FIRST).  Group A with FIRST keeps the first block's weights in
    // the same registers: Wr[p][k] = high part (p = 0) / residual (p = 1) of 16-wide k chunk k = 0..2.
    bf16x8 Wr[9][K::KC];
    if (FIRST && grp == 0) {
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int k = 0; k < 3; ++k) Wr[p][k] = ((const bf16x8 *)wfragA)[((cb * 2 + p) * 3 + k) * 64 + lane];
    } else {
        load_weight_frags<C>(Wr, grp == 0 ? wfragA : wfragB, cb, lane);
    }

    const int vb = xcd_virtual_block(blockIdx.x, gridDim.x);
    const int n_begin = vb * st.ipw, n_end = min(g.n_img, n_begin + st.ipw);
    if (n_begin >= n_end) return;
    const int S = (g.h + 1) / 2;
    const int J = WIDE ? g.colblks : 1;           // column blocks of a tile
    const size_t img_bytes = (size_t)g.h * g.w * C * 2;
    const uint32_t row_bytes = (uint32_t)(g.w * C * 2);
    const lrow_t in_base = lds_address(ring_in) + (xb * 32 + px) * K::PS + half * 16;
    const lrow_t mid_base = lds_address(ring_mid) + (xb * 32 + px) * K::PS + half * 16;
    const int sample_phase = min(3, g.strips - 1);
    auto slot_of = [](int y) { return (y + 2) & (kPairRing - 1); };

    // Loads of input row y of image n into its ring slot by the four wavefronts of one group: piece q of
    // the row by wavefront q mod 4.  What a lane loads within a row does not change: byte offset of its
    // slot in an image row (kSlotZero: zeros; kSlotNone: no slot - the last piece of a row is partial, the
    // next row starts right behind it).
    constexpr int QPW = (PIECES + 3) / 4;
    // per lane and piece: byte offset of the lane's slot in an image row for column block 0 (negative for the
    // halo column left of the tile), or a mark far below zero: no slot (the last piece of a row is partial, the
    // next row starts right behind it), or one of a pixel's padding slots (always zero)
    constexpr int32_t kSlotNone = INT32_MIN, kSlotPad = INT32_MIN / 2;
    int32_t lane_off[QPW];
#pragma unroll
    for (int k = 0; k < QPW; ++k) {
        const int sl = (w4 + 4 * k) * 64 + lane;
        const int col = sl / K::SPP, cpos = sl - col * K::SPP;
        lane_off[k] = sl >= SLOTS ? kSlotNone : (cpos < C / 8 ? ((col - 1) * C + cpos * 8) * 2 : kSlotPad);
    }
    auto issue_row = [&](int n, int blk, int y, int vrow) { // vrow: the row's place in the stream of units (see the main loop)
        const bool rowok = y >= 0 && y < g.h;
        const uint8_t *rowp = in + (size_t)n * img_bytes + (size_t)(rowok ? y : 0) * row_bytes; // same for the whole workgroup
        const int32_t xoff = blk * (kTileW * C * 2);
        uint8_t *dst = ring_in + slot_of(vrow) * ROWB;
#pragma unroll
        for (int k = 0; k < QPW; ++k) {
            const int q = w4 + 4 * k;
            if (q < PIECES) {
                const int32_t o = lane_off[k] + xoff; // the marks stay far below zero
                const uint8_t *p = (rowok && (uint32_t)o < row_bytes) ? rowp + o : zeros;
                if (lane_off[k] != kSlotNone)
                    __builtin_amdgcn_global_load_lds((gptr_t)p, (lptr_t)(dst + q * 1024), 16, 0, 0);
            }
        }
    };
    // s_initA[o] = biasA[o] + sum_c rsum[c][o] * mean_n[c], by the four wavefronts of group A
    auto prepare_init = [&](int n) {
        constexpr int OPW = C / 4, PARTS = 64 / OPW, CP = C / PARTS;
        const int ln = pin_in_loop(tid & 63);
        const int o = w4 * OPW + ln % OPW, part = ln / OPW;
        float d = 0.f;
        if (st.tin && st.rsum) {
            if (ln < C) {
                float sum = 0.f, cnt = 0.f;
                for (int s2 = 0; s2 < st.in_slots; ++s2) {
                    const float *rec = st.tin + ((int64_t)n * st.in_slots + s2) * stat_rec(C, 1);
                    sum += rec[ln];
                    cnt += rec[C];
                }
                s_mean[w4][ln] = cnt > 0.f ? sum / cnt : 0.f;
            }
#pragma unroll 4
            for (int k = 0; k < CP; ++k) {
                const int c = part * CP + k;
                d = fmaf(st.rsum[c * C + o], s_mean[w4][c], d);
            }
#pragma unroll
            for (int sh = OPW; sh < 64; sh <<= 1) d += __shfl_xor(d, sh);
        }
        if (part == 0) s_initA[o] = biasA[o] + d;
    };
    // FIRST: rows of the raw tile -> normalised bf16 pixels in s_pix, by the 256 threads of group A.
    // Element e of a row pair: row e / 198, channel (e % 198) / 66, staged column (e % 198) % 66.
    constexpr int kRowElems = 3 * kHaloW;
    const int plane = src.H * src.W;
    // The load is unconditional (coordinates clamped into the tile, the value dropped later when it lies
    // outside) and fetches the aligned dword that holds the byte (it never leaves the byte's page): a load under
    // a lane mask, or a byte load with its widening, would be waited for on the spot, and a step would then
    // contain two round trips to memory instead of hiding them behind its matrix work.
    auto pixel_fetch = [&](const uint8_t *tile0, int x0, int y0, int e, bool &inside, uint32_t &shift) -> uint32_t {
        const int ec = min(e, 2 * kRowElems - 1);
        const int row = ec / kRowElems, rem = ec - row * kRowElems;
        const int c = rem / kHaloW, col = rem - c * kHaloW;
        const int ty = y0 + row, tx = x0 + col - 1;
        inside = e < 2 * kRowElems && ty >= 0 && ty < g.h && tx >= 0 && tx < g.w;
        const int tyc = clampi(ty, 0, g.h - 1), txc = clampi(tx, 0, g.w - 1);
        const uintptr_t p = (uintptr_t)(tile0 + ((int64_t)c * plane + (int64_t)tyc * src.W + txc));
        shift = (uint32_t)(p & 3u) * 8u;
        typedef const uint32_t __attribute__((address_space(1))) *global_word_t; // a global load, not a flat one
        return *(global_word_t)(p & ~(uintptr_t)3);
    };
    auto pixel_store = [&](int y0, int e, uint32_t word, uint32_t shift, bool inside) { // y0: place of the first row in the stream of images
        asm volatile("" : "+v"(word)); // the value is first looked at here, not where it was asked for
        if (e < 2 * kRowElems) {
            const int row = e / kRowElems, rem = e - row * kRowElems;
            const int c = rem / kHaloW, col = rem - c * kHaloW;
            // the byte itself, exact as bf16: the normalisation lives in the weights (see conv_first_kernel)
            const float f = inside ? (float)((word >> shift) & 0xffu) : 0.f;
            s_pix[slot_of(y0 + row)][col][c] = __builtin_bit_cast(uint16_t, (bf16_t)f);
            if (c == 0) s_pix[slot_of(y0 + row)][col][3] = inside ? (uint16_t)0x3F80 : (uint16_t)0; // 1 inside the tile
        }
    };

    // ---- once per workgroup: biases, the halo columns of the intermediate ring, statistics
    if (grp == kFinishGroup) {
        if (lane < 32) {
#pragma unroll
            for (int q = 0; q < NQ; ++q) s_stat[w4][q][lane] = 0.f;
        }
        if (lane == 0) s_cnt[w4] = 0.f;
    }
    if (grp == 1) {
        if (tid - 256 < C) s_biasB[tid - 256] = biasB[tid - 256];
    } else if (FIRST) {
        if (tid < C) s_initA[tid] = biasA[tid];
    }
    if (!WIDE) // (WIDE: pixels 0 and 1 are rewritten in every step, 2 .. 65 by group A)
    for (int i = tid; i < kPairRing * 2 * (K::PS / 16); i += 512) { // columns -1 and w.. stay zero for good
        const int row = i / (2 * (K::PS / 16)), rem = i - row * 2 * (K::PS / 16);
        const int side = rem / (K::PS / 16), sl = rem - side * (K::PS / 16);
        *(u32x4 *)(ring_mid + row * ROWB + (side ? (kHaloW - 1) : 0) * K::PS + sl * 16) = (u32x4){0u, 0u, 0u, 0u};
    }

    // The units (image, column block) of a workgroup form one stream of row pairs: unit u takes P = S + 1 steps
    // (S row pairs and the pair of padding rows below the tile, which is also the padding row above the next
    // unit), and virtual row 2 P u + y stands for row y of unit u in both rings.  In step sigma group A is at
    // position sigma of the stream, group B at sigma - 2, the epilogue of B's rows at sigma - 3, the loads at
    // sigma + 2: nothing drains between units.
    struct Pos {
        int i, b, s; // image within the workgroup, column block within the image, step within the unit
    };
    const int P = S + 1;
    const int n_cnt = n_end - n_begin;
    auto pos_of = [P, J](int sigma) {
        const int u = sigma >= 0 ? sigma / P : -((P - 1 - sigma) / P);
        const int i = u >= 0 ? u / J : -((J - 1 - u) / J);
        return Pos{i, u - i * J, sigma - u * P};
    };
    auto advance = [P, J](Pos &p) {
        if (__builtin_expect(++p.s == P, 0)) { // once per unit: kept out of the way of the other steps
            p.s = 0;
            if (++p.b == J) {
                p.b = 0;
                ++p.i;
            }
        }
    };
    auto next_unit = [J](const Pos &p) { return p.b + 1 == J ? Pos{p.i + 1, 0, 0} : Pos{p.i, p.b + 1, 0}; };
    Pos pa = pos_of(0), pb = pos_of(-2), pf = pos_of(-3), pl = pos_of(2), p1 = pos_of(1);
    auto tile_origin = [&](int n) {
        int oy = 0, ox = 0;
        if (src.off) {
            oy = clampi(src.off[2 * n], 0, src.H - g.h);
            ox = clampi(src.off[2 * n + 1], 0, src.W - g.w);
        }
        return src.img + (int64_t)n * 3 * plane + (int64_t)oy * src.W + ox;
    };

    // ---- before the first step: correction of the first image, its input rows -1 .. 4 (FIRST: -1 .. 2),
    //      intermediate row -1 = zero
    const uint8_t *tile0 = nullptr;
    if (FIRST) {
        tile0 = tile_origin(n_begin);
        if (grp == 0) {
#pragma unroll 1
            for (int y0 = -1; y0 <= 1; y0 += 2)
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    bool inside;
                    uint32_t shift;
                    const uint32_t v = pixel_fetch(tile0, 0, y0, tid + 256 * k, inside, shift);
                    pixel_store(y0, tid + 256 * k, v, shift, inside);
                }
        }
    } else {
#pragma unroll 1
        for (int v = -1 + grp; v <= 4; v += 2) { // first, so that they travel while the correction is computed
            const int u = (v + 1) / (2 * P);     // a tile of one or two rows: rows 3, 4 of the stream are the next unit's
            const int i = u / J;
            if (i < n_cnt) issue_row(n_begin + i, u - i * J, v - 2 * P * u, v);
        }
        if (grp == 0) prepare_init(n_begin);
    }
    if (grp == 1)
        for (int i = tid - 256; i < SLOTS; i += 256) *(u32x4 *)(ring_mid + slot_of(-1) * ROWB + i * 16) = (u32x4){0u, 0u, 0u, 0u};
    __builtin_amdgcn_s_waitcnt(kWaitVm0);
    __syncthreads();

    // LASTB: the nine border-aware channel sums of the last block's output (see strip_statistics) from the two
    // rows in `a`.  The sum over the whole tile, the only one every pixel goes into, is kept in a register per
    // lane: the 16 channel values of a lane (both rows added) go through one butterfly over the 32 pixel lanes,
    // after which every lane holds the sum of one channel and adds it to its running total (run_sum; written to
    // the record when the image is done).  First / last column: the one lane that holds it adds its 16 values
    // to the LDS accumulators, in the wavefronts that contain such a column only.  First / last row and the four
    // corners: the same for that row alone, in the (two) steps that contain those rows.
    float run_sum = 0.f;
    auto last_block_statistics = [&](const f32x16 (&a)[RW], const float *si, int x, int x0w, int j, int pxl, int hf) {
        float *stat = &s_stat[w4][0][hf * 16]; // + sum index * 32 + channel
        const bool colok = (uint32_t)x < (uint32_t)g.w;
        const bool allcols = x0w >= 0 && x0w + 32 <= g.w; // same for the whole wavefront
        const bool row1 = 2 * j + 1 < g.h;                // (row 2j always lies in the tile)
        const bool has_first = x0w <= 0 && x0w + 32 > 0, has_last = x0w <= g.w - 1 && g.w - 1 < x0w + 32;
        float bias[16], t[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 bq = *(const f32x4 *)(si + 4 * q);
            bias[4 * q] = bq[0]; bias[4 * q + 1] = bq[1]; bias[4 * q + 2] = bq[2]; bias[4 * q + 3] = bq[3];
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float r1 = fmaxf(a[1][v] + bias[v], 0.f);
            t[v] = fmaxf(a[0][v] + bias[v], 0.f) + (row1 ? r1 : 0.f);
        }
        if (!allcols) {
#pragma unroll
            for (int v = 0; v < 16; ++v) t[v] = colok ? t[v] : 0.f;
        }
        auto column = [&](float *dst, const float (&val)[16], bool pred) { // one lane's 16 values into 16 accumulators
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float four[4] = {val[4 * q], val[4 * q + 1], val[4 * q + 2], val[4 * q + 3]};
                lds_accumulate4(dst + 4 * q, four, pred);
            }
        };
        if (has_first) column(stat + 3 * 32, t, x == 0);
        if (has_last) column(stat + 4 * 32, t, x == g.w - 1);
        run_sum += reduce16_over_half(t, pxl);
        const int rl = g.h - 1 - 2 * j; // the tile's last row, counted from this pair's first
        if (j == 0 || rl < RW) { // the tile's first and / or last row is one of the two
#pragma unroll 1
            for (int which = 0; which < 2; ++which) {
                if (which == 0 ? j != 0 : (rl < 0 || rl >= RW)) continue;
                const bool second = which == 1 && rl == 1;
                float rv[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float av = second ? a[1][v] : a[0][v];
                    rv[v] = colok ? fmaxf(av + bias[v], 0.f) : 0.f;
                }
                const float y = reduce16_over_half(rv, pxl);
                if ((pxl & 1) == 0) { // (an LDS add, as in lds_accumulate4)
                    const lrow_t ad = lds_address(stat + (1 + which) * 32 + reduce16_index(pxl));
                    asm volatile("ds_add_f32 %0, %1" : : "v"(ad), "v"(y) : "memory");
                }
                if (has_first) column(stat + (5 + 2 * which) * 32, rv, x == 0);
                if (has_last) column(stat + (6 + 2 * which) * 32, rv, x == g.w - 1);
            }
        }
    };

    // bias, ReLU, bf16, stores (or nothing: LASTB) and statistics of output rows 2j, 2j+1 of column block blk of
    // image n held in `a`; after the last row pair of an image its channel sums go to its records and the
    // accumulators are cleared
    auto finish = [&](const f32x16 (&a)[RW], int n, int blk, int j) {
        const int ln = pin_in_loop(tid & 63);
        const int pxl = ln & 31, hf = ln >> 5;
        const int x_lo = blk * kTileW - kSkew;     // first of the workgroup's 64 output columns (-1 in block 0 of a wide tile)
        const int x = x_lo + xb * 32 + pxl;
        const float *si = &s_biasB[cb * 32 + hf * 16];
        if (!LASTB) {
            // address = uniform start of the row pair + what the lane adds
            bf16_t *rows = out + ((size_t)n * g.h + 2 * j) * ((size_t)g.w * C);
            const int le = x * C + cb * 32 + hf * 16;
            const int rstride = g.w * C;
            const uint32_t dbase = dither16(x, 2 * j);
            const bool full = 2 * j + RW <= g.h && x_lo >= 0 && x_lo + kTileW <= g.w; // same for the whole workgroup
            if (full) { // the common case: straight-line code, no predicates
#pragma unroll
                for (int hq = 0; hq < 2; ++hq) {
                    const f32x4 b0 = *(const f32x4 *)(si + 8 * hq), b1 = *(const f32x4 *)(si + 8 * hq + 4);
#pragma unroll
                    for (int r = 0; r < RW; ++r) {
                        const uint32_t dth = dbase ^ ((uint32_t)r << 15); // the pair's second row: half a step apart
                        u32x4 pk;
                        pk[0] = pack_bf16_relu(a[r][8 * hq + 0] + b0[0], a[r][8 * hq + 1] + b0[1], dth, true);
                        pk[1] = pack_bf16_relu(a[r][8 * hq + 2] + b0[2], a[r][8 * hq + 3] + b0[3], dth, true);
                        pk[2] = pack_bf16_relu(a[r][8 * hq + 4] + b1[0], a[r][8 * hq + 5] + b1[1], dth, true);
                        pk[3] = pack_bf16_relu(a[r][8 * hq + 6] + b1[2], a[r][8 * hq + 7] + b1[3], dth, true);
                        *(u32x4 *)(rows + (le + r * rstride + 8 * hq)) = pk;
                    }
                }
            } else {
#pragma unroll
                for (int hq = 0; hq < 2; ++hq) {
                    const f32x4 b0 = *(const f32x4 *)(si + 8 * hq), b1 = *(const f32x4 *)(si + 8 * hq + 4);
#pragma unroll
                    for (int r = 0; r < RW; ++r) {
                        const uint32_t dth = dbase ^ ((uint32_t)r << 15); // the pair's second row: half a step apart
                        u32x4 pk;
                        pk[0] = pack_bf16_relu(a[r][8 * hq + 0] + b0[0], a[r][8 * hq + 1] + b0[1], dth, true);
                        pk[1] = pack_bf16_relu(a[r][8 * hq + 2] + b0[2], a[r][8 * hq + 3] + b0[3], dth, true);
                        pk[2] = pack_bf16_relu(a[r][8 * hq + 4] + b1[0], a[r][8 * hq + 5] + b1[1], dth, true);
                        pk[3] = pack_bf16_relu(a[r][8 * hq + 6] + b1[2], a[r][8 * hq + 7] + b1[3], dth, true);
                        if (2 * j + r < g.h && (uint32_t)x < (uint32_t)g.w) *(u32x4 *)(rows + (le + r * rstride + 8 * hq)) = pk;
                    }
                }
            }
        }
        if (LASTB) {
            if (st.tout) last_block_statistics(a, si, x, x_lo + xb * 32, j, pxl, hf);
        } else if (st.tout && ((j >> 1) & 7) == sample_phase) { // (the rows conv_mid would sample)
            strip_statistics<RW, false>(a, si, &s_stat[w4][0][hf * 16], x, 2 * j, g.h, g.w, pxl);
        }
        if (st.tout && (LASTB || ((j >> 1) & 7) == sample_phase)) {
            if (cb == 0 && ln == 0) {
                const int rows = max(0, min(RW, g.h - 2 * j));
                const int cols = max(0, min(x_lo + xb * 32 + 32, g.w) - max(x_lo + xb * 32, 0));
                s_cnt[w4] += (float)(rows * cols);
            }
        }
        if (st.tout && j == S - 1 && blk == J - 1) { // what this wavefront gathered for the image (its own part of s_stat)
            if (LASTB) { // the whole-tile sums lived in a register: one channel per lane
                if ((pxl & 1) == 0) s_stat[w4][0][hf * 16 + reduce16_index(pxl)] = run_sum;
                run_sum = 0.f;
            }
            float *rec = st.tout + ((int64_t)n * st.out_slots + xb) * stat_rec(C, NQ);
            if (ln < 32) {
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    rec[q * C + cb * 32 + ln] = s_stat[w4][q][ln];
                    s_stat[w4][q][ln] = 0.f;
                }
            }
            if (cb == 0 && ln == 0) {
                rec[NQ * C] = s_cnt[w4];
                s_cnt[w4] = 0.f;
            }
        }
    };

    // FIRST, group A: where in the pixel ring this lane's two taps of every k chunk lie (chunk k, half hf: taps
    // 4k + 2hf and 4k + 2hf + 1; beyond 8: zero weights, tap 8 re-read): row offset dy and byte offset of
    // column xl + dx, fixed for the lifetime of the workgroup
    int tap_dy[3][2], tap_col8[3][2];
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int j2 = 0; j2 < 2; ++j2) {
            int tap = 4 * k + 2 * half + j2;
            tap = tap > 8 ? 8 : tap;
            tap_dy[k][j2] = tap / 3;
            tap_col8[k][j2] = (xb * 32 + px + tap % 3) * 8;
        }
    // WIDE, group A: the last two columns (62, 63) of the intermediate rows written in this step, read back from
    // the ring (the wavefront's own writes) and stored to the seam rows at `rows` (null: nothing to hand over).
    // Issued behind the step's wait for global memory, so that the wait never has to sit out these stores.
    auto seam_flush = [&](uint8_t *rows, int sg) {
        if (!rows || xb != 1) return;
        const int ln = pin_in_loop(tid & 63);
        const int pxl = ln & 31, hf = ln >> 5;
        if (pxl >= 30) {
#pragma unroll
            for (int r = 0; r < RW; ++r)
#pragma unroll
                for (int hq = 0; hq < 2; ++hq) {
                    const u32x4 v = *(const u32x4 *)(ring_mid + slot_of(2 * sg + r) * ROWB + (1 + kSkew + 32 + pxl) * K::PS + (cb * 32 + hf * 16 + 8 * hq) * 2);
                    *(u32x4 *)(rows + r * kSeamRowBytes + (pxl - 30) * (C * 2) + (cb * 32 + hf * 16 + 8 * hq) * 2) = v;
                }
        }
    };
    // !FIRST, group A, in the middle of its step (between its matrix work and its epilogue): what the wavefront
    // issued a step ago - the two input rows of the step after this one, the seam columns - is waited for, then the
    // two rows needed two steps from now are put on their way: rows 2s+1, 2s+2 of the unit of step sg + 2, or rows
    // -1, 0 of the unit after it when that step is the one of the padding rows.  Their ring slots were last read in
    // the step before this one.  In the middle of the step, not at its end: the vector-memory instructions of a
    // compute unit queue up behind each other, and group B's stores at the start of the next step - the critical
    // path - would otherwise wait behind these twenty loads.
    auto input_loads = [&](int sg) {
        __builtin_amdgcn_s_waitcnt(kWaitVm0);
        if (pl.i < n_cnt) {
            const bool nxt = pl.s == S;
            const Pos lu = nxt ? next_unit(pl) : pl;
            if (lu.i < n_cnt) {
                issue_row(n_begin + lu.i, lu.b, (nxt ? -1 : 2 * pl.s + 1), 2 * sg + 5);
                issue_row(n_begin + lu.i, lu.b, (nxt ? -1 : 2 * pl.s + 1) + 1, 2 * sg + 6);
            }
        }
    };
    // WIDE: ring pixels 0 and 1 of the intermediate rows group A writes in this step: the two columns left of its
    // block, from the seam of the block before (zeros in block 0 and in the padding rows); 2 x 9 slots per row,
    // straight into LDS.  One wavefront issues them at the start of the step - a wavefront of the group that is
    // not the step's critical path: vector-memory instructions of a compute unit queue up behind each other, and
    // right after the barrier the queue still holds what was issued at the end of the previous step - and waits
    // for them before the step's barrier.
    const size_t seam_half = (size_t)(2 * S) * kSeamRowBytes; // one of a workgroup's two seam buffers
    auto seam_loads = [&](int sg) {
        if (w4 != 0 || pa.i >= n_cnt) return;
        const int ln = pin_in_loop(tid & 63);
        const bool have = pa.b > 0 && pa.s < S;
        const uint8_t *sp = st.seam + ((size_t)blockIdx.x * 2 + ((pa.b & 1) ^ 1)) * seam_half + (size_t)(2 * pa.s) * kSeamRowBytes;
        const int spx = ln / K::SPP, sslot = ln - spx * K::SPP;
#pragma unroll
        for (int r = 0; r < RW; ++r) {
            const uint8_t *p = (have && sslot < C / 8) ? sp + r * kSeamRowBytes + spx * (C * 2) + sslot * 16 : zeros;
            if (ln < 2 * K::SPP)
                __builtin_amdgcn_global_load_lds((gptr_t)p, (lptr_t)(ring_mid + slot_of(2 * sg + r) * ROWB), 16, 0, 0);
        }
    };
    f32x16 acc[RW];
    const int n_steps = n_cnt * J * P + 2;
#pragma unroll 1
    for (int sg = 0; sg < n_steps; ++sg) {
        const bool fin = pf.i >= 0 && pf.i < n_cnt && pf.s < S; // rows accumulated in the previous step wait for their epilogue
        uint8_t *seam_rows_step = nullptr;
        if (grp == 0) {
            const int ln = pin_in_loop(tid & 63);
            const int pxl = ln & 31, hf = ln >> 5;
            const int xl = xb * 32 + pxl;          // this lane's column within the block
            const int x = pa.b * kTileW + xl;      // and within the tile
            uint8_t *seam_rows = nullptr;          // WIDE: where the seam columns of this step's rows go, if anywhere
            if (WIDE && !FIRST) seam_loads(sg);    // (waited for at the end of the step, with this group's other loads)
            // FIRST: the raw pixels of virtual rows 2sg+3, 2sg+4 (window of step sg+1) start their way into registers
            uint32_t pv[2] = {0, 0}, psh[2] = {0, 0};
            bool pin[2] = {false, false};
            bool fetch = false;
            if (FIRST && p1.i < n_cnt) {
                int y0 = 2 * p1.s + 1, fb = p1.b;
                fetch = true;
                if (p1.s == S) { // rows -1, 0 of the next unit
                    const Pos nu = next_unit(p1);
                    fetch = nu.i < n_cnt;
                    y0 = -1;
                    fb = nu.b;
                    if (fetch && nu.b == 0) tile0 = tile_origin(n_begin + nu.i);
                }
                if (fetch) {
#pragma unroll
                    for (int k = 0; k < 2; ++k) pv[k] = pixel_fetch(tile0, fb * kTileW, y0, tid + 256 * k, pin[k], psh[k]);
                }
            }
            if (pa.i < n_cnt && pa.s < S) {
                if (FIRST) {
                    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int r = 0; r < RW; ++r) {
                        const int vy = 2 * sg + r;
                        bf16x8 bfrag[3];
#pragma unroll
                        for (int k = 0; k < 3; ++k) {
                            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                            u32x2 two[2];
#pragma unroll
                            for (int j2 = 0; j2 < 2; ++j2) {
                                const int slot = (vy + 1 + tap_dy[k][j2]) & (kPairRing - 1); // slot_of(vy - 1 + dy)
                                two[j2] = *(const u32x2 *)((const uint8_t *)&s_pix[0][0][0] + slot * (kHaloW * 8) + tap_col8[k][j2]);
                            }
                            const u32x4 both = {two[0][0], two[0][1], two[1][0], two[1][1]};
                            bfrag[k] = __builtin_bit_cast(bf16x8, both);
                        }
                        acc[r] = mfma32(Wr[0][0], bfrag[0], zero);
                        acc[r] = mfma32(Wr[0][1], bfrag[1], acc[r]);
                        acc[r] = mfma32(Wr[0][2], bfrag[2], acc[r]);
#pragma unroll
                        for (int k = 0; k < 3; ++k) acc[r] = mfma32(Wr[1][k], bfrag[k], acc[r]);
                    }
                } else {
                    lrow_t rowp[RW + 2];
#pragma unroll
                    for (int r = 0; r < RW + 2; ++r) rowp[r] = in_base + (uint32_t)slot_of(2 * sg - 1 + r) * ROWB;
                    strip_mma<C, RW, false, false, true>(rowp, Wr, acc, RW);
                    input_loads(sg);
                }
                // epilogue: + bias and correction, ReLU, bf16 -> intermediate ring (zeros outside the tile)
                const float *si = &s_initA[cb * 32 + hf * 16];
                const uint32_t dbase = dither16(x, 2 * pa.s);
                // WIDE: the last two columns of the block also go to the seam (seam_flush below): the workgroup's
                // own (for its next column block) or the image's (the tile's last two columns, for conv_seam_kernel)
                if (WIDE) {
                    if (pa.b + 1 < J) seam_rows = st.seam + ((size_t)blockIdx.x * 2 + (pa.b & 1)) * seam_half;
                    else if (st.seam_last) seam_rows = st.seam_last + (size_t)(n_begin + pa.i) * seam_half;
                    if (seam_rows) seam_rows += (size_t)(2 * pa.s) * kSeamRowBytes;
                }
#pragma unroll
                for (int hq = 0; hq < 2; ++hq) {
                    const f32x4 b0 = *(const f32x4 *)(si + 8 * hq), b1 = *(const f32x4 *)(si + 8 * hq + 4);
#pragma unroll
                    for (int r = 0; r < RW; ++r) {
                        const int y = 2 * pa.s + r;
                        const uint32_t dth = dbase ^ ((uint32_t)r << 15);
                        u32x4 pk;
                        pk[0] = pack_bf16_relu(acc[r][8 * hq + 0] + b0[0], acc[r][8 * hq + 1] + b0[1], dth, true);
                        pk[1] = pack_bf16_relu(acc[r][8 * hq + 2] + b0[2], acc[r][8 * hq + 3] + b0[3], dth, true);
                        pk[2] = pack_bf16_relu(acc[r][8 * hq + 4] + b1[0], acc[r][8 * hq + 5] + b1[1], dth, true);
                        pk[3] = pack_bf16_relu(acc[r][8 * hq + 6] + b1[2], acc[r][8 * hq + 7] + b1[3], dth, true);
                        if (y >= g.h || x >= g.w) pk = (u32x4){0u, 0u, 0u, 0u};
                        *(u32x4 *)(ring_mid + slot_of(2 * sg + r) * ROWB + (1 + kSkew + xl) * K::PS + (cb * 32 + hf * 16 + 8 * hq) * 2) = pk;
                    }
                }
            } else if (pa.i < n_cnt) { // the rows below the tile: zero padding of the second block (and above the next image)
                if (!FIRST) input_loads(sg);
#pragma unroll
                for (int r = 0; r < RW; ++r)
#pragma unroll
                    for (int hq = 0; hq < 2; ++hq)
                        *(u32x4 *)(ring_mid + slot_of(2 * sg + r) * ROWB + (1 + kSkew + xl) * K::PS + (cb * 32 + hf * 16 + 8 * hq) * 2) =
                            (u32x4){0u, 0u, 0u, 0u};
                if (!FIRST && pa.b == J - 1 && pa.i + 1 < n_cnt) prepare_init(n_begin + pa.i + 1); // nobody reads s_initA in this step
            }
            // WIDE: once per step this group waits for all of its global memory traffic, at a point where it has
            // to wait for its loads anyway; the stores of the previous step are then known to be done, among them
            // the seam rows, which are read back a whole unit - at least two steps - after they were written.
            if (FIRST && WIDE) __builtin_amdgcn_s_waitcnt(kWaitVm0);
            if (FIRST && fetch) { // their slots were last read two steps ago; before the stores below, which need not be waited for
#pragma unroll
                for (int k = 0; k < 2; ++k) pixel_store(2 * sg + 3, tid + 256 * k, pv[k], psh[k], pin[k]);
            }
            if (FIRST && WIDE) seam_flush(seam_rows, sg);
            seam_rows_step = seam_rows;
            if (FIRST && fin) { // the rows group B accumulated in the previous step
                const float *srcx = &s_accx[((((sg - 3) & 1) * 4 + w4) * 8) * 256 + ln * 4];
                f32x16 a[RW];
#pragma unroll
                for (int r = 0; r < RW; ++r)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const f32x4 v = *(const f32x4 *)(srcx + (r * 4 + q) * 256);
                        a[r][4 * q] = v[0]; a[r][4 * q + 1] = v[1]; a[r][4 * q + 2] = v[2]; a[r][4 * q + 3] = v[3];
                    }
                finish(a, n_begin + pf.i, pf.b, pf.s);
            }
        } else {
            const int ln = pin_in_loop(tid & 63);
            if (WIDE && FIRST) seam_loads(sg); // (group A is the critical path of this variant)
            if (!FIRST && fin) finish(acc, n_begin + pf.i, pf.b, pf.s); // the rows accumulated in the previous step
            if (pb.i >= 0 && pb.i < n_cnt && pb.s < S) {
                lrow_t rowp[RW + 2];
#pragma unroll
                for (int r = 0; r < RW + 2; ++r) rowp[r] = mid_base + (uint32_t)slot_of(2 * (sg - 2) - 1 + r) * ROWB;
                strip_mma<C, RW, false, false, true>(rowp, Wr, acc, RW);
                if (FIRST) { // group A finishes these rows in the next step
                    float *dst = &s_accx[((((sg - 2) & 1) * 4 + w4) * 8) * 256 + ln * 4];
#pragma unroll
                    for (int r = 0; r < RW; ++r)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            *(f32x4 *)(dst + (r * 4 + q) * 256) = (f32x4){acc[r][4 * q], acc[r][4 * q + 1], acc[r][4 * q + 2], acc[r][4 * q + 3]};
                }
            }
        }
        // End of the step
        if (!FIRST && WIDE && grp == 0) seam_flush(seam_rows_step, sg);
        if (WIDE && FIRST && grp == 1 && w4 == 0) __builtin_amdgcn_s_waitcnt(kWaitVm0); // the seam columns have landed
        lds_barrier();
        advance(pa);
        advance(pb);
        advance(pf);
        advance(pl);
        advance(p1);
    }
}

// The last output column of a fused launch on a tile whose width is a multiple of 64 (see conv_pair_kernel,
// WIDE): out[r][w-1] from the intermediate columns w-2, w-1 that group A left in the per-image seam buffer; the
// column right of them is the zero padding, so only the taps dx = 0, 1 count.  One workgroup of two wavefronts
// (one per 32 output channels) per 32 rows of an image; a lane's pixel is a row.  Operands come straight from
// global memory: the launch is a fraction of a percent of the fused one's work.
// LASTB: instead of activations the column's share of the nine border-aware channel sums, one record per
// workgroup (record rec_first + its index within the image).
template <int C, bool LASTB>
__global__ __launch_bounds__(128) void conv_seam_kernel(const uint8_t *__restrict__ seam_last, ConvGeom g,
                                                        const bf16_t *__restrict__ wfragB, const float *__restrict__ biasB,
                                                        float *__restrict__ tout, int out_slots, int rec_first,
                                                        bf16_t *__restrict__ out)
{
    typedef MidCfg<C> K;
    __shared__ float s_rec[LASTB ? stat_rec(C, 9) : 1];
    const int lane = threadIdx.x & 63;
    const int cb = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int px = lane & 31, half = lane >> 5;
    const int tiles = (g.h + 31) / 32;
    const int n = blockIdx.x / tiles, t = blockIdx.x - n * tiles;
    const int r = t * 32 + px; // this lane's output row
    const uint8_t *sl = seam_last + (size_t)n * (2 * ((g.h + 1) / 2)) * kSeamRowBytes;
    const bf16x8 *wp = (const bf16x8 *)wfragB + (size_t)cb * 9 * K::KC * 64 + lane;
    if (LASTB) {
        for (int i = threadIdx.x; i < stat_rec(C, 9); i += 128) s_rec[i] = 0.f;
        __syncthreads();
    }
    // all operands are asked for before the first is used (unconditional loads from a clamped row; what lies
    // outside the tile is dropped afterwards): the launch is bound by memory latency, not by its 24 matrix instructions
    u32x4 bv[3][2][K::KC];
    bf16x8 av[3][2][K::KC];
#pragma unroll
    for (int dy = 0; dy < 3; ++dy) {
        const int yc = clampi(r + dy - 1, 0, g.h - 1);
#pragma unroll
        for (int dx = 0; dx < 2; ++dx)
#pragma unroll
            for (int kc = 0; kc < K::KC; ++kc) {
                bv[dy][dx][kc] = *(const u32x4 *)(sl + (size_t)yc * kSeamRowBytes + dx * (C * 2) + (kc * 16 + half * 8) * 2);
                av[dy][dx][kc] = wp[((dy * 3 + dx) * K::KC + kc) * 64];
            }
    }
    f32x16 sum = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int dy = 0; dy < 3; ++dy) {
        const int y = r + dy - 1;
        const bool ok = y >= 0 && y < g.h;
#pragma unroll
        for (int dx = 0; dx < 2; ++dx)
#pragma unroll
            for (int kc = 0; kc < K::KC; ++kc) {
                const u32x4 b = ok ? bv[dy][dx][kc] : (u32x4){0u, 0u, 0u, 0u};
                sum = mfma32(av[dy][dx][kc], __builtin_bit_cast(bf16x8, b), sum);
            }
    }
    const float *bp = biasB + cb * 32 + half * 16;
    float val[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) val[v] = sum[v] + bp[v];
    if constexpr (!LASTB) {
        if (r < g.h) {
            bf16_t *dst = out + (((size_t)n * g.h + r) * g.w + (g.w - 1)) * C + cb * 32 + half * 16;
            u32x4 lo, hi;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                lo[v] = pack_bf16_relu(val[2 * v], val[2 * v + 1], dither16(g.w - 1, r), true);
                hi[v] = pack_bf16_relu(val[8 + 2 * v], val[8 + 2 * v + 1], dither16(g.w - 1, r), true);
            }
            *(u32x4 *)dst = lo;
            *(u32x4 *)(dst + 8) = hi;
        }
    } else if (tout) {
        // sums 0 (everything) and 4 (last column): all rows; 1 and 6 (first row, its right corner): row 0;
        // 2 and 8 (last row, its right corner): row h-1.  Every entry has one writer.
        const int ch = cb * 32 + half * 16;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float a = r < g.h ? fmaxf(val[v], 0.f) : 0.f;
            const float tot = half_sum(a);
            if (px == kSumLane) {
                s_rec[0 * C + ch + v] = tot;
                s_rec[4 * C + ch + v] = tot;
            }
            if (r == 0) {
                s_rec[1 * C + ch + v] = a;
                s_rec[6 * C + ch + v] = a;
            }
            if (r == g.h - 1) {
                s_rec[2 * C + ch + v] = a;
                s_rec[8 * C + ch + v] = a;
            }
        }
        if (threadIdx.x == 0) s_rec[9 * C] = (float)max(0, min(32, g.h - t * 32));
        __syncthreads();
        float *rec = tout + ((int64_t)n * out_slots + rec_first + t) * stat_rec(C, 9);
        for (int i = threadIdx.x; i < stat_rec(C, 9); i += 128) rec[i] = s_rec[i];
    }
}

// Final conv C -> 64 output channels per grid.y slice, summed over the pixels of one (image, column
// block).  partial[n][colblk*2 + xb][slice*64 + cb*32 + half*16 + v]
template <int C, bool RELU>
__global__ __launch_bounds__(256, 2) void conv_final_kernel(const uint8_t *__restrict__ ws, size_t in_off,
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
    lrow_t rowp[RW + 2];
#pragma unroll
    for (int r = 0; r < RW + 2; ++r) rowp[r] = lds_address(lds) + r * K::ROWB + (xb * 32 + px) * K::PS + half * 16;
    const size_t img_bytes = (size_t)g.h * g.w * C * 2;

    for (int t = t_begin; t < t_end; ++t) {
        const int colblk = t % g.colblks;
        const int n = t / g.colblks;
        const int x0 = colblk * kTileW;
        const int x = x0 + xb * 32 + px;

        f32x16 sum[2];
#pragma unroll
        for (int v = 0; v < 16; ++v) { sum[0][v] = 0.f; sum[1][v] = 0.f; }

        __syncthreads();
        issue_strip_loads<C>(lds, ws, ws + in_off + (size_t)n * img_bytes, g.h, g.w, 0, x0, wave, lane);
        for (int strip = 0; strip < g.strips; ++strip) {
            const int y0 = strip * kRows;
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (!RELU) {
                if (g.h - y0 >= RW) strip_mma<C, RW, true, false>(rowp, Wr, sum, RW);
                else strip_mma<C, RW, true, true>(rowp, Wr, sum, g.h - y0);
                __syncthreads();
                if (strip + 1 < g.strips)
                    issue_strip_loads<C>(lds, ws, ws + in_off + (size_t)n * img_bytes, g.h, g.w, y0 + kRows, x0, wave, lane);
            } else {
                f32x16 acc[RW];
#pragma unroll
                for (int r = 0; r < RW; ++r)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[r][v] = bias16[v];
                strip_mma<C, RW, false>(rowp, Wr, acc, RW);
                __syncthreads();
                if (strip + 1 < g.strips)
                    issue_strip_loads<C>(lds, ws, ws + in_off + (size_t)n * img_bytes, g.h, g.w, y0 + kRows, x0, wave, lane);
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
// The normalisation is folded into the weights, so that the operands of the matrix cores are exact:
//   sum_c w[c] * (p_c / 255 - mean_c) / std_c  =  sum_c (w[c] / (255 std_c)) * p_c  +  (- sum_c w[c] mean_c / std_c) * 1
// A workgroup stages the (4+2) x (64+2) window of the tile as pixels of 4 bf16 channels (8 bytes) in LDS: the
// three bytes as they are (0..255 are exact in bf16) and a fourth channel that is 1 inside the tile; whatever
// lies outside the tile is four zeros, which is the zero padding of the normalised domain exactly (the
// constant term vanishes with the indicator).  The weights of the four channels are kept as bf16 high part +
// bf16 residual, i.e. to about 16 bits.  K = 9 taps x 4 channels = 36, padded to 48 = three 16-wide k chunks;
// a lane's 8 k values of a chunk are two taps, i.e. two 8-byte LDS reads.  A wavefront computes one 32-channel
// output block for one (C = 32) or two (C = 64) rows of the strip.
// ------------------------------------------------------------------------------------------------
constexpr int kFirstPix = (kRows + 2) * kHaloW;

template <int C>
__global__ __launch_bounds__(256, 4) void conv_first_kernel(TileSrc src, ConvGeom g, const bf16_t *__restrict__ wfrag,
                                                         const float *__restrict__ bias, float *__restrict__ tout,
                                                         int out_slots, int per, bf16_t *__restrict__ out)
{
    constexpr int NCB = C / 32;
    __shared__ __attribute__((aligned(16))) uint16_t lds[kFirstPix * 4];
    __shared__ __attribute__((aligned(16))) float s_stat[4][32]; // per wavefront, the 32 channels of its block
    __shared__ float s_cnt[4];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int px = lane & 31, half = lane >> 5;

    // a wavefront owns one 32-channel output block and NCB of the strip's rows
    const int cb = wave % NCB;
    const int rbase = (wave / NCB) * NCB;
    // weights as bf16 high part + bf16 residual: this layer is tiny, so it is computed to ~16 bits
    bf16x8 Wr[2][3];
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int q = 0; q < 3; ++q) Wr[p][q] = ((const bf16x8 *)wfrag)[((cb * 2 + p) * 3 + q) * 64 + lane];
    f32x16 bias16;
    {
        const float4 *bp = (const float4 *)(bias + cb * 32 + half * 16);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 bq = bp[q];
            bias16[4 * q] = bq.x; bias16[4 * q + 1] = bq.y; bias16[4 * q + 2] = bq.z; bias16[4 * q + 3] = bq.w;
        }
    }

    // LDS byte offsets (relative to the lane's output pixel) of the two taps of each k chunk:
    // chunk q, half h -> taps 4q + 2h and 4q + 2h + 1; taps >= 9 carry zero weights and re-read tap 8.
    int toff[3][2];
#pragma unroll
    for (int q = 0; q < 3; ++q)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            int tap = 4 * q + 2 * half + j;
            tap = tap > 8 ? 8 : tap;
            toff[q][j] = ((tap / 3) * kHaloW + tap % 3) * 8;
        }
    for (int i = tid; i < 4 * 32; i += 256) (&s_stat[0][0])[i] = 0.f;
    if (tid < 4) s_cnt[tid] = 0.f;

    const int plane = src.H * src.W;

    const int tpi = g.strips * g.colblks;
    const int total = g.n_img * tpi;
    const int t_begin = blockIdx.x * per;
    const int t_end = min(total, t_begin + per);
    const int out_slot = per >= tpi ? 0 : (t_begin % tpi) / per;

    auto flush = [&](int n) {
        __syncthreads();
        float *rec = tout + ((int64_t)n * out_slots + out_slot) * stat_rec(C, 1);
        if (tid < C) {
            float v = 0.f;
#pragma unroll
            for (int w2 = 0; w2 < 4; ++w2)
                if (w2 % NCB == tid / 32) v += s_stat[w2][tid & 31];
            rec[tid] = v;
        }
        if (tid == 0) rec[C] = s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
        __syncthreads();
        for (int i = tid; i < 4 * 32; i += 256) (&s_stat[0][0])[i] = 0.f;
        if (tid < 4) s_cnt[tid] = 0.f;
        __syncthreads();
    };

    int cur_n = -1;
    for (int t = t_begin; t < t_end; ++t) {
        const int colblk = t % g.colblks;
        const int strip = (t / g.colblks) % g.strips;
        const int n = t / tpi;
        const int y0 = strip * kRows, x0 = colblk * kTileW;
        if (n != cur_n) {
            if (cur_n >= 0 && tout) flush(cur_n);
            cur_n = n;
        }
        int oy = 0, ox = 0;
        if (src.off) {
            oy = clampi(src.off[2 * n], 0, src.H - g.h);
            ox = clampi(src.off[2 * n + 1], 0, src.W - g.w);
        }
        const uint8_t *tile0 = src.img + (int64_t)n * 3 * plane + (int64_t)oy * src.W + ox;

        __syncthreads(); // previous strip fully consumed
#pragma unroll
        for (int it = 0; it < (kFirstPix * 3 + 255) / 256; ++it) {
            const int idx = tid + it * 256;
            if (idx < kFirstPix * 3) {
                const int c = idx / kFirstPix, p = idx - c * kFirstPix;
                const int row = p / kHaloW, col = p - row * kHaloW;
                const int ty = y0 - 1 + row, tx = x0 - 1 + col;
                const bool inside = ty >= 0 && ty < g.h && tx >= 0 && tx < g.w;
                float v = 0.f;
                if (inside) v = (float)tile0[(int64_t)c * plane + (int64_t)ty * src.W + tx];
                lds[p * 4 + c] = __builtin_bit_cast(uint16_t, (bf16_t)v);
                if (c == 0) lds[p * 4 + 3] = inside ? (uint16_t)0x3F80 : (uint16_t)0;
            }
        }
        __syncthreads();

        const bool sample = tout && (strip & 7) == min(3, g.strips - 1);
#pragma unroll
        for (int rr = 0; rr < NCB; ++rr) {
            const int row = rbase + rr;
            const int y = y0 + row;
            if (y >= g.h) continue; // same for the whole wavefront
#pragma unroll
            for (int xb = 0; xb < 2; ++xb) {
                const int x = x0 + xb * 32 + px;
                const uint8_t *lp = (const uint8_t *)lds + (row * kHaloW + xb * 32 + px) * 8;
                bf16x8 bfrag[3];
#pragma unroll
                for (int q = 0; q < 3; ++q) {
                    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                    const u32x2 lo = *(const u32x2 *)(lp + toff[q][0]);
                    const u32x2 hi = *(const u32x2 *)(lp + toff[q][1]);
                    const u32x4 both = {lo[0], lo[1], hi[0], hi[1]};
                    bfrag[q] = __builtin_bit_cast(bf16x8, both);
                }
                const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                f32x16 sum = mfma32(Wr[0][0], bfrag[0], zero);
                sum = mfma32(Wr[0][1], bfrag[1], sum);
                sum = mfma32(Wr[0][2], bfrag[2], sum);
#pragma unroll
                for (int q = 0; q < 3; ++q) sum = mfma32(Wr[1][q], bfrag[q], sum);
                f32x16 acc;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[v] = sum[v] + bias16[v];
                if (x < g.w)
                    store_tile_bf16(out + (((int64_t)n * g.h + y) * g.w + x) * C + cb * 32 + half * 16, acc, dither16(x, y), true);
                if (sample) {
                    float tv[16];
#pragma unroll
                    for (int v = 0; v < 16; ++v) tv[v] = half_sum(x < g.w ? fmaxf(acc[v], 0.f) : 0.f);
                    lds_accumulate(&s_stat[wave][half * 16], tv, px == kSumLane);
                    if (cb == 0 && lane == 0) s_cnt[wave] += (float)max(0, min(32, g.w - (x0 + xb * 32)));
                }
            }
        }
    }
    if (cur_n >= 0 && tout) flush(cur_n);
}

// ------------------------------------------------------------------------------------------------
// Head for the linear tail: the nine border-aware channel sums of the last block -> final conv + global
// average pool in closed form (fp32 weights) -> linear -> logits -> bits -> symbols.
//   pooled[o] = 1/(h w) * sum_{c,dy,dx} Wf[o][c][dy][dx] * S[c][dy][dx],
//   S[c][dy][dx] = sum of channel c over the input pixels that tap (dy,dx) reaches with zero padding
//                = whole - excluded row - excluded column + their corner
//   (dy = 0 never reaches the last row, dy = 2 never the first; same for dx and columns).
// IPB images per block share every weight read.
// ------------------------------------------------------------------------------------------------
constexpr int kHeadIpb = 1;   // images per block (a launch of a few hundred images should reach every compute unit)
constexpr int kHeadKParts = 8; // the k = (channel, tap) range is cut in eight, one part per 64 threads
constexpr int kHeadThreads = 64 * kHeadKParts;

__global__ __launch_bounds__(kHeadThreads) void head_kernel(const float *__restrict__ recs, int slots, int C, int n_img,
                                                   int n_bits, int nbp, float inv_hw,
                                                   const float *__restrict__ wft /*[C*9][nbp]*/,
                                                   const float *__restrict__ fbias, const float *__restrict__ lin_w,
                                                   const float *__restrict__ lin_b, float *__restrict__ logits,
                                                   uint8_t *__restrict__ bits, uint8_t *__restrict__ symbols, int m)
{
    __shared__ float Q[kHeadIpb][9][64];
    __shared__ float S[kHeadIpb][9 * 64]; // [c*9 + tap]
    __shared__ float part[kHeadKParts][kHeadIpb][128];
    __shared__ float pooled[kHeadIpb][128];
    __shared__ uint8_t sbit[kHeadIpb][128];
    const int tid = threadIdx.x;
    const int64_t n0 = (int64_t)blockIdx.x * kHeadIpb;
    const int rec = stat_rec(C, 9);
    for (int idx = tid; idx < kHeadIpb * 9 * C; idx += kHeadThreads) {
        const int i = idx / (9 * C), r = idx - i * 9 * C; // r = q*C + c
        float v = 0.f;
        if (n0 + i < n_img)
            for (int s2 = 0; s2 < slots; ++s2) v += recs[((n0 + i) * slots + s2) * rec + r];
        Q[i][r / C][r % C] = v;
    }
    __syncthreads();
    for (int idx = tid; idx < kHeadIpb * C; idx += kHeadThreads) {
        const int i = idx / C, c = idx - i * C;
        const float T = Q[i][0][c], R0 = Q[i][1][c], Rl = Q[i][2][c], C0 = Q[i][3][c], Cl = Q[i][4][c];
        const float c00 = Q[i][5][c], c0l = Q[i][6][c], cl0 = Q[i][7][c], cll = Q[i][8][c];
#pragma unroll
        for (int dy = 0; dy < 3; ++dy)
#pragma unroll
            for (int dx = 0; dx < 3; ++dx) {
                const float rex = dy == 0 ? Rl : (dy == 2 ? R0 : 0.f);
                const float cex = dx == 0 ? Cl : (dx == 2 ? C0 : 0.f);
                float corner = 0.f;
                if (dy == 0 && dx == 0) corner = cll;
                if (dy == 0 && dx == 2) corner = cl0;
                if (dy == 2 && dx == 0) corner = c0l;
                if (dy == 2 && dx == 2) corner = c00;
                S[i][c * 9 + dy * 3 + dx] = T - rex - cex + corner;
            }
    }
    __syncthreads();
    // final conv + pool: thread (kp, ol) sums its quarter of k for outputs ol, ol + 64
    {
        const int kp = tid >> 6, ol = tid & 63;
        const int klen = (C * 9) / kHeadKParts, k0 = kp * klen;
        for (int o = ol; o < nbp; o += 64) {
            float acc[kHeadIpb];
#pragma unroll
            for (int i = 0; i < kHeadIpb; ++i) acc[i] = 0.f;
#pragma unroll 8
            for (int k = k0; k < k0 + klen; ++k) {
                const float wv = wft[(int64_t)k * nbp + o];
#pragma unroll
                for (int i = 0; i < kHeadIpb; ++i) acc[i] = fmaf(wv, S[i][k], acc[i]);
            }
#pragma unroll
            for (int i = 0; i < kHeadIpb; ++i) part[kp][i][o] = acc[i];
        }
    }
    __syncthreads();
    for (int idx = tid; idx < kHeadIpb * n_bits; idx += kHeadThreads) {
        const int i = idx / n_bits, o = idx - i * n_bits;
        float v = 0.f;
#pragma unroll
        for (int kp = 0; kp < kHeadKParts; ++kp) v += part[kp][i][o];
        pooled[i][o] = v * inv_hw + (fbias ? fbias[o] : 0.f);
    }
    __syncthreads();
    for (int idx = tid; idx < kHeadIpb * n_bits; idx += kHeadThreads) {
        const int i = idx / n_bits, o = idx - i * n_bits;
        float z = lin_b ? lin_b[o] : 0.f;
        for (int k = 0; k < n_bits; ++k) z = fmaf(lin_w[o * n_bits + k], pooled[i][k], z);
        const uint8_t bt = z > 0.f ? 1 : 0;
        sbit[i][o] = bt;
        if (n0 + i < n_img) {
            if (logits) logits[(n0 + i) * n_bits + o] = z;
            if (bits) bits[(n0 + i) * n_bits + o] = bt;
        }
    }
    __syncthreads();
    if (symbols) {
        const int nsym = n_bits / m;
        for (int idx = tid; idx < kHeadIpb * nsym; idx += kHeadThreads) {
            const int i = idx / nsym, j = idx - i * nsym;
            if (n0 + i < n_img) {
                int sym = 0;
                for (int u = 0; u < m; ++u) sym |= (int)sbit[i][j * m + u] << (m - 1 - u);
                symbols[(n0 + i) * nsym + j] = (uint8_t)sym;
            }
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
                             float *tout, const Partition &part, bf16_t *out, hipStream_t s)
{
    if (C == 64)
        hipLaunchKernelGGL(conv_first_kernel<64>, dim3(part.blocks), dim3(256), 0, s, src, g, wfrag, bias, tout,
                           part.slots, part.per, out);
    else
        hipLaunchKernelGGL(conv_first_kernel<32>, dim3(part.blocks), dim3(256), 0, s, src, g, wfrag, bias, tout,
                           part.slots, part.per, out);
    return hipGetLastError();
}

hipError_t launch_conv_mid(const uint8_t *ws, size_t in_off, const ConvGeom &g, int C, const bf16_t *wfrag,
                           const float *bias, const float *tin, int in_slots, const float *rsum, float *tout,
                           const Partition &part, bool last, bf16_t *out, hipStream_t s)
{
    StatArgs st{tin, in_slots, rsum, tout, part.slots, part.per};
    const dim3 grid(part.blocks), block(64 * kMidWaves);
    if (C == 64) {
        if (last) hipLaunchKernelGGL((conv_mid_kernel<64, MODE_LAST>), grid, block, 0, s, ws, in_off, g, wfrag, bias, st, out);
        else hipLaunchKernelGGL((conv_mid_kernel<64, MODE_MID>), grid, block, 0, s, ws, in_off, g, wfrag, bias, st, out);
    } else {
        if (last) hipLaunchKernelGGL((conv_mid_kernel<32, MODE_LAST>), grid, block, 0, s, ws, in_off, g, wfrag, bias, st, out);
        else hipLaunchKernelGGL((conv_mid_kernel<32, MODE_MID>), grid, block, 0, s, ws, in_off, g, wfrag, bias, st, out);
    }
    return hipGetLastError();
}

bool conv_pair_supported(int C, const ConvGeom &g) { return C == 64 && g.colblks >= 1; }

int conv_pair_records_per_image(const ConvGeom &g, bool last)
{
    const bool seam_column = g.colblks > 1 && g.w % kTileW == 0; // conv_seam_kernel adds records of its own
    return kPairSub + ((last && seam_column) ? (g.h + 31) / 32 : 0);
}

size_t conv_pair_seam_bytes(const ConvGeom &g, int num_cu)
{
    if (g.colblks <= 1) return 0;
    const size_t half = (size_t)(2 * ((g.h + 1) / 2)) * kSeamRowBytes;
    return half * (2 * (size_t)num_cu + (g.w % kTileW == 0 ? (size_t)g.n_img : 0));
}

template <bool FIRST, bool LASTB>
static void launch_pair_variant(bool wide, dim3 grid, hipStream_t s, const uint8_t *zeros, const uint8_t *in, const TileSrc &src,
                                const ConvGeom &g, const bf16_t *wfrag_a, const bf16_t *wfrag_b, const float *bias_a,
                                const float *bias_b, const PairArgs &st, bf16_t *out)
{
    if (wide) hipLaunchKernelGGL((conv_pair_kernel<64, FIRST, LASTB, true>), grid, dim3(512), 0, s, zeros, in, src, g, wfrag_a, wfrag_b, bias_a, bias_b, st, out);
    else hipLaunchKernelGGL((conv_pair_kernel<64, FIRST, LASTB, false>), grid, dim3(512), 0, s, zeros, in, src, g, wfrag_a, wfrag_b, bias_a, bias_b, st, out);
}

hipError_t launch_conv_pair(const uint8_t *zeros, const uint8_t *in, const TileSrc *first, const ConvGeom &g, int C,
                            const bf16_t *wfrag_a, const bf16_t *wfrag_b, const float *bias_a, const float *bias_b,
                            const float *tin, int in_slots, const float *rsum_a, float *tout, bool last, int num_cu,
                            uint8_t *seam, bf16_t *out, hipStream_t s)
{
    if (!conv_pair_supported(C, g)) return hipErrorInvalidValue;
    const bool wide = g.colblks > 1;
    const bool seam_column = wide && g.w % kTileW == 0;
    if (wide && !seam) return hipErrorInvalidValue;
    const int ipw = (g.n_img + num_cu - 1) / num_cu;
    const dim3 grid((g.n_img + ipw - 1) / ipw);
    if ((int)grid.x > num_cu) return hipErrorInvalidValue; // the seam buffer holds num_cu workgroups
    const size_t half = (size_t)(2 * ((g.h + 1) / 2)) * kSeamRowBytes;
    uint8_t *seam_last = seam_column ? seam + 2 * (size_t)num_cu * half : nullptr;
    const int out_slots = conv_pair_records_per_image(g, last);
    PairArgs st{tin, in_slots, rsum_a, tout, out_slots, ipw, seam, seam_last};
    const TileSrc src = first ? *first : TileSrc{};
    if (first) {
        if (last) launch_pair_variant<true, true>(wide, grid, s, zeros, in, src, g, wfrag_a, wfrag_b, bias_a, bias_b, st, out);
        else launch_pair_variant<true, false>(wide, grid, s, zeros, in, src, g, wfrag_a, wfrag_b, bias_a, bias_b, st, out);
    } else {
        if (last) launch_pair_variant<false, true>(wide, grid, s, zeros, in, src, g, wfrag_a, wfrag_b, bias_a, bias_b, st, out);
        else launch_pair_variant<false, false>(wide, grid, s, zeros, in, src, g, wfrag_a, wfrag_b, bias_a, bias_b, st, out);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !seam_column) return e;
    const dim3 sgrid((unsigned)g.n_img * (unsigned)((g.h + 31) / 32));
    if (last) hipLaunchKernelGGL((conv_seam_kernel<64, true>), sgrid, dim3(128), 0, s, seam_last, g, wfrag_b, bias_b, tout, out_slots, kPairSub, out);
    else hipLaunchKernelGGL((conv_seam_kernel<64, false>), sgrid, dim3(128), 0, s, seam_last, g, wfrag_b, bias_b, tout, out_slots, kPairSub, out);
    return hipGetLastError();
}

hipError_t launch_head(const float *recs, int slots, int C, int64_t n_img, int n_bits, int nbp, float inv_hw,
                       const float *wft, const float *fbias, const float *lin_w, const float *lin_b, float *logits,
                       uint8_t *bits, uint8_t *symbols, int m, hipStream_t s)
{
    if (n_img <= 0) return hipSuccess;
    const unsigned blocks = (unsigned)((n_img + kHeadIpb - 1) / kHeadIpb);
    hipLaunchKernelGGL(head_kernel, dim3(blocks), dim3(kHeadThreads), 0, s, recs, slots, C, (int)n_img, n_bits, nbp, inv_hw, wft,
                       fbias, lin_w, lin_b, logits, bits, symbols, m);
    return hipGetLastError();
}

// Tiles are dealt to workgroups in contiguous runs of `per`; `per` divides the tiles of one image or is
// a multiple of them, so a workgroup never holds two partial images and an image is touched by exactly
// `slots` workgroups.
Partition make_partition(int64_t n_img, int tiles_per_image, int target_blocks, int sub)
{
    Partition p{};
    p.sub = sub;
    const int64_t total = n_img * tiles_per_image;
    int64_t want = (total + target_blocks - 1) / target_blocks;
    if (want < 1) want = 1;
    if (want >= tiles_per_image) {
        p.per = (int)((want + tiles_per_image - 1) / tiles_per_image) * tiles_per_image;
        p.slots = 1;
    } else {
        int d = (int)want;
        while (tiles_per_image % d) ++d;
        p.per = d;
        p.slots = tiles_per_image / d;
    }
    p.blocks = (int)((total + p.per - 1) / p.per);
    return p;
}

size_t stat_record_floats(int C, int nq) { return (size_t)stat_rec(C, nq); }

int conv_mid_records_per_workgroup(int C) { return kMidWaves / (C / 32); }

hipError_t launch_conv_final(const uint8_t *ws, size_t in_off, const ConvGeom &g, int C, int nbp,
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
