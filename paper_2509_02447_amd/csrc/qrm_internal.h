// Internal declarations shared by the HIP sources of libqrm (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/qrm.h"

namespace qrm {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kRows = 4;     // output rows per strip of the conv kernels
constexpr int kTileW = 64;   // output columns per strip
constexpr int kHaloW = kTileW + 2;
constexpr int kMaxPart = 64; // upper bound on pooled partial sums per image handled by the linear kernel

// Geometry of one extractor pass over a micro-batch.
struct ConvGeom {
    int n_img;      // images in this launch
    int h, w;       // tile height / width (conv domain)
    int strips;     // ceil(h / kRows)
    int colblks;    // ceil(w / kTileW)
};

// Source of the first convolution: raw u8 planes of the whole image plus tile origin.
struct TileSrc {
    const uint8_t *img; // [N,3,H,W]
    const int32_t *off; // [N,2] (y,x) or nullptr
    int H, W;
    float mean[3], inv_std[3];
};

// ---- launchers (each enqueues on `s`, returns hipGetLastError()) ----------

hipError_t launch_extract_tiles(const uint8_t *img, int64_t N, int H, int W, const int32_t *off, int tile,
                                uint8_t *out, hipStream_t s);

// How the tiles of a launch are dealt to workgroups (see make_partition).
struct Partition {
    int per;    // tiles per workgroup
    int slots;  // workgroups that touch one image
    int sub;    // statistics records a workgroup writes per image; records per image = slots * sub
    int blocks; // grid size
};
Partition make_partition(int64_t n_img, int tiles_per_image, int target_blocks, int sub = 1);
int conv_mid_records_per_workgroup(int C);
size_t stat_record_floats(int C, int nq); // floats per statistics record holding nq sums per channel

// conv1: crop + normalise + conv3x3 (3 -> C, bf16 high + residual weights) + bias + ReLU -> bf16 NHWC;
// tout (optional): sampled channel sums of the output, [n_img][part.slots][stat_record_floats(C,1)]
hipError_t launch_conv_first(const TileSrc &src, const ConvGeom &g, int C, const bf16_t *wfrag, const float *bias,
                             float *tout, const Partition &part, bf16_t *out, hipStream_t s);

// conv3x3 C -> C + bias + ReLU, bf16 NHWC in/out.  The input is addressed as ws + in_off + image * its bytes
// (+ 32-bit offsets inside an image); the first kZeroBytes of ws must be zero: the source of the zero padding.
// tin / in_slots / rsum: channel sums of the input (in_slots records per image) and the summed weight-rounding
// residual [c_in][c_out] used
// to correct the bias (either may be null).  tout: statistics of the output.  last: no activations are
// written, tout receives the nine border-aware sums per channel (stat_record_floats(C,9) per record).
constexpr size_t kZeroBytes = 256;
hipError_t launch_conv_mid(const uint8_t *ws, size_t in_off, const ConvGeom &g, int C, const bf16_t *wfrag,
                           const float *bias, const float *tin, int in_slots, const float *rsum, float *tout,
                           const Partition &part, bool last, bf16_t *out, hipStream_t s);

// Two consecutive blocks in one launch, the activations between them staying in LDS (C = 64:
// conv_pair_supported; tiles wider than 64 columns are walked through in column blocks and need `seam`,
// conv_pair_seam_bytes() bytes of scratch).  zeros: kZeroBytes of zeros; in: the input activations.
// first != nullptr: the first of the two is the network's first block (raw u8 tiles, wfrag_a / bias_a of that
// block; in / tin / rsum_a unused); otherwise both are C -> C blocks and tin / in_slots / rsum_a are as for
// launch_conv_mid (first block only: the second block's weights are rounded so that it needs no correction).
// last: the second block is the network's last one (no activations written, nine sums per channel in the
// records).  tout: channel sums of the output, conv_pair_records_per_image() records per image.
bool conv_pair_supported(int C, const ConvGeom &g);
int conv_pair_records_per_image(const ConvGeom &g, bool last);
size_t conv_pair_seam_bytes(const ConvGeom &g, int num_cu);
hipError_t launch_conv_pair(const uint8_t *zeros, const uint8_t *in, const TileSrc *first, const ConvGeom &g, int C,
                            const bf16_t *wfrag_a, const bf16_t *wfrag_b, const float *bias_a, const float *bias_b,
                            const float *tin, int in_slots, const float *rsum_a, float *tout, bool last, int num_cu,
                            uint8_t *seam, bf16_t *out, hipStream_t s);

// nine channel sums of the last block -> final conv + average pool in closed form -> linear -> logits,
// bits, symbols.  wft: final conv weights fp32, [C*9][nbp] (k = c*9 + tap major)
hipError_t launch_head(const float *recs, int slots, int C, int64_t n_img, int n_bits, int nbp, float inv_hw,
                       const float *wft, const float *fbias, const float *lin_w, const float *lin_b, float *logits,
                       uint8_t *bits, uint8_t *symbols, int m, hipStream_t s);

// final conv3x3 C -> nbp (n_bits padded to 32s) (+bias, optional ReLU) + sum over pixels -> partial sums
// partial: f32 [n_img][colblks*2][nbp]
hipError_t launch_conv_final(const uint8_t *ws, size_t in_off, const ConvGeom &g, int C, int nbp,
                             const bf16_t *wfrag, const float *bias, int relu, float *partial, int num_cu,
                             hipStream_t s);

// pooled = sum(partials)/(h*w); logits = lin_w * pooled + lin_b; bits; symbols (MSB first, m bits each)
// fbias: optional bias of the final convolution, added to the pooled value
hipError_t launch_linear_pack(const float *partial, int n_part, int nbp, int64_t n_img, int n_bits, float inv_hw,
                              const float *fbias, const float *lin_w, const float *lin_b, float *logits, uint8_t *bits,
                              uint8_t *symbols, int m, hipStream_t s);

// bf16 NHWC -> f32 NCHW (diagnostic)
hipError_t launch_nhwc_to_nchw(const bf16_t *in, int64_t n_img, int h, int w, int C, float *out, hipStream_t s);

struct RsParams {
    int m, q, n, k, two_t, fcr;
    const uint8_t *exp2; // device, [2*(q-1)] alpha^i
    const uint8_t *log;  // device, [q], log[0] unused
};

// Key verification: `key` device [k] symbols; matches null = no verification.
struct KeyArgs {
    const uint8_t *key = nullptr;
    int tau = 0;
    int32_t *matches = nullptr; // [N] number of message bits equal to the key's
    uint8_t *detected = nullptr; // [N] matches >= tau, or null
};

hipError_t launch_rs_decode(const RsParams &p, const uint8_t *sym, int64_t N, uint8_t *msg, uint8_t *cw, int8_t *nerr,
                            const KeyArgs &key, hipStream_t s);
// matches / detected for messages already in memory (msg device [N,k])
hipError_t launch_verify(const RsParams &p, const uint8_t *msg, int64_t N, const KeyArgs &key, hipStream_t s);

// Variance-based tile selection: origin of the first window with the largest weighted sum of channel variances.
// off_yx device [N,2]; scores device [N, nH*nW] or null; w: channel weights.
bool select_tiles_supported(int H, int W, int win, int stride);
hipError_t launch_select_tiles_variance(const uint8_t *img, int64_t N, int H, int W, int win, int stride,
                                        const double w[3], int32_t *off_yx, double *scores, hipStream_t s);

// Fused pre-processing: raw u8 [N,H_in,W_in,3] -> resize (shorter side x) -> centre crop x -> planar u8
// [N,3,T,T], the whole crop (T = x) or a tile of it at off (device [N,2] or null).
bool preprocess_supported(int H_in, int W_in, int x, int T);
hipError_t launch_preprocess(const uint8_t *raw, int64_t N, int H_in, int W_in, int x, const int32_t *off, int T,
                             uint8_t *out, hipStream_t s);

// host-side helpers
uint16_t f32_to_bf16_rne(float f);

} // namespace qrm
