/*
 * qrm.h - C ABI of the MI355X (gfx950) batched watermark-detection library.
 *
 * The library computes, for a batch of images, what the detection stage of the
 * paper computes per image (Section 4.3 "Detection with Reed-Solomon
 * Correction"): one l x l tile is cropped from the image and normalised
 * (Table 1: toTensor, normalize; tile strategies random / random grid / fixed),
 * the convolutional extractor H_D turns the tile into N soft bits (Section
 * 4.1), the soft bits are thresholded at zero, grouped into m-bit symbols and
 * Reed-Solomon decoded over GF(2^m) (Appendix B).  Per image the caller gets
 * the triple the paper's decoder returns (Appendix B, after "Berlekamp-Welch
 * Decoding"): corrected message, corrected codeword, number of corrected
 * symbols.
 *
 * Conventions common to every call
 *   - Pointers named d_* are DEVICE pointers owned by the caller; everything
 *     else is HOST memory.  The library never frees or keeps caller memory,
 *     except that a context copies (and converts) the weights at creation.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work on it and return without waiting.
 *   - Return value is a qrm_status; nothing aborts or throws.  On anything but
 *     QRM_OK no kernel of that call has been launched unless stated, and
 *     qrm_last_error() describes the reason.
 *   - N == 0 is a successful no-op.
 *   - A context belongs to one device and one host thread at a time.  Work on
 *     up to QRM_MAX_STREAMS different streams may be in flight: each stream
 *     gets its own workspace inside the context and keeps it from call to
 *     call.  When more streams than that have been used, a stream not seen
 *     before takes over the workspace whose last call lies furthest back; its
 *     work is ordered (on the device) behind that call, so results stay
 *     correct, and streams that no longer exist cost nothing.
 *     qrm_release_stream hands a stream's workspace back explicitly.
 */
#ifndef QRM_H
#define QRM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QRM_MAX_STREAMS 8

#if defined(__GNUC__)
#define QRM_API __attribute__((visibility("default")))
#else
#define QRM_API
#endif

typedef struct qrm_ctx qrm_ctx; /* opaque, library-owned */

typedef enum {
    QRM_OK = 0,
    QRM_E_INVALID = 1,     /* bad argument (NULL pointer, shape, code parameters) */
    QRM_E_UNSUPPORTED = 2, /* valid but outside what the kernels are built for */
    QRM_E_NOMEM = 3,       /* workspace allocation failed */
    QRM_E_DEVICE = 4       /* a HIP call failed */
} qrm_status;

/*
 * The extractor H_D (Section 4.1: a HiDDeN-style convolutional extractor that maps a
 * tile to N soft bits).  Architecture, as fixed by the benchmark configurations:
 *   block b = 0..n_blocks-1 : conv3x3 (stride 1, zero pad 1, no flip) -> *scale + bias -> ReLU
 *                             block 0 maps in_ch -> channels, the others channels -> channels
 *   final conv3x3 channels -> n_bits (optional affine, optional ReLU), global average pool,
 *   linear n_bits x n_bits (+ bias), logits.
 * The input is normalised as x = (u8/255 - mean[c]) / std[c]; padding is zero in the
 * normalised domain and never looks outside the tile.
 * All pointers are HOST fp32 arrays, read during qrm_create only.
 */
typedef struct {
    int32_t in_ch;       /* 3 */
    int32_t n_blocks;    /* >= 1 */
    int32_t channels;    /* 32 or 64 */
    int32_t n_bits;      /* 1..128 */
    const float *conv_w; /* OIHW, concatenated: [C,in_ch,3,3], (n_blocks-1) x [C,C,3,3], [n_bits,C,3,3] */
    const float *scale;  /* [n_blocks*C] (+ n_bits more if final_affine); NULL = all ones */
    const float *bias;   /* same length as scale; NULL = all zeros */
    int32_t final_affine; /* 1: scale/bias carry n_bits extra entries applied to the final conv */
    int32_t final_relu;  /* 1: ReLU after the final conv (0 in every benchmark configuration) */
    const float *lin_w;  /* [n_bits,n_bits] row-major (out,in) */
    const float *lin_b;  /* [n_bits] or NULL */
    float mean[3], std[3];
} qrm_extractor_desc;

/*
 * The Reed-Solomon code (Appendix B "Notation"): m-bit symbols, length n <= 2^m - 1, k message
 * symbols, t = (n-k)/2 correctable symbol errors.  Narrow-sense BCH view: the generator
 * polynomial has roots alpha^fcr .. alpha^(fcr+2t-1), alpha = x.  n < 2^m - 1 is the shortened
 * code (the highest powers are dropped).  Symbol 0 of a word is the highest-degree coefficient;
 * the message occupies the first k symbols.
 */
typedef struct {
    int32_t m;          /* 2..8 */
    uint32_t prim_poly; /* e.g. 0x13 for m=4, 0x11D for m=8; must be primitive */
    int32_t n, k;       /* 0 < k < n <= 2^m - 1, n - k even, (n-k)/2 <= 8 */
    int32_t fcr;        /* first consecutive root, >= 0 (1 in the benchmark configurations); taken mod 2^m - 1 */
} qrm_rs_desc;

/*
 * Create a context on `device`.  Either descriptor may be NULL; calls that need the missing half
 * then return QRM_E_INVALID.  Weights are converted to bf16 MFMA operand layout (folded scale) and
 * uploaded; GF(2^m) log/antilog tables are built and uploaded.
 * Errors: QRM_E_INVALID for NULL out pointer / inconsistent descriptor (n > 2^m-1, odd n-k, non-
 * primitive polynomial, channels not 32/64, ...), QRM_E_UNSUPPORTED for t > 8, QRM_E_DEVICE.
 * On failure *out is NULL and qrm_last_error(NULL) holds the message.
 */
QRM_API qrm_status qrm_create(const qrm_extractor_desc *ext, const qrm_rs_desc *rs, int device, qrm_ctx **out);

/* Waits for the context's streams, frees its device memory.  NULL is ignored. */
QRM_API void qrm_destroy(qrm_ctx *ctx);

/* Message of the last failing call on `ctx` (or of the last failing qrm_create if ctx == NULL).
 * The string is owned by the library and valid until the next failing call. */
QRM_API const char *qrm_last_error(const qrm_ctx *ctx);

/*
 * Images per internal micro-batch of the extractor (the activations of one micro-batch ping-pong
 * between two workspace buffers).  0 restores the default: half a GiB of activations per buffer,
 * e.g. 1024 images for 64 x 64 tiles and 64 channels.
 */
QRM_API qrm_status qrm_set_micro_batch(qrm_ctx *ctx, int32_t images);

/*
 * Tells the context that `stream` will not be used with it again (e.g. before the caller destroys the
 * stream): waits for the context's last call on that stream and marks its workspace free for another
 * stream; the memory is kept for reuse.  A stream the context has never seen is a successful no-op.
 */
QRM_API qrm_status qrm_release_stream(qrm_ctx *ctx, void *stream);

/* Bytes of device workspace one stream of this context needs for a call with these sizes. */
QRM_API size_t qrm_workspace_bytes(const qrm_ctx *ctx, int64_t N, int32_t tile_h, int32_t tile_w);

/*
 * Tile crop (Section 4.3; Table 1 "Tile"): d_tiles[i][c][y][x] = d_images[i][c][oy+y][ox+x] with
 * (oy,ox) = d_off_yx[i] clamped to [0,H-tile] x [0,W-tile] (all three tiling strategies reduce to
 * an origin).  d_images u8 [N,3,H,W] planar; d_off_yx i32 [N,2] or NULL (= origin 0,0);
 * d_tiles u8 [N,3,tile,tile].  Bit-exact copy.
 * Errors: QRM_E_INVALID if tile <= 0, tile > H, tile > W, or a required pointer is NULL.
 */
QRM_API qrm_status qrm_extract_tiles(qrm_ctx *ctx, const uint8_t *d_images, int64_t N, int32_t H, int32_t W,
                             const int32_t *d_off_yx, int32_t tile, uint8_t *d_tiles, void *stream);

/*
 * Fused pre-processing (Table 1: resizeto(x), centercrop(x), toTensor; Appendix A "Kernel Fusion for
 * Preprocessing": the raw buffer is consumed in one pass).  Normalisation is not done here: the
 * extractor's first convolution applies it.
 * d_raw u8 [N,H_in,W_in,3], interleaved colours (a decoded image buffer); all images of a call have
 * the same size.  The shorter side is resized to `size`, the longer one to floor(size * long / short);
 * bilinear, pixel centres at half-integers, no anti-aliasing filter, source coordinates clamped to the
 * image; the centre size x size window starts at ((H_r - size) / 2, (W_r - size) / 2) (integer division).
 * Fixed point: the fraction of a source coordinate is rounded to 11 bits (w1 = round(frac * 2048),
 * w0 = 2048 - w1), the four products pixel * wy * wx are summed exactly, then (sum + 2^21) >> 22.
 * tile = 0: d_out u8 [N,3,size,size], the whole pre-processed image (input of qrm_detect).
 * tile > 0: d_out u8 [N,3,tile,tile], only the tile at d_off_yx i32 [N,2] (NULL = origin 0,0; clamped
 * to [0, size - tile]) of that image (input of qrm_extractor_forward); the rest is never computed.
 * Errors: QRM_E_INVALID (sizes <= 0, tile > size, NULL pointer), QRM_E_UNSUPPORTED (a raw or resized
 * side above 16384, a window wider than 1024).
 */
QRM_API qrm_status qrm_preprocess(qrm_ctx *ctx, const uint8_t *d_raw, int64_t N, int32_t H_in, int32_t W_in,
                                  int32_t size, const int32_t *d_off_yx, int32_t tile, uint8_t *d_out,
                                  void *stream);

/*
 * Variance-based tile selection (Listing 1, the user-defined strategy `select_patch`): windows of
 * tile x tile pixels at `stride` (the listing: 64 and 32), the variance of every window per channel,
 * summed over the channels; the window with the largest sum is the image's tile.  Readings: argmax over
 * all windows, the first in row-major order on ties; unbiased variance; the image as the extractor sees
 * it, i.e. channel c divided by std_c, so that its variance counts with weight w_c = inv_std_c^2
 * (inv_std_c = (float)(1.0 / std_c) as stored at qrm_create; w = 1 when the context has no extractor).
 * Exact form: with n = tile^2, S1 = sum x, S2 = sum x^2 over the window's raw bytes of channel c,
 * V_c = n S2 - S1^2 (an integer = n (n-1) variance), score = ((V_0 w_0) + V_1 w_1) + V_2 w_2 in IEEE
 * float64, each product and sum rounded once.
 * d_images u8 [N,3,H,W]; d_off_yx i32 [N,2] (y, x) receives the origins, ready for qrm_detect;
 * d_scores f64 [N, nH*nW] or NULL, nH = (H-tile)/stride + 1, nW likewise, windows in row-major order.
 * Errors: QRM_E_INVALID (tile or stride <= 0, tile > H or W, NULL pointer), QRM_E_UNSUPPORTED (tile not
 * a multiple of stride, tile > 512, stride > 256, more than 1024 stride x stride cells under the windows).
 */
QRM_API qrm_status qrm_select_tiles_variance(qrm_ctx *ctx, const uint8_t *d_images, int64_t N, int32_t H,
                                             int32_t W, int32_t tile, int32_t stride, int32_t *d_off_yx,
                                             double *d_scores, void *stream);

/*
 * Extractor forward pass on raw tiles (Section 4.1, m' = H_D(tile); hard bit = (logit > 0)).
 * d_tiles u8 [N,3,h,w] raw bytes, normalised inside the first convolution.
 * d_logits f32 [N,n_bits]; d_bits u8 [N,n_bits] with values 0/1, may be NULL.
 * Errors: QRM_E_INVALID (no extractor in ctx, NULL pointer, h or w < 1), QRM_E_UNSUPPORTED (the
 * activations of one tile, h*w*channels*2 bytes, exceed 1900 MiB), QRM_E_NOMEM.
 */
QRM_API qrm_status qrm_extractor_forward(qrm_ctx *ctx, const uint8_t *d_tiles, int64_t N, int32_t h, int32_t w,
                                 float *d_logits, uint8_t *d_bits, void *stream);

/*
 * Diagnostic companion of qrm_extractor_forward: runs blocks 0..n_run-1 only (1 <= n_run <=
 * n_blocks) and writes that block's output activations, converted from the internal bf16 NHWC
 * layout, to d_act f32 [N,channels,h,w].  Same kernels as the full pass.
 */
QRM_API qrm_status qrm_extractor_blocks(qrm_ctx *ctx, const uint8_t *d_tiles, int64_t N, int32_t h, int32_t w,
                                int32_t n_run, float *d_act, void *stream);

/*
 * Batched bounded-distance Reed-Solomon decoding (Appendix B; same function as the paper's
 * Berlekamp-Welch decoder, computed by syndromes, Berlekamp-Massey, Chien search and Forney).
 * d_symbols u8 [N,n], one symbol per byte (bits above m are ignored).
 * d_msg u8 [N,k]; d_codeword u8 [N,n] or NULL; d_nerr i8 [N]: number of corrected symbols 0..t,
 * or -1 when no codeword lies within distance t - then d_msg / d_codeword carry the received
 * symbols unchanged.  An uncorrectable word is not an error status.
 * Errors: QRM_E_INVALID (no code in ctx, NULL pointer, N < 0).
 */
QRM_API qrm_status qrm_rs_decode(qrm_ctx *ctx, const uint8_t *d_symbols, int64_t N,
                         uint8_t *d_msg, uint8_t *d_codeword, int8_t *d_nerr, void *stream);

/*
 * The whole detection path of Section 4.3 ("Detection with Reed-Solomon Correction") on a batch resident
 * in device memory: crop + normalise fused into the first convolution, extractor, threshold, MSB-first
 * bit->symbol packing (symbol j = bits j*m .. j*m+m-1), RS decode.  Requires n_bits == n*m.
 * d_images u8 [N,3,H,W]; d_off_yx i32 [N,2] or NULL; tile = l.
 * d_logits f32 [N,n_bits] or NULL; d_bits u8 [N,n_bits] or NULL;
 * d_msg u8 [N,k]; d_codeword u8 [N,n] or NULL; d_nerr i8 [N].
 * Errors: as above, plus QRM_E_INVALID when n_bits != n*m.
 */
QRM_API qrm_status qrm_detect(qrm_ctx *ctx, const uint8_t *d_images, int64_t N, int32_t H, int32_t W,
                      const int32_t *d_off_yx, int32_t tile,
                      float *d_logits, uint8_t *d_bits,
                      uint8_t *d_msg, uint8_t *d_codeword, int8_t *d_nerr, void *stream);

/*
 * qrm_detect for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same results as qrm_detect, but the workspace
 * (activation buffers of a micro-batch, channel statistics, packed symbols) is a fixed array of
 * QRM_STATIC_SCRATCH_BYTES inside the library's device image instead of memory taken from the context, and
 * the call neither allocates nor frees anything, creates no event or stream, and records no memset (the
 * array's block of zeros is cleared by a kernel).  The micro-batch is the largest one that fits the array
 * (e.g. 56 images of 64 x 64 tiles at 64 channels); qrm_set_micro_batch and the profiling switch do not apply.
 * Every call on a device shares that device's one array (each device holds its own copy until the process
 * ends): calls that overlap in time on one device, on whatever streams or contexts, race.  Calls on one
 * stream, one after the other, are safe.
 * Errors: as qrm_detect, plus QRM_E_UNSUPPORTED when the sizes do not fit the array (a single tile's
 * activations, tile*tile*channels*2 bytes, must fit twice beside N*n symbol bytes: tiles up to about
 * 500 x 500 at 64 channels), QRM_E_DEVICE when the array's address could not be looked up at qrm_create.
 */
#define QRM_STATIC_SCRATCH_BYTES (64u << 20)
QRM_API qrm_status qrm_detect_static(qrm_ctx *ctx, const uint8_t *d_images, int64_t N, int32_t H, int32_t W,
                                     const int32_t *d_off_yx, int32_t tile,
                                     float *d_logits, uint8_t *d_bits,
                                     uint8_t *d_msg, uint8_t *d_codeword, int8_t *d_nerr, void *stream);

/*
 * Key verification (Section 4.3: the RS-corrected message is compared with the predetermined key;
 * Listing 1, `verify(recovered_key, secret_key)`; Table 2: the false-positive rate is held at 1e-6).
 * An image that carries no watermark yields message bits that agree with the key like fair coin
 * flips, so the number of agreeing bits among the K = k*m message bits is Binomial(K, 1/2).
 *
 * qrm_key_threshold: host-only, no context.  Returns the smallest tau in 0..n_bits+1 with
 * P(Binomial(n_bits, 1/2) >= tau) <= fpr (n_bits+1 means that no image can pass), or -1 for
 * n_bits outside 1..2040 or fpr negative / NaN.  For 48 bits and 1e-6 it returns 41.
 *
 * qrm_set_key: h_key HOST u8 [k], one m-bit symbol per byte in the message's order (bits above m are
 * ignored); tau as above.  Copies the key to the device synchronously; must not be called while calls
 * that verify are still running on any stream.  Errors: QRM_E_INVALID (no code in ctx, NULL, tau
 * outside 0..k*m+1).
 *
 * qrm_verify_key: d_msg u8 [N,k] (e.g. the output of qrm_rs_decode) -> d_matches i32 [N] = number
 * of message bits equal to the key's (k*m for the key itself); d_detected u8 [N] = (matches >= tau),
 * may be NULL.  A word whose decoding failed is judged on its uncorrected message symbols.
 * Errors: QRM_E_INVALID (no key set, NULL pointer, N < 0).
 *
 * qrm_detect_verify: qrm_detect with the comparison done in the decoder's epilogue; arguments as
 * qrm_detect plus d_matches (required) and d_detected (may be NULL).
 */
QRM_API int32_t qrm_key_threshold(int32_t n_bits, double fpr);
QRM_API qrm_status qrm_set_key(qrm_ctx *ctx, const uint8_t *h_key, int32_t tau);
QRM_API qrm_status qrm_verify_key(qrm_ctx *ctx, const uint8_t *d_msg, int64_t N, int32_t *d_matches,
                                  uint8_t *d_detected, void *stream);
QRM_API qrm_status qrm_detect_verify(qrm_ctx *ctx, const uint8_t *d_images, int64_t N, int32_t H, int32_t W,
                                     const int32_t *d_off_yx, int32_t tile,
                                     float *d_logits, uint8_t *d_bits,
                                     uint8_t *d_msg, uint8_t *d_codeword, int8_t *d_nerr,
                                     int32_t *d_matches, uint8_t *d_detected, void *stream);

/*
 * Adaptive stream / micro-batch planner (Section 5, "Adaptive multi-channel horizontal fusion", Algorithm 1;
 * cost model at the end of Section 5: a stage whose warm-up time for a baseline batch b0 on one stream was t
 * takes t / s * m / b0 for a micro-batch m on s streams).  Host-only, no context, touches no device.
 * h_t HOST f64 [n_stages]: warm-up seconds per stage (> 0); h_u HOST f64 [n_stages]: bytes one sample holds
 * in that stage (>= 0); B: global batch; b0: the batch the warm-up ran on; P: stream budget over all stages
 * (>= n_stages); M_cap: memory cap in bytes for sum s[k] * m[k] * u[k]; eps: the smallest drop of the
 * bottleneck latency (seconds) worth another stream; tau: the search ends after tau scans without such a drop.
 * Outputs (HOST, caller's): h_s i32 [n_stages] streams per stage; h_m i64 [n_stages] micro-batch per stage;
 * h_J (may be NULL) predicted bottleneck latency max_k t[k] / s[k] * m[k] / b0 of the plan; h_accepted (may be
 * NULL) number of streams handed out beyond one per stage.  Steps: one stream per stage and the largest
 * uniform micro-batch <= B that fits; greedy search (the stage whose extra stream lowers the bottleneck most,
 * first stage on ties, inside both budgets); leveling (stages at most half as slow as the bottleneck get
 * min(B / sum s, 2 m) samples if that is more than they have and still fits).
 * Errors: QRM_E_INVALID (NULL pointer, n_stages outside 1..QRM_PLAN_MAX_STAGES, non-positive time, negative
 * or NaN size, P < n_stages, B, b0 or tau < 1), QRM_E_UNSUPPORTED (not even one sample per stage fits M_cap).
 */
#define QRM_PLAN_MAX_STAGES 64
QRM_API qrm_status qrm_plan_streams(int32_t n_stages, const double *h_t, const double *h_u, int64_t B, int64_t b0,
                                    int32_t P, double M_cap, double eps, int32_t tau, int32_t *h_s, int64_t *h_m,
                                    double *h_J, int32_t *h_accepted);

/*
 * The same path for a batch that lives in HOST memory, streamed through the GPU in chunks (the
 * pipelined detection of Section 5: the transfer of one mini-batch overlaps the kernels of another;
 * Section 7 streams up to a million images this way).  The context owns three (default-priority)
 * streams, one per role: uploads follow each other back to back on the first, the kernels of a chunk
 * run on the second once its upload is done, its results go home on the third.  `depth` (1..
 * QRM_MAX_STREAMS) is the number of chunks in flight = staging buffers on the device
 * (depth * chunk_images * 3*H*W bytes): 1 serialises, 2 overlaps upload and kernels, 3 adds slack.
 * h_chunks: n_chunks HOST pointers, each to u8 [chunk_images,3,H,W]; the same buffer may appear more
 * than once (a caller that refills a few buffers round-robin).  For copies that overlap with kernels
 * the buffers must be page-locked (hipHostMalloc); pageable memory works but serialises.
 * h_off_chunks: n_chunks HOST pointers to i32 [chunk_images,2], or NULL (= origin 0,0 everywhere).
 * h_msg u8 [n_chunks*chunk_images,k]; h_codeword u8 [n_chunks*chunk_images,n] or NULL;
 * h_nerr i8 [n_chunks*chunk_images]: HOST buffers, chunk after chunk.
 * The call returns when every chunk is done.  Errors: as qrm_detect, plus QRM_E_INVALID for depth
 * outside 1..QRM_MAX_STREAMS, chunk_images <= 0, n_chunks < 0 or a NULL chunk pointer.
 */
QRM_API qrm_status qrm_detect_host(qrm_ctx *ctx, const uint8_t *const *h_chunks, int32_t n_chunks,
                                   int32_t chunk_images, int32_t H, int32_t W,
                                   const int32_t *const *h_off_chunks, int32_t tile, int32_t depth,
                                   uint8_t *h_msg, uint8_t *h_codeword, int8_t *h_nerr);

/*
 * Per-launch timing, for benchmarks: while enabled, every kernel launch of qrm_detect / qrm_detect_verify /
 * qrm_extractor_forward on this context is bracketed by two hipEvents recorded on the stream it is launched
 * on, and filed under one of the kinds below.  qrm_profile_enable(ctx, on) switches the recording and clears
 * what was recorded.  qrm_profile_read waits for the recorded events of one kind and returns their summed
 * duration in milliseconds, the number of launches and their algorithmic FLOPs (2*9*C_in*C_out*h*w per image
 * and convolution block; 0 for the kinds that are not convolutions); it does not clear.  Any output pointer
 * may be NULL.  Errors: QRM_E_INVALID for a kind outside 0..QRM_PROFILE_KINDS-1.
 */
enum {
    QRM_PROFILE_PAIR_FIRST = 0,  /* fused launch: the network's first block + the C -> C block after it */
    QRM_PROFILE_PAIR_MID = 1,    /* fused launch: two C -> C blocks, activations written */
    QRM_PROFILE_PAIR_LAST = 2,   /* fused launch whose second block is the network's last (channel sums only) */
    QRM_PROFILE_BLOCK_FIRST = 3, /* the first block alone */
    QRM_PROFILE_BLOCK_MID = 4,   /* one C -> C block alone */
    QRM_PROFILE_BLOCK_LAST = 5,  /* the last block alone */
    QRM_PROFILE_HEAD = 6,        /* final convolution + pool + linear + threshold + symbol packing */
    QRM_PROFILE_RS_DECODE = 7,   /* Reed-Solomon decoding */
    QRM_PROFILE_KINDS = 8
};
QRM_API qrm_status qrm_profile_enable(qrm_ctx *ctx, int32_t on);
QRM_API qrm_status qrm_profile_read(qrm_ctx *ctx, int32_t kind, double *ms_total, int64_t *launches, double *flops);
/*
 * The time line of the last qrm_detect_host call made while profiling was enabled (that call records five events
 * per chunk instead of two per launch): ms[i*5 + 0..4] = upload start, upload end, kernels start, kernels end,
 * download end of chunk i, in milliseconds since the first upload started, for the first min(max_chunks, chunks)
 * chunks; *n_chunks receives the number of chunks that call had.  "kernels start" is when the kernel stream
 * reached the chunk, i.e. after the waits for its upload and for its output buffer.
 */
QRM_API qrm_status qrm_profile_read_chunks(qrm_ctx *ctx, int32_t max_chunks, double *ms, int32_t *n_chunks);

/* Library version string, e.g. "qrm 0.1 gfx950". */
QRM_API const char *qrm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* QRM_H */
