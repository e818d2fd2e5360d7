// Host-side state of a libqrm context and the helpers its entry points share (qrm_api.hip, qrm_noalloc.hip,
// qrm_diag.hip).  Nothing here is visible outside the library.
#pragma once

#include <string>
#include <vector>

#include "qrm_internal.h"

// A workspace of the context: the device memory the kernels of one caller stream work in.
struct QrmSlot {
    bool used = false;
    hipStream_t stream = nullptr; // the stream it serves while `used`
    void *ws = nullptr;
    size_t bytes = 0;
    hipEvent_t done = nullptr;    // recorded behind the last kernel of every call that used the workspace
    uint64_t last_use = 0;        // value of the context's call counter at that call
};

struct qrm_ctx {
    int device = 0;
    int num_cu = 256;
    bool has_ext = false, has_rs = false;
    // extractor
    int n_blocks = 0, C = 0, n_bits = 0, nbp = 0, final_relu = 0, final_affine = 0;
    float mean[3] = {0, 0, 0}, inv_std[3] = {1, 1, 1};
    void *d_weights = nullptr;  // one allocation: all fragments, biases, linear layer
    const qrm::bf16_t *d_w_first = nullptr;
    std::vector<const qrm::bf16_t *> d_w_mid;
    const qrm::bf16_t *d_w_final = nullptr;
    const float *d_bias = nullptr;        // [n_blocks*C]
    const float *d_bias_final = nullptr;  // [nbp] or null
    const float *d_lin_w = nullptr, *d_lin_b = nullptr;
    const float *d_rsum = nullptr;        // [(n_blocks-1)][C][C] weight-rounding residual sums of the C -> C layers
    const float *d_wft = nullptr;         // final conv, fp32, [C*9][nbp]
    bool collapse = false;                // final conv + pool evaluated in closed form from channel sums
    bool pairable = false;                // weights are prepared for the fused schedule (see qrm_create)
    // code
    qrm::RsParams rs{};
    void *d_tables = nullptr;             // 1 KiB: antilog table, log table at 512, key symbols at 768
    bool has_key = false;
    int key_tau = 0;
    // workspaces: one per caller stream in use, plus the kernel stream of qrm_detect_host
    int micro_batch = 0; // 0 = default
    QrmSlot slots[QRM_MAX_STREAMS + 1];
    uint64_t use_clock = 0;
    int diag_flags = 0;  // QRM_DIAG_* (include/qrm_diag.h); 0 in production
    // optional per-launch timing of the convolution kernels (hipEvents on the launch stream)
    bool profile = false;
    struct Timed {
        hipEvent_t start = nullptr, stop = nullptr;
        int kind = 0;      // QRM_PROFILE_* class of the launch
        double flops = 0;  // algorithmic FLOPs of the launch
    };
    std::vector<Timed> timed;  // pool of event pairs; the first timed_used are recorded
    size_t timed_used = 0;
    bool in_host_pipeline = false; // qrm_detect_host is running: its chunks are timed as wholes, not launch by launch
    struct ChunkTimes {
        hipEvent_t ev[5] = {nullptr, nullptr, nullptr, nullptr, nullptr}; // upload start / end, kernels start / end, download end
    };
    std::vector<ChunkTimes> chunk_times; // pool; the first chunks_timed are recorded (last qrm_detect_host call)
    size_t chunks_timed = 0;
    // chunked host -> device pipeline of qrm_detect_host, created on first use: one stream per role
    // (upload, kernels, download) and a ring of staging buffers with the events that hand them on
    struct Stage {
        uint8_t *d_img = nullptr;  // [chunk,3,H,W]
        int32_t *d_off = nullptr;  // [chunk,2]
        uint8_t *d_out = nullptr;  // msg [chunk,k] | codeword [chunk,n] | nerr [chunk]
        size_t img_bytes = 0, out_bytes = 0, off_bytes = 0;
        hipEvent_t uploaded = nullptr, computed = nullptr, downloaded = nullptr;
    };
    Stage stages[QRM_MAX_STREAMS];
    hipStream_t s_up = nullptr, s_run = nullptr, s_down = nullptr;
    std::string err;
};

namespace qrm {

qrm_status fail(qrm_ctx *c, qrm_status st, const std::string &msg);
qrm_status hip_fail(qrm_ctx *c, hipError_t e, const char *what);

// Where the parts of a workspace lie (byte offsets from its base are the running sums, in this order: the
// block of zeros, two activation buffers, partial sums of the final convolution, two statistics buffers, the
// columns a fused launch on wide tiles hands from one column block to the next, symbols).
struct WsLayout {
    size_t act, partial, stats, seam, symbols, total;
    int mb, n_part;
};
// act_budget: bytes one activation buffer may take (0: the context's micro-batch setting decides)
WsLayout ws_layout(const qrm_ctx *c, int64_t N, int h, int w, bool want_symbols, size_t act_budget = 0);

// Runs the extractor over [N] tiles taken from `src` (whole images + origins, or raw tiles) in the workspace at
// `base` laid out as L.  n_run < 0: full pass -> logits / bits / symbols.  n_run >= 1: stop after that many
// blocks -> d_act.  may_time: launches may be bracketed by events when the context's profiling is on.
qrm_status run_extractor(qrm_ctx *c, uint8_t *base, const WsLayout &L, TileSrc src, int64_t N, int h, int w, int n_run,
                         float *d_logits, uint8_t *d_bits, uint8_t *d_symbols, int m_sym, float *d_act, bool may_time,
                         hipStream_t s);

// Argument checks shared by the entry points that run the whole detection path.
qrm_status check_detect_args(qrm_ctx *c, const uint8_t *d_images, int64_t N, int32_t H, int32_t W, int32_t tile,
                             uint8_t *d_msg, int8_t *d_nerr, bool verify, int32_t *d_matches);

// qrm_noalloc.hip: looks up the device address of the static workspace on `device` (which must be current)
hipError_t static_scratch_init(int device);

inline size_t symbols_offset(const WsLayout &L) { return kZeroBytes + 2 * L.act + L.partial + 2 * L.stats + L.seam; }

} // namespace qrm
