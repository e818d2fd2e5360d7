// C ABI of libqrm: context, weight / table preparation, workspace, and the entry points that chain the
// kernels of the detection path (Section 4.3 of the paper; kernels in extractor.hip, rs_decode.hip,
// tiles.hip).  Host code only; no arithmetic of the method runs on the CPU after qrm_create.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <string>
#include <vector>

#include <stdlib.h>
#include "qrm_ctx.h"
#include "../../include/qrm_diag.h"

using namespace qrm;

namespace qrm {

uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) return (uint16_t)((u >> 16) | ((u & 0xffffu) ? 0x40u : 0u)); // inf / nan
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

} // namespace qrm

namespace {

std::string g_create_error;

size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// MFMA row r of a 32-row weight fragment carries output channel perm32(r) of its block, so that the
// 16 accumulators of a lane are 16 consecutive channels.
int perm32(int r) { return 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3); }

} // namespace

namespace qrm {

qrm_status fail(qrm_ctx *c, qrm_status st, const std::string &msg)
{
    if (c) c->err = msg; else g_create_error = msg;
    return st;
}

qrm_status hip_fail(qrm_ctx *c, hipError_t e, const char *what)
{
    return fail(c, QRM_E_DEVICE, std::string(what) + ": " + hipGetErrorString(e));
}

} // namespace qrm

namespace {

// Non-negative integers of a few thousand bits, just enough for exact binomial tails.
struct Big {
    std::vector<uint32_t> w; // little endian, no leading zero words
    explicit Big(uint64_t v = 0)
    {
        if (v & 0xffffffffu || v >> 32) w.push_back((uint32_t)v);
        if (v >> 32) w.push_back((uint32_t)(v >> 32));
    }
    void trim() { while (!w.empty() && w.back() == 0) w.pop_back(); }
    void add(const Big &o)
    {
        if (w.size() < o.w.size()) w.resize(o.w.size(), 0);
        uint64_t carry = 0;
        for (size_t i = 0; i < w.size(); ++i) {
            carry += (uint64_t)w[i] + (i < o.w.size() ? o.w[i] : 0u);
            w[i] = (uint32_t)carry;
            carry >>= 32;
        }
        if (carry) w.push_back((uint32_t)carry);
    }
    void mul_small(uint32_t f)
    {
        uint64_t carry = 0;
        for (auto &x : w) {
            carry += (uint64_t)x * f;
            x = (uint32_t)carry;
            carry >>= 32;
        }
        if (carry) w.push_back((uint32_t)carry);
        trim();
    }
    void div_small(uint32_t d) // the remainder is dropped (callers divide exactly)
    {
        uint64_t rem = 0;
        for (size_t i = w.size(); i-- > 0;) {
            const uint64_t cur = (rem << 32) | w[i];
            w[i] = (uint32_t)(cur / d);
            rem = cur % d;
        }
        trim();
    }
    void shl(int bits)
    {
        if (w.empty() || bits <= 0) return;
        const int words = bits / 32, r = bits % 32;
        std::vector<uint32_t> o(w.size() + words + 1, 0);
        for (size_t i = 0; i < w.size(); ++i) {
            const uint64_t v = (uint64_t)w[i] << r;
            o[i + words] |= (uint32_t)v;
            o[i + words + 1] |= (uint32_t)(v >> 32);
        }
        w.swap(o);
        trim();
    }
    int cmp(const Big &o) const
    {
        if (w.size() != o.w.size()) return w.size() < o.w.size() ? -1 : 1;
        for (size_t i = w.size(); i-- > 0;)
            if (w[i] != o.w[i]) return w[i] < o.w[i] ? -1 : 1;
        return 0;
    }
};

// ---- weights -> MFMA A-fragment order ------------------------------------------------------------
// fragment element (blk, tap, kc, lane, e): output channel blk*32 + perm32(lane%32),
// input channel kc*16 + (lane/32)*8 + e.  w is OIHW [cout][cin][3][3]; rows >= cout are zero.
float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

// bf16 values of one layer's (scaled) weights, [o][ci][tap].  cancel = false: each weight rounded to nearest
// even.  cancel = true: error feedback over the taps of every (o, ci) pair - each tap is rounded after the
// residual of the taps before it has been added - so that the residuals sum to (almost) nothing: the part of
// the rounding error that acts on the mean activation, the only part that global average pooling does not
// wash out, is gone without any correction term.  Two refinements, both measured on structured tiles: the
// taps are taken largest first, so that what is left over at the end is a fraction of the smallest weight's
// rounding step, not of a typical one; and the taps with dy + dx even and those with dy + dx odd form two
// chains of their own, so that the residuals also cancel against an activation map that alternates from
// pixel to pixel (a one-pixel checkerboard keeps that structure through every layer).
std::vector<uint16_t> round_layer(const float *w, const float *scale, int cout, int cin, bool cancel)
{
    std::vector<uint16_t> r((size_t)cout * cin * 9);
    for (int o = 0; o < cout; ++o)
        for (int ci = 0; ci < cin; ++ci) {
            const size_t base = ((size_t)o * cin + ci) * 9;
            float v[9];
            int order[9];
            for (int tap = 0; tap < 9; ++tap) {
                v[tap] = w[base + tap] * (scale ? scale[o] : 1.f);
                order[tap] = tap;
            }
            if (cancel) std::stable_sort(order, order + 9, [&](int a, int b) { return fabsf(v[a]) > fabsf(v[b]); });
            double carry[2] = {0.0, 0.0};
            for (int k = 0; k < 9; ++k) {
                const int tap = order[k];
                const int chain = (tap / 3 + tap % 3) & 1;
                const float target = cancel ? (float)((double)v[tap] + carry[chain]) : v[tap];
                r[base + tap] = f32_to_bf16_rne(target);
                carry[chain] += (double)v[tap] - (double)bf16_to_f32(r[base + tap]);
            }
        }
    return r;
}

void pack_mid(const std::vector<uint16_t> &r, int cout, int cout_pad, int cin, std::vector<uint16_t> &dst)
{
    const int KC = cin / 16;
    for (int blk = 0; blk < cout_pad / 32; ++blk)
        for (int tap = 0; tap < 9; ++tap)
            for (int kc = 0; kc < KC; ++kc)
                for (int lane = 0; lane < 64; ++lane)
                    for (int e = 0; e < 8; ++e) {
                        const int o = blk * 32 + perm32(lane & 31);
                        const int ci = kc * 16 + (lane >> 5) * 8 + e;
                        dst.push_back(o < cout ? r[((size_t)o * cin + ci) * 9 + tap] : (uint16_t)0);
                    }
}

// first layer: k = q*16 + (lane/32)*8 + e  ->  tap = k/4 (0..8, beyond: zero), channel = k%4.
// The kernels feed the raw bytes p_c (exact in bf16) and a fourth channel that is 1 inside the tile, so the
// normalisation x_c = (p_c / 255 - mean_c) / std_c is folded into the weights: channel c < 3 carries
// w / (255 std_c), channel 3 carries - sum_c w mean_c / std_c (per tap).
// Per output block two fragment sets: bf16(v) and bf16(v - bf16(v)).
void pack_first(const float *w, const float *scale, int cout, const float *mean, const float *std, std::vector<uint16_t> &dst)
{
    for (int blk = 0; blk < cout / 32; ++blk)
        for (int part = 0; part < 2; ++part)
            for (int q = 0; q < 3; ++q)
                for (int lane = 0; lane < 64; ++lane)
                    for (int e = 0; e < 8; ++e) {
                        const int o = blk * 32 + perm32(lane & 31);
                        const int k = q * 16 + (lane >> 5) * 8 + e;
                        const int tap = k / 4, ch = k % 4;
                        double v = 0.0;
                        if (tap < 9) {
                            const double sc = scale ? (double)scale[o] : 1.0;
                            if (ch < 3) v = (double)w[((size_t)o * 3 + ch) * 9 + tap] * sc / (255.0 * (double)std[ch]);
                            else
                                for (int c = 0; c < 3; ++c)
                                    v -= (double)w[((size_t)o * 3 + c) * 9 + tap] * sc * (double)mean[c] / (double)std[c];
                        }
                        const uint16_t hi = f32_to_bf16_rne((float)v);
                        dst.push_back(part == 0 ? hi : f32_to_bf16_rne((float)(v - (double)bf16_to_f32(hi))));
                    }
}

// rsum[o][c] = sum over the 9 taps of (w*scale - bf16(w*scale)): what the bf16 weights leave out, as it
// acts on a spatially constant input
// appended as [c_in][c_out]: the lanes of the kernel that applies it run over c_out
void residual_sums(const float *w, const float *scale, const std::vector<uint16_t> &r, int C, std::vector<float> &dst)
{
    for (int ci = 0; ci < C; ++ci)
        for (int o = 0; o < C; ++o) {
            double s = 0.0;
            for (int tap = 0; tap < 9; ++tap) {
                const size_t i = ((size_t)o * C + ci) * 9 + tap;
                s += (double)(w[i] * (scale ? scale[o] : 1.f)) - (double)bf16_to_f32(r[i]);
            }
            dst.push_back((float)s);
        }
}

// One image's activations must stay below this many bytes: the kernels address a pixel inside an image with
// 32-bit byte offsets.
constexpr size_t kMaxImageActBytes = (size_t)1900 << 20;

int default_micro_batch(const qrm_ctx *c, int h, int w)
{
    // Half a GiB of activations per buffer: measured best for the fused pairs (1024 images at 64 x 64: four per
    // compute unit, which the workgroups walk through without draining) and for the single-block kernel on wide
    // tiles (256 images at 128 x 128, 64 at 256 x 256: ~16 k strips per launch).  Cache residency of the two
    // buffers (128 MiB each) measured worse in both cases.
    const size_t per_img = (size_t)h * w * c->C * 2;
    size_t mb = ((size_t)512 << 20) / (per_img ? per_img : 1);
    if (mb < 64) mb = 64;
    // The fused kernels give every compute unit whole images: tiles wider than one column block (where an image
    // is a long run of work) get at least one image per compute unit, as long as a buffer stays below 4 GiB.
    if (c->pairable && w > kTileW && mb < (size_t)c->num_cu && (size_t)c->num_cu * per_img <= ((size_t)4 << 30)) mb = c->num_cu;
    if (mb > 8192) mb = 8192;
    return (int)mb;
}

// Whether a launch of cnt images of h x w runs the fused schedule (two blocks per launch).  Narrow tiles always
// do; wide ones only when the launch has images for at least half of the compute units (a workgroup of the fused
// kernel takes whole images; the single-block kernel deals strips).
bool use_fused(const qrm_ctx *c, int cnt, int w, int blocks)
{
    if ((c->diag_flags & QRM_DIAG_NO_FUSED_PAIRS) || !c->pairable || blocks < 2) return false;
    if (w <= kTileW || (c->diag_flags & QRM_DIAG_FUSE_ALWAYS)) return true;
    return 2 * cnt >= c->num_cu;
}

int effective_micro_batch(const qrm_ctx *c, int64_t N, int h, int w, size_t act_budget)
{
    const size_t per_img = (size_t)h * w * c->C * 2;
    int mb = c->micro_batch > 0 ? c->micro_batch : default_micro_batch(c, h, w);
    if (act_budget) mb = (int)std::min<size_t>(act_budget / (per_img ? per_img : 1), 65536);
    if ((int64_t)mb > N) mb = (int)(N > 0 ? N : 1);
    if (per_img > kMaxImageActBytes) mb = 0; // the kernels address a pixel inside an image with 32-bit offsets
    return mb; // 0: not even one image fits
}

int tiles_per_image(int h, int w) { return ((h + kRows - 1) / kRows) * ((w + kTileW - 1) / kTileW); }
int first_blocks(const qrm_ctx *c) { return 8 * c->num_cu; }
int mid_blocks(const qrm_ctx *c) { return c->num_cu; } // one persistent workgroup per CU

} // namespace

namespace qrm {

WsLayout ws_layout(const qrm_ctx *c, int64_t N, int h, int w, bool want_symbols, size_t act_budget)
{
    WsLayout L{};
    if (c->has_ext) {
        L.mb = effective_micro_batch(c, N, h, w, act_budget);
        L.n_part = ((w + kTileW - 1) / kTileW) * 2;
        L.act = align_up((size_t)L.mb * h * w * c->C * 2);
        L.partial = align_up((size_t)L.mb * L.n_part * c->nbp * 4);
        // statistics records: sized for the fullest micro-batch and for the ragged last one
        const int tpi = tiles_per_image(h, w);
        size_t recs = 0;
        const int64_t counts[2] = {L.mb, L.mb ? N % L.mb : 0};
        for (int64_t cnt : counts) {
            if (cnt <= 0) continue;
            const Partition pf = make_partition(cnt, tpi, first_blocks(c));
            const Partition pm = make_partition(cnt, tpi, mid_blocks(c), conv_mid_records_per_workgroup(c->C));
            const ConvGeom g{(int)cnt, h, w, (h + kRows - 1) / kRows, (w + kTileW - 1) / kTileW};
            const int rp = c->pairable ? conv_pair_records_per_image(g, true) : 0;
            const int rf = pf.slots * pf.sub, rm = pm.slots * pm.sub;
            const size_t r = (size_t)cnt * std::max(rp, std::max(rf, rm));
            if (r > recs) recs = r;
            if (c->pairable) L.seam = std::max(L.seam, align_up(conv_pair_seam_bytes(g, c->num_cu)));
        }
        L.stats = align_up(recs * stat_record_floats(c->C, 9) * 4);
    }
    L.symbols = (want_symbols && c->has_rs) ? align_up((size_t)N * c->rs.n) : 0;
    L.total = kZeroBytes + 2 * L.act + L.partial + 2 * L.stats + L.seam + L.symbols;
    return L;
}

} // namespace qrm

namespace {

// Hands the caller's stream its workspace of at least `bytes` bytes.  A stream keeps its workspace from call
// to call.  A stream not seen before takes a free one, or - when all are taken - the one whose last call lies
// furthest back: the new stream is then made to wait (on the device) for that call to finish, so nothing is
// overwritten while in use, whether or not the old stream still exists.
qrm_status get_slot(qrm_ctx *c, hipStream_t s, size_t bytes, QrmSlot **out)
{
    QrmSlot *slot = nullptr;
    for (auto &sl : c->slots)
        if (sl.used && sl.stream == s) { slot = &sl; break; }
    if (!slot) {
        for (auto &sl : c->slots) // a free one, preferably one whose memory is already large enough
            if (!sl.used && (!slot || (slot->bytes < bytes && sl.bytes > slot->bytes))) slot = &sl;
        if (!slot)
            for (auto &sl : c->slots)
                if (!slot || sl.last_use < slot->last_use) slot = &sl;
        if (slot->done && slot->last_use) {
            hipError_t e = hipStreamWaitEvent(s, slot->done, 0);
            if (e != hipSuccess) return hip_fail(c, e, "hipStreamWaitEvent(workspace hand-over)");
        }
        slot->used = true;
        slot->stream = s;
    }
    slot->last_use = ++c->use_clock;
    if (!slot->done) {
        hipError_t e = hipEventCreateWithFlags(&slot->done, hipEventDisableTiming);
        if (e != hipSuccess) return hip_fail(c, e, "hipEventCreateWithFlags");
    }
    if (slot->bytes < bytes) {
        if (slot->ws) {
            // everything that used the old memory is behind `done` (calls on earlier streams) or on s itself
            hipError_t e = hipEventSynchronize(slot->done);
            if (e == hipSuccess) e = hipStreamSynchronize(s);
            if (e != hipSuccess) return hip_fail(c, e, "hipStreamSynchronize");
            (void)hipFree(slot->ws);
            slot->ws = nullptr;
            slot->bytes = 0;
        }
        hipError_t e = hipMalloc(&slot->ws, bytes);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            char buf[128];
            snprintf(buf, sizeof buf, "workspace allocation of %zu bytes failed", bytes);
            return fail(c, QRM_E_NOMEM, buf);
        }
        slot->bytes = bytes;
        // Diagnostic (qrm_diag_set_flags): a new workspace filled with 0xFF bytes (NaN as bf16 / fp32), so that
        // a kernel reading something no kernel wrote shows up in the results.
        if (c->diag_flags & QRM_DIAG_POISON_WORKSPACE) {
            const int fill = (c->diag_flags >> 8) & 0xFF; // another fill byte may ride in bits 8..15
            e = hipMemsetAsync(slot->ws, fill ? fill : 0xFF, bytes, s);
            if (e != hipSuccess) return hip_fail(c, e, "hipMemsetAsync(workspace poison)");
        }
        // The block of zeros the convolutions read their padding from; written once per allocation, on
        // the stream of the kernels that read it (the stream may not synchronise with the null stream).
        e = hipMemsetAsync(slot->ws, 0, kZeroBytes, s);
        if (e != hipSuccess) return hip_fail(c, e, "hipMemsetAsync(workspace zero block)");
    }
    *out = slot;
    return QRM_OK;
}

// behind the last kernel of a call: whoever takes the workspace over waits for this
qrm_status slot_done(qrm_ctx *c, QrmSlot *slot, hipStream_t s)
{
    hipError_t e = hipEventRecord(slot->done, s);
    if (e != hipSuccess) return hip_fail(c, e, "hipEventRecord");
    return QRM_OK;
}

// Event pair around one launch while profiling is on (null otherwise).
qrm_ctx::Timed *time_begin(qrm_ctx *c, bool may_time, int kind, double flops, hipStream_t s)
{
    if (!c->profile || !may_time || c->in_host_pipeline) return nullptr;
    if (c->timed_used == c->timed.size()) {
        qrm_ctx::Timed t;
        if (hipEventCreate(&t.start) != hipSuccess) return nullptr;
        if (hipEventCreate(&t.stop) != hipSuccess) { (void)hipEventDestroy(t.start); return nullptr; }
        c->timed.push_back(t);
    }
    qrm_ctx::Timed *t = &c->timed[c->timed_used++];
    t->kind = kind;
    t->flops = flops;
    (void)hipEventRecord(t->start, s);
    return t;
}
void time_end(qrm_ctx::Timed *t, hipStream_t s)
{
    if (t) (void)hipEventRecord(t->stop, s);
}

} // namespace

namespace qrm {

qrm_status run_extractor(qrm_ctx *c, uint8_t *base, const WsLayout &L, TileSrc src, int64_t N, int h, int w, int n_run,
                         float *d_logits, uint8_t *d_bits, uint8_t *d_symbols, int m_sym, float *d_act, bool may_time,
                         hipStream_t s)
{
    const size_t buf_off[2] = {kZeroBytes, kZeroBytes + L.act};
    uint8_t *seam = base + kZeroBytes + 2 * L.act + L.partial + 2 * L.stats;
    bf16_t *buf[2] = {(bf16_t *)(base + buf_off[0]), (bf16_t *)(base + buf_off[1])};
    float *partial = (float *)(base + kZeroBytes + 2 * L.act);
    float *tb[2] = {(float *)(base + kZeroBytes + 2 * L.act + L.partial),
                    (float *)(base + kZeroBytes + 2 * L.act + L.partial + L.stats)};
    const int nsym = (d_symbols && m_sym > 0) ? c->n_bits / m_sym : 0;
    const uint8_t *img0 = src.img;
    const int32_t *off0 = src.off;
    const int tpi = tiles_per_image(h, w);
    const float inv_hw = 1.0f / ((float)h * (float)w);
    const double block_flops = 2.0 * 9.0 * c->C * c->C * (double)h * w;   // one C -> C block, one image
    const double first_flops = 2.0 * 9.0 * 3 * c->C * (double)h * w;      // the first block, one image
    hipError_t e;
    for (int64_t n0 = 0; n0 < N; n0 += L.mb) {
        const int cnt = (int)((N - n0 < L.mb) ? (N - n0) : L.mb);
        ConvGeom g{cnt, h, w, (h + kRows - 1) / kRows, (w + kTileW - 1) / kTileW};
        const Partition pf = make_partition(cnt, tpi, first_blocks(c));
        const Partition pm = make_partition(cnt, tpi, mid_blocks(c), conv_mid_records_per_workgroup(c->C));
        src.img = img0 + n0 * 3 * (int64_t)src.H * src.W;
        src.off = off0 ? off0 + 2 * n0 : nullptr;
        int cur = 0, tcur = 0, in_slots = pf.slots * pf.sub;
        const int blocks = n_run > 0 ? n_run : c->n_blocks; // blocks to run: the first one and C -> C layers m = b - 1
        // Fused schedule (64 channels; see use_fused): [first + layer 0], (1,2), (3,4), ..; what is left over
        // runs alone.
        const bool fused = use_fused(c, cnt, w, blocks) && conv_pair_supported(c->C, g);
        auto is_last = [&](int b) { return n_run < 0 && c->collapse && b == c->n_blocks - 1; };
        int b = 1;
        if (fused) {
            qrm_ctx::Timed *t = time_begin(c, may_time, is_last(1) ? QRM_PROFILE_PAIR_LAST : QRM_PROFILE_PAIR_FIRST,
                                           (first_flops + block_flops) * cnt, s);
            e = launch_conv_pair(base, nullptr, &src, g, c->C, c->d_w_first, c->d_w_mid[0], c->d_bias, c->d_bias + (size_t)c->C, nullptr,
                                 0, nullptr, tb[tcur], is_last(1), c->num_cu, seam, buf[cur], s);
            if (e != hipSuccess) return hip_fail(c, e, "conv_pair (first) launch");
            time_end(t, s);
            in_slots = conv_pair_records_per_image(g, is_last(1));
            b = 2;
        } else {
            qrm_ctx::Timed *t = time_begin(c, may_time, QRM_PROFILE_BLOCK_FIRST, first_flops * cnt, s);
            e = launch_conv_first(src, g, c->C, c->d_w_first, c->d_bias, tb[tcur], pf, buf[cur], s);
            if (e != hipSuccess) return hip_fail(c, e, "conv_first launch");
            time_end(t, s);
        }
        while (b < blocks) {
            const int m = b - 1;
            const bool pair = fused && (m & 1) == 1 && b + 1 < blocks;
            const float *rsum = c->d_rsum + (size_t)m * c->C * c->C;
            if (pair) {
                qrm_ctx::Timed *t = time_begin(c, may_time, is_last(b + 1) ? QRM_PROFILE_PAIR_LAST : QRM_PROFILE_PAIR_MID,
                                               2.0 * block_flops * cnt, s);
                e = launch_conv_pair(base, base + buf_off[cur], nullptr, g, c->C, c->d_w_mid[m], c->d_w_mid[m + 1],
                                     c->d_bias + (size_t)b * c->C, c->d_bias + (size_t)(b + 1) * c->C, tb[tcur], in_slots, rsum,
                                     tb[tcur ^ 1], is_last(b + 1), c->num_cu, seam, buf[cur ^ 1], s);
                if (e != hipSuccess) return hip_fail(c, e, "conv_pair launch");
                time_end(t, s);
                in_slots = conv_pair_records_per_image(g, is_last(b + 1));
            } else {
                qrm_ctx::Timed *t = time_begin(c, may_time, is_last(b) ? QRM_PROFILE_BLOCK_LAST : QRM_PROFILE_BLOCK_MID,
                                               block_flops * cnt, s);
                e = launch_conv_mid(base, buf_off[cur], g, c->C, c->d_w_mid[m], c->d_bias + (size_t)b * c->C, tb[tcur], in_slots,
                                    rsum, tb[tcur ^ 1], pm, is_last(b), buf[cur ^ 1], s);
                if (e != hipSuccess) return hip_fail(c, e, "conv_mid launch");
                time_end(t, s);
                in_slots = pm.slots * pm.sub;
            }
            cur ^= 1;
            tcur ^= 1;
            b += pair ? 2 : 1;
        }
        if (n_run > 0) {
            e = launch_nhwc_to_nchw(buf[cur], cnt, h, w, c->C, d_act + n0 * (int64_t)c->C * h * w, s);
            if (e != hipSuccess) return hip_fail(c, e, "nhwc_to_nchw launch");
            continue;
        }
        float *lg = d_logits ? d_logits + n0 * c->n_bits : nullptr;
        uint8_t *bt = d_bits ? d_bits + n0 * c->n_bits : nullptr;
        uint8_t *sy = nsym ? d_symbols + n0 * nsym : nullptr;
        qrm_ctx::Timed *t = time_begin(c, may_time, QRM_PROFILE_HEAD, 0.0, s);
        if (c->collapse) {
            e = launch_head(tb[tcur], in_slots, c->C, cnt, c->n_bits, c->nbp, inv_hw, c->d_wft, c->d_bias_final,
                            c->d_lin_w, c->d_lin_b, lg, bt, sy, m_sym > 0 ? m_sym : 1, s);
            if (e != hipSuccess) return hip_fail(c, e, "head launch");
        } else {
            e = launch_conv_final(base, buf_off[cur], g, c->C, c->nbp, c->d_w_final, c->d_bias_final, c->final_relu,
                                  partial, c->num_cu, s);
            if (e != hipSuccess) return hip_fail(c, e, "conv_final launch");
            e = launch_linear_pack(partial, L.n_part, c->nbp, cnt, c->n_bits, inv_hw,
                                   c->final_relu ? nullptr : c->d_bias_final, c->d_lin_w, c->d_lin_b, lg, bt, sy,
                                   m_sym > 0 ? m_sym : 1, s);
            if (e != hipSuccess) return hip_fail(c, e, "linear_pack launch");
        }
        time_end(t, s);
    }
    return QRM_OK;
}

} // namespace qrm

namespace {

bool build_gf_tables(int m, uint32_t poly, std::vector<uint8_t> &exp2, std::vector<uint8_t> &lg)
{
    const int q = 1 << m, ord = q - 1;
    exp2.assign(2 * ord, 0);
    lg.assign(q, 0);
    uint32_t x = 1;
    for (int i = 0; i < ord; ++i) {
        if (i > 0 && x == 1) return false; // alpha's order is too small: not primitive
        exp2[i] = exp2[i + ord] = (uint8_t)x;
        lg[x] = (uint8_t)i;
        x <<= 1;
        if (x & (uint32_t)q) x ^= poly;
        if (x >= (uint32_t)q) return false; // polynomial does not have degree m
    }
    return x == 1;
}

} // namespace

extern "C" {

const char *qrm_version(void) { return "qrm 0.1 gfx950"; }

const char *qrm_last_error(const qrm_ctx *ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

qrm_status qrm_create(const qrm_extractor_desc *ext, const qrm_rs_desc *rs, int device, qrm_ctx **out)
{
    if (!out) return fail(nullptr, QRM_E_INVALID, "out is NULL");
    *out = nullptr;
    if (!ext && !rs) return fail(nullptr, QRM_E_INVALID, "both descriptors are NULL");
    if (ext) {
        if (ext->in_ch != 3) return fail(nullptr, QRM_E_UNSUPPORTED, "in_ch must be 3");
        if (ext->channels != 32 && ext->channels != 64) return fail(nullptr, QRM_E_INVALID, "channels must be 32 or 64");
        if (ext->n_blocks < 1 || ext->n_blocks > 64) return fail(nullptr, QRM_E_INVALID, "n_blocks out of range");
        if (ext->n_bits < 1 || ext->n_bits > 128) return fail(nullptr, QRM_E_INVALID, "n_bits out of range (1..128)");
        if (!ext->conv_w || !ext->lin_w) return fail(nullptr, QRM_E_INVALID, "conv_w / lin_w is NULL");
        if ((ext->scale == nullptr) != (ext->bias == nullptr) && ext->final_affine)
            return fail(nullptr, QRM_E_INVALID, "final_affine needs both scale and bias");
        for (int i = 0; i < 3; ++i)
            if (!(ext->std[i] > 0.f)) return fail(nullptr, QRM_E_INVALID, "std must be positive");
    }
    std::vector<uint8_t> exp2, lg;
    if (rs) {
        if (rs->m < 2 || rs->m > 8) return fail(nullptr, QRM_E_INVALID, "m must be in 2..8");
        const int q = 1 << rs->m;
        if (rs->n > q - 1) return fail(nullptr, QRM_E_INVALID, "n exceeds 2^m - 1");
        if (rs->k <= 0 || rs->k >= rs->n) return fail(nullptr, QRM_E_INVALID, "need 0 < k < n");
        if ((rs->n - rs->k) & 1) return fail(nullptr, QRM_E_INVALID, "n - k must be even");
        if (rs->fcr < 0) return fail(nullptr, QRM_E_INVALID, "fcr must be >= 0");
        if ((rs->n - rs->k) / 2 > 8) return fail(nullptr, QRM_E_UNSUPPORTED, "t > 8 is not built");
        if (!build_gf_tables(rs->m, rs->prim_poly, exp2, lg))
            return fail(nullptr, QRM_E_INVALID, "prim_poly is not a primitive polynomial of degree m");
    }
    hipError_t e = hipSetDevice(device);
    if (e != hipSuccess) return hip_fail(nullptr, e, "hipSetDevice");
    // once per device, with that device current: the address of the static workspace of qrm_detect_static
    // (a failure is reported by that entry point, not here)
    (void)static_scratch_init(device);
    (void)hipGetLastError();

    qrm_ctx *c = new qrm_ctx();
    c->device = device;
    int cu = 0;
    if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && cu > 0) c->num_cu = cu;

    if (ext) {
        const int C = ext->channels, nb = ext->n_blocks, nbits = ext->n_bits;
        const int nbp = (nbits + 63) / 64 * 64;
        c->has_ext = true;
        c->n_blocks = nb; c->C = C; c->n_bits = nbits; c->nbp = nbp;
        c->final_relu = ext->final_relu ? 1 : 0;
        c->final_affine = (ext->final_affine && ext->scale && ext->bias) ? 1 : 0;
        for (int i = 0; i < 3; ++i) { c->mean[i] = ext->mean[i]; c->inv_std[i] = (float)(1.0 / (double)ext->std[i]); }

        std::vector<uint16_t> frag;
        std::vector<size_t> frag_off; // element offsets: first, mids..., final
        const float *w = ext->conv_w;
        frag_off.push_back(frag.size());
        pack_first(w, ext->scale, C, ext->mean, ext->std, frag);
        w += (size_t)C * 3 * 9;
        c->collapse = nb >= 2 && !c->final_relu;
        // Fused schedule (launch_conv_pair; C = 64): [first block + C -> C layer 0],
        // then C -> C layers (1,2), (3,4), ..; a layer left over runs alone.  The second block of a fused
        // launch - the even C -> C layers - cannot have its bias corrected with channel means of its input
        // (that input never exists as a whole image): those layers get residual-cancelling rounding instead.
        c->pairable = C == 64;
        std::vector<std::vector<uint16_t>> rounded; // per C -> C layer
        for (int b = 1; b < nb; ++b) {
            const int m = b - 1;
            rounded.push_back(round_layer(w, ext->scale ? ext->scale + (size_t)b * C : nullptr, C, C, c->pairable && (m & 1) == 0));
            frag_off.push_back(frag.size());
            pack_mid(rounded.back(), C, C, C, frag);
            w += (size_t)C * C * 9;
        }
        frag_off.push_back(frag.size());
        pack_mid(round_layer(w, c->final_affine ? ext->scale + (size_t)nb * C : nullptr, nbits, C, false), nbits, nbp, C, frag);

        std::vector<float> fl; // biases [nb*C], final bias [nbp], lin_w, lin_b, residual sums, final conv (fp32)
        for (int i = 0; i < nb * C; ++i) fl.push_back(ext->bias ? ext->bias[i] : 0.f);
        const size_t off_fb = fl.size();
        for (int i = 0; i < nbp; ++i) fl.push_back((c->final_affine && i < nbits) ? ext->bias[(size_t)nb * C + i] : 0.f);
        const size_t off_lw = fl.size();
        for (int i = 0; i < nbits * nbits; ++i) fl.push_back(ext->lin_w[i]);
        const size_t off_lb = fl.size();
        for (int i = 0; i < nbits; ++i) fl.push_back(ext->lin_b ? ext->lin_b[i] : 0.f);
        while (fl.size() % 4) fl.push_back(0.f);
        const size_t off_rs = fl.size();
        {
            const float *wm = ext->conv_w + (size_t)C * 3 * 9;
            for (int b = 1; b < nb; ++b) {
                residual_sums(wm, ext->scale ? ext->scale + (size_t)b * C : nullptr, rounded[b - 1], C, fl);
                wm += (size_t)C * C * 9;
            }
        }
        const size_t off_wft = fl.size();
        {
            const float *wf = ext->conv_w + (size_t)C * 3 * 9 + (size_t)(nb - 1) * C * C * 9;
            for (int k = 0; k < C * 9; ++k)          // k = c*9 + tap, the OIHW order within one output
                for (int o = 0; o < nbp; ++o)
                    fl.push_back(o < nbits ? wf[(size_t)o * C * 9 + k] * (c->final_affine ? ext->scale[(size_t)nb * C + o] : 1.f)
                                           : 0.f);
        }

        const size_t frag_bytes = align_up(frag.size() * 2);
        const size_t total = frag_bytes + align_up(fl.size() * 4);
        e = hipMalloc(&c->d_weights, total);
        if (e != hipSuccess) { delete c; return hip_fail(nullptr, e, "hipMalloc(weights)"); }
        e = hipMemcpy(c->d_weights, frag.data(), frag.size() * 2, hipMemcpyHostToDevice);
        if (e == hipSuccess)
            e = hipMemcpy((uint8_t *)c->d_weights + frag_bytes, fl.data(), fl.size() * 4, hipMemcpyHostToDevice);
        if (e != hipSuccess) { (void)hipFree(c->d_weights); delete c; return hip_fail(nullptr, e, "hipMemcpy(weights)"); }
        const bf16_t *fb = (const bf16_t *)c->d_weights;
        c->d_w_first = fb + frag_off[0];
        for (int b = 1; b < nb; ++b) c->d_w_mid.push_back(fb + frag_off[b]);
        c->d_w_final = fb + frag_off[nb];
        const float *flb = (const float *)((uint8_t *)c->d_weights + frag_bytes);
        c->d_bias = flb;
        c->d_bias_final = c->final_affine ? flb + off_fb : nullptr;
        c->d_lin_w = flb + off_lw;
        c->d_lin_b = flb + off_lb;
        c->d_rsum = flb + off_rs;
        c->d_wft = flb + off_wft;
    }
    if (rs) {
        c->has_rs = true;
        const int q = 1 << rs->m;
        e = hipMalloc(&c->d_tables, 1024);
        if (e != hipSuccess) { if (c->d_weights) (void)hipFree(c->d_weights); delete c; return hip_fail(nullptr, e, "hipMalloc(tables)"); }
        e = hipMemcpy(c->d_tables, exp2.data(), exp2.size(), hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMemcpy((uint8_t *)c->d_tables + 512, lg.data(), lg.size(), hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            (void)hipFree(c->d_tables);
            if (c->d_weights) (void)hipFree(c->d_weights);
            delete c;
            return hip_fail(nullptr, e, "hipMemcpy(tables)");
        }
        // alpha has order q - 1: only fcr mod (q - 1) matters, and the kernels multiply it by positions in 32 bits
        c->rs = RsParams{rs->m, q, rs->n, rs->k, rs->n - rs->k, rs->fcr % (q - 1), (const uint8_t *)c->d_tables,
                         (const uint8_t *)c->d_tables + 512};
    }
    *out = c;
    return QRM_OK;
}

void qrm_destroy(qrm_ctx *c)
{
    if (!c) return;
    (void)hipSetDevice(c->device);
    for (auto &sl : c->slots) {
        // the caller's stream may be gone by now: the event behind the workspace's last call is what is waited for
        if (sl.done) {
            if (sl.last_use) (void)hipEventSynchronize(sl.done);
            (void)hipEventDestroy(sl.done);
        }
        if (sl.ws) (void)hipFree(sl.ws);
    }
    for (auto &t : c->timed) {
        (void)hipEventDestroy(t.start);
        (void)hipEventDestroy(t.stop);
    }
    for (auto &ct : c->chunk_times)
        for (hipEvent_t ev : ct.ev)
            if (ev) (void)hipEventDestroy(ev);
    for (hipStream_t s : {c->s_up, c->s_run, c->s_down})
        if (s) (void)hipStreamSynchronize(s);
    for (auto &sg : c->stages) {
        if (sg.d_img) (void)hipFree(sg.d_img);
        if (sg.d_off) (void)hipFree(sg.d_off);
        if (sg.d_out) (void)hipFree(sg.d_out);
        for (hipEvent_t ev : {sg.uploaded, sg.computed, sg.downloaded})
            if (ev) (void)hipEventDestroy(ev);
    }
    for (hipStream_t s : {c->s_up, c->s_run, c->s_down})
        if (s) (void)hipStreamDestroy(s);
    if (c->d_weights) (void)hipFree(c->d_weights);
    if (c->d_tables) (void)hipFree(c->d_tables);
    delete c;
}

qrm_status qrm_release_stream(qrm_ctx *c, void *stream)
{
    if (!c) return QRM_E_INVALID;
    hipError_t e = hipSetDevice(c->device);
    if (e != hipSuccess) return hip_fail(c, e, "hipSetDevice");
    for (auto &sl : c->slots)
        if (sl.used && sl.stream == (hipStream_t)stream) {
            if (sl.done && sl.last_use) {
                e = hipEventSynchronize(sl.done);
                if (e != hipSuccess) return hip_fail(c, e, "hipEventSynchronize");
            }
            sl.used = false;
            sl.stream = nullptr;
            sl.last_use = 0; // idle: the next stream takes it without waiting
        }
    return QRM_OK;
}

qrm_status qrm_profile_enable(qrm_ctx *c, int32_t on)
{
    if (!c) return QRM_E_INVALID;
    c->profile = on != 0;
    c->timed_used = 0;
    return QRM_OK;
}

qrm_status qrm_profile_read(qrm_ctx *c, int32_t kind, double *ms_total, int64_t *launches, double *flops)
{
    if (!c) return QRM_E_INVALID;
    if (kind < 0 || kind >= QRM_PROFILE_KINDS) return fail(c, QRM_E_INVALID, "kind is one of the QRM_PROFILE_* values");
    double ms = 0.0, fl = 0.0;
    int64_t cnt = 0;
    for (size_t i = 0; i < c->timed_used; ++i) {
        const qrm_ctx::Timed &t = c->timed[i];
        if (t.kind != kind) continue;
        hipError_t e = hipEventSynchronize(t.stop);
        float dt = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&dt, t.start, t.stop);
        if (e != hipSuccess) return hip_fail(c, e, "hipEventElapsedTime");
        ms += dt;
        fl += t.flops;
        ++cnt;
    }
    if (ms_total) *ms_total = ms;
    if (launches) *launches = cnt;
    if (flops) *flops = fl;
    return QRM_OK;
}

qrm_status qrm_profile_read_chunks(qrm_ctx *c, int32_t max_chunks, double *ms, int32_t *n_chunks)
{
    if (!c) return QRM_E_INVALID;
    if (max_chunks < 0 || (max_chunks > 0 && !ms)) return fail(c, QRM_E_INVALID, "ms is NULL");
    const int n = (int)std::min<size_t>(c->chunks_timed, (size_t)max_chunks);
    if (n_chunks) *n_chunks = (int32_t)c->chunks_timed;
    if (n == 0) return QRM_OK;
    hipEvent_t base = c->chunk_times[0].ev[0];
    for (int i = 0; i < n; ++i)
        for (int k = 0; k < 5; ++k) {
            hipError_t e = hipEventSynchronize(c->chunk_times[i].ev[k]);
            float t = 0.f;
            if (e == hipSuccess) e = hipEventElapsedTime(&t, base, c->chunk_times[i].ev[k]);
            if (e != hipSuccess) return hip_fail(c, e, "hipEventElapsedTime");
            ms[i * 5 + k] = t;
        }
    return QRM_OK;
}

qrm_status qrm_set_micro_batch(qrm_ctx *c, int32_t images)
{
    if (!c) return QRM_E_INVALID;
    if (images < 0 || images > 65536) return fail(c, QRM_E_INVALID, "micro batch must be in 0..65536");
    c->micro_batch = images;
    return QRM_OK;
}

size_t qrm_workspace_bytes(const qrm_ctx *c, int64_t N, int32_t tile_h, int32_t tile_w)
{
    if (!c || N <= 0 || tile_h <= 0 || tile_w <= 0) return 0;
    return ws_layout(c, N, tile_h, tile_w, true).total;
}

qrm_status qrm_extract_tiles(qrm_ctx *c, const uint8_t *d_images, int64_t N, int32_t H, int32_t W,
                             const int32_t *d_off_yx, int32_t tile, uint8_t *d_tiles, void *stream)
{
    if (!c) return QRM_E_INVALID;
    if (N < 0) return fail(c, QRM_E_INVALID, "N < 0");
    if (tile <= 0 || H <= 0 || W <= 0 || tile > H || tile > W) return fail(c, QRM_E_INVALID, "need 0 < tile <= H, W");
    if (N == 0) return QRM_OK;
    if (!d_images || !d_tiles) return fail(c, QRM_E_INVALID, "d_images / d_tiles is NULL");
    hipError_t e = hipSetDevice(c->device);
    if (e != hipSuccess) return hip_fail(c, e, "hipSetDevice");
    e = launch_extract_tiles(d_images, N, H, W, d_off_yx, tile, d_tiles, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(c, e, "extract_tiles launch");
    return QRM_OK;
}

qrm_status qrm_preprocess(qrm_ctx *c, const uint8_t *d_raw, int64_t N, int32_t H_in, int32_t W_in, int32_t size,
                          const int32_t *d_off_yx, int32_t tile, uint8_t *d_out, void *stream)
{
    if (!c) return QRM_E_INVALID;
    if (N < 0) return fail(c, QRM_E_INVALID, "N < 0");
    if (H_in <= 0 || W_in <= 0 || size <= 0 || tile < 0 || tile > size)
        return fail(c, QRM_E_INVALID, "need H_in, W_in, size > 0 and 0 <= tile <= size");
    const int T = tile ? tile : size;
    if (!preprocess_supported(H_in, W_in, size, T))
        return fail(c, QRM_E_UNSUPPORTED, "raw and resized sides up to 16384, windows up to 1024 columns");
    if (N == 0) return QRM_OK;
    if (!d_raw || !d_out) return fail(c, QRM_E_INVALID, "d_raw / d_out is NULL");
    hipError_t e = hipSetDevice(c->device);
    if (e != hipSuccess) return hip_fail(c, e, "hipSetDevice");
    e = launch_preprocess(d_raw, N, H_in, W_in, size, tile ? d_off_yx : nullptr, T, d_out, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(c, e, "preprocess launch");
    return QRM_OK;
}

qrm_status qrm_select_tiles_variance(qrm_ctx *c, const uint8_t *d_images, int64_t N, int32_t H, int32_t W,
                                     int32_t tile, int32_t stride, int32_t *d_off_yx, double *d_scores, void *stream)
{
    if (!c) return QRM_E_INVALID;
    if (N < 0) return fail(c, QRM_E_INVALID, "N < 0");
    if (tile <= 0 || stride <= 0 || H <= 0 || W <= 0 || tile > H || tile > W)
        return fail(c, QRM_E_INVALID, "need 0 < tile <= H, W and stride > 0");
    if (!select_tiles_supported(H, W, tile, stride))
        return fail(c, QRM_E_UNSUPPORTED, "tile must be a multiple of stride, tile <= 512, stride <= 256, at most 1024 cells");
    if (N == 0) return QRM_OK;
    if (!d_images || !d_off_yx) return fail(c, QRM_E_INVALID, "d_images / d_off_yx is NULL");
    hipError_t e = hipSetDevice(c->device);
    if (e != hipSuccess) return hip_fail(c, e, "hipSetDevice");
    // the extractor sees channel c scaled by 1/std_c: its variance counts with the square of that
    double w[3] = {1.0, 1.0, 1.0};
    if (c->has_ext)
        for (int i = 0; i < 3; ++i) w[i] = (double)c->inv_std[i] * (double)c->inv_std[i];
    e = launch_select_tiles_variance(d_images, N, H, W, tile, stride, w, d_off_yx, d_scores, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(c, e, "select_tiles launch");
    return QRM_OK;
}

static qrm_status extractor_common(qrm_ctx *c, const uint8_t *d_tiles, int64_t N, int32_t h, int32_t w, int n_run,
                                   float *d_logits, uint8_t *d_bits, float *d_act, void *stream)
{
    if (!c) return QRM_E_INVALID;
    if (!c->has_ext) return fail(c, QRM_E_INVALID, "context has no extractor");
    if (N < 0) return fail(c, QRM_E_INVALID, "N < 0");
    if (h < 1 || w < 1 || h > 16384 || w > 16384) return fail(c, QRM_E_INVALID, "tile size out of range");
    if (N == 0) return QRM_OK;
    if (!d_tiles) return fail(c, QRM_E_INVALID, "d_tiles is NULL");
    hipError_t e = hipSetDevice(c->device);
    if (e != hipSuccess) return hip_fail(c, e, "hipSetDevice");
    hipStream_t s = (hipStream_t)stream;
    WsLayout L = ws_layout(c, N, h, w, false);
    if (L.mb < 1) return fail(c, QRM_E_UNSUPPORTED, "the activations of one tile exceed 1900 MiB");
    QrmSlot *slot = nullptr;
    qrm_status st = get_slot(c, s, L.total, &slot);
    if (st != QRM_OK) return st;
    TileSrc src{d_tiles, nullptr, h, w, {c->mean[0], c->mean[1], c->mean[2]},
                {c->inv_std[0], c->inv_std[1], c->inv_std[2]}};
    st = run_extractor(c, (uint8_t *)slot->ws, L, src, N, h, w, n_run, d_logits, d_bits, nullptr, 0, d_act, true, s);
    const qrm_status st2 = slot_done(c, slot, s); // also after an error: kernels may have been enqueued
    return st != QRM_OK ? st : st2;
}

qrm_status qrm_extractor_forward(qrm_ctx *c, const uint8_t *d_tiles, int64_t N, int32_t h, int32_t w,
                                 float *d_logits, uint8_t *d_bits, void *stream)
{
    if (c && N > 0 && !d_logits) return fail(c, QRM_E_INVALID, "d_logits is NULL");
    return extractor_common(c, d_tiles, N, h, w, -1, d_logits, d_bits, nullptr, stream);
}

qrm_status qrm_extractor_blocks(qrm_ctx *c, const uint8_t *d_tiles, int64_t N, int32_t h, int32_t w, int32_t n_run,
                                float *d_act, void *stream)
{
    if (c && c->has_ext && (n_run < 1 || n_run > c->n_blocks)) return fail(c, QRM_E_INVALID, "n_run out of range");
    if (c && N > 0 && !d_act) return fail(c, QRM_E_INVALID, "d_act is NULL");
    return extractor_common(c, d_tiles, N, h, w, n_run, nullptr, nullptr, d_act, stream);
}

qrm_status qrm_rs_decode(qrm_ctx *c, const uint8_t *d_symbols, int64_t N, uint8_t *d_msg, uint8_t *d_codeword,
                         int8_t *d_nerr, void *stream)
{
    if (!c) return QRM_E_INVALID;
    if (!c->has_rs) return fail(c, QRM_E_INVALID, "context has no Reed-Solomon code");
    if (N < 0) return fail(c, QRM_E_INVALID, "N < 0");
    if (N == 0) return QRM_OK;
    if (!d_symbols || !d_msg || !d_nerr) return fail(c, QRM_E_INVALID, "d_symbols / d_msg / d_nerr is NULL");
    hipError_t e = hipSetDevice(c->device);
    if (e != hipSuccess) return hip_fail(c, e, "hipSetDevice");
    e = launch_rs_decode(c->rs, d_symbols, N, d_msg, d_codeword, d_nerr, KeyArgs{}, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(c, e, "rs_decode launch");
    return QRM_OK;
}

int32_t qrm_key_threshold(int32_t n_bits, double fpr)
{
    if (n_bits < 1 || n_bits > 8 * 255 || !(fpr >= 0.0)) return -1;
    // Exact integer arithmetic: P(X >= tau) <= fpr  <=>  sum_{j >= tau} C(K,j) <= fpr * 2^K, and a double
    // is an integer times a power of two, so both sides are integers (after a common shift).
    const int K = n_bits;
    if (fpr >= 1.0) return 0;
    if (fpr == 0.0) return K + 1;
    int e2 = 0;
    const double fr = frexp(fpr, &e2);                       // fpr = fr * 2^e2, 0.5 <= fr < 1
    const uint64_t mant = (uint64_t)ldexp(fr, 53);           // fpr = mant * 2^(e2-53)
    const int sh = K + e2 - 53;                              // fpr * 2^K = mant * 2^sh
    Big rhs(mant), tail(0), term(1);                         // term = C(K,K)
    if (sh >= 0) rhs.shl(sh);
    int tau = K + 1;
    for (int j = K; j >= 0; --j) {
        tail.add(term);
        Big lhs = tail;
        if (sh < 0) lhs.shl(-sh);
        if (lhs.cmp(rhs) > 0) break;
        tau = j;
        term.mul_small((uint32_t)j);                         // C(K,j-1) = C(K,j) * j / (K-j+1), exactly
        term.div_small((uint32_t)(K - j + 1));
    }
    return tau;
}

qrm_status qrm_set_key(qrm_ctx *c, const uint8_t *h_key, int32_t tau)
{
    if (!c) return QRM_E_INVALID;
    if (!c->has_rs) return fail(c, QRM_E_INVALID, "context has no Reed-Solomon code");
    if (!h_key) return fail(c, QRM_E_INVALID, "h_key is NULL");
    if (tau < 0 || tau > c->rs.k * c->rs.m + 1) return fail(c, QRM_E_INVALID, "tau outside 0 .. k*m+1");
    hipError_t e = hipSetDevice(c->device);
    if (e != hipSuccess) return hip_fail(c, e, "hipSetDevice");
    uint8_t masked[256] = {0};
    for (int i = 0; i < c->rs.k; ++i) masked[i] = (uint8_t)(h_key[i] & (c->rs.q - 1));
    e = hipMemcpy((uint8_t *)c->d_tables + 768, masked, 256, hipMemcpyHostToDevice);
    if (e != hipSuccess) return hip_fail(c, e, "hipMemcpy(key)");
    c->has_key = true;
    c->key_tau = tau;
    return QRM_OK;
}

qrm_status qrm_verify_key(qrm_ctx *c, const uint8_t *d_msg, int64_t N, int32_t *d_matches, uint8_t *d_detected,
                          void *stream)
{
    if (!c) return QRM_E_INVALID;
    if (!c->has_rs || !c->has_key) return fail(c, QRM_E_INVALID, "context has no code or no key (qrm_set_key)");
    if (N < 0) return fail(c, QRM_E_INVALID, "N < 0");
    if (N == 0) return QRM_OK;
    if (!d_msg || !d_matches) return fail(c, QRM_E_INVALID, "d_msg / d_matches is NULL");
    hipError_t e = hipSetDevice(c->device);
    if (e != hipSuccess) return hip_fail(c, e, "hipSetDevice");
    const KeyArgs key{(const uint8_t *)c->d_tables + 768, c->key_tau, d_matches, d_detected};
    e = launch_verify(c->rs, d_msg, N, key, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(c, e, "verify launch");
    return QRM_OK;
}

} // extern "C"

namespace qrm {

qrm_status check_detect_args(qrm_ctx *c, const uint8_t *d_images, int64_t N, int32_t H, int32_t W, int32_t tile,
                             uint8_t *d_msg, int8_t *d_nerr, bool verify, int32_t *d_matches)
{
    if (!c->has_ext || !c->has_rs) return fail(c, QRM_E_INVALID, "context needs both an extractor and a code");
    if (verify && !c->has_key) return fail(c, QRM_E_INVALID, "context has no key (qrm_set_key)");
    if (verify && N > 0 && !d_matches) return fail(c, QRM_E_INVALID, "d_matches is NULL");
    if (c->n_bits != c->rs.n * c->rs.m) return fail(c, QRM_E_INVALID, "n_bits != n * m");
    if (N < 0) return fail(c, QRM_E_INVALID, "N < 0");
    if (tile <= 0 || H <= 0 || W <= 0 || tile > H || tile > W || H > 16384 || W > 16384)
        return fail(c, QRM_E_INVALID, "need 0 < tile <= H, W <= 16384");
    if (N > 0 && (!d_images || !d_msg || !d_nerr)) return fail(c, QRM_E_INVALID, "d_images / d_msg / d_nerr is NULL");
    return QRM_OK;
}

} // namespace qrm

static qrm_status detect_common(qrm_ctx *c, const uint8_t *d_images, int64_t N, int32_t H, int32_t W,
                                const int32_t *d_off_yx, int32_t tile, float *d_logits, uint8_t *d_bits,
                                uint8_t *d_msg, uint8_t *d_codeword, int8_t *d_nerr, bool verify, int32_t *d_matches,
                                uint8_t *d_detected, void *stream)
{
    if (!c) return QRM_E_INVALID;
    qrm_status st = check_detect_args(c, d_images, N, H, W, tile, d_msg, d_nerr, verify, d_matches);
    if (st != QRM_OK) return st;
    if (N == 0) return QRM_OK;
    hipError_t e = hipSetDevice(c->device);
    if (e != hipSuccess) return hip_fail(c, e, "hipSetDevice");
    hipStream_t s = (hipStream_t)stream;
    WsLayout L = ws_layout(c, N, tile, tile, true);
    if (L.mb < 1) return fail(c, QRM_E_UNSUPPORTED, "the activations of one tile exceed 1900 MiB");
    QrmSlot *slot = nullptr;
    st = get_slot(c, s, L.total, &slot);
    if (st != QRM_OK) return st;
    uint8_t *d_sym = (uint8_t *)slot->ws + symbols_offset(L);
    TileSrc src{d_images, d_off_yx, H, W, {c->mean[0], c->mean[1], c->mean[2]},
                {c->inv_std[0], c->inv_std[1], c->inv_std[2]}};
    st = run_extractor(c, (uint8_t *)slot->ws, L, src, N, tile, tile, -1, d_logits, d_bits, d_sym, c->rs.m, nullptr, true, s);
    if (st == QRM_OK) {
        KeyArgs key{};
        if (verify) key = KeyArgs{(const uint8_t *)c->d_tables + 768, c->key_tau, d_matches, d_detected};
        qrm_ctx::Timed *t = time_begin(c, true, QRM_PROFILE_RS_DECODE, 0.0, s);
        e = launch_rs_decode(c->rs, d_sym, N, d_msg, d_codeword, d_nerr, key, s);
        if (e != hipSuccess) st = hip_fail(c, e, "rs_decode launch");
        time_end(t, s);
    }
    const qrm_status st2 = slot_done(c, slot, s); // also after an error: kernels may have been enqueued
    return st != QRM_OK ? st : st2;
}

extern "C" {

qrm_status qrm_detect(qrm_ctx *c, const uint8_t *d_images, int64_t N, int32_t H, int32_t W, const int32_t *d_off_yx,
                      int32_t tile, float *d_logits, uint8_t *d_bits, uint8_t *d_msg, uint8_t *d_codeword,
                      int8_t *d_nerr, void *stream)
{
    return detect_common(c, d_images, N, H, W, d_off_yx, tile, d_logits, d_bits, d_msg, d_codeword, d_nerr, false,
                         nullptr, nullptr, stream);
}

qrm_status qrm_detect_verify(qrm_ctx *c, const uint8_t *d_images, int64_t N, int32_t H, int32_t W,
                             const int32_t *d_off_yx, int32_t tile, float *d_logits, uint8_t *d_bits, uint8_t *d_msg,
                             uint8_t *d_codeword, int8_t *d_nerr, int32_t *d_matches, uint8_t *d_detected,
                             void *stream)
{
    return detect_common(c, d_images, N, H, W, d_off_yx, tile, d_logits, d_bits, d_msg, d_codeword, d_nerr, true,
                         d_matches, d_detected, stream);
}

// Grows *p to at least `need` bytes (contents are not kept).
static qrm_status grow(qrm_ctx *c, void **p, size_t *have, size_t need, hipStream_t s)
{
    if (*have >= need) return QRM_OK;
    if (*p) {
        hipError_t e = hipStreamSynchronize(s);
        if (e != hipSuccess) return hip_fail(c, e, "hipStreamSynchronize");
        (void)hipFree(*p);
        *p = nullptr;
        *have = 0;
    }
    hipError_t e = hipMalloc(p, need);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(c, QRM_E_NOMEM, "staging buffer allocation failed");
    }
    *have = need;
    return QRM_OK;
}

qrm_status qrm_detect_host(qrm_ctx *c, const uint8_t *const *h_chunks, int32_t n_chunks, int32_t chunk_images, int32_t H,
                           int32_t W, const int32_t *const *h_off_chunks, int32_t tile, int32_t depth, uint8_t *h_msg,
                           uint8_t *h_codeword, int8_t *h_nerr)
{
    if (!c) return QRM_E_INVALID;
    if (!c->has_ext || !c->has_rs) return fail(c, QRM_E_INVALID, "context needs both an extractor and a code");
    if (n_chunks < 0 || chunk_images <= 0) return fail(c, QRM_E_INVALID, "need n_chunks >= 0 and chunk_images > 0");
    if (depth < 1 || depth > QRM_MAX_STREAMS) return fail(c, QRM_E_INVALID, "depth out of range");
    if (tile <= 0 || H <= 0 || W <= 0 || tile > H || tile > W || H > 16384 || W > 16384)
        return fail(c, QRM_E_INVALID, "need 0 < tile <= H, W <= 16384");
    if (c->n_bits != c->rs.n * c->rs.m) return fail(c, QRM_E_INVALID, "n_bits != n * m");
    if (n_chunks == 0) return QRM_OK;
    if (!h_chunks || !h_msg || !h_nerr) return fail(c, QRM_E_INVALID, "h_chunks / h_msg / h_nerr is NULL");
    for (int i = 0; i < n_chunks; ++i)
        if (!h_chunks[i] || (h_off_chunks && !h_off_chunks[i])) return fail(c, QRM_E_INVALID, "NULL chunk pointer");
    hipError_t e = hipSetDevice(c->device);
    if (e != hipSuccess) return hip_fail(c, e, "hipSetDevice");

    const size_t img_bytes = (size_t)chunk_images * 3 * H * W, off_bytes = (size_t)chunk_images * 2 * sizeof(int32_t);
    const int k = c->rs.k, n = c->rs.n;
    const size_t msg_bytes = (size_t)chunk_images * k, cw_bytes = (size_t)chunk_images * n;
    const size_t out_bytes = msg_bytes + cw_bytes + (size_t)chunk_images;
    const int used = depth < n_chunks ? depth : n_chunks;
    for (hipStream_t *s : {&c->s_up, &c->s_run, &c->s_down})
        if (!*s) {
            e = hipStreamCreateWithFlags(s, hipStreamNonBlocking); // default priority
            if (e != hipSuccess) return hip_fail(c, e, "hipStreamCreateWithFlags");
        }
    for (int j = 0; j < used; ++j) {
        qrm_ctx::Stage &sg = c->stages[j];
        for (hipEvent_t *ev : {&sg.uploaded, &sg.computed, &sg.downloaded})
            if (!*ev) {
                e = hipEventCreateWithFlags(ev, hipEventDisableTiming);
                if (e != hipSuccess) return hip_fail(c, e, "hipEventCreateWithFlags");
            }
        qrm_status st = grow(c, (void **)&sg.d_img, &sg.img_bytes, img_bytes, c->s_run);
        if (st == QRM_OK) st = grow(c, (void **)&sg.d_off, &sg.off_bytes, off_bytes, c->s_run);
        if (st == QRM_OK) st = grow(c, (void **)&sg.d_out, &sg.out_bytes, out_bytes, c->s_run);
        if (st != QRM_OK) return st;
    }
    // Three streams, one per role.  Uploads follow each other back to back on s_up (the link is the
    // scarce resource: it should never idle and never be shared by two copies); the kernels of chunk i
    // run on s_run once its upload is done; its results go home on s_down.  Chunk i uses staging buffer
    // i mod depth, which is free again when the kernels (input) and the download (output) of chunk
    // i - depth are done.  Copies of all streams pass through the copy engines in the order they were
    // submitted and a download waits for its kernels: the download of chunk i-1 is submitted after the
    // upload of chunk i, so that it never holds up an upload that could already run.
    qrm_status st = QRM_OK;
    // while profiling is on, five events per chunk: upload start / end, kernels start / end, download end
    const bool timeline = c->profile;
    c->chunks_timed = 0;
    if (timeline) {
        while (c->chunk_times.size() < (size_t)n_chunks) {
            qrm_ctx::ChunkTimes ct;
            for (hipEvent_t &ev : ct.ev) {
                e = hipEventCreate(&ev);
                if (e != hipSuccess) return hip_fail(c, e, "hipEventCreate");
            }
            c->chunk_times.push_back(ct);
        }
    }
    auto mark = [&](int i, int k, hipStream_t s) { if (timeline) (void)hipEventRecord(c->chunk_times[i].ev[k], s); };
    c->in_host_pipeline = true;
    auto download = [&](int i) -> hipError_t {
        qrm_ctx::Stage &sg = c->stages[i % used];
        const uint8_t *d_msg = sg.d_out, *d_cw = sg.d_out + msg_bytes, *d_ne = sg.d_out + msg_bytes + cw_bytes;
        hipError_t err = hipStreamWaitEvent(c->s_down, sg.computed, 0);
        if (err == hipSuccess)
            err = hipMemcpyAsync(h_msg + (size_t)i * msg_bytes, d_msg, msg_bytes, hipMemcpyDeviceToHost, c->s_down);
        if (err == hipSuccess && h_codeword)
            err = hipMemcpyAsync(h_codeword + (size_t)i * cw_bytes, d_cw, cw_bytes, hipMemcpyDeviceToHost, c->s_down);
        if (err == hipSuccess)
            err = hipMemcpyAsync(h_nerr + (size_t)i * chunk_images, d_ne, chunk_images, hipMemcpyDeviceToHost, c->s_down);
        if (err == hipSuccess) err = hipEventRecord(sg.downloaded, c->s_down);
        mark(i, 4, c->s_down);
        return err;
    };
    int submitted = 0; // chunks whose kernels are enqueued
    for (int i = 0; i < n_chunks && st == QRM_OK; ++i) {
        qrm_ctx::Stage &sg = c->stages[i % used];
        uint8_t *d_msg = sg.d_out, *d_cw = sg.d_out + msg_bytes;
        int8_t *d_ne = (int8_t *)(sg.d_out + msg_bytes + cw_bytes);
        e = hipSuccess;
        if (i >= used) e = hipStreamWaitEvent(c->s_up, sg.computed, 0); // the kernels of chunk i - depth have read d_img
        mark(i, 0, c->s_up);
        if (e == hipSuccess) e = hipMemcpyAsync(sg.d_img, h_chunks[i], img_bytes, hipMemcpyHostToDevice, c->s_up);
        if (e == hipSuccess && h_off_chunks)
            e = hipMemcpyAsync(sg.d_off, h_off_chunks[i], off_bytes, hipMemcpyHostToDevice, c->s_up);
        if (e == hipSuccess) e = hipEventRecord(sg.uploaded, c->s_up);
        mark(i, 1, c->s_up);
        if (e == hipSuccess) e = hipStreamWaitEvent(c->s_run, sg.uploaded, 0);
        if (e == hipSuccess && i >= used) e = hipStreamWaitEvent(c->s_run, sg.downloaded, 0); // d_out is free again
        mark(i, 2, c->s_run);
        if (e != hipSuccess) { st = hip_fail(c, e, "upload of a chunk"); break; }
        st = qrm_detect(c, sg.d_img, chunk_images, H, W, h_off_chunks ? sg.d_off : nullptr, tile, nullptr, nullptr, d_msg,
                        h_codeword ? d_cw : nullptr, d_ne, c->s_run);
        if (st != QRM_OK) break;
        e = hipEventRecord(sg.computed, c->s_run);
        if (e != hipSuccess) { st = hip_fail(c, e, "hipEventRecord"); break; }
        mark(i, 3, c->s_run);
        submitted = i + 1;
        // The download of a chunk must be submitted before the kernels of the next chunk that shares its
        // staging buffer (their wait on `downloaded` above refers to the event as recorded by then).  With
        // two or more buffers that is the chunk before this one, submitted behind this chunk's upload; with
        // a single buffer it is this chunk itself.
        const int due = used == 1 ? i : i - 1;
        if (due >= 0) {
            e = download(due);
            if (e != hipSuccess) st = hip_fail(c, e, "download of a chunk");
        }
    }
    if (st == QRM_OK && submitted >= 1 && used > 1) {
        e = download(submitted - 1);
        if (e != hipSuccess) st = hip_fail(c, e, "download of a chunk");
    }
    // the call returns when every chunk is done (also after an error: nothing of ours stays in flight)
    for (hipStream_t s : {c->s_up, c->s_run, c->s_down}) {
        e = hipStreamSynchronize(s);
        if (e != hipSuccess && st == QRM_OK) st = hip_fail(c, e, "hipStreamSynchronize");
    }
    c->in_host_pipeline = false;
    if (timeline && st == QRM_OK) c->chunks_timed = (size_t)submitted;
    return st;
}

} // extern "C"
