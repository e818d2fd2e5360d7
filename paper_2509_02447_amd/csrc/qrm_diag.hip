// Diagnostic entry points (include/qrm_diag.h): flags for A/B runs and a probe of the matrix pipes.  Bench and
// test tooling; nothing of the detection path lives here.
#include <math.h>

#include <vector>

#include "qrm_ctx.h"
#include "../../include/qrm_diag.h"

using namespace qrm;

namespace qrm {
namespace {

// What the matrix pipes sustain with nothing else going on.  Eight wavefronts per CU issue
// v_mfma_f32_32x32x16_bf16 back to back on four operand sets taken from `src` (8192 floats: 4096 for the A
// side, 4096 for the B side).  The clock of the part follows its power budget, and the power of a matrix
// instruction follows the data: zeros run at the published rate, random data do not.
__global__ __launch_bounds__(512) void matrix_rate_kernel(const float *__restrict__ src, int iters, float *__restrict__ out)
{
    bf16x8 a[4], b[4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a[s][i] = (bf16_t)src[((s * 8 + i) * 512 + threadIdx.x) % 4096];
            b[s][i] = (bf16_t)src[((s * 8 + i) * 512 + threadIdx.x) % 4096 + 4096];
        }
    f32x16 acc[4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[s][i] = 0.f;
#pragma unroll 1
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int s = 0; s < 4; ++s) acc[s] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s], b[s], acc[s], 0, 0, 0);
    }
    out[blockIdx.x * 512 + threadIdx.x] = acc[0][0] + acc[1][1] + acc[2][2] + acc[3][3];
}

hipError_t launch_matrix_rate(const float *src, int iters, int blocks, float *out, hipStream_t s)
{
    hipLaunchKernelGGL(matrix_rate_kernel, dim3(blocks), dim3(512), 0, s, src, iters, out);
    return hipGetLastError();
}

} // namespace
} // namespace qrm

extern "C" {

qrm_status qrm_diag_set_flags(qrm_ctx *c, int32_t flags)
{
    if (!c) return QRM_E_INVALID;
    if (flags & ~(QRM_DIAG_NO_FUSED_PAIRS | QRM_DIAG_POISON_WORKSPACE | QRM_DIAG_FUSE_ALWAYS | 0xFF00)) return fail(c, QRM_E_INVALID, "unknown diagnostic flag");
    c->diag_flags = flags;
    return QRM_OK;
}

qrm_status qrm_diag_matrix_rate(qrm_ctx *c, int32_t data, double *tflops)
{
    if (!c) return QRM_E_INVALID;
    if (data < 0 || data > 2 || !tflops) return fail(c, QRM_E_INVALID, "data is 0 (zeros), 1 (a constant) or 2 (random); tflops must not be NULL");
    hipError_t e = hipSetDevice(c->device);
    if (e != hipSuccess) return hip_fail(c, e, "hipSetDevice");
    // operands: A side like rounded weights (normal, small), B side like activations after a ReLU
    std::vector<float> h(8192);
    uint64_t state = 0x9E3779B97F4A7C15ull;
    auto uni = [&]() {
        state = state * 6364136223846793005ull + 1442695040888963407ull;
        return ((double)(state >> 11) + 1.0) / 9007199254740994.0;
    };
    for (int i = 0; i < 8192; ++i) {
        const double n = sqrt(-2.0 * log(uni())) * cos(6.283185307179586 * uni());
        h[i] = data == 0 ? 0.f : data == 1 ? 1.5f : (float)(i >= 4096 ? (n > 0 ? n : 0.0) : 0.06 * n);
    }
    const int blocks = c->num_cu, iters = 8000, reps = 3;
    float *d_src = nullptr, *d_out = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    e = hipMalloc((void **)&d_src, h.size() * 4);
    if (e == hipSuccess) e = hipMalloc((void **)&d_out, (size_t)blocks * 512 * 4);
    if (e == hipSuccess) e = hipMemcpy(d_src, h.data(), h.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    if (e == hipSuccess) e = launch_matrix_rate(d_src, iters, blocks, d_out, nullptr); // warm-up
    if (e == hipSuccess) e = hipEventRecord(e0, nullptr);
    for (int r = 0; r < reps && e == hipSuccess; ++r) e = launch_matrix_rate(d_src, iters, blocks, d_out, nullptr);
    if (e == hipSuccess) e = hipEventRecord(e1, nullptr);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (d_src) (void)hipFree(d_src);
    if (d_out) (void)hipFree(d_out);
    if (e != hipSuccess) return hip_fail(c, e, "matrix rate probe");
    const double flops = (double)reps * blocks * 8 * (double)iters * 4 * 32768.0; // 2 * 32 * 32 * 16 per instruction
    *tflops = flops / ((double)ms * 1e-3) / 1e12;
    return QRM_OK;
}


} // extern "C"
