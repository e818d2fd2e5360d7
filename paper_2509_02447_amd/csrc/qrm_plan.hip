// Adaptive stream / micro-batch planner: host code only (Section 5, "Adaptive multi-channel horizontal
// fusion", Algorithm 1, with the cost model printed at the end of that section).
//
// A pipeline of K stages processes a global batch B; stage k took t[k] seconds for a baseline batch b0 on one
// stream during warm-up and holds u[k] bytes per sample.  On s streams a micro-batch of m samples is predicted
// to take t[k] / s * m / b0.  The planner hands the stream budget P to the stages one stream at a time, always
// where the bottleneck latency drops most, inside the memory cap, and then raises the micro-batch of stages
// that are much faster than the bottleneck.
//
// Readings where the algorithm leaves something open:
//  * the uniform micro-batch of step 1 is the largest m <= B whose one-stream-per-stage footprint fits;
//  * a candidate of the search must also keep sum s[k] <= P (the text's stream cap);
//  * of equally good candidates the first stage wins (strict comparison);
//  * "much faster than the bottleneck" means at most half of it, "memory allows" that the cap still holds
//    with the new micro-batch, and the micro-batch only ever grows (the bound min(m_unit, 2 m[k]) is
//    ignored when it lies below m[k]);
//  * the bottleneck the leveling compares with is the one the search ended on.
// Every expression is evaluated in double, left to right as written, without fused multiply-add: the integer
// decisions (which stage gets a stream, whether a micro-batch fits) depend on it.
#include <cstdint>
#include <vector>

#include "../../include/qrm.h"

#pragma clang fp contract(off)

namespace {

double stage_time(double t_k, int32_t s_k, int64_t m_k, int64_t b0)
{
    return t_k / (double)s_k * (double)m_k / (double)b0;
}

double memory_in_use(const std::vector<int32_t> &s, const std::vector<int64_t> &m, const double *u)
{
    double total = 0.0;
    for (size_t k = 0; k < s.size(); ++k) total = total + (double)((int64_t)s[k] * m[k]) * u[k];
    return total;
}

double bottleneck(const double *t, const std::vector<int32_t> &s, const std::vector<int64_t> &m, int64_t b0)
{
    double J = stage_time(t[0], s[0], m[0], b0);
    for (size_t k = 1; k < s.size(); ++k) {
        const double v = stage_time(t[k], s[k], m[k], b0);
        if (v > J) J = v;
    }
    return J;
}

} // namespace

extern "C" qrm_status qrm_plan_streams(int32_t n_stages, const double *h_t, const double *h_u, int64_t B, int64_t b0,
                                       int32_t P, double M_cap, double eps, int32_t tau, int32_t *h_s, int64_t *h_m,
                                       double *h_J, int32_t *h_accepted)
{
    const int32_t K = n_stages;
    if (K < 1 || K > QRM_PLAN_MAX_STAGES || !h_t || !h_u || !h_s || !h_m || B < 1 || b0 < 1 || P < K || tau < 1)
        return QRM_E_INVALID;
    if (B > (int64_t)1 << 40 || b0 > (int64_t)1 << 40 || P > 1 << 20) return QRM_E_INVALID; // (products stay exact)
    for (int32_t k = 0; k < K; ++k)
        if (!(h_t[k] > 0.0) || !(h_u[k] >= 0.0)) return QRM_E_INVALID; // (NaN fails both)
    if (!(eps >= 0.0) || !(M_cap >= 0.0)) return QRM_E_INVALID;

    // Step 1: one stream per stage, the largest uniform micro-batch that fits
    std::vector<int32_t> s(K, 1);
    std::vector<int64_t> m(K, 1);
    const double per_sample = memory_in_use(s, m, h_u);
    int64_t m0 = B;
    if (per_sample > 0.0 && M_cap / per_sample < (double)B) m0 = (int64_t)(M_cap / per_sample);
    auto uniform = [&](int64_t v) { for (auto &x : m) x = v; return memory_in_use(s, m, h_u); };
    while (m0 >= 1 && uniform(m0) > M_cap) --m0;
    while (m0 < B && uniform(m0 + 1) <= M_cap) ++m0;
    if (m0 < 1) return QRM_E_UNSUPPORTED; // not even one sample per stage fits the cap
    uniform(m0);
    double J = bottleneck(h_t, s, m, b0);
    int32_t stall = 0, accepted = 0;

    // Step 2: adaptive search
    while (stall < tau) {
        double gain = 0.0;
        int32_t best = -1;
        int64_t streams = 0;
        for (int32_t k = 0; k < K; ++k) streams += s[k];
        for (int32_t k = 0; k < K; ++k) {
            s[k] += 1;
            if (streams + 1 <= P && memory_in_use(s, m, h_u) <= M_cap) {
                const double delta = J - bottleneck(h_t, s, m, b0);
                if (delta > gain) {
                    gain = delta;
                    best = k;
                }
            }
            s[k] -= 1;
        }
        if (gain > eps) {
            s[best] += 1;
            J = bottleneck(h_t, s, m, b0);
            stall = 0;
            ++accepted;
        } else {
            ++stall;
        }
    }

    // Step 3: micro-batch leveling
    int64_t u_s = 0;
    for (int32_t k = 0; k < K; ++k) u_s += s[k];
    const int64_t m_unit = B / u_s > 1 ? B / u_s : 1;
    for (int32_t k = 0; k < K; ++k) {
        if (2.0 * stage_time(h_t[k], s[k], m[k], b0) <= J) {
            const int64_t m_new = m_unit < 2 * m[k] ? m_unit : 2 * m[k];
            if (m_new > m[k]) {
                const int64_t keep = m[k];
                m[k] = m_new;
                if (!(memory_in_use(s, m, h_u) <= M_cap)) m[k] = keep;
            }
        }
    }
    for (int32_t k = 0; k < K; ++k) {
        h_s[k] = s[k];
        h_m[k] = m[k];
    }
    if (h_J) *h_J = bottleneck(h_t, s, m, b0);
    if (h_accepted) *h_accepted = accepted;
    return QRM_OK;
}
