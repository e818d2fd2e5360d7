// Batched bounded-distance Reed-Solomon decoding over GF(2^m) for gfx950.
//
// Function computed (Appendix B of the paper): for every received word, the unique codeword within
// t = (n-k)/2 symbol errors, the message in its first k symbols and the number of corrected symbols,
// or a failure flag.  The paper's decoder is Berlekamp-Welch on the CPU; this kernel reaches the same
// result through syndromes -> Berlekamp-Massey -> Chien search -> Forney.
//
// Mapping of the group kernel (short codes with t <= 2 use the lane-per-word kernel further down): a group of
// G lanes owns one codeword (G = 16 for n <= 16, so a 64-wide wavefront decodes four words; G = 64 otherwise, each lane then holds ceil(n/64) symbols).  Lane i of the group holds
// symbol i, i.e. the coefficient of x^(n-1-i).  Syndromes are XOR-reduced across the group (packed
// four per 32-bit word), the short serial Berlekamp-Massey recursion is replicated in every lane, and
// Chien search and Forney run one position per lane.  Log / antilog tables live in LDS.  No lane ever
// leaves the main path early, so cross-lane operations always see a full wavefront.
//
// Key verification (Section 4.3: the corrected message is compared with the predetermined key) rides in
// the decoder's epilogue when a key is given: every lane counts the bits of its message symbol that
// agree with the key's, the group adds the counts, lane 0 writes the count and (count >= tau).  The
// same count for messages already in memory is `verify_kernel`, a plain streaming pass.
#include "qrm_internal.h"

namespace qrm {

namespace {

struct Gf {
    const uint8_t *exp2; // LDS, alpha^i for i in [0, 2*ord)
    const uint8_t *log;  // LDS
    int ord;
    __device__ __forceinline__ int mul(int a, int b) const { return (a && b) ? exp2[log[a] + log[b]] : 0; }
    __device__ __forceinline__ int inv(int a) const { return exp2[ord - log[a]]; } // a != 0
    // a * alpha^e, 0 <= e < ord
    __device__ __forceinline__ int mul_pow(int a, int e) const { return a ? exp2[log[a] + e] : 0; }
};

template <int G>
__device__ __forceinline__ uint32_t group_xor(uint32_t v)
{
#pragma unroll
    for (int off = G / 2; off >= 1; off >>= 1) v ^= (uint32_t)__shfl_xor((int)v, off, G);
    return v;
}

template <int G>
__device__ __forceinline__ int group_count(bool pred, int lane)
{
    unsigned long long mask = __ballot(pred);
    if (G == 64) return __popcll(mask);
    int sh = (lane & 63) / G * G;
    return __popcll((mask >> sh) & ((1ull << G) - 1ull));
}

template <int G>
__device__ __forceinline__ int group_add(int v)
{
#pragma unroll
    for (int off = G / 2; off >= 1; off >>= 1) v += __shfl_xor(v, off, G);
    return v;
}

template <int G, int TMAX, int SPL>
__global__ __launch_bounds__(256) void rs_decode_kernel(RsParams p, const uint8_t *__restrict__ sym, int64_t N,
                                                        uint8_t *__restrict__ msg, uint8_t *__restrict__ cw,
                                                        int8_t *__restrict__ nerr, KeyArgs key)
{
    __shared__ uint8_t s_exp[512];
    __shared__ uint8_t s_log[256];
    __shared__ uint8_t s_key[256];
    const int tid = threadIdx.x;
    const int ord = p.q - 1;
    const bool with_key = key.matches != nullptr; // the same for every lane
    for (int i = tid; i < 2 * ord; i += 256) s_exp[i] = p.exp2[i];
    for (int i = tid; i < p.q; i += 256) s_log[i] = p.log[i];
    s_key[tid] = (with_key && tid < p.k) ? key.key[tid] : 0;
    __syncthreads();
    Gf gf{s_exp, s_log, ord};

    constexpr int GPB = 256 / G; // codewords per block per iteration
    const int lane_g = tid % G;
    const int n = p.n, k = p.k, two_t = p.two_t, t = p.two_t / 2;
    const int64_t stride = (int64_t)gridDim.x * GPB;
    const int64_t iters = (N + stride - 1) / stride; // same for every lane: no early exit

    for (int64_t it = 0; it < iters; ++it) {
        const int64_t w = it * stride + (int64_t)blockIdx.x * GPB + tid / G;
        const bool valid = w < N;

        // ---- load symbols, per-lane syndrome terms
        int r[SPL];
        uint32_t Spk[(2 * TMAX + 3) / 4];
#pragma unroll
        for (int j = 0; j < (2 * TMAX + 3) / 4; ++j) Spk[j] = 0;
#pragma unroll
        for (int s = 0; s < SPL; ++s) {
            const int i = lane_g + s * G;
            int v = 0;
            if (valid && i < n) v = sym[w * n + i] & (p.q - 1);
            r[s] = v;
            if (v) {
                const int lv = s_log[v];
                const int pw = n - 1 - i;         // this symbol multiplies x^pw, pw < ord
                int e = (p.fcr * pw) % ord;       // exponent of alpha^(fcr*pw)
#pragma unroll
                for (int j = 0; j < 2 * TMAX; ++j) {
                    if (j < two_t) Spk[j / 4] ^= (uint32_t)s_exp[lv + e] << (8 * (j % 4));
                    e += pw;
                    if (e >= ord) e -= ord;
                }
            }
        }
        int S[2 * TMAX];
#pragma unroll
        for (int j = 0; j < (2 * TMAX + 3) / 4; ++j) Spk[j] = group_xor<G>(Spk[j]);
#pragma unroll
        for (int j = 0; j < 2 * TMAX; ++j) S[j] = (Spk[j / 4] >> (8 * (j % 4))) & 0xff;

        // ---- Berlekamp-Massey (replicated in every lane of the group)
        int Lam[TMAX + 1], Bp[TMAX + 1];
#pragma unroll
        for (int i = 0; i <= TMAX; ++i) { Lam[i] = (i == 0); Bp[i] = (i == 0); }
        int L = 0;
#pragma unroll
        for (int rr = 0; rr < 2 * TMAX; ++rr) {
            if (rr < two_t) {
                int d = S[rr];
#pragma unroll
                for (int i = 1; i <= TMAX; ++i)
                    if (i <= rr && i <= L) d ^= gf.mul(Lam[i], S[rr - i]);
                // xB = x * B (top coefficient falls off only when the word is uncorrectable anyway)
                int xB[TMAX + 1];
                xB[0] = 0;
#pragma unroll
                for (int i = 1; i <= TMAX; ++i) xB[i] = Bp[i - 1];
                if (d == 0) {
#pragma unroll
                    for (int i = 0; i <= TMAX; ++i) Bp[i] = xB[i];
                } else {
                    const bool grow = 2 * L <= rr;
                    const int dinv = gf.inv(d);
#pragma unroll
                    for (int i = 0; i <= TMAX; ++i) {
                        const int old = Lam[i];
                        Lam[i] = old ^ gf.mul(d, xB[i]);
                        Bp[i] = grow ? gf.mul(dinv, old) : xB[i];
                    }
                    if (grow) L = rr + 1 - L;
                }
            }
        }
        bool fail = L > t;
        // degree of Lam must equal L
        {
            int top = 0;
#pragma unroll
            for (int i = 1; i <= TMAX; ++i)
                if (i == L) top = Lam[i];
            if (L > 0 && L <= t && top == 0) fail = true;
        }

        // ---- Omega = S(x) Lam(x) mod x^(2t)
        int Om[2 * TMAX];
#pragma unroll
        for (int i = 0; i < 2 * TMAX; ++i) {
            int o = 0;
#pragma unroll
            for (int j = 0; j <= TMAX; ++j)
                if (j <= i && j <= L) o ^= gf.mul(Lam[j], S[i - j]);
            Om[i] = (i < two_t) ? o : 0;
        }

        // ---- Chien search + Forney, one position per lane
        int ev[SPL];
        int nroots = 0;
        bool bad = false;
#pragma unroll
        for (int s = 0; s < SPL; ++s) {
            const int i = lane_g + s * G;
            const int pw = n - 1 - i;
            const bool in_word = i < n;
            const int xe = in_word ? (pw == 0 ? 0 : ord - pw) : 0; // exponent of X^-1 = alpha^-pw
            int lam_x = Lam[0], den = 0, num = Om[0];
            int e = 0;                                            // exponent of X^-j, built incrementally
#pragma unroll
            for (int j = 1; j < 2 * TMAX; ++j) {
                e += xe;
                if (e >= ord) e -= ord;
                if (j <= TMAX) {
                    if (j <= L) lam_x ^= gf.mul_pow(Lam[j], e);
                }
                if (j < two_t) num ^= gf.mul_pow(Om[j], e);
            }
            // Lam'(x) = sum over odd j of Lam[j] x^(j-1)
            e = 0;
#pragma unroll
            for (int j = 1; j <= TMAX; ++j) {
                if ((j & 1) && j <= L) den ^= gf.mul_pow(Lam[j], e);
                e += xe;
                if (e >= ord) e -= ord;
            }
            const bool root = in_word && !fail && L > 0 && lam_x == 0;
            nroots += group_count<G>(root, tid);
            int val = 0;
            if (root) {
                if (den == 0) {
                    bad = true;
                } else {
                    val = gf.mul(num, gf.inv(den));
                    // times X^(1-fcr) = alpha^(pw*(1-fcr))
                    int ex = (pw * (1 - p.fcr)) % ord;
                    if (ex < 0) ex += ord;
                    val = gf.mul_pow(val, ex);
                    if (val == 0) bad = true;
                }
            }
            ev[s] = val;
        }
        if (nroots != L) fail = true;
        if (group_count<G>(bad, tid) != 0) fail = true;

        // ---- write back
        int agree = 0;
#pragma unroll
        for (int s = 0; s < SPL; ++s) {
            const int i = lane_g + s * G;
            if (valid && i < n) {
                const uint8_t out = (uint8_t)(fail ? r[s] : (r[s] ^ ev[s]));
                if (cw) cw[w * n + i] = out;
                if (i < k) {
                    msg[w * k + i] = out;
                    agree += p.m - __popc((unsigned)(out ^ s_key[i]) & (unsigned)(p.q - 1));
                }
            }
        }
        if (valid && lane_g == 0) nerr[w] = (int8_t)(fail ? -1 : L);
        if (with_key) {
            agree = group_add<G>(agree);
            if (valid && lane_g == 0) {
                key.matches[w] = agree;
                if (key.detected) key.detected[w] = (uint8_t)(agree >= key.tau);
            }
        }
    }
}

// Short codes (n <= 16): one word per LANE.  The group kernel above repeats the serial recursion of
// Berlekamp-Massey on all lanes of a word and is bound by the vector ALUs; here nothing is repeated: a lane reads
// its word (adjacent lanes read adjacent words), forms the 2t syndromes (exponents are the same for all lanes,
// so they live in scalar registers), runs the recursion once, evaluates the locator at the n positions, and does
// Forney only at the (at most t) roots it found.  Same decisions, same outputs as the group kernel.
template <int TMAX>
__global__ __launch_bounds__(256) void rs_decode_lane_kernel(RsParams p, const uint8_t *__restrict__ sym, int64_t N,
                                                             uint8_t *__restrict__ msg, uint8_t *__restrict__ cw,
                                                             int8_t *__restrict__ nerr, KeyArgs key)
{
    constexpr int NMAX = 16;
    __shared__ uint8_t s_exp[512];
    __shared__ uint8_t s_log[256];
    __shared__ uint8_t s_key[256];
    const int tid = threadIdx.x;
    const int ord = p.q - 1;
    const bool with_key = key.matches != nullptr; // the same for every lane
    for (int i = tid; i < 2 * ord; i += 256) s_exp[i] = p.exp2[i];
    for (int i = tid; i < p.q; i += 256) s_log[i] = p.log[i];
    s_key[tid] = (with_key && tid < p.k) ? key.key[tid] : 0;
    __syncthreads();
    Gf gf{s_exp, s_log, ord};
    const int n = p.n, k = p.k, two_t = p.two_t, t = p.two_t / 2;
    const int64_t w = (int64_t)blockIdx.x * 256 + tid;
    if (w >= N) return; // no cross-lane operation below
    const uint8_t *src = sym + w * n;

    // ---- symbols and syndromes
    int r[NMAX];
    int S[2 * TMAX];
#pragma unroll
    for (int j = 0; j < 2 * TMAX; ++j) S[j] = 0;
#pragma unroll
    for (int i = 0; i < NMAX; ++i) {
        r[i] = 0;
        if (i < n) {
            const int v = src[i] & (p.q - 1);
            r[i] = v;
            const int pw = n - 1 - i;       // this symbol multiplies x^pw, pw < ord
            int e = (p.fcr * pw) % ord;     // exponent of alpha^(fcr*pw): the same in every lane
            const int lv = s_log[v];
#pragma unroll
            for (int j = 0; j < 2 * TMAX; ++j) {
                if (j < two_t) S[j] ^= v ? s_exp[lv + e] : 0;
                e += pw;
                if (e >= ord) e -= ord;
            }
        }
    }

    // ---- Berlekamp-Massey
    int Lam[TMAX + 1], Bp[TMAX + 1];
#pragma unroll
    for (int i = 0; i <= TMAX; ++i) { Lam[i] = (i == 0); Bp[i] = (i == 0); }
    int L = 0;
#pragma unroll
    for (int rr = 0; rr < 2 * TMAX; ++rr) {
        if (rr < two_t) {
            int d = S[rr];
#pragma unroll
            for (int i = 1; i <= TMAX; ++i)
                if (i <= rr && i <= L) d ^= gf.mul(Lam[i], S[rr - i]);
            int xB[TMAX + 1];
            xB[0] = 0;
#pragma unroll
            for (int i = 1; i <= TMAX; ++i) xB[i] = Bp[i - 1];
            const bool grow = d != 0 && 2 * L <= rr;
            const int dinv = d ? gf.inv(d) : 0;
#pragma unroll
            for (int i = 0; i <= TMAX; ++i) {
                const int old = Lam[i];
                Lam[i] = old ^ gf.mul(d, xB[i]);              // d = 0: unchanged
                Bp[i] = grow ? gf.mul(dinv, old) : xB[i];
            }
            if (grow) L = rr + 1 - L;
        }
    }
    bool fail = L > t;
    {
        int top = 0;
#pragma unroll
        for (int i = 1; i <= TMAX; ++i)
            if (i == L) top = Lam[i];
        if (L > 0 && L <= t && top == 0) fail = true;
    }

    // ---- Omega = S(x) Lam(x) mod x^(2t)
    int Om[2 * TMAX];
#pragma unroll
    for (int i = 0; i < 2 * TMAX; ++i) {
        int o = 0;
#pragma unroll
        for (int j = 0; j <= TMAX; ++j)
            if (j <= i && j <= L) o ^= gf.mul(Lam[j], S[i - j]);
        Om[i] = (i < two_t) ? o : 0;
    }

    // ---- Chien search over the n positions (exponents are the same in every lane), roots remembered
    int lamlog[TMAX + 1];
#pragma unroll
    for (int j = 1; j <= TMAX; ++j) lamlog[j] = s_log[Lam[j]];
    int nroots = 0;
    int rootpos[TMAX];
#pragma unroll
    for (int q2 = 0; q2 < TMAX; ++q2) rootpos[q2] = 0;
#pragma unroll
    for (int i = 0; i < NMAX; ++i) {
        if (i < n) {
            const int pw = n - 1 - i;
            const int xe = pw == 0 ? 0 : ord - pw; // exponent of X^-1 = alpha^-pw
            int lam_x = Lam[0];
            int e = 0;
#pragma unroll
            for (int j = 1; j <= TMAX; ++j) {
                e += xe;
                if (e >= ord) e -= ord;
                if (j <= L && Lam[j]) lam_x ^= s_exp[lamlog[j] + e];
            }
            const bool root = !fail && L > 0 && lam_x == 0;
            if (root) {
#pragma unroll
                for (int q2 = 0; q2 < TMAX; ++q2)
                    if (q2 == nroots) rootpos[q2] = i;
                ++nroots;
            }
        }
    }
    if (nroots != L) fail = true;

    // ---- Forney at the roots
    int evpos[TMAX], evval[TMAX];
#pragma unroll
    for (int q2 = 0; q2 < TMAX; ++q2) {
        evpos[q2] = -1;
        evval[q2] = 0;
        if (!fail && q2 < nroots && q2 < L) {
            const int i = rootpos[q2];
            const int pw = n - 1 - i;
            const int xe = pw == 0 ? 0 : ord - pw;
            int num = Om[0], den = 0;
            int e = 0;
#pragma unroll
            for (int j = 1; j < 2 * TMAX; ++j) {
                e += xe;
                if (e >= ord) e -= ord;
                if (j < two_t) num ^= gf.mul_pow(Om[j], e);
            }
            e = 0;
#pragma unroll
            for (int j = 1; j <= TMAX; ++j) {
                if ((j & 1) && j <= L) den ^= gf.mul_pow(Lam[j], e);
                e += xe;
                if (e >= ord) e -= ord;
            }
            int val = 0;
            if (den != 0) {
                val = gf.mul(num, gf.inv(den));
                int ex = (pw * (1 - p.fcr)) % ord;
                if (ex < 0) ex += ord;
                val = gf.mul_pow(val, ex);
            }
            if (val == 0) fail = true; // zero denominator or zero error value: not a valid correction
            evpos[q2] = i;
            evval[q2] = val;
        }
    }

    // ---- write back
    int agree = 0;
#pragma unroll
    for (int i = 0; i < NMAX; ++i) {
        if (i < n) {
            int out = r[i];
            if (!fail) {
#pragma unroll
                for (int q2 = 0; q2 < TMAX; ++q2)
                    if (evpos[q2] == i) out ^= evval[q2];
            }
            if (cw) cw[w * n + i] = (uint8_t)out;
            if (i < k) {
                msg[w * k + i] = (uint8_t)out;
                agree += p.m - __popc((unsigned)(out ^ s_key[i]) & (unsigned)(p.q - 1));
            }
        }
    }
    nerr[w] = (int8_t)(fail ? -1 : L);
    if (with_key) {
        key.matches[w] = agree;
        if (key.detected) key.detected[w] = (uint8_t)(agree >= key.tau);
    }
}

// Agreement of stored messages with the key: one word per lane, V bytes of it per load.
template <typename V>
__global__ __launch_bounds__(256) void verify_kernel(const uint8_t *__restrict__ msg, int64_t N, int k, int m,
                                                     KeyArgs key)
{
    __shared__ V s_key[256 / sizeof(V)];
    const int per = k / (int)sizeof(V);
    if ((int)threadIdx.x < per) s_key[threadIdx.x] = reinterpret_cast<const V *>(key.key)[threadIdx.x];
    __syncthreads();
    V mask = 0;
#pragma unroll
    for (int b = 0; b < (int)sizeof(V); ++b) mask |= (V)((1u << m) - 1u) << (8 * b);
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x; w < N; w += stride) {
        const V *src = reinterpret_cast<const V *>(msg + w * k);
        int differ = 0;
        for (int j = 0; j < per; ++j) differ += __popcll((unsigned long long)((src[j] ^ s_key[j]) & mask));
        const int agree = k * m - differ;
        key.matches[w] = agree;
        if (key.detected) key.detected[w] = (uint8_t)(agree >= key.tau);
    }
}

template <int G, int TMAX, int SPL>
hipError_t launch_one(const RsParams &p, const uint8_t *sym, int64_t N, uint8_t *msg, uint8_t *cw, int8_t *nerr,
                      const KeyArgs &key, hipStream_t s)
{
    constexpr int GPB = 256 / G;
    int64_t blocks = (N + GPB - 1) / GPB;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL((rs_decode_kernel<G, TMAX, SPL>), dim3((unsigned)blocks), dim3(256), 0, s, p, sym, N, msg, cw,
                       nerr, key);
    return hipGetLastError();
}

template <int TMAX>
hipError_t launch_t(const RsParams &p, const uint8_t *sym, int64_t N, uint8_t *msg, uint8_t *cw, int8_t *nerr,
                    const KeyArgs &key, hipStream_t s)
{
    if constexpr (TMAX <= 2) if (p.n <= 16) { // short codes: one word per lane
        const int64_t blocks = (N + 255) / 256;
        const int64_t kMaxGrid = 1LL << 30;
        for (int64_t b0 = 0; b0 < blocks; b0 += kMaxGrid) {
            const int64_t cnt = blocks - b0 < kMaxGrid ? blocks - b0 : kMaxGrid;
            const int64_t w0 = b0 * 256;
            KeyArgs k2 = key;
            if (k2.matches) k2.matches += w0;
            if (k2.detected) k2.detected += w0;
            hipLaunchKernelGGL(rs_decode_lane_kernel<TMAX>, dim3((unsigned)cnt), dim3(256), 0, s, p, sym + w0 * p.n,
                               N - w0, msg + w0 * p.k, cw ? cw + w0 * p.n : nullptr, nerr + w0, k2);
        }
        return hipGetLastError();
    }
    if (p.n <= 16) return launch_one<16, TMAX, 1>(p, sym, N, msg, cw, nerr, key, s);
    if (p.n <= 64) return launch_one<64, TMAX, 1>(p, sym, N, msg, cw, nerr, key, s);
    if (p.n <= 128) return launch_one<64, TMAX, 2>(p, sym, N, msg, cw, nerr, key, s);
    return launch_one<64, TMAX, 4>(p, sym, N, msg, cw, nerr, key, s);
}

} // namespace

hipError_t launch_rs_decode(const RsParams &p, const uint8_t *sym, int64_t N, uint8_t *msg, uint8_t *cw, int8_t *nerr,
                            const KeyArgs &key, hipStream_t s)
{
    if (N <= 0) return hipSuccess;
    const int t = p.two_t / 2;
    if (t <= 2) return launch_t<2>(p, sym, N, msg, cw, nerr, key, s);
    if (t <= 4) return launch_t<4>(p, sym, N, msg, cw, nerr, key, s);
    return launch_t<8>(p, sym, N, msg, cw, nerr, key, s);
}

hipError_t launch_verify(const RsParams &p, const uint8_t *msg, int64_t N, const KeyArgs &key, hipStream_t s)
{
    if (N <= 0) return hipSuccess;
    int64_t blocks = (N + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    const dim3 grid((unsigned)blocks), block(256);
    // wide loads need every word (and the key) to start on a multiple of the load width
    const uintptr_t a = (uintptr_t)msg | (uintptr_t)key.key;
    if (p.k % 8 == 0 && a % 8 == 0)
        hipLaunchKernelGGL(verify_kernel<uint64_t>, grid, block, 0, s, msg, N, p.k, p.m, key);
    else if (p.k % 4 == 0 && a % 4 == 0)
        hipLaunchKernelGGL(verify_kernel<uint32_t>, grid, block, 0, s, msg, N, p.k, p.m, key);
    else
        hipLaunchKernelGGL(verify_kernel<uint8_t>, grid, block, 0, s, msg, N, p.k, p.m, key);
    return hipGetLastError();
}

} // namespace qrm
