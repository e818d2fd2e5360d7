/*
 * CPU oracle for batched watermark detection.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of what the detection path
 * computes: tile crop, per-channel normalisation, a 3x3 convolutional
 * bit-extractor in fp64, hard-bit thresholding, bit->symbol packing and
 * bounded-distance Reed-Solomon decoding over GF(2^m).  It shares no code with
 * the HIP library and must never be called from the product path; only tests,
 * the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * What follows the paper and what is a reading of it:
 *   - detection flow (Section 4.3): one l x l tile of the image goes through
 *     the extractor H_D, the raw bits are RS-corrected;
 *   - hard bit = sign of the soft bit (Section 4.1); here bit = (logit > 0);
 *   - RS notation (Appendix B, "Notation"): (n,k,t), t = floor((n-k)/2),
 *     m-bit symbols, n <= 2^m - 1; the decoder returns corrected message,
 *     corrected codeword and the number of symbol errors corrected
 *     (Appendix B, end of "Berlekamp-Welch Decoding");
 *   - the paper decodes with Berlekamp-Welch; this oracle implements the same
 *     function (unique codeword within Hamming distance t of the received
 *     word, else failure) through the syndrome / Berlekamp-Massey / Chien /
 *     Forney chain on the narrow-sense BCH view of the code.  Both are
 *     bounded-distance decoders of the same code, so they agree on every
 *     input; the tests pin this against an exhaustive nearest-codeword search.
 *   - conventions where the paper is silent: bits are packed MSB first; symbol 0
 *     is the highest-degree coefficient; message first, parity last; a shortened
 *     code drops the highest powers; the field generator is alpha = x (= 2).
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py against
 * closed forms, exhaustive search, textbook values or an independent library
 * routine; the bit order / symbol order convention alone is self-consistent
 * only ("parity unpinned" against any external system).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_MAXQ 256
#define ORC_MAX2T 254

typedef struct {
    int m, q, n, k, two_t, fcr;
    int exp[2 * ORC_MAXQ]; /* exp[i] = alpha^i, i in [0, 2(q-1)) */
    int log[ORC_MAXQ];     /* log[alpha^i] = i, log[0] unused */
} orc_rs;

/* ---------------------------------------------------------------- field */

static int gf_mul(const orc_rs *f, int a, int b)
{
    if (a == 0 || b == 0) return 0;
    return f->exp[f->log[a] + f->log[b]];
}

static int gf_inv(const orc_rs *f, int a) /* a != 0 */
{
    return f->exp[(f->q - 1 - f->log[a]) % (f->q - 1)];
}

static int gf_alpha_pow(const orc_rs *f, long e)
{
    long ord = f->q - 1;
    e %= ord;
    if (e < 0) e += ord;
    return f->exp[e];
}

/* returns 0 on success */
int orc_rs_init(orc_rs *f, int m, unsigned prim_poly, int n, int k, int fcr)
{
    if (m < 2 || m > 8) return 1;
    int q = 1 << m;
    if (n > q - 1 || k <= 0 || k >= n || ((n - k) & 1) || fcr < 0) return 1;
    f->m = m; f->q = q; f->n = n; f->k = k; f->two_t = n - k; f->fcr = fcr;
    memset(f->log, 0, sizeof f->log);
    int x = 1;
    for (int i = 0; i < q - 1; i++) {
        if (i > 0 && x == 1) return 2; /* alpha has order < q-1: polynomial not primitive */
        f->exp[i] = x;
        f->exp[i + q - 1] = x;
        f->log[x] = i;
        x <<= 1;
        if (x & q) x ^= (int)prim_poly;
    }
    if (x != 1) return 2; /* alpha is not primitive for this polynomial */
    return 0;
}

/* tables out, for the tests */
int orc_gf_tables(int m, unsigned prim_poly, int32_t *exp_out /*[2^m-1]*/, int32_t *log_out /*[2^m]*/)
{
    orc_rs f;
    int rc = orc_rs_init(&f, m, prim_poly, (1 << m) - 1, (1 << m) - 3, 1);
    if (rc) return rc;
    for (int i = 0; i < f.q - 1; i++) exp_out[i] = f.exp[i];
    for (int i = 0; i < f.q; i++) log_out[i] = i ? f.log[i] : -1;
    return 0;
}

int orc_gf_mul(int m, unsigned prim_poly, int a, int b)
{
    orc_rs f;
    if (orc_rs_init(&f, m, prim_poly, (1 << m) - 1, (1 << m) - 3, 1)) return -1;
    return gf_mul(&f, a, b);
}

/* ---------------------------------------------------------------- encoder */

/* g(x) = prod_{j=0}^{2t-1} (x - alpha^{fcr+j}); g[i] = coefficient of x^i, g[2t] = 1 */
static void rs_generator(const orc_rs *f, int *g)
{
    int two_t = f->two_t;
    memset(g, 0, sizeof(int) * (two_t + 1));
    g[0] = 1;
    for (int j = 0; j < two_t; j++) {
        int root = gf_alpha_pow(f, f->fcr + j);
        /* g <- g * (x + root) */
        for (int i = j + 1; i >= 1; i--) g[i] = g[i - 1] ^ gf_mul(f, g[i], root);
        g[0] = gf_mul(f, g[0], root);
    }
}

int orc_rs_generator(int m, unsigned prim_poly, int n, int k, int fcr, int32_t *g_out /*[n-k+1]*/)
{
    orc_rs f;
    int g[ORC_MAX2T + 1];
    int rc = orc_rs_init(&f, m, prim_poly, n, k, fcr);
    if (rc) return rc;
    rs_generator(&f, g);
    for (int i = 0; i <= f.two_t; i++) g_out[i] = g[i];
    return 0;
}

/* Systematic encoding: codeword(x) = msg(x) x^{2t} + (msg(x) x^{2t} mod g(x)).
 * Symbol 0 is the coefficient of x^{n-1}. */
static void rs_encode_one(const orc_rs *f, const int *g, const uint8_t *msg, uint8_t *cw)
{
    int n = f->n, k = f->k, two_t = f->two_t;
    int rem[ORC_MAXQ];
    /* dividend, highest power first: rem[i] is the coefficient of x^{n-1-i} */
    for (int i = 0; i < n; i++) rem[i] = i < k ? (msg[i] & (f->q - 1)) : 0;
    for (int i = 0; i < k; i++) {           /* long division by the monic g */
        int lead = rem[i];
        if (lead == 0) continue;
        for (int j = 0; j <= two_t; j++)    /* subtract lead * x^{..} * g */
            rem[i + j] ^= gf_mul(f, lead, g[two_t - j]);
    }
    for (int i = 0; i < k; i++) cw[i] = msg[i] & (f->q - 1);
    for (int i = k; i < n; i++) cw[i] = (uint8_t)rem[i];
}

int orc_rs_encode(int m, unsigned prim_poly, int n, int k, int fcr,
                  const uint8_t *msgs, int64_t count, uint8_t *cws)
{
    orc_rs f;
    int g[ORC_MAX2T + 1];
    int rc = orc_rs_init(&f, m, prim_poly, n, k, fcr);
    if (rc) return rc;
    rs_generator(&f, g);
    for (int64_t i = 0; i < count; i++) rs_encode_one(&f, g, msgs + i * k, cws + i * n);
    return 0;
}

/* ---------------------------------------------------------------- decoder */

/* S[j] = r(alpha^{fcr+j}), j = 0..2t-1, with r(x) = sum_i sym[i] x^{n-1-i} */
static void rs_syndromes(const orc_rs *f, const uint8_t *sym, int *S)
{
    for (int j = 0; j < f->two_t; j++) {
        int s = 0;
        for (int i = 0; i < f->n; i++) {
            int r = sym[i] & (f->q - 1);
            s ^= gf_mul(f, r, gf_alpha_pow(f, (long)(f->fcr + j) * (f->n - 1 - i)));
        }
        S[j] = s;
    }
}

int orc_rs_syndromes(int m, unsigned prim_poly, int n, int k, int fcr,
                     const uint8_t *syms, int64_t count, uint8_t *S_out /*[count, n-k]*/)
{
    orc_rs f;
    int S[ORC_MAX2T];
    int rc = orc_rs_init(&f, m, prim_poly, n, k, fcr);
    if (rc) return rc;
    for (int64_t i = 0; i < count; i++) {
        rs_syndromes(&f, syms + i * n, S);
        for (int j = 0; j < f.two_t; j++) S_out[i * f.two_t + j] = (uint8_t)S[j];
    }
    return 0;
}

static int poly_eval(const orc_rs *f, const int *p, int deg, int x)
{
    int y = 0;
    for (int i = deg; i >= 0; i--) y = gf_mul(f, y, x) ^ p[i]; /* Horner */
    return y;
}

/* Bounded-distance decoding.  Returns the number of corrected symbols (0..t) or -1.
 * On failure msg/cw are the received symbols unchanged. */
static int rs_decode_one(const orc_rs *f, const uint8_t *recv, uint8_t *msg, uint8_t *cw)
{
    int n = f->n, k = f->k, two_t = f->two_t, t = two_t / 2;
    int S[ORC_MAX2T];
    uint8_t work[ORC_MAXQ];
    for (int i = 0; i < n; i++) work[i] = recv[i] & (f->q - 1);

#define ORC_FAIL() do { \
        for (int i_ = 0; i_ < n; i_++) { uint8_t v_ = recv[i_] & (f->q - 1); \
            if (cw) cw[i_] = v_; if (i_ < k) msg[i_] = v_; } \
        return -1; } while (0)

    rs_syndromes(f, work, S);
    int any = 0;
    for (int j = 0; j < two_t; j++) any |= S[j];
    if (!any) {
        for (int i = 0; i < n; i++) { if (cw) cw[i] = work[i]; if (i < k) msg[i] = work[i]; }
        return 0;
    }

    /* Berlekamp-Massey: shortest LFSR (connection polynomial Lam, length L) generating S */
    int Lam[ORC_MAX2T + 2], B[ORC_MAX2T + 2], T[ORC_MAX2T + 2];
    memset(Lam, 0, sizeof Lam); memset(B, 0, sizeof B);
    Lam[0] = 1; B[0] = 1;
    int L = 0, shift = 1, b = 1;
    for (int r = 0; r < two_t; r++) {
        int d = S[r];
        for (int i = 1; i <= L; i++) d ^= gf_mul(f, Lam[i], S[r - i]);
        if (d == 0) {
            shift++;
        } else {
            int coef = gf_mul(f, d, gf_inv(f, b));
            memcpy(T, Lam, sizeof Lam);
            for (int i = 0; i + shift <= two_t; i++) Lam[i + shift] ^= gf_mul(f, coef, B[i]);
            if (2 * L <= r) {
                L = r + 1 - L;
                memcpy(B, T, sizeof B);
                b = d;
                shift = 1;
            } else {
                shift++;
            }
        }
    }
    if (L > t) ORC_FAIL();
    if (Lam[L] == 0) ORC_FAIL(); /* degree below L: cannot have L roots */

    /* Chien search: error at power p (symbol index n-1-p) iff Lam(alpha^{-p}) = 0 */
    int pos[ORC_MAX2T], nroots = 0;
    for (int p = 0; p < n; p++) {
        if (poly_eval(f, Lam, L, gf_alpha_pow(f, -p)) == 0) {
            if (nroots < L) pos[nroots] = p;
            nroots++;
        }
    }
    if (nroots != L) ORC_FAIL();

    /* Forney: Omega = S(x) Lam(x) mod x^{2t}, S(x) = sum_j S[j] x^j;
     * e_p = X_p^{1-fcr} Omega(X_p^{-1}) / Lam'(X_p^{-1}),  X_p = alpha^p */
    int Om[ORC_MAX2T];
    for (int i = 0; i < two_t; i++) {
        int o = 0;
        for (int j = 0; j <= i && j <= L; j++) o ^= gf_mul(f, Lam[j], S[i - j]);
        Om[i] = o;
    }
    int dLam[ORC_MAX2T + 1]; /* formal derivative, characteristic 2 */
    for (int i = 0; i < L; i++) dLam[i] = ((i + 1) & 1) ? Lam[i + 1] : 0;
    for (int r = 0; r < L; r++) {
        int p = pos[r];
        int xinv = gf_alpha_pow(f, -p);
        int num = poly_eval(f, Om, two_t - 1, xinv);
        int den = poly_eval(f, dLam, L - 1, xinv);
        if (den == 0) ORC_FAIL();
        int e = gf_mul(f, num, gf_inv(f, den));
        e = gf_mul(f, e, gf_alpha_pow(f, (long)p * (1 - f->fcr)));
        if (e == 0) ORC_FAIL();
        work[n - 1 - p] ^= (uint8_t)e;
    }
    /* belt and braces: the corrected word must be a codeword */
    rs_syndromes(f, work, S);
    for (int j = 0; j < two_t; j++) if (S[j]) ORC_FAIL();

    for (int i = 0; i < n; i++) { if (cw) cw[i] = work[i]; if (i < k) msg[i] = work[i]; }
    return L;
#undef ORC_FAIL
}

int orc_rs_decode(int m, unsigned prim_poly, int n, int k, int fcr,
                  const uint8_t *syms, int64_t count,
                  uint8_t *msgs /*[count,k]*/, uint8_t *cws /*[count,n] or NULL*/, int8_t *nerr /*[count]*/)
{
    orc_rs f;
    int rc = orc_rs_init(&f, m, prim_poly, n, k, fcr);
    if (rc) return rc;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; i++)
        nerr[i] = (int8_t)rs_decode_one(&f, syms + i * n, msgs + i * k, cws ? cws + i * n : NULL);
    return 0;
}

/* ---------------------------------------------------------------- tiles */

static int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

/* T[c][i][j] = I[c][y+i][x+j], (y,x) clamped so the tile lies inside the image */
int orc_extract_tiles(const uint8_t *images, int64_t N, int H, int W,
                      const int32_t *off_yx /*[N,2] or NULL = (0,0)*/, int tile, uint8_t *tiles)
{
    if (tile <= 0 || tile > H || tile > W) return 1;
    for (int64_t n = 0; n < N; n++) {
        int y = off_yx ? clampi(off_yx[2 * n], 0, H - tile) : 0;
        int x = off_yx ? clampi(off_yx[2 * n + 1], 0, W - tile) : 0;
        for (int c = 0; c < 3; c++)
            for (int i = 0; i < tile; i++)
                for (int j = 0; j < tile; j++)
                    tiles[((n * 3 + c) * tile + i) * tile + j] =
                        images[((n * 3 + c) * (int64_t)H + y + i) * W + x + j];
    }
    return 0;
}

/* ---------------------------------------------------------------- extractor */

typedef struct {
    int in_ch, n_blocks, channels, n_bits, final_relu;
    const float *conv_w;  /* OIHW concatenated */
    const float *scale;   /* [n_blocks*C] then optionally [n_bits]; NULL => 1 */
    const float *bias;    /* same; NULL => 0 */
    int has_final_affine; /* scale/bias carry n_bits extra entries for the final conv */
    const float *lin_w;   /* [n_bits,n_bits] (out,in) */
    const float *lin_b;   /* [n_bits] or NULL */
    float mean[3], std[3];
} orc_extractor;

/* out[o][i][j] = sum_{c,di,dj} w[o][c][di][dj] * in[c][i+di-1][j+dj-1], zero outside the tile
 * (stride 1, pad 1, cross-correlation), then out = out*scale[o] + bias[o], then optional ReLU */
static void conv3x3(const double *in, int cin, int h, int w, const float *wt, int cout,
                    const float *scale, const float *bias, int relu, double *out)
{
    for (int o = 0; o < cout; o++)
        for (int i = 0; i < h; i++)
            for (int j = 0; j < w; j++) {
                double acc = 0.0;
                for (int c = 0; c < cin; c++)
                    for (int di = 0; di < 3; di++) {
                        int ii = i + di - 1;
                        if (ii < 0 || ii >= h) continue;
                        for (int dj = 0; dj < 3; dj++) {
                            int jj = j + dj - 1;
                            if (jj < 0 || jj >= w) continue;
                            acc += (double)wt[((o * cin + c) * 3 + di) * 3 + dj] *
                                   in[((int64_t)c * h + ii) * w + jj];
                        }
                    }
                if (scale) acc *= (double)scale[o];
                if (bias) acc += (double)bias[o];
                if (relu && acc < 0.0) acc = 0.0;
                out[((int64_t)o * h + i) * w + j] = acc;
            }
}

/* one tile [in_ch,h,w] u8 -> logits[n_bits] (fp64).  acts_out (optional) receives the
 * output of every block, [n_blocks][C][h][w]; pooled_out (optional) the pooled features. */
static int extractor_one(const orc_extractor *e, const uint8_t *tile, int h, int w,
                         double *logits, double *acts_out, double *pooled_out)
{
    int C = e->channels, nb = e->n_blocks;
    int64_t hw = (int64_t)h * w;
    int cmax = C > e->n_bits ? C : e->n_bits;
    if (e->in_ch > cmax) cmax = e->in_ch;
    double *a = (double *)malloc(sizeof(double) * cmax * hw);
    double *b = (double *)malloc(sizeof(double) * cmax * hw);
    if (!a || !b) { free(a); free(b); return 3; }

    /* normalise: x = (u8/255 - mean_c) / std_c */
    for (int c = 0; c < e->in_ch; c++)
        for (int64_t p = 0; p < hw; p++)
            a[c * hw + p] = ((double)tile[c * hw + p] / 255.0 - (double)e->mean[c]) / (double)e->std[c];

    const float *wt = e->conv_w;
    int cin = e->in_ch;
    for (int blk = 0; blk < nb; blk++) {
        conv3x3(a, cin, h, w, wt, C, e->scale ? e->scale + blk * C : NULL,
                e->bias ? e->bias + blk * C : NULL, 1, b);
        if (acts_out) memcpy(acts_out + (int64_t)blk * C * hw, b, sizeof(double) * C * hw);
        wt += (int64_t)C * cin * 9;
        cin = C;
        double *tmp = a; a = b; b = tmp;
    }
    /* final conv C -> n_bits: no ReLU unless asked; affine only if supplied */
    conv3x3(a, cin, h, w, wt, e->n_bits,
            (e->has_final_affine && e->scale) ? e->scale + nb * C : NULL,
            (e->has_final_affine && e->bias) ? e->bias + nb * C : NULL, e->final_relu, b);

    /* global average pool, then linear */
    double *pooled = (double *)malloc(sizeof(double) * e->n_bits);
    for (int o = 0; o < e->n_bits; o++) {
        double s = 0.0;
        for (int64_t p = 0; p < hw; p++) s += b[o * hw + p];
        pooled[o] = s / (double)hw;
    }
    if (pooled_out) memcpy(pooled_out, pooled, sizeof(double) * e->n_bits);
    for (int o = 0; o < e->n_bits; o++) {
        double z = e->lin_b ? (double)e->lin_b[o] : 0.0;
        for (int i = 0; i < e->n_bits; i++) z += (double)e->lin_w[o * e->n_bits + i] * pooled[i];
        logits[o] = z;
    }
    free(pooled); free(a); free(b);
    return 0;
}

static void fill_extractor(orc_extractor *e, int in_ch, int n_blocks, int channels, int n_bits,
                           int final_relu, int has_final_affine,
                           const float *conv_w, const float *scale, const float *bias,
                           const float *lin_w, const float *lin_b, const float *mean, const float *std)
{
    e->in_ch = in_ch; e->n_blocks = n_blocks; e->channels = channels; e->n_bits = n_bits;
    e->final_relu = final_relu; e->has_final_affine = has_final_affine;
    e->conv_w = conv_w; e->scale = scale; e->bias = bias; e->lin_w = lin_w; e->lin_b = lin_b;
    for (int c = 0; c < 3; c++) { e->mean[c] = mean[c]; e->std[c] = std[c]; }
}

/* tiles u8 [N,in_ch,h,w] -> logits f64 [N,n_bits], bits u8 [N,n_bits] (logit > 0).
 * acts_out optional, only meaningful for N == 1.  Threads over images. */
int orc_extractor_forward(int in_ch, int n_blocks, int channels, int n_bits, int final_relu,
                          int has_final_affine,
                          const float *conv_w, const float *scale, const float *bias,
                          const float *lin_w, const float *lin_b, const float *mean, const float *std,
                          const uint8_t *tiles, int64_t N, int h, int w,
                          double *logits, uint8_t *bits, double *acts_out, double *pooled_out)
{
    orc_extractor e;
    if (in_ch < 1 || in_ch > 3) return 1;
    fill_extractor(&e, in_ch, n_blocks, channels, n_bits, final_relu, has_final_affine,
                   conv_w, scale, bias, lin_w, lin_b, mean, std);
    int rc = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t n = 0; n < N; n++) {
        int r = extractor_one(&e, tiles + n * in_ch * (int64_t)h * w, h, w, logits + n * n_bits,
                              (acts_out && N == 1) ? acts_out : NULL,
                              pooled_out ? pooled_out + n * n_bits : NULL);
        if (r) {
#pragma omp atomic write
            rc = r;
        }
        if (bits)
            for (int o = 0; o < n_bits; o++) bits[n * n_bits + o] = logits[n * n_bits + o] > 0.0;
    }
    return rc;
}

/* s_j = sum_{u<m} bit[j*m+u] << (m-1-u)  (MSB first) */
int orc_bits_to_symbols(const uint8_t *bits, int64_t N, int n_bits, int m, uint8_t *syms /*[N, n_bits/m]*/)
{
    if (m < 1 || m > 8 || n_bits % m) return 1;
    int n = n_bits / m;
    for (int64_t i = 0; i < N; i++)
        for (int j = 0; j < n; j++) {
            int s = 0;
            for (int u = 0; u < m; u++) s |= (bits[i * n_bits + j * m + u] ? 1 : 0) << (m - 1 - u);
            syms[i * n + j] = (uint8_t)s;
        }
    return 0;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
