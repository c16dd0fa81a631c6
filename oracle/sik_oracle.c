/*
 * Self-Indexing KV cache -- CPU oracle.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, fp64
 * implementation of the decode-time path of "Self-Indexing KVCache: Predicting
 * Sparse Attention from Compressed Keys", written step by step in the paper's
 * order and notation so it can be checked against the paper by eye.  Only the
 * tests, the smoke check and the benchmark's CPU-baseline leg may call it.
 * It shares no code with the HIP library and includes none of its headers.
 *
 * Conventions
 *   K, V : [B, Hkv, Lmax, D] 16-bit floats given as raw uint16 bit patterns,
 *          dtype 0 = IEEE binary16 (fp16), 1 = bfloat16.
 *   q    : [B, Hq, D] same dtype.  Query head hq reads KV head hq / (Hq/Hkv).
 *   mu   : [B, Hkv, D] fp32            (channel means, section "Entropy-Aware
 *                                       Normalization", K' = K - mu)
 *   codes: [B, Hkv, Lmax, D/8] uint8   (packed sign bits, 16 B per 128-d key)
 *   codebook: [B, Hkv, G, 16, 4] fp32, counts [B, Hkv, G, 16] int32, G = D/4
 *          (section "Codebook Construction", centroid = cluster mean)
 *   table: [B, Hq, G, 16] fp64         (section "Compressed-Domain Top-k
 *                                       Retrieval", query . centroid)
 *   scores:[B, Hq, Lmax] fp64          (sum of table entries per key)
 *   idx  : [B, Hq, k] int32, -1 = empty slot
 *   out  : [B, Hq, D] fp64
 *   seq_len: [B] int32 on the host, tokens currently valid per sequence.
 *
 * Every function returns 0, or -1 on an argument it cannot handle.
 * All arithmetic is fp64 on values widened exactly from their 16-bit form.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 1;

/* Number of host threads the (batch, head) loops may use; 1 = serial. */
int sik_oracle_set_threads(int n)
{
    if (n < 1) n = 1;
#ifdef _OPENMP
    g_threads = n;
#else
    g_threads = 1;
#endif
    return g_threads;
}

int sik_oracle_get_threads(void) { return g_threads; }

/* ---- exact widening of the two 16-bit formats --------------------------- */

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
static double fp16_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);              /* zero and subnormals */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(f | 0x400), e - 25); /* (1 + f/1024) * 2^(e-15) */
    return sign ? -v : v;
}

/* bfloat16 is the upper half of an IEEE binary32. */
static double bf16_to_double(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static inline double widen(uint16_t h, int dtype)
{
    return dtype == 0 ? fp16_to_double(h) : bf16_to_double(h);
}

/* Exposed so that a test can pin the conversions against numpy / torch. */
int sik_oracle_widen(const uint16_t *x, int dtype, int64_t n, double *out)
{
    if (dtype != 0 && dtype != 1) return -1;
    for (int64_t i = 0; i < n; ++i) out[i] = widen(x[i], dtype);
    return 0;
}

static int bad_shape(int B, int Hkv, int Lmax, int D)
{
    return B < 1 || Hkv < 1 || Lmax < 1 || D < 8 || (D % 8) != 0;
}

/* ---- channel mean: mu_d = (1/L) sum_i K[i,d]  (normalisation equation) --- */
int sik_oracle_mean(const uint16_t *K, int dtype, int B, int Hkv, int Lmax, int D,
                    const int32_t *seq_len, float *mu)
{
    if (bad_shape(B, Hkv, Lmax, D) || (dtype != 0 && dtype != 1)) return -1;
#pragma omp parallel for collapse(2) num_threads(g_threads)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h) {
            int L = seq_len[b];
            const uint16_t *Kh = K + ((int64_t)b * Hkv + h) * Lmax * D;
            for (int d = 0; d < D; ++d) {
                double s = 0.0;
                for (int i = 0; i < L; ++i) s += widen(Kh[(int64_t)i * D + d], dtype);
                mu[((int64_t)b * Hkv + h) * D + d] = L > 0 ? (float)(s / (double)L) : 0.0f;
            }
        }
    return 0;
}

/* ---- sign pattern and 4-bit Code, packed two codes per byte ---------------
 * sign: bit = 1 when K >= mu (so K' = K - mu is "+"), else 0; the comparison
 * is done on the values themselves, no subtraction is rounded.
 * Code of a 4-d sub-vector = sum_i bit_i * 2^(4-i), i = 1..4: the first
 * element is the most significant bit.  Byte j of a token holds Code of group
 * 2j in its high nibble and Code of group 2j+1 in its low nibble.
 * Encodes tokens [t0, t0+n) of every (b, h); other tokens are left untouched. */
int sik_oracle_encode(const uint16_t *K, int dtype, int B, int Hkv, int Lmax, int D,
                      int t0, int n, const float *mu, uint8_t *codes)
{
    if (bad_shape(B, Hkv, Lmax, D) || (dtype != 0 && dtype != 1)) return -1;
    if (t0 < 0 || n < 0 || t0 + n > Lmax) return -1;
    int G = D / 4;
#pragma omp parallel for collapse(2) num_threads(g_threads)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h) {
            int64_t bh = (int64_t)b * Hkv + h;
            const uint16_t *Kh = K + bh * Lmax * D;
            const float *muh = mu + bh * D;
            uint8_t *ch = codes + bh * Lmax * (D / 8);
            for (int i = t0; i < t0 + n; ++i)
                for (int g = 0; g < G; g += 2) {
                    int code[2];
                    for (int c = 0; c < 2; ++c) {
                        int v = 0;
                        for (int e = 0; e < 4; ++e) {
                            int d = 4 * (g + c) + e;
                            int bit = widen(Kh[(int64_t)i * D + d], dtype) >= (double)muh[d];
                            v += bit << (3 - e);
                        }
                        code[c] = v;
                    }
                    ch[(int64_t)i * (D / 8) + g / 2] = (uint8_t)((code[0] << 4) | code[1]);
                }
        }
    return 0;
}

static inline int code_of(const uint8_t *tok, int g)
{
    uint8_t byte = tok[g >> 1];
    return (g & 1) ? (byte & 0xf) : (byte >> 4);
}

/* ---- one-pass sign clustering: centroid c_j = mean of the members of C_j --
 * Members are the centred sub-vectors K'_i^(g) = K_i^(g) - mu^(g) whose Code is
 * j (the codes passed in).  An empty cluster gets a zero centroid, count 0. */
int sik_oracle_codebook(const uint16_t *K, int dtype, int B, int Hkv, int Lmax, int D,
                        const int32_t *seq_len, const float *mu, const uint8_t *codes,
                        float *codebook, int32_t *counts)
{
    if (bad_shape(B, Hkv, Lmax, D) || (dtype != 0 && dtype != 1)) return -1;
    int G = D / 4;
#pragma omp parallel for collapse(2) num_threads(g_threads)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h) {
            int64_t bh = (int64_t)b * Hkv + h;
            int L = seq_len[b];
            const uint16_t *Kh = K + bh * Lmax * D;
            const float *muh = mu + bh * D;
            const uint8_t *ch = codes + bh * Lmax * (D / 8);
            for (int g = 0; g < G; ++g) {
                double sum[16][4];
                int32_t cnt[16];
                memset(sum, 0, sizeof sum);
                memset(cnt, 0, sizeof cnt);
                for (int i = 0; i < L; ++i) {
                    int j = code_of(ch + (int64_t)i * (D / 8), g);
                    cnt[j] += 1;
                    for (int e = 0; e < 4; ++e) {
                        int d = 4 * g + e;
                        sum[j][e] += widen(Kh[(int64_t)i * D + d], dtype) - (double)muh[d];
                    }
                }
                for (int j = 0; j < 16; ++j) {
                    counts[(bh * G + g) * 16 + j] = cnt[j];
                    for (int e = 0; e < 4; ++e)
                        codebook[((bh * G + g) * 16 + j) * 4 + e] =
                            cnt[j] > 0 ? (float)(sum[j][e] / (double)cnt[j]) : 0.0f;
                }
            }
        }
    return 0;
}

/* ---- lookup table: Table^(g)[j] = q^(g) . c_j^(g) ------------------------ */
int sik_oracle_table(const uint16_t *q, int dtype, int B, int Hkv, int Hq, int D,
                     const float *codebook, double *table)
{
    if (B < 1 || Hkv < 1 || Hq < 1 || Hq % Hkv || D % 8 || (dtype != 0 && dtype != 1)) return -1;
    int G = D / 4, R = Hq / Hkv;
    for (int b = 0; b < B; ++b)
        for (int hq = 0; hq < Hq; ++hq) {
            int64_t bh = (int64_t)b * Hkv + hq / R;
            const uint16_t *qh = q + ((int64_t)b * Hq + hq) * D;
            for (int g = 0; g < G; ++g)
                for (int j = 0; j < 16; ++j) {
                    double t = 0.0;
                    for (int e = 0; e < 4; ++e)
                        t += widen(qh[4 * g + e], dtype) *
                             (double)codebook[((bh * G + g) * 16 + j) * 4 + e];
                    table[(((int64_t)b * Hq + hq) * G + g) * 16 + j] = t;
                }
        }
    return 0;
}

/* ---- LUT-GEMV: score(q, k_i) = sum_g Table^(g)[Code(K'_i)^(g)] ------------
 * Written for tokens i < seq_len[b]; the rest of each row is left untouched. */
int sik_oracle_score(const double *table, const uint8_t *codes, int B, int Hkv, int Hq,
                     int Lmax, int D, const int32_t *seq_len, double *scores)
{
    if (bad_shape(B, Hkv, Lmax, D) || Hq < 1 || Hq % Hkv) return -1;
    int G = D / 4, R = Hq / Hkv;
#pragma omp parallel for collapse(2) num_threads(g_threads)
    for (int b = 0; b < B; ++b)
        for (int hq = 0; hq < Hq; ++hq) {
            int L = seq_len[b];
            const uint8_t *ch = codes + ((int64_t)b * Hkv + hq / R) * Lmax * (D / 8);
            const double *T = table + ((int64_t)b * Hq + hq) * G * 16;
            double *s = scores + ((int64_t)b * Hq + hq) * Lmax;
            for (int i = 0; i < L; ++i) {
                double acc = 0.0;
                for (int g = 0; g < G; ++g)
                    acc += T[g * 16 + code_of(ch + (int64_t)i * (D / 8), g)];
                s[i] = acc;
            }
        }
    return 0;
}

/* ---- top-k: the k largest scores of each query head ----------------------
 * Ties go to the smaller token index.  Output is ordered by decreasing score;
 * when k exceeds the number of valid tokens every token is returned and the
 * remaining slots hold -1. */
typedef struct { double s; int32_t i; } sik_pair;

static int pair_cmp(const void *a, const void *b)
{
    const sik_pair *x = (const sik_pair *)a, *y = (const sik_pair *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->i > y->i) - (x->i < y->i);
}

int sik_oracle_topk(const double *scores, int B, int Hq, int Lmax, const int32_t *seq_len,
                    int k, int32_t *idx)
{
    if (B < 1 || Hq < 1 || Lmax < 1 || k < 1) return -1;
    int fail = 0;
#pragma omp parallel for collapse(2) num_threads(g_threads)
    for (int b = 0; b < B; ++b)
        for (int hq = 0; hq < Hq; ++hq) {
            int L = seq_len[b];
            const double *s = scores + ((int64_t)b * Hq + hq) * Lmax;
            int32_t *o = idx + ((int64_t)b * Hq + hq) * k;
            sik_pair *p = (sik_pair *)malloc(sizeof(sik_pair) * (size_t)(L > 0 ? L : 1));
            if (!p) { fail = 1; continue; }
            for (int i = 0; i < L; ++i) { p[i].s = s[i]; p[i].i = i; }
            qsort(p, (size_t)L, sizeof(sik_pair), pair_cmp);
            for (int r = 0; r < k; ++r) o[r] = r < L ? p[r].i : -1;
            free(p);
        }
    return fail ? -1 : 0;
}

/* ---- sparse attention: out = softmax(q K_S^T / sqrt(D)) V_S --------------
 * over the selected set S = idx (entries < 0 skipped, repeats count as
 * repeats), on the stored 16-bit K and V rows.  scale <= 0 means 1/sqrt(D).
 * An empty selection gives a zero row. */
int sik_oracle_sparse_attn(const uint16_t *q, const uint16_t *K, const uint16_t *V, int dtype,
                           int B, int Hkv, int Hq, int Lmax, int D, const int32_t *idx, int k,
                           double scale, double *out)
{
    if (bad_shape(B, Hkv, Lmax, D) || Hq < 1 || Hq % Hkv || k < 1) return -1;
    if (dtype != 0 && dtype != 1) return -1;
    int R = Hq / Hkv;
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)D);
    int fail = 0;
#pragma omp parallel for collapse(2) num_threads(g_threads)
    for (int b = 0; b < B; ++b)
        for (int hq = 0; hq < Hq; ++hq) {
            int64_t bh = (int64_t)b * Hkv + hq / R;
            const uint16_t *qh = q + ((int64_t)b * Hq + hq) * D;
            const uint16_t *Kh = K + bh * Lmax * D;
            const uint16_t *Vh = V + bh * Lmax * D;
            const int32_t *S = idx + ((int64_t)b * Hq + hq) * k;
            double *o = out + ((int64_t)b * Hq + hq) * D;
            double *z = (double *)malloc(sizeof(double) * (size_t)k);
            if (!z) { fail = 1; continue; }
            double zmax = -INFINITY;
            for (int r = 0; r < k; ++r) {
                if (S[r] < 0 || S[r] >= Lmax) { z[r] = -INFINITY; continue; }
                double dot = 0.0;
                for (int d = 0; d < D; ++d)
                    dot += widen(qh[d], dtype) * widen(Kh[(int64_t)S[r] * D + d], dtype);
                z[r] = dot * scale;
                if (z[r] > zmax) zmax = z[r];
            }
            double denom = 0.0;
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            for (int r = 0; r < k; ++r) {
                if (S[r] < 0 || S[r] >= Lmax) continue;
                double p = exp(z[r] - zmax);
                denom += p;
                for (int d = 0; d < D; ++d) o[d] += p * widen(Vh[(int64_t)S[r] * D + d], dtype);
            }
            if (denom > 0.0)
                for (int d = 0; d < D; ++d) o[d] /= denom;
            free(z);
        }
    return fail ? -1 : 0;
}

/* ---- append: copy one new K and V row per (b, h) to row seq_len[b] -------- */
int sik_oracle_append_rows(uint16_t *K, uint16_t *V, const uint16_t *k_new, const uint16_t *v_new,
                           int B, int Hkv, int Lmax, int D, const int32_t *seq_len)
{
    if (bad_shape(B, Hkv, Lmax, D)) return -1;
    for (int b = 0; b < B; ++b) {
        if (seq_len[b] < 0 || seq_len[b] >= Lmax) return -1;
        for (int h = 0; h < Hkv; ++h) {
            int64_t bh = (int64_t)b * Hkv + h;
            memcpy(K + (bh * Lmax + seq_len[b]) * D, k_new + bh * D, sizeof(uint16_t) * (size_t)D);
            memcpy(V + (bh * Lmax + seq_len[b]) * D, v_new + bh * D, sizeof(uint16_t) * (size_t)D);
        }
    }
    return 0;
}

/* ==========================================================================
 * 2-bit token-wise magnitude quantisation (section "Token-Wise Quantization
 * Format") -- the compressed K/V form that sparse attention reads instead of
 * the 16-bit rows.
 *
 * Like everything else in this file it is the paper's function evaluated in
 * fp64 on exactly widened inputs, with true divisions; only the values the
 * format STORES are rounded (qs and zp to IEEE binary16, alpha to binary32).
 *
 * Per token, each run of 32 consecutive channels is one quantisation group
 * with B = 2 bits (quantisation equation):
 *     zp = fp16(min x),  qs = fp16((max x - min x) / (2^B - 1))   (stored)
 *     Q(x) = clamp(round((x - zp) / qs), 0, 2^B - 1), round = nearest, ties to
 *            even; qs = 0 (constant group) gives Q = 0
 *     D(x) = qs * Q(x) + zp                                 (dequantisation)
 * with the STORED (fp16-rounded) qs and zp on both sides of the format, so
 * that D inverts Q consistently.
 * For V, x is the value itself.  For K (normalisation equation of the same
 * section), x = |K'| / alpha with K' = K - mu (mu the stored fp32 mean),
 * alpha_d = max over the fitted tokens of |K'_d| stored as fp32, and
 * alpha_d = 0 gives x = 0.  The sign of K' is not quantised: it is the sign
 * bit of the 1-bit code.  The dequantised key is  s * alpha * D(x),  s = +1
 * where the code bit is 1.
 *
 * An implementation in lower precision takes the same decisions except where
 * (x - zp) / qs falls within its own rounding error of a half-integer (or a
 * stored parameter within its rounding error of a binary16 rounding boundary);
 * the parity tests state that band and count the exceptions.
 * ========================================================================== */

/* fp64 -> IEEE binary16 bits in ONE rounding (nearest, ties to even), with
 * subnormals and overflow to infinity. */
static uint16_t double_to_fp16_bits(double v)
{
    uint16_t sign = (uint16_t)(signbit(v) ? 0x8000u : 0u);
    if (isnan(v)) return (uint16_t)(sign | 0x7e00u);
    if (isinf(v)) return (uint16_t)(sign | 0x7c00u);
    double a = fabs(v);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                  /* a = m * 2^e, 0.5 <= m < 1: a in [2^(e-1), 2^e) */
    int ulp_exp = (e - 1 < -14 ? -14 : e - 1) - 10;  /* spacing of fp16 numbers around a */
    double steps = nearbyint(ldexp(a, -ulp_exp));    /* default rounding mode: ties to even */
    double r = ldexp(steps, ulp_exp);
    if (r >= 65520.0) return (uint16_t)(sign | 0x7c00u);
    if (r < ldexp(1.0, -14)) return (uint16_t)(sign | (uint16_t)steps); /* subnormal or zero */
    int re;
    double rm = frexp(r, &re);                       /* r = rm * 2^re */
    uint16_t frac = (uint16_t)((rm * 2.0 - 1.0) * 1024.0);
    return (uint16_t)(sign | ((uint16_t)(re - 1 + 15) << 10) | frac);
}

/* Exposed so that a test can pin the conversion against numpy (binary32 and fp64 inputs). */
int sik_oracle_to_fp16(const float *x, int64_t n, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = double_to_fp16_bits((double)x[i]);
    return 0;
}

int sik_oracle_f64_to_fp16(const double *x, int64_t n, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = double_to_fp16_bits(x[i]);
    return 0;
}

/* ---- alpha_d = max_i |K'_{i,d}| over the tokens i < seq_len[b] ----------- */
int sik_oracle_alpha(const uint16_t *K, int dtype, int B, int Hkv, int Lmax, int D,
                     const int32_t *seq_len, const float *mu, float *alpha)
{
    if (bad_shape(B, Hkv, Lmax, D) || (dtype != 0 && dtype != 1)) return -1;
#pragma omp parallel for collapse(2) num_threads(g_threads)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h) {
            int64_t bh = (int64_t)b * Hkv + h;
            const uint16_t *Kh = K + bh * Lmax * D;
            for (int d = 0; d < D; ++d) {
                double a = 0.0;
                for (int i = 0; i < seq_len[b]; ++i) {
                    double kp = widen(Kh[(int64_t)i * D + d], dtype) - (double)mu[bh * D + d];
                    if (fabs(kp) > a) a = fabs(kp);
                }
                alpha[bh * D + d] = (float)a;     /* stored as fp32 */
            }
        }
    return 0;
}

/* One group of 32 values: stored parameters and 2-bit codes (quantisation equation, B = 2). */
static void quantize_group(const double *x, uint16_t *param /* qs, zp */, uint8_t *code)
{
    double lo = x[0], hi = x[0];
    for (int e = 1; e < 32; ++e) {
        if (x[e] < lo) lo = x[e];
        if (x[e] > hi) hi = x[e];
    }
    lo = lo + 0.0;                        /* a zero minimum is stored as +0 whatever the signs of the zeros */
    param[0] = double_to_fp16_bits((hi - lo) / 3.0);
    param[1] = double_to_fp16_bits(lo);
    double qs = fp16_to_double(param[0]);
    double zp = fp16_to_double(param[1]);
    for (int e = 0; e < 32; ++e) {
        if (!(qs > 0.0)) { code[e] = 0; continue; }
        double r = nearbyint((x[e] - zp) / qs);      /* default rounding mode: ties to even */
        code[e] = (uint8_t)(r < 0.0 ? 0 : (r > 3.0 ? 3 : (int)r));
    }
}

/* ---- quantise tokens [t0, t0+n) of every (b, h) --------------------------
 * kq, vq   : [B, Hkv, Lmax, D] uint8, values 0..3
 * kpar,vpar: [B, Hkv, Lmax, D/32, 2] uint16 = fp16 bits of (qs, zp)          */
int sik_oracle_quantize_kv(const uint16_t *K, const uint16_t *V, int dtype, int B, int Hkv,
                           int Lmax, int D, int t0, int n, const float *mu, const float *alpha,
                           uint8_t *kq, uint16_t *kpar, uint8_t *vq, uint16_t *vpar)
{
    if (bad_shape(B, Hkv, Lmax, D) || D % 32 || (dtype != 0 && dtype != 1)) return -1;
    if (t0 < 0 || n < 0 || t0 + n > Lmax) return -1;
    int NG = D / 32;
#pragma omp parallel for collapse(2) num_threads(g_threads)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h) {
            int64_t bh = (int64_t)b * Hkv + h;
            for (int i = t0; i < t0 + n; ++i) {
                int64_t row = bh * Lmax + i;
                for (int g = 0; g < NG; ++g) {
                    double xk[32], xv[32];
                    for (int e = 0; e < 32; ++e) {
                        int d = 32 * g + e;
                        double kp = widen(K[row * D + d], dtype) - (double)mu[bh * D + d];
                        double a = (double)alpha[bh * D + d];
                        xk[e] = a > 0.0 ? fabs(kp) / a : 0.0;      /* normalisation equation */
                        xv[e] = widen(V[row * D + d], dtype);
                    }
                    quantize_group(xk, kpar + (row * NG + g) * 2, kq + row * D + 32 * g);
                    quantize_group(xv, vpar + (row * NG + g) * 2, vq + row * D + 32 * g);
                }
            }
        }
    return 0;
}

/* One token of one (b, h): Kd = s * alpha * (qs Q + zp), Vd = qs Q + zp, in fp64.
 * code16: the token's 16 sign bytes; kq/vq: its D 2-bit codes; kpar/vpar: its D/32 (qs, zp) pairs. */
static void dequant_row(const uint8_t *code16, const uint8_t *kq, const uint16_t *kpar,
                        const uint8_t *vq, const uint16_t *vpar, const float *alpha, int D,
                        double *Kd, double *Vd)
{
    for (int d = 0; d < D; ++d) {
        int g = d / 32;
        double kqs = fp16_to_double(kpar[2 * g]), kzp = fp16_to_double(kpar[2 * g + 1]);
        double vqs = fp16_to_double(vpar[2 * g]), vzp = fp16_to_double(vpar[2 * g + 1]);
        int bit = (code16[d / 8] >> (7 - d % 8)) & 1;
        double mag = (double)alpha[d] * (kqs * (double)kq[d] + kzp);
        Kd[d] = bit ? mag : -mag;
        Vd[d] = vqs * (double)vq[d] + vzp;
    }
}

/* ---- dequantise tokens [t0, t0+n) of every (b, h) (for tests) ------------ */
int sik_oracle_dequant_kv(const uint8_t *codes, const uint8_t *kq, const uint16_t *kpar,
                          const uint8_t *vq, const uint16_t *vpar, const float *alpha, int B,
                          int Hkv, int Lmax, int D, int t0, int n, double *Kd, double *Vd)
{
    if (bad_shape(B, Hkv, Lmax, D) || D % 32) return -1;
    if (t0 < 0 || n < 0 || t0 + n > Lmax) return -1;
    int NG = D / 32;
    for (int64_t bh = 0; bh < (int64_t)B * Hkv; ++bh)
        for (int i = t0; i < t0 + n; ++i) {
            int64_t row = bh * Lmax + i;
            dequant_row(codes + row * (D / 8), kq + row * D, kpar + row * NG * 2, vq + row * D,
                        vpar + row * NG * 2, alpha + bh * D, D, Kd + row * D, Vd + row * D);
        }
    return 0;
}

/* ---- sparse attention over the dequantised rows --------------------------
 * Same softmax as sik_oracle_sparse_attn; the key is the centred K' (the
 * dropped q . mu is one constant per query and cancels in the softmax). */
int sik_oracle_sparse_attn_q2(const uint16_t *q, int dtype, const uint8_t *codes, const uint8_t *kq,
                              const uint16_t *kpar, const uint8_t *vq, const uint16_t *vpar,
                              const float *alpha, int B, int Hkv, int Hq, int Lmax, int D,
                              const int32_t *idx, int k, double scale, double *out)
{
    if (bad_shape(B, Hkv, Lmax, D) || D % 32 || Hq < 1 || Hq % Hkv || k < 1) return -1;
    if (dtype != 0 && dtype != 1) return -1;
    int R = Hq / Hkv, NG = D / 32;
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)D);
    int fail = 0;
#pragma omp parallel for collapse(2) num_threads(g_threads)
    for (int b = 0; b < B; ++b)
        for (int hq = 0; hq < Hq; ++hq) {
            int64_t bh = (int64_t)b * Hkv + hq / R;
            const uint16_t *qh = q + ((int64_t)b * Hq + hq) * D;
            const int32_t *S = idx + ((int64_t)b * Hq + hq) * k;
            double *o = out + ((int64_t)b * Hq + hq) * D;
            double *z = (double *)malloc(sizeof(double) * (size_t)k);
            double *kd = (double *)malloc(sizeof(double) * (size_t)D * 2);
            if (!z || !kd) { fail = 1; free(z); free(kd); continue; }
            double *vd = kd + D;
            double zmax = -INFINITY;
            for (int pass = 0; pass < 2; ++pass) {   /* pass 0: logits and their maximum; pass 1: weighted sum */
                double denom = 0.0;
                if (pass == 1)
                    for (int d = 0; d < D; ++d) o[d] = 0.0;
                for (int r = 0; r < k; ++r) {
                    if (S[r] < 0 || S[r] >= Lmax) { z[r] = -INFINITY; continue; }
                    int64_t row = bh * Lmax + S[r];
                    dequant_row(codes + row * (D / 8), kq + row * D, kpar + row * NG * 2, vq + row * D,
                                vpar + row * NG * 2, alpha + bh * D, D, kd, vd);
                    if (pass == 0) {
                        double dot = 0.0;
                        for (int d = 0; d < D; ++d) dot += widen(qh[d], dtype) * kd[d];
                        z[r] = dot * scale;
                        if (z[r] > zmax) zmax = z[r];
                    } else {
                        double p = exp(z[r] - zmax);
                        denom += p;
                        for (int d = 0; d < D; ++d) o[d] += p * vd[d];
                    }
                }
                if (pass == 1 && denom > 0.0)
                    for (int d = 0; d < D; ++d) o[d] /= denom;
            }
            free(z);
            free(kd);
        }
    return fail ? -1 : 0;
}

/* ---- sparse attention with full-precision forced rows next to records ----
 * ("Full Precision Sink Tokens": a fixed set of tokens kept in 16 bits that always takes part
 * in the sparse attention computation.)  The softmax runs over the union of
 *   - the selected tokens idx[b,hq,:] (entries < 0 skipped), read from the 2-bit fields, and
 *   - the forced rows fK, fV [B,Hkv,nf,D] (16-bit), row j counted when fvalid[b,h,j] != 0.
 * The records hold the centred key K' = K - mu, so a forced key is centred the same way,
 * K_f - mu, before its dot product (one softmax needs one common shift). */
int sik_oracle_sparse_attn_q2_forced(const uint16_t *q, int dtype, const uint8_t *codes,
                                     const uint8_t *kq, const uint16_t *kpar, const uint8_t *vq,
                                     const uint16_t *vpar, const float *alpha, const float *mu,
                                     const uint16_t *fK, const uint16_t *fV, const uint8_t *fvalid,
                                     int nf, int B, int Hkv, int Hq, int Lmax, int D,
                                     const int32_t *idx, int k, double scale, double *out)
{
    if (bad_shape(B, Hkv, Lmax, D) || D % 32 || Hq < 1 || Hq % Hkv || k < 1 || nf < 0) return -1;
    if (dtype != 0 && dtype != 1) return -1;
    int R = Hq / Hkv, NG = D / 32;
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)D);
    int fail = 0;
#pragma omp parallel for collapse(2) num_threads(g_threads)
    for (int b = 0; b < B; ++b)
        for (int hq = 0; hq < Hq; ++hq) {
            int64_t bh = (int64_t)b * Hkv + hq / R;
            const uint16_t *qh = q + ((int64_t)b * Hq + hq) * D;
            const int32_t *S = idx + ((int64_t)b * Hq + hq) * k;
            double *o = out + ((int64_t)b * Hq + hq) * D;
            int n = k + nf;
            double *z = (double *)malloc(sizeof(double) * (size_t)n);
            double *kd = (double *)malloc(sizeof(double) * (size_t)D * 2);
            if (!z || !kd) { fail = 1; free(z); free(kd); continue; }
            double *vd = kd + D;
            double zmax = -INFINITY;
            for (int pass = 0; pass < 2; ++pass) {
                double denom = 0.0;
                if (pass == 1)
                    for (int d = 0; d < D; ++d) o[d] = 0.0;
                for (int r = 0; r < n; ++r) {
                    if (r < k) {                         /* a selected token, from its record */
                        if (S[r] < 0 || S[r] >= Lmax) { z[r] = -INFINITY; continue; }
                        int64_t row = bh * Lmax + S[r];
                        dequant_row(codes + row * (D / 8), kq + row * D, kpar + row * NG * 2, vq + row * D,
                                    vpar + row * NG * 2, alpha + bh * D, D, kd, vd);
                    } else {                             /* a forced row, 16-bit, centred */
                        int j = r - k;
                        if (!fvalid[bh * nf + j]) { z[r] = -INFINITY; continue; }
                        for (int d = 0; d < D; ++d) {
                            kd[d] = widen(fK[(bh * nf + j) * D + d], dtype) - (double)mu[bh * D + d];
                            vd[d] = widen(fV[(bh * nf + j) * D + d], dtype);
                        }
                    }
                    if (pass == 0) {
                        double dot = 0.0;
                        for (int d = 0; d < D; ++d) dot += widen(qh[d], dtype) * kd[d];
                        z[r] = dot * scale;
                        if (z[r] > zmax) zmax = z[r];
                    } else {
                        double p = exp(z[r] - zmax);
                        denom += p;
                        for (int d = 0; d < D; ++d) o[d] += p * vd[d];
                    }
                }
                if (pass == 1 && denom > 0.0)
                    for (int d = 0; d < D; ++d) o[d] /= denom;
            }
            free(z);
            free(kd);
        }
    return fail ? -1 : 0;
}
