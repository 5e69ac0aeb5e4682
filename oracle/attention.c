/*
 * CPU oracle for masked multi-head attention -- TEST INFRASTRUCTURE ONLY.
 *
 * Nothing in the product path may call this file; it exists so that tests, the
 * smoke check and the benchmark's cpu_baseline leg have an independent, slow,
 * obviously correct answer to compare the HIP kernels against.  It shares no
 * code, header, table or format with the HIP library.
 *
 * What it computes (scaled dot-product attention with a mask, Sec. 2.1.1 of the
 * paper; a mask entry of 0 means "this key is skipped", Sec. 3.2 / Sec. 4.2.2):
 *
 *   A_i     = { j : M[i][j] = 1 }
 *   s_ij    = scale * sum_k Q[i][k] * K[j][k]                  for j in A_i
 *   p_ij    = exp(s_ij - max_j s_ij) / sum_j' exp(s_ij' - max) for j in A_i
 *   O[i][:] = sum_{j in A_i} p_ij * V[j][:]
 *   A_i empty  ->  O[i][:] = 0   (stated convention; the paper is silent)
 *
 * Two plain passes per query row over the DENSE mask, all arithmetic in fp64,
 * no tiling, no running max, no sparse format.  The fast path's blocked online
 * softmax (Algorithm 1 of the paper) must reach this same result up to rounding.
 *
 * Inputs are raw IEEE binary16 or bfloat16 bit patterns; they are widened to
 * fp64 exactly before any arithmetic.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* exact binary16 -> double */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int f = h & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);             /* zero or subnormal: f * 2^-24 */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(f | 0x400), e - 25); /* (1024 + f) * 2^(e-15-10) */
    return sign ? -v : v;
}

/* exact bfloat16 -> double (bfloat16 is the top half of a binary32) */
static double bf16_bits_to_double(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static void widen(const uint16_t *src, double *dst, size_t n, int dtype)
{
    for (size_t t = 0; t < n; ++t)
        dst[t] = dtype == 0 ? half_bits_to_double(src[t]) : bf16_bits_to_double(src[t]);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* One query row: writes d outputs; if probs != NULL also writes the S
 * probabilities (0 at masked positions). */
static void attend_row(const double *q, const double *K, const double *V, const uint8_t *mrow,
                       int S, int d, double scale, double *s, double *out, double *probs)
{
    double mx = -INFINITY;
    int any = 0;
    for (int j = 0; j < S; ++j) {
        if (!mrow[j]) continue;
        double acc = 0.0;
        const double *k = K + (size_t)j * d;
        for (int t = 0; t < d; ++t) acc += q[t] * k[t];
        s[j] = scale * acc;
        if (!any || s[j] > mx) mx = s[j];
        any = 1;
    }
    for (int t = 0; t < d; ++t) out[t] = 0.0;
    if (probs) for (int j = 0; j < S; ++j) probs[j] = 0.0;
    if (!any) return;                          /* fully masked row -> zeros */
    double denom = 0.0;
    for (int j = 0; j < S; ++j)
        if (mrow[j]) denom += exp(s[j] - mx);
    for (int j = 0; j < S; ++j) {
        if (!mrow[j]) continue;
        double p = exp(s[j] - mx) / denom;
        if (probs) probs[j] = p;
        const double *v = V + (size_t)j * d;
        for (int t = 0; t < d; ++t) out[t] += p * v[t];
    }
}

/*
 * The definition above does not need as many queries as keys (cross-attention, a decoding step
 * against cached keys, or simply a sample of the query rows of a long sequence):
 * Q:       [B][H][Sq][d] bit patterns (dtype 0 = binary16, 1 = bfloat16), packed.
 * K, V:    [B][H][Sk][d].
 * mask:    [Bm][Hm][Sq][Sk] bytes, nonzero = attend; Bm in {1,B}, Hm in {1,H}.
 * O:       [B][H][Sq][d] doubles.
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int oracle_masked_attention_rect(const uint16_t *Q, const uint16_t *K, const uint16_t *V, int dtype,
                                 const uint8_t *mask, int Bm, int Hm,
                                 int B, int H, int Sq, int Sk, int d, double scale, double *O)
{
    if (!Q || !K || !V || !mask || !O || B < 1 || H < 1 || Sq < 1 || Sk < 1 || d < 1) return -1;
    if ((Bm != 1 && Bm != B) || (Hm != 1 && Hm != H) || (dtype != 0 && dtype != 1)) return -1;
    size_t nq = (size_t)B * H * Sq * d, nk = (size_t)B * H * Sk * d;
    double *q = malloc(nq * sizeof *q), *k = malloc(nk * sizeof *k), *v = malloc(nk * sizeof *v);
    if (!q || !k || !v) { free(q); free(k); free(v); return -1; }
    widen(Q, q, nq, dtype);
    widen(K, k, nk, dtype);
    widen(V, v, nk, dtype);
    int fail = 0;
    long rows = (long)B * H * Sq;
#pragma omp parallel
    {
        double *s = malloc((size_t)Sk * sizeof *s);
        if (!s) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 16)
        for (long r = 0; r < rows; ++r) {
            if (!s) continue;
            int i = (int)(r % Sq);
            int h = (int)((r / Sq) % H);
            int b = (int)(r / ((long)Sq * H));
            size_t bhq = ((size_t)b * H + h) * Sq * d, bhk = ((size_t)b * H + h) * Sk * d;
            const uint8_t *mrow = mask +
                ((((size_t)(Bm == 1 ? 0 : b)) * Hm + (Hm == 1 ? 0 : h)) * Sq + i) * (size_t)Sk;
            attend_row(q + bhq + (size_t)i * d, k + bhk, v + bhk, mrow, Sk, d, scale, s,
                       O + bhq + (size_t)i * d, NULL);
        }
        free(s);
    }
    free(q); free(k); free(v);
    return fail ? -1 : 0;
}

/* Self-attention: as many queries as keys, mask [Bm][Hm][S][S]. */
int oracle_masked_attention(const uint16_t *Q, const uint16_t *K, const uint16_t *V, int dtype,
                            const uint8_t *mask, int Bm, int Hm,
                            int B, int H, int S, int d, double scale, double *O)
{
    return oracle_masked_attention_rect(Q, K, V, dtype, mask, Bm, Hm, B, H, S, S, d, scale, O);
}

/* Probabilities of a single query row (b, h, i): probs[S].  For invariant tests. */
int oracle_row_probs(const uint16_t *Q, const uint16_t *K, const uint16_t *V, int dtype,
                     const uint8_t *mask, int Bm, int Hm, int B, int H, int S, int d,
                     double scale, int b, int h, int i, double *probs, double *out)
{
    if (b < 0 || b >= B || h < 0 || h >= H || i < 0 || i >= S) return -1;
    size_t bh = ((size_t)b * H + h) * S * d;
    double *q = malloc((size_t)d * sizeof *q);
    double *k = malloc((size_t)S * d * sizeof *k);
    double *v = malloc((size_t)S * d * sizeof *v);
    double *s = malloc((size_t)S * sizeof *s);
    if (!q || !k || !v || !s) { free(q); free(k); free(v); free(s); return -1; }
    widen(Q + bh + (size_t)i * d, q, d, dtype);
    widen(K + bh, k, (size_t)S * d, dtype);
    widen(V + bh, v, (size_t)S * d, dtype);
    const uint8_t *mrow = mask +
        ((((size_t)(Bm == 1 ? 0 : b)) * Hm + (Hm == 1 ? 0 : h)) * S + i) * (size_t)S;
    attend_row(q, k, v, mrow, S, d, scale, s, out, probs);
    free(q); free(k); free(v); free(s);
    return 0;
}

/* Exact widening exposed for the conversion pins. */
double oracle_f16_to_f64(uint16_t h) { return half_bits_to_double(h); }
double oracle_bf16_to_f64(uint16_t h) { return bf16_bits_to_double(h); }
