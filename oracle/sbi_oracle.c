/*
 * CPU oracle for the small-batch inference GeMM  Y[B,N] = epilogue(X[B,K] . W[K,N] + bias).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct definition the GPU
 * library is checked against.  It shares no code, header, table or constant with the HIP
 * path and must never be called from it.
 *
 * What it follows.  The paper (Sec. III-C, "SBI-GeMM") states the operation only as a
 * "skinny matrix multiplication" of a small batch of activations with a layer's weight
 * matrix, and Sec. III-D names "bias and residual addition" as the fused tail of a
 * transformer layer.  The method is a faster way to reach the plain matrix product, so
 * the oracle is that definition written out:
 *
 *     acc[b,n] = sum_{k=0}^{K-1} X[b,k] * W[k,n]          fp64, k ascending
 *     v        = acc[b,n] (+ bias[n])
 *     GeLU:      v = 0.5 * v * (1 + erf(v / sqrt 2))        exact-erf form, libm erf
 *     residual:  v = v + R[b,n]
 *     Y[b,n]   = fp16(v)                                    ONE round-to-nearest-even step
 *
 * All tensors are IEEE binary16 bit patterns (uint16_t), row-major, contiguous.
 * fp16*fp16 products are exact in fp64 and the fp64 sum has relative error about
 * K*2^-53, so before the final rounding this is "the exact result" at fp16 resolution.
 * No blocking, fusion or reordering changes any output: the only blocking is over
 * independent columns (each output still sums k = 0..K-1 in order).
 *
 * Every function here is pinned by tests/test_oracle_*.py (brute-force rational
 * arithmetic, identity / one-hot weights, linearity, GeLU closed forms, exhaustive
 * fp16 round trips; layer-norm and the INT8 functions: hand-worked cases, exact integer
 * brute force, reduction to the fp16 GeMM where the scales are 1; decode attention: closed-form
 * weight patterns, invariances, an exact rational case): no part is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* epilogue selector: bit 0 = add bias, bit 1 = GeLU, bit 2 = add residual */
#define ORACLE_EPI_BIAS 1
#define ORACLE_EPI_GELU 2
#define ORACLE_EPI_RES  4

/* binary16 bit pattern -> double (exact: every fp16 value is a double) */
double sbi_oracle_half_to_double(uint16_t h)
{
    const int sign = (h >> 15) & 1;
    const int exp  = (h >> 10) & 0x1f;
    const int man  = h & 0x3ff;
    double v;
    if (exp == 0)        v = ldexp((double)man, -24);              /* zero / subnormal */
    else if (exp == 31)  v = man ? NAN : INFINITY;
    else                 v = ldexp((double)(man | 0x400), exp - 25); /* 1.man * 2^(exp-15) */
    return sign ? -v : v;
}

/* double -> binary16 bit pattern, a single round-to-nearest-even step (never via float) */
uint16_t sbi_oracle_double_to_half(double v)
{
    uint64_t bits;
    memcpy(&bits, &v, sizeof bits);
    const uint16_t sign = (uint16_t)((bits >> 63) << 15);
    const int      bexp = (int)((bits >> 52) & 0x7ff);
    const uint64_t man  = bits & ((1ull << 52) - 1);

    if (bexp == 0x7ff) return (uint16_t)(sign | (man ? 0x7e00 : 0x7c00));  /* NaN / inf */
    if (bexp == 0)     return sign;            /* fp64 zero or subnormal: far below 2^-25 */

    const int e = bexp - 1023;                 /* v = 1.man * 2^e */
    if (e > 15) return (uint16_t)(sign | 0x7c00);

    if (e >= -14) {                            /* fp16 normal range: keep 10 fraction bits */
        uint64_t q   = man >> 42;
        uint64_t rem = man & ((1ull << 42) - 1);
        uint64_t half = 1ull << 41;
        uint32_t out = (uint32_t)(((uint32_t)(e + 15) << 10) | (uint32_t)q);
        if (rem > half || (rem == half && (q & 1))) out += 1;   /* carry may reach exponent / inf */
        return (uint16_t)(sign | out);
    }
    /* fp16 subnormal range: count units of 2^-24 */
    const int shift = 42 + (-14 - e);          /* >= 43 */
    if (shift >= 64) return sign;
    const uint64_t full = (1ull << 52) | man;
    uint64_t q    = full >> shift;
    uint64_t rem  = full & ((1ull << shift) - 1);
    uint64_t half = 1ull << (shift - 1);
    if (rem > half || (rem == half && (q & 1))) q += 1;          /* may become 0x400 = min normal */
    return (uint16_t)(sign | (uint16_t)q);
}

/* exact-erf GeLU in fp64 */
double sbi_oracle_gelu(double v)
{
    return 0.5 * v * (1.0 + erf(v / sqrt(2.0)));
}

/*
 * Layer normalisation of each row of X [B,K] (fp16 bits) in fp64, the operation the paper
 * fuses in front of the QKV and the intermediate (FFN1) GeMM (Sec. III-D, regions 1 and 3;
 * the layer-norm itself is the standard one it cites: per-row mean and biased variance over
 * the K features):
 *     mean = (1/K) sum_k x[k]        var = (1/K) sum_k (x[k] - mean)^2
 *     y[k] = (x[k] - mean) / sqrt(var + eps) * gamma[k] + beta[k]
 * The result is rounded once to fp16, because it is the fp16 operand of the GeMM that follows.
 * `pre` (optional, [B,K] doubles) receives y before that rounding.
 */
int sbi_oracle_layernorm(const uint16_t* X, const uint16_t* gamma, const uint16_t* beta, double eps,
                         int64_t B, int64_t K, uint16_t* out, double* pre)
{
    if (!X || !gamma || !beta || !out || B <= 0 || K <= 0 || !(eps >= 0.0)) return -1;
    for (int64_t b = 0; b < B; ++b) {
        const uint16_t* x = X + b * K;
        double mean = 0.0;
        for (int64_t k = 0; k < K; ++k) mean += sbi_oracle_half_to_double(x[k]);
        mean /= (double)K;
        double var = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double d = sbi_oracle_half_to_double(x[k]) - mean;
            var += d * d;
        }
        var /= (double)K;
        const double rstd = 1.0 / sqrt(var + eps);
        for (int64_t k = 0; k < K; ++k) {
            const double y = (sbi_oracle_half_to_double(x[k]) - mean) * rstd *
                             sbi_oracle_half_to_double(gamma[k]) + sbi_oracle_half_to_double(beta[k]);
            if (pre) pre[b * K + k] = y;
            out[b * K + k] = sbi_oracle_double_to_half(y);
        }
    }
    return 0;
}

/*
 * INT8 path (paper Sec. III-D, "Support for Different Data Types": an INT8 GeMM with a quantize
 * operation fused before it and the de-quantisation fused after it).  The paper gives no
 * quantisation formula; the reading taken here is the plain symmetric one, per row of the
 * activations (per token) and per column of the weights (per output channel):
 *
 *     amax  = max_j |v_j|              inv = 127 / amax          scale = amax / 127
 *     q_j   = clamp(rint(v_j * inv), -127, 127)                   (amax = 0: q = 0, scale = 0)
 *
 * The code q_j is an INTEGER decided by floating point, so its arithmetic is fixed exactly and
 * is the kernel's: IEEE binary32, `inv` and `scale` one correctly rounded division each, one
 * correctly rounded multiplication, round-half-to-even to an integer.  (fp16 inputs are exact
 * in binary32.)  Everything after the codes is exact or fp64:
 *
 *     acc[b,n] = sum_k Xq[b,k] * Wq[k,n]                          exact integer
 *     v        = acc * sx[b] * sw[n] (+ bias) -> GeLU -> + residual   fp64, as in sbi_oracle_gemm
 *     Y        = fp16(v)                                           one RNE step
 */
static void quantize_line(const uint16_t* v, int64_t n, int64_t stride, int8_t* q, float* scale)
{
    float amax = 0.0f;
    for (int64_t j = 0; j < n; ++j) {
        const float a = fabsf((float)sbi_oracle_half_to_double(v[j * stride]));
        if (a > amax) amax = a;
    }
    if (!(amax > 0.0f)) {
        for (int64_t j = 0; j < n; ++j) q[j * stride] = 0;
        *scale = 0.0f;
        return;
    }
    const volatile float inv = 127.0f / amax;
    *scale = amax / 127.0f;
    for (int64_t j = 0; j < n; ++j) {
        const volatile float p = (float)sbi_oracle_half_to_double(v[j * stride]) * inv;   /* binary32 product */
        float r = rintf(p);                       /* current rounding mode: to nearest, ties to even */
        if (r > 127.0f) r = 127.0f;
        if (r < -127.0f) r = -127.0f;
        q[j * stride] = (int8_t)r;
    }
}

/* X [B,K] fp16 bits -> Xq [B,K] int8 and sx [B]: one scale per row */
int sbi_oracle_quantize_rows(const uint16_t* X, int64_t B, int64_t K, int8_t* Xq, float* sx)
{
    if (!X || !Xq || !sx || B <= 0 || K <= 0) return -1;
    for (int64_t b = 0; b < B; ++b) quantize_line(X + b * K, K, 1, Xq + b * K, sx + b);
    return 0;
}

/* W [K,N] fp16 bits -> Wq [K,N] int8 and sw [N]: one scale per column */
int sbi_oracle_quantize_columns(const uint16_t* W, int64_t K, int64_t N, int8_t* Wq, float* sw)
{
    if (!W || !Wq || !sw || K <= 0 || N <= 0) return -1;
    for (int64_t n = 0; n < N; ++n) quantize_line(W + n, K, N, Wq + n, sw + n);
    return 0;
}

/* The INT8 GeMM on given codes and scales.  Xq [B,K], Wq [K,N] int8; sx [B], sw [N] binary32. */
int sbi_oracle_gemm_i8(const int8_t* Xq, const float* sx, const int8_t* Wq, const float* sw,
                       const uint16_t* bias, const uint16_t* R, int epi, int64_t B, int64_t K, int64_t N,
                       uint16_t* Y, double* pre)
{
    if (!Xq || !sx || !Wq || !sw || !Y || B <= 0 || K <= 0 || N <= 0) return -1;
    if ((epi & ORACLE_EPI_BIAS) && !bias) return -1;
    if ((epi & ORACLE_EPI_RES) && !R) return -1;
    if (epi & ~7) return -1;
    int64_t* acc = (int64_t*)malloc(sizeof(int64_t) * (size_t)N);
    if (!acc) return -1;
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t n = 0; n < N; ++n) acc[n] = 0;
        for (int64_t k = 0; k < K; ++k) {
            const int64_t x = Xq[b * K + k];
            if (x == 0) continue;
            const int8_t* w = Wq + k * N;
            for (int64_t n = 0; n < N; ++n) acc[n] += x * (int64_t)w[n];
        }
        for (int64_t n = 0; n < N; ++n) {
            double v = (double)acc[n] * (double)sx[b] * (double)sw[n];
            if (epi & ORACLE_EPI_BIAS) v += sbi_oracle_half_to_double(bias[n]);
            if (epi & ORACLE_EPI_GELU) v = sbi_oracle_gelu(v);
            if (epi & ORACLE_EPI_RES)  v += sbi_oracle_half_to_double(R[b * N + n]);
            if (pre) pre[b * N + n] = v;
            Y[b * N + n] = sbi_oracle_double_to_half(v);
        }
    }
    free(acc);
    return 0;
}

/*
 * Single-token attention with a key/value cache (paper Sec. III-D region 2, "transposition plus
 * attention", for the token-generation phase of Sec. IV in which "the new computation only
 * depends on a single previously generated token" and everything older is re-used from the
 * cache).  The paper relies on the standard scaled dot-product attention; written out for one
 * new token per sequence:
 *
 *   qkv   [B][3][H][d]   the QKV GeMM's output row of the new token: query, key, value per head
 *   Kc,Vc [B][H][S][d]   caches holding `pos` earlier tokens per sequence (positions 0..pos-1)
 *
 *   1. "transposition": the new key and value go to position `pos` of their head's cache
 *      (token-major [3][H][d] -> head-major [H][S][d]), bit for bit;
 *   2. s_j = scale * sum_e q[e] * K[j][e]                    j = 0..pos      (fp64)
 *   3. p_j = exp(s_j - max_j s_j) / sum_j exp(s_j - max_j s_j)
 *   4. out[b][h*d + e] = fp16( sum_j p_j * V[j][e] )         token-major again, one rounding
 *
 * No mask is needed: a cache only ever holds the past.  `pre` (optional, [B][H*d] doubles)
 * receives the outputs before the rounding.
 */
int sbi_oracle_attn_decode(const uint16_t* qkv, uint16_t* Kc, uint16_t* Vc, int64_t B, int64_t H, int64_t d,
                           int64_t S, int64_t pos, double scale, uint16_t* out, double* pre)
{
    if (!qkv || !Kc || !Vc || !out || B <= 0 || H <= 0 || d <= 0 || S <= 0 || pos < 0 || pos >= S) return -1;
    double* sc = (double*)malloc(sizeof(double) * (size_t)(pos + 1));
    if (!sc) return -1;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t h = 0; h < H; ++h) {
            const uint16_t* q = qkv + ((b * 3 + 0) * H + h) * d;
            const uint16_t* kn = qkv + ((b * 3 + 1) * H + h) * d;
            const uint16_t* vn = qkv + ((b * 3 + 2) * H + h) * d;
            uint16_t* K = Kc + (b * H + h) * S * d;
            uint16_t* V = Vc + (b * H + h) * S * d;
            memcpy(K + pos * d, kn, sizeof(uint16_t) * (size_t)d);
            memcpy(V + pos * d, vn, sizeof(uint16_t) * (size_t)d);
            double mx = -INFINITY;
            for (int64_t j = 0; j <= pos; ++j) {
                double a = 0.0;
                for (int64_t e = 0; e < d; ++e)
                    a += sbi_oracle_half_to_double(q[e]) * sbi_oracle_half_to_double(K[j * d + e]);
                sc[j] = a * scale;
                if (sc[j] > mx) mx = sc[j];
            }
            double den = 0.0;
            for (int64_t j = 0; j <= pos; ++j) { sc[j] = exp(sc[j] - mx); den += sc[j]; }
            for (int64_t e = 0; e < d; ++e) {
                double a = 0.0;
                for (int64_t j = 0; j <= pos; ++j) a += sc[j] * sbi_oracle_half_to_double(V[j * d + e]);
                a /= den;
                if (pre) pre[b * H * d + h * d + e] = a;
                out[b * H * d + h * d + e] = sbi_oracle_double_to_half(a);
            }
        }
    free(sc);
    return 0;
}

void sbi_oracle_half_to_double_array(const uint16_t* h, double* d, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) d[i] = sbi_oracle_half_to_double(h[i]);
}

void sbi_oracle_double_to_half_array(const double* d, uint16_t* h, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) h[i] = sbi_oracle_double_to_half(d[i]);
}

int sbi_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * The GeMM.  X [B,K], W [K,N], bias [N] or NULL, R [B,N] or NULL, Y [B,N] (fp16 bits).
 * `pre` (optional, [B,N] doubles) receives v before the final fp16 rounding.
 * `threads` <= 0 means "all cores".  Returns 0, or -1 on a bad argument.
 * Columns are processed in independent blocks of CB; each output sums k = 0..K-1 in order.
 */
int sbi_oracle_gemm(const uint16_t* X, const uint16_t* W, const uint16_t* bias,
                    const uint16_t* R, int epi, int64_t B, int64_t K, int64_t N,
                    uint16_t* Y, double* pre, int threads)
{
    if (!X || !W || !Y || B <= 0 || K <= 0 || N <= 0) return -1;
    if ((epi & ORACLE_EPI_BIAS) && !bias) return -1;
    if ((epi & ORACLE_EPI_RES) && !R) return -1;
    if (epi & ~7) return -1;

    enum { CB = 128 };
    double* Xd = (double*)malloc(sizeof(double) * (size_t)B * (size_t)K);
    if (!Xd) return -1;
    sbi_oracle_half_to_double_array(X, Xd, B * K);

    const int64_t nblocks = (N + CB - 1) / CB;
#ifdef _OPENMP
    if (threads <= 0) threads = omp_get_max_threads();
#else
    threads = 1;
#endif
    int failed = 0;

#pragma omp parallel num_threads(threads)
    {
        double* acc  = (double*)malloc(sizeof(double) * (size_t)B * CB);
        double  wrow[CB];
        if (!acc) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t blk = 0; blk < nblocks; ++blk) {
            if (!acc) continue;
            const int64_t n0 = blk * CB;
            const int     nb = (int)((N - n0 < CB) ? (N - n0) : CB);
            for (int64_t i = 0; i < B * CB; ++i) acc[i] = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                const uint16_t* wr = W + k * N + n0;
                for (int j = 0; j < nb; ++j) wrow[j] = sbi_oracle_half_to_double(wr[j]);
                for (int64_t b = 0; b < B; ++b) {
                    const double x = Xd[b * K + k];
                    double* a = acc + b * CB;
                    for (int j = 0; j < nb; ++j) a[j] += x * wrow[j];
                }
            }
            for (int64_t b = 0; b < B; ++b) {
                for (int j = 0; j < nb; ++j) {
                    const int64_t n = n0 + j;
                    double v = acc[b * CB + j];
                    if (epi & ORACLE_EPI_BIAS) v += sbi_oracle_half_to_double(bias[n]);
                    if (epi & ORACLE_EPI_GELU) v = sbi_oracle_gelu(v);
                    if (epi & ORACLE_EPI_RES)  v += sbi_oracle_half_to_double(R[b * N + n]);
                    if (pre) pre[b * N + n] = v;
                    Y[b * N + n] = sbi_oracle_double_to_half(v);
                }
            }
        }
        free(acc);
    }
    free(Xd);
    return failed ? -1 : 0;
}
