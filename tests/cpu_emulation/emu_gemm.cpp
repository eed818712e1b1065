// Driver: one GeMM through sbi_gemm_ex / sbi_gemm_ln with explicit tuning, CPU-emulated kernel, ASan.
#include "sbi_gemm.h"
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

// exactly `bytes` bytes (the sanitizer then sees any access past the end), aligned as the ABI asks
static void* exact_alloc(size_t align, size_t bytes)
{
    void* p = nullptr;
    if (posix_memalign(&p, align < sizeof(void*) ? sizeof(void*) : align, bytes ? bytes : 1) != 0) abort();
    return p;
}
static _Float16* halfs(size_t n, std::mt19937& rng, float sigma, float mean = 0.f)
{
    _Float16* p = (_Float16*)exact_alloc(256, n * 2);
    std::normal_distribution<float> d(mean, sigma);
    for (size_t i = 0; i < n; ++i) p[i] = (_Float16)d(rng);
    return p;
}
static void* layout(const _Float16* W, int64_t K, int64_t N)
{
    const size_t bytes = sbi_gemm_layout_bytes(K, N);
    unsigned char* buf = (unsigned char*)exact_alloc(256, bytes);
    memset(buf, 0, bytes);
    const int64_t KS = (((K + 31) / 32) + 7) / 8 * 8;
    _Float16* out = (_Float16*)(buf + 256);
    for (int64_t k = 0; k < K; ++k)
        for (int64_t n = 0; n < N; ++n) {
            const int64_t p = n / 64, t = (n % 64) / 16, i = n % 16, ks = k / 32, g = (k % 32) / 8, e = k % 8;
            out[((((p * KS + ks) * 4 + t) * 64 + (g * 16 + i)) * 8) + e] = W[k * N + n];
        }
    return buf;
}
// symmetric int8 codes of n values with stride `stride` (binary32 decisions, as the library documents)
static float quantize_line(const _Float16* v, int64_t n, int64_t stride, signed char* q)
{
    float amax = 0.f;
    for (int64_t j = 0; j < n; ++j) amax = std::fmax(amax, std::fabs((float)v[j * stride]));
    if (!(amax > 0.f)) { for (int64_t j = 0; j < n; ++j) q[j * stride] = 0; return 0.f; }
    const volatile float inv = 127.0f / amax;
    for (int64_t j = 0; j < n; ++j) {
        const volatile float pr = (float)v[j * stride] * inv;
        float r = std::rint(pr);
        r = std::fmin(std::fmax(r, -127.f), 127.f);
        q[j * stride] = (signed char)r;
    }
    return amax / 127.0f;
}

static void* layout_i8(const signed char* Wq, int64_t K, int64_t N)
{
    const size_t bytes = sbi_gemm_i8_layout_bytes(K, N);
    unsigned char* buf = (unsigned char*)exact_alloc(256, bytes);
    memset(buf, 0, bytes);
    const int64_t KS = (((K + 63) / 64) + 7) / 8 * 8;
    signed char* out = (signed char*)(buf + 256);
    for (int64_t k = 0; k < K; ++k)
        for (int64_t n = 0; n < N; ++n) {
            const int64_t p = n / 64, t = (n % 64) / 16, i = n % 16, ks = k / 64, g = (k % 64) / 16, e = k % 16;
            out[((((p * KS + ks) * 4 + t) * 64 + (g * 16 + i)) * 16) + e] = Wq[k * N + n];
        }
    return buf;
}

int main(int argc, char** argv)
{
    if (argc < 9) { fprintf(stderr, "usage: B K N waves depth split panels ln\n"); return 9; }
    const int B = atoi(argv[1]); const int64_t K = atoll(argv[2]), N = atoll(argv[3]);
    sbi_tuning t = {SBI_PATH_MFMA, atoi(argv[6]), atoi(argv[4]), atoi(argv[5]), 0, atoi(argv[7]), 0};
    const int mode = atoi(argv[8]);         // 0 plain, 1 layer-norm, 2 int8, 3 plain + emitted moments, 4 layer-norm fed by moments,
                                            // 5 layer-norm in front of int8
    const int ln = mode == 1 || mode == 4 || mode == 5, i8 = mode == 2 || mode == 5;
    if (t.waves == 0) t.path = SBI_PATH_AUTO;
    std::mt19937 rng(7);
    _Float16* W = halfs((size_t)K * N, rng, 0.02f);
    void* Wl = layout(W, K, N);
    _Float16* bias = halfs(N, rng, 0.02f);
    _Float16* X = halfs((size_t)B * K, rng, 1.0f, ln ? 0.5f : 0.f);
    _Float16* R = halfs((size_t)B * N, rng, 1.0f);
    _Float16 *g1 = halfs(K, rng, 0.1f, 1.f), *b1 = halfs(K, rng, 0.1f);
    _Float16* Y = (_Float16*)exact_alloc(4, (size_t)B * N * 2);
    memset(Y, 0xFF, (size_t)B * N * 2);
    sbi_plan pl;
    sbi_tuning tp = t; tp.layernorm = ln; tp.int8 = i8;
    std::vector<signed char> Wq, Xq;
    std::vector<float> sw, sx;
    void* Wl8 = nullptr;
    float* swd = nullptr;
    if (i8) {
        Wq.resize((size_t)K * N); sw.resize(N); Xq.resize((size_t)B * K); sx.resize(B);
        for (int64_t n = 0; n < N; ++n) sw[n] = quantize_line(W + n, K, N, Wq.data() + n);
        std::vector<_Float16> xn16((size_t)B * K);
        for (int b = 0; b < B; ++b) {       // mode 5: the rows that are quantised are the normalised ones, rounded to fp16
            const _Float16* x = X + (size_t)b * K;
            double mean = 0, var = 0;
            for (int64_t k = 0; k < K; ++k) mean += (double)x[k];
            mean /= K;
            for (int64_t k = 0; k < K; ++k) var += ((double)x[k] - mean) * ((double)x[k] - mean);
            var /= K;
            for (int64_t k = 0; k < K; ++k)
                xn16[(size_t)b * K + k] = ln ? (_Float16)(((double)x[k] - mean) * (1.0 / std::sqrt(var + (double)1e-5f)) * (double)g1[k] + (double)b1[k]) : x[k];
        }
        for (int b = 0; b < B; ++b) sx[b] = quantize_line(xn16.data() + (size_t)b * K, K, 1, Xq.data() + (size_t)b * K);
        Wl8 = layout_i8(Wq.data(), K, N);
        swd = (float*)exact_alloc(4, (size_t)N * 4);
        memcpy(swd, sw.data(), (size_t)N * 4);
    }
    sbi_status st = sbi_gemm_plan(B, K, N, &tp, &pl);
    if (st) { fprintf(stderr, "plan: %s\n", sbi_status_string(st)); return 1; }
    fprintf(stderr, "B=%d K=%ld N=%ld ln=%d: w=%d d=%d pw=%d S=%d ksps=%d kc=%d grid=%d lds=%ld ws=%ld\n", B, (long)K, (long)N, ln,
            pl.waves, pl.depth, pl.panels, pl.split_k, pl.ksteps_per_split, pl.ksteps_per_chunk, pl.grid, (long)pl.lds_bytes, (long)pl.workspace_bytes);
    const size_t wsb = pl.workspace_bytes;
    void* ws = exact_alloc(256, wsb ? wsb : 256);
    memset(ws, 0, wsb ? wsb : 256);
    sbi_layernorm l = {g1, b1, 1e-5f, nullptr};
    const int64_t Pn = (N + 63) / 64, Pk = (K + 63) / 64;
    float* mom_out = (float*)exact_alloc(8, (size_t)B * Pn * 8);
    float* mom_in = (float*)exact_alloc(8, (size_t)B * Pk * 8);
    if (mode == 4) {                         // what a producing GeMM would have left for these rows
        if (K % 64) { fprintf(stderr, "mode 4 needs K %% 64 == 0\n"); return 9; }
        for (int b = 0; b < B; ++b)
            for (int64_t pp = 0; pp < Pk; ++pp) {
                double m = 0, q = 0;
                for (int j = 0; j < 64; ++j) m += (double)X[(size_t)b * K + pp * 64 + j];
                m /= 64;
                for (int j = 0; j < 64; ++j) { const double d = (double)X[(size_t)b * K + pp * 64 + j] - m; q += d * d; }
                mom_in[((size_t)b * Pk + pp) * 2] = (float)m;
                mom_in[((size_t)b * Pk + pp) * 2 + 1] = (float)q;
            }
        l.moments = mom_in;
    }
    if (mode == 3) st = sbi_gemm_moments(Wl, K, N, X, B, nullptr, bias, R, SBI_EPI_BIAS_RESIDUAL, Y, mom_out, ws, wsb, nullptr, &t);
    else if (i8 && ln) st = sbi_gemm_i8_ln(Wl8, swd, K, N, X, B, &l, bias, R, SBI_EPI_BIAS_RESIDUAL, Y, ws, wsb, nullptr, &t);
    else if (i8) st = sbi_gemm_i8(Wl8, swd, K, N, X, B, bias, R, SBI_EPI_BIAS_RESIDUAL, Y, ws, wsb, nullptr, &t);
    else if (ln) st = sbi_gemm_ln(Wl, K, N, X, B, &l, bias, R, SBI_EPI_BIAS_RESIDUAL, Y, ws, wsb, nullptr, &t);
    else st = sbi_gemm_ex(Wl, K, N, X, B, bias, R, SBI_EPI_BIAS_RESIDUAL, Y, ws, wsb, nullptr, &t);
    fprintf(stderr, "status %d (%s)\n", (int)st, sbi_status_string(st));
    if (st) return 1;
    if (!getenv("EMU_BLOCKS")) {
        double worst = 0;
        for (int b = 0; b < B; ++b) {
            std::vector<double> xn(K);
            const _Float16* x = X + (size_t)b * K;
            double mean = 0, var = 0;
            for (int64_t k = 0; k < K; ++k) mean += (double)x[k];
            mean /= K;
            for (int64_t k = 0; k < K; ++k) var += ((double)x[k] - mean) * ((double)x[k] - mean);
            var /= K;
            for (int64_t k = 0; k < K; ++k)
                xn[k] = ln ? (double)(_Float16)(((double)x[k] - mean) / std::sqrt(var + 1e-5) * (double)g1[k] + (double)b1[k]) : (double)x[k];
            for (int64_t n = 0; n < N; ++n) {
                double acc = 0;
                if (i8) {
                    long long s = 0;
                    for (int64_t k = 0; k < K; ++k) s += (long long)Xq[(size_t)b * K + k] * (long long)Wq[k * N + n];
                    acc = (double)s * (double)sx[b] * (double)sw[n];
                } else {
                    for (int64_t k = 0; k < K; ++k) acc += xn[k] * (double)W[k * N + n];
                }
                acc += (double)bias[n] + (double)R[(size_t)b * N + n];
                const double err = std::fabs((double)Y[(size_t)b * N + n] - acc);
                if (!(err <= worst)) worst = err;
            }
        }
        fprintf(stderr, "max abs error vs fp64 reference: %g\n", worst);
        if (!(worst < 6e-3)) return 2;
        if (mode == 3) {
            double werr = 0;
            for (int b = 0; b < B; ++b)
                for (int64_t pp = 0; pp < Pn; ++pp) {
                    const int64_t n0 = pp * 64, n1 = (n0 + 64 < N) ? n0 + 64 : N;
                    double m = 0, q = 0;
                    for (int64_t n = n0; n < n1; ++n) m += (double)Y[(size_t)b * N + n];
                    m /= (double)(n1 - n0);
                    for (int64_t n = n0; n < n1; ++n) { const double d = (double)Y[(size_t)b * N + n] - m; q += d * d; }
                    werr = std::fmax(werr, std::fabs(mom_out[((size_t)b * Pn + pp) * 2] - m) / (1e-6 + std::fabs(m)));
                    werr = std::fmax(werr, std::fabs(mom_out[((size_t)b * Pn + pp) * 2 + 1] - q) / (1e-5 + q));
                }
            fprintf(stderr, "max relative error of the emitted moments: %g\n", werr);
            if (!(werr < 1e-3)) return 3;
        }
    }
    return 0;
}
