// Driver: one transformer layer's grouped launch (optionally with fused layer-norms) through the
// real host code and the CPU-emulated kernel, all buffers malloc'ed at their exact sizes.
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
    _Float16* p = (_Float16*)exact_alloc(256, n * 2);   // exact byte size
    std::normal_distribution<float> d(mean, sigma);
    for (size_t i = 0; i < n; ++i) p[i] = (_Float16)d(rng);
    return p;
}

// host pre-layout following the documented format
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

int main(int argc, char** argv)
{
    const int B = argc > 1 ? atoi(argv[1]) : 1;
    const int64_t h = argc > 2 ? atoll(argv[2]) : 4096;
    const int ln = argc > 3 ? atoi(argv[3]) : 1;
    const int check = argc > 4 ? atoi(argv[4]) : 0;     // 1: all blocks ran, compare with a reference
    const int64_t Ks[4] = {h, h, h, 4 * h}, Ns[4] = {3 * h, h, 4 * h, h};
    std::mt19937 rng(1234);
    _Float16 *W[4], *bias[4], *X[4], *Y[4];
    void* Wl[4];
    for (int g = 0; g < 4; ++g) {
        W[g] = halfs((size_t)Ks[g] * Ns[g], rng, 0.02f);
        Wl[g] = layout(W[g], Ks[g], Ns[g]);
        bias[g] = halfs(Ns[g], rng, 0.02f);
        X[g] = halfs((size_t)B * Ks[g], rng, 1.0f, (g == 0 || g == 2) ? 0.5f : 0.f);
        Y[g] = (_Float16*)exact_alloc(4, (size_t)B * Ns[g] * 2);
        memset(Y[g], 0xFF, (size_t)B * Ns[g] * 2);
    }
    _Float16* R = halfs((size_t)B * h, rng, 1.0f);
    _Float16 *g1 = halfs(h, rng, 0.1f, 1.f), *b1 = halfs(h, rng, 0.1f), *g2 = halfs(h, rng, 0.1f, 1.f), *b2 = halfs(h, rng, 0.1f);
    sbi_layer L;
    memset(&L, 0, sizeof L);
    L.Wqkv = Wl[0]; L.Wout = Wl[1]; L.Wffn1 = Wl[2]; L.Wffn2 = Wl[3];
    L.bqkv = bias[0]; L.bout = bias[1]; L.bffn1 = bias[2]; L.bffn2 = bias[3];
    L.h = h; L.n_qkv = 3 * h; L.k_out = h; L.n_ffn1 = 4 * h; L.k_ffn2 = 4 * h; L.ffn1_gelu = 1;
    if (ln) { L.ln1_gamma = g1; L.ln1_beta = b1; L.ln2_gamma = g2; L.ln2_beta = b2; L.ln_eps = 1e-5f; }
    const size_t wsb = sbi_layer_workspace_bytes(&L, B);
    void* ws = exact_alloc(256, wsb ? wsb : 256);
    memset(ws, 0, wsb ? wsb : 256);
    sbi_plan plans[4]; int32_t grid = 0;
    sbi_layer_plan(&L, B, 0, plans, &grid);
    fprintf(stderr, "B=%d h=%ld ln=%d grid=%d waves=%d depth=%d lds=%ld ws=%zu\n", B, (long)h, ln, grid, plans[0].waves,
            plans[0].depth, (long)plans[0].lds_bytes, wsb);
    const sbi_status st = sbi_layer_gemms(&L, B, X[0], X[1], X[2], X[3], R, Y[0], Y[1], Y[2], Y[3], ws, wsb, nullptr);
    fprintf(stderr, "status %d (%s)\n", (int)st, sbi_status_string(st));
    if (st != SBI_OK) return 1;
    if (check) {
        double worst = 0;
        for (int g = 0; g < 4; ++g) {
            std::vector<double> xn((size_t)B * Ks[g]);
            for (int b = 0; b < B; ++b) {
                const _Float16* x = X[g] + (size_t)b * Ks[g];
                const bool use = ln && (g == 0 || g == 2);
                double mean = 0, var = 0;
                for (int64_t k = 0; k < Ks[g]; ++k) mean += (double)x[k];
                mean /= Ks[g];
                for (int64_t k = 0; k < Ks[g]; ++k) var += ((double)x[k] - mean) * ((double)x[k] - mean);
                var /= Ks[g];
                const _Float16 *ga = g == 0 ? g1 : g2, *be = g == 0 ? b1 : b2;
                for (int64_t k = 0; k < Ks[g]; ++k)
                    xn[(size_t)b * Ks[g] + k] = use ? (double)(_Float16)(((double)x[k] - mean) / std::sqrt(var + 1e-5) * (double)ga[k] + (double)be[k])
                                                    : (double)x[k];
            }
            for (int b = 0; b < B; ++b)
                for (int64_t n = 0; n < Ns[g]; ++n) {
                    double acc = 0;
                    for (int64_t k = 0; k < Ks[g]; ++k) acc += xn[(size_t)b * Ks[g] + k] * (double)W[g][k * Ns[g] + n];
                    acc += (double)bias[g][n];
                    if (g == 2) acc = 0.5 * acc * (1 + std::erf(acc / std::sqrt(2.0)));
                    if (g == 3) acc += (double)R[(size_t)b * h + n];
                    const double got = (double)Y[g][(size_t)b * Ns[g] + n];
                    const double err = std::fabs(got - acc);
                    if (!(err <= worst)) worst = err;
                }
        }
        fprintf(stderr, "max abs error vs fp64 reference: %g\n", worst);
        if (!(worst < 4e-3)) return 2;
    }
    unsigned* c = (unsigned*)ws;
    for (size_t i = 0; i < 65536 && i * 4 < wsb; ++i) if (c[i]) { fprintf(stderr, "counter %zu = %u\n", i, c[i]); break; }
    return 0;
}
