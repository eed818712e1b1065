// Driver: single-token attention with a KV cache through the real host code and the CPU-emulated
// kernel, all buffers malloc'ed at their exact sizes; result against an fp64 reference.
#include "sbi_gemm.h"
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

static void* exact_alloc(size_t align, size_t bytes)
{
    void* p = nullptr;
    if (posix_memalign(&p, align < sizeof(void*) ? sizeof(void*) : align, bytes ? bytes : 1) != 0) abort();
    return p;
}

int main(int argc, char** argv)
{
    if (argc < 6) { fprintf(stderr, "usage: B H d S pos [ragged]\n"); return 9; }
    const int64_t B = atoll(argv[1]); const int H = atoi(argv[2]), d = atoi(argv[3]);
    const int64_t S = atoll(argv[4]), bound = atoll(argv[5]);
    const bool ragged = argc > 6 && atoi(argv[6]) != 0;
    std::mt19937 rng(11);
    // ragged: one position per sequence through sbi_attn_decode_ragged - the first at the bound, one at
    // 0, one out of range on either side (the kernel forces those to the ends of 0 .. bound), the rest drawn
    int32_t* pos_of = (int32_t*)exact_alloc(4, (size_t)B * 4);
    std::vector<int64_t> pos_eff(B, bound);
    for (int64_t b = 0; ragged && b < B; ++b) {
        int64_t v = b == 0 ? bound : b == 1 ? 0 : b == 2 ? bound + 7 : b == 3 ? -3 : (int64_t)(rng() % (uint64_t)(bound + 1));
        pos_of[b] = (int32_t)v;
        pos_eff[b] = v < 0 ? 0 : v > bound ? bound : v;
    }
    std::normal_distribution<float> nd(0.f, 1.f);
    const size_t nq = (size_t)B * 3 * H * d, nc = (size_t)B * H * S * d;
    _Float16* qkv = (_Float16*)exact_alloc(16, nq * 2);
    _Float16* Kc = (_Float16*)exact_alloc(16, nc * 2);
    _Float16* Vc = (_Float16*)exact_alloc(16, nc * 2);
    _Float16* out = (_Float16*)exact_alloc(16, (size_t)B * H * d * 2);
    for (size_t i = 0; i < nq; ++i) qkv[i] = (_Float16)nd(rng);
    for (size_t i = 0; i < nc; ++i) { Kc[i] = (_Float16)nd(rng); Vc[i] = (_Float16)nd(rng); }
    std::vector<_Float16> K0(Kc, Kc + nc), V0(Vc, Vc + nc);
    const size_t wsb = sbi_attn_decode_workspace_bytes(B, H, d, S);
    void* ws = exact_alloc(256, wsb ? wsb : 256);
    memset(ws, 0, wsb ? wsb : 256);
    const sbi_status st = ragged ? sbi_attn_decode_ragged(qkv, Kc, Vc, B, H, d, S, pos_of, bound, 0.0f, out, wsb ? ws : nullptr, wsb, nullptr)
                                 : sbi_attn_decode(qkv, Kc, Vc, B, H, d, S, bound, 0.0f, out, wsb ? ws : nullptr, wsb, nullptr);
    fprintf(stderr, "B=%ld H=%d d=%d S=%ld pos=%ld ragged=%d ws=%zu status %d (%s)\n", (long)B, H, d, (long)S, (long)bound,
            (int)ragged, wsb, (int)st, sbi_status_string(st));
    if (st) return 1;
    double worst = 0;
    const double scale = 1.0 / std::sqrt((double)d);
    for (int64_t b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            const int64_t pos = pos_eff[b];
            const _Float16* q = qkv + ((b * 3 + 0) * H + h) * d;
            const _Float16* kn = qkv + ((b * 3 + 1) * H + h) * d;
            const _Float16* vn = qkv + ((b * 3 + 2) * H + h) * d;
            const size_t base = ((size_t)b * H + h) * S * d;
            std::vector<double> sc(pos + 1);
            double mx = -1e300;
            for (int64_t j = 0; j <= pos; ++j) {
                double a = 0;
                for (int e = 0; e < d; ++e) a += (double)q[e] * (double)(j == pos ? kn[e] : K0[base + j * d + e]);
                sc[j] = a * scale; mx = std::fmax(mx, sc[j]);
            }
            double den = 0;
            for (auto& v : sc) { v = std::exp(v - mx); den += v; }
            for (int e = 0; e < d; ++e) {
                double a = 0;
                for (int64_t j = 0; j <= pos; ++j) a += sc[j] * (double)(j == pos ? vn[e] : V0[base + j * d + e]);
                worst = std::fmax(worst, std::fabs(a / den - (double)out[(size_t)b * H * d + h * d + e]));
            }
            // the transposition: the new row is in the cache, nothing else changed
            if (memcmp(Kc + base + pos * d, kn, d * 2) || memcmp(Vc + base + pos * d, vn, d * 2)) { fprintf(stderr, "cache row not written\n"); return 3; }
            for (int64_t j = 0; j < S; ++j)
                if (j != pos && (memcmp(Kc + base + j * d, K0.data() + base + j * d, d * 2) || memcmp(Vc + base + j * d, V0.data() + base + j * d, d * 2))) {
                    fprintf(stderr, "cache row %ld changed\n", (long)j); return 3;
                }
        }
    fprintf(stderr, "max abs error vs fp64 reference: %g\n", worst);
    if (!(worst < 3e-3)) return 2;
    const unsigned* c = (const unsigned*)ws;
    for (size_t i = 0; wsb && i < (size_t)B * H; ++i) if (c[i]) { fprintf(stderr, "counter %zu left at %u\n", i, c[i]); return 4; }
    return 0;
}
