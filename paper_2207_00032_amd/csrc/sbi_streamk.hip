// Work-balanced ("stream-K") matrix-core kernel for the small-batch GeMM on gfx950, able to
// run the independent GeMMs of a transformer layer as ONE launch.
//
// The laid-out weights of all problems of a launch form one long sequence of 4 KiB units
// (one k-step of one 64-column panel; inside a problem the units are contiguous in memory).
// That sequence is cut into equal contiguous ranges, one per wavefront, so every wavefront -
// and therefore every CU - streams the same number of bytes from HBM whatever the shapes are.
// A wavefront is an independent worker: no LDS, no block barrier.  It keeps DEPTH units in
// flight in a register ring; a unit is the A operand of four v_mfma_f32_16x16x32_f16 (64
// columns x 32 k), the B operand (X, up to 16 batch rows per MFMA, 16 bytes per lane) is
// loaded straight from global memory with the same ring (it stays in L2: every panel re-reads
// it).  Ranges start and end on multiples of 8 units and every panel has a multiple of 8
// k-steps, so a ring round never straddles a panel.
//
// When a wavefront's range covers a whole panel the epilogue (bias, exact-erf GeLU, residual,
// fp16 rounding) runs from registers.  A panel cut by a range boundary is finished by the
// paper's second level of tiling (Sec. III-C "Tiling Strategies": split the input dimension
// and reduce across tiles): each wavefront parks its partial tile in the workspace, counts its
// arrival at the end of its range, and the wavefront that arrives last sums the slabs in range
// order - deterministic - and runs the epilogue.  Nobody ever waits for another wavefront.
#include "sbi_common.h"

namespace sbi {

__device__ __forceinline__ float sk_gelu(float v)
{
    return 0.5f * v * (1.0f + erff(v * 0.70710678118654752440f));
}

__device__ __forceinline__ void sk_store_pair(float* dst, float s0, float s1)
{
    const unsigned long long bits = ((unsigned long long)__builtin_bit_cast(unsigned int, s1) << 32) |
                                    (unsigned long long)__builtin_bit_cast(unsigned int, s0);
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(dst), bits, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void sk_load_pair(const float* src, float& s0, float& s1)
{
    const unsigned long long bits = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(src),
                                                      __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s0 = __builtin_bit_cast(float, (unsigned int)(bits & 0xffffffffull));
    s1 = __builtin_bit_cast(float, (unsigned int)(bits >> 32));
}

// Epilogue + fp16 store of four consecutive columns n0..n0+3 of batch row b.
__device__ __forceinline__ void sk_finish4(const SkProblem& q, int b, int n0, float (&v)[4])
{
    if (n0 >= q.N) return;
    const int flags = q.flags;
    const int64_t off = (int64_t)b * q.N + n0;
    if (q.fast) {
        typedef _Float16 half4 __attribute__((ext_vector_type(4)));
        if (flags & kEpiBias) {
            const half4 bv = *reinterpret_cast<const half4*>(q.bias + n0);
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] += (float)bv[r];
        }
        if (flags & kEpiGelu) {
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] = sk_gelu(v[r]);
        }
        if (flags & kEpiRes) {
            const half4 rv = *reinterpret_cast<const half4*>(q.R + off);
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] += (float)rv[r];
        }
        half4 out = {(_Float16)v[0], (_Float16)v[1], (_Float16)v[2], (_Float16)v[3]};
        *reinterpret_cast<half4*>(q.Y + off) = out;
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int n = n0 + r;
            if (n >= q.N) continue;
            float x = v[r];
            if (flags & kEpiBias) x += (float)q.bias[n];
            if (flags & kEpiGelu) x = sk_gelu(x);
            if (flags & kEpiRes) x += (float)q.R[off + r];
            q.Y[off + r] = (_Float16)x;
        }
    }
}

// Epilogue + store of one panel from the MFMA result layout: lane (g4, i) holds, for tile t
// and row block m, columns panel*64 + t*16 + 4*g4 .. +3 of batch row m*16 + i.
template <int MB>
__device__ __forceinline__ void sk_epilogue_store(const SkProblem& q, int B, int panel,
                                                  const floatx4 (&acc)[kPanelTiles][MB], int g4, int i)
{
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        const int b = m * 16 + i;
        if (b >= B) continue;
#pragma unroll
        for (int t = 0; t < kPanelTiles; ++t) {
            float v[4] = {acc[t][m][0], acc[t][m][1], acc[t][m][2], acc[t][m][3]};
            sk_finish4(q, b, panel * kPanelN + t * kTileN + 4 * g4, v);
        }
    }
}

// Finish a panel that several wavefronts contributed to: the B x 64 tile is spread flat over
// the 64 lanes (4 columns each); every lane sums its piece over the slabs of wavefronts
// wf..wl in that order (so the result does not depend on who does it), requesting the slabs
// eight at a time so their latencies overlap, then runs the epilogue.
__device__ __forceinline__ void sk_fixup(const SkParams& p, const SkProblem& q, int panel, int wf, int wl, int lane)
{
    constexpr int kBatch = 8;
    const int pieces = p.B * (kPanelN / 4);
    for (int e = lane; e < pieces; e += 64) {
        const int b = e >> 4;
        const int c4 = (e & 15) * 4;
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        for (int w0 = wf; w0 <= wl; w0 += kBatch) {
            float t0[kBatch], t1[kBatch], t2[kBatch], t3[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int ww = min(w0 + j, wl);          // repeats of the last slab are dropped below
                const int slab = (ww == wf) ? 2 * ww + 1 : 2 * ww;
                const float* src = p.partials + ((int64_t)slab * p.B + b) * kPanelN + c4;
                sk_load_pair(src, t0[j], t1[j]);
                sk_load_pair(src + 2, t2[j], t3[j]);
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                if (w0 + j <= wl) { v[0] += t0[j]; v[1] += t1[j]; v[2] += t2[j]; v[3] += t3[j]; }
            }
        }
        sk_finish4(q, b, panel * kPanelN + c4, v);
    }
}

template <int MB, int NW, int DEPTH>
__global__ __launch_bounds__(NW * 64) void sbi_streamk_kernel(const SkParams p)
{
    static_assert(kStepGroup % DEPTH == 0, "a ring round must not straddle a panel");
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int w = blockIdx.x * NW + wave;            // this wavefront's index in the launch
    const int g4 = lane >> 4;                        // k group inside a k-step
    const int i = lane & 15;                         // column inside a tile (A) / batch row (B operand)
    const int u0 = w * p.upw;
    if (u0 >= p.U) return;
    const int cnt = min(p.upw, p.U - u0);            // a multiple of 8
    const int rounds = cnt / DEPTH;

    int row[MB];                                     // rows beyond B re-read row B-1 (never stored)
#pragma unroll
    for (int m = 0; m < MB; ++m) row[m] = min(m * 16 + i, p.B - 1);

    // ---- request cursor: (problem, unit inside the problem) of the next round to request
    int gf = 0;
    while (gf + 1 < p.G && u0 >= p.prob[gf + 1].unit_base) ++gf;
    int ulf = u0 - p.prob[gf].unit_base;
    const u32x4* Wf = p.prob[gf].Wl;
    const _Float16* Xf = p.prob[gf].X;
    int Kf = p.prob[gf].K;
    int KSf = p.prob[gf].KS;
    int unitsf = p.prob[gf].P * KSf;
    int ksf = ulf % KSf;

    // ---- consume cursor
    int gc = gf;
    int KSc = KSf;
    int Pc = p.prob[gf].P;
    int pc = ulf / KSf;
    int ksc = ksf;
    int seg_first = ksf;                             // k-step at which this wave's part of the panel began

    u32x4 wr[DEPTH][kPanelTiles];
    u32x4 xr[DEPTH][MB];
    floatx4 acc[kPanelTiles][MB];
#pragma unroll
    for (int t = 0; t < kPanelTiles; ++t)
#pragma unroll
        for (int m = 0; m < MB; ++m) acc[t][m] = floatx4{0.f, 0.f, 0.f, 0.f};

    // partial panels this wave must report at the end of its range
    int head_g = -1, head_p = 0, tail_g = -1, tail_p = 0;

#define SK_REQUEST(d)                                                                              \
    {                                                                                              \
        const u32x4* wsrc = Wf + (int64_t)(ulf + (d)) * (kPanelTiles * 64) + lane;                 \
        _Pragma("unroll") for (int t = 0; t < kPanelTiles; ++t)                                    \
            wr[d][t] = __builtin_nontemporal_load(wsrc + t * 64);                                  \
        const int kk = min((ksf + (d)) * kTileK + kChunkK * g4, Kf - kChunkK);                     \
        _Pragma("unroll") for (int m = 0; m < MB; ++m)                                             \
            xr[d][m] = *reinterpret_cast<const u32x4*>(Xf + (int64_t)row[m] * Kf + kk);            \
    }
#define SK_ADVANCE_REQUEST()                                                                       \
    {                                                                                              \
        ulf += DEPTH;                                                                              \
        ksf += DEPTH;                                                                              \
        if (ksf == KSf) ksf = 0;                                                                   \
        if (ulf == unitsf && gf + 1 < p.G) {                                                       \
            ++gf;                                                                                  \
            Wf = p.prob[gf].Wl; Xf = p.prob[gf].X; Kf = p.prob[gf].K; KSf = p.prob[gf].KS;         \
            unitsf = p.prob[gf].P * KSf; ulf = 0; ksf = 0;                                         \
        }                                                                                          \
    }
#define SK_CONSUME(d)                                                                              \
    {                                                                                              \
        _Pragma("unroll") for (int t = 0; t < kPanelTiles; ++t) {                                  \
            const half8 wf = __builtin_bit_cast(half8, wr[d][t]);                                  \
            _Pragma("unroll") for (int m = 0; m < MB; ++m)                                         \
                acc[t][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(                                \
                    wf, __builtin_bit_cast(half8, xr[d][m]), acc[t][m], 0, 0, 0);                  \
        }                                                                                          \
    }
    // End of a round: if the panel (or the range) ends here, finish or park the tile.
#define SK_ROUND_DONE(last_round)                                                                  \
    {                                                                                              \
        ksc += DEPTH;                                                                              \
        const bool panel_end = (ksc == KSc);                                                       \
        if (panel_end || (last_round)) {                                                           \
            if (panel_end && seg_first == 0) {                                                     \
                sk_epilogue_store<MB>(p.prob[gc], p.B, pc, acc, g4, i);                            \
            } else {                                                                               \
                const int slab = (seg_first > 0) ? 2 * w : 2 * w + 1;                              \
                if (seg_first > 0) { head_g = gc; head_p = pc; } else { tail_g = gc; tail_p = pc; } \
                float* dst = p.partials + (int64_t)slab * p.B * kPanelN;                           \
                _Pragma("unroll") for (int m = 0; m < MB; ++m) {                                   \
                    const int b = m * 16 + i;                                                      \
                    if (b < p.B) {                                                                 \
                        _Pragma("unroll") for (int t = 0; t < kPanelTiles; ++t) {                  \
                            float* d2 = dst + (int64_t)b * kPanelN + t * kTileN + 4 * g4;          \
                            sk_store_pair(d2, acc[t][m][0], acc[t][m][1]);                         \
                            sk_store_pair(d2 + 2, acc[t][m][2], acc[t][m][3]);                     \
                        }                                                                          \
                    }                                                                              \
                }                                                                                  \
            }                                                                                      \
            _Pragma("unroll") for (int t = 0; t < kPanelTiles; ++t)                                \
                _Pragma("unroll") for (int m = 0; m < MB; ++m) acc[t][m] = floatx4{0.f, 0.f, 0.f, 0.f}; \
            if (panel_end) {                                                                       \
                ksc = 0; seg_first = 0; ++pc;                                                      \
                if (pc == Pc && gc + 1 < p.G) { ++gc; pc = 0; KSc = p.prob[gc].KS; Pc = p.prob[gc].P; } \
            }                                                                                      \
        }                                                                                          \
    }

    // ---- the stream
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) SK_REQUEST(d)
    SK_ADVANCE_REQUEST()
    for (int r = 0; r + 1 < rounds; ++r) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            SK_CONSUME(d)
            SK_REQUEST(d)
            __builtin_amdgcn_sched_barrier(0);
        }
        SK_ADVANCE_REQUEST()
        SK_ROUND_DONE(false)
    }
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) SK_CONSUME(d)
    SK_ROUND_DONE(true)
#undef SK_REQUEST
#undef SK_ADVANCE_REQUEST
#undef SK_CONSUME
#undef SK_ROUND_DONE

    if (head_g < 0 && tail_g < 0) return;

    // ---- arrivals: all of this wave's partial tiles have been acknowledged before it is counted
    wait_stores_acknowledged();
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        const int g = which == 0 ? head_g : tail_g;
        const int pn = which == 0 ? head_p : tail_p;
        if (g < 0) continue;
        const SkProblem& q = p.prob[g];
        const int ub = q.unit_base + pn * q.KS;
        const int wf = ub / p.upw;
        const int wl = (ub + q.KS - 1) / p.upw;
        const int nseg = wl - wf + 1;
        unsigned int* ctr = p.counters + q.panel_base + pn;
        unsigned int old = 0;
        if (lane == 0) old = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        old = __builtin_amdgcn_readfirstlane(old);
        if (old != (unsigned int)(nseg - 1)) continue;
        // last to arrive: sum the slabs in range order, then the epilogue
        sk_fixup(p, q, pn, wf, wl, lane);
        if (lane == 0) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <int MB, int NW, int DEPTH>
static int launch_one(const SkParams& p, int grid, hipStream_t st)
{
    hipLaunchKernelGGL((sbi_streamk_kernel<MB, NW, DEPTH>), dim3(grid), dim3(NW * 64), 0, st, p);
    return (int)hipGetLastError();
}

template <int NW, int DEPTH>
static int launch_mb(const SkParams& p, int grid, hipStream_t st)
{
    switch ((p.B + 15) / 16) {
        case 1: return launch_one<1, NW, DEPTH>(p, grid, st);
        case 2: return launch_one<2, NW, DEPTH>(p, grid, st);
        case 3: return launch_one<3, NW, DEPTH>(p, grid, st);
        case 4: return launch_one<4, NW, DEPTH>(p, grid, st);
    }
    return (int)hipErrorInvalidValue;
}

int launch_streamk(const SkParams& p, int waves, int depth, int grid, hipStream_t st)
{
    if (waves == 4 && depth == 4) return launch_mb<4, 4>(p, grid, st);
    if (waves == 4 && depth == 8) return launch_mb<4, 8>(p, grid, st);
    if (waves == 8 && depth == 4) return launch_mb<8, 4>(p, grid, st);
    if (waves == 8 && depth == 8) return launch_mb<8, 8>(p, grid, st);
    return (int)hipErrorInvalidValue;
}

}  // namespace sbi
