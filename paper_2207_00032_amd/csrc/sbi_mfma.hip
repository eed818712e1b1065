// Matrix-core streaming kernel for the small-batch GeMM on gfx950.
//
// One block owns one 64-column panel of W and a contiguous range of k-steps (32 rows of W
// each); its NW wavefronts take the k-steps of that range round-robin, so the block as a
// whole walks a contiguous run of the laid-out weights and every byte of W is loaded from
// HBM exactly once, by one 128-bit load of one lane.  Each loaded 1 KiB tile is directly
// the A operand of v_mfma_f32_16x16x32_f16 (rows = 16 columns of W, K = 32); the B operand
// is the X tile (up to 16 batch rows per MFMA) read from LDS.  Each wavefront keeps DEPTH
// k-steps (DEPTH x 4 KiB) of W in flight in a register ring.
//
// The paper tiles the output dimension first and splits the input dimension only when the
// output is too narrow to fill the machine (Sec. III-C, "Tiling Strategies"); the same two
// levels appear here as panels (grid) x k-split (waves of a block, then blocks of a panel).
#include <cstring>

#include "sbi_block.h"

namespace sbi {

// Per-wave contraction state: PW 64-column x (MB*16)-row fp32 tiles in MFMA result layout.
// LN: the X pieces in LDS are raw; each is layer-normalised (fp32, rounded once to fp16) right
// before it becomes the MFMA operand, with the row statistics of this lane's batch rows held
// in registers and the k-step's gamma and beta pieces read from LDS next to the X chunk.
template <int MB, int PW, bool LN>
struct MfmaOp {
    floatx4 acc[kPanelTiles * PW][MB];
    int xoff[MB];     // this lane's 16-byte slot inside a k-step's X block
    floatx2 st[LN ? MB : 1];
    int goff, boff;   // this lane's gamma piece inside a k-step's gamma block; beta: boff further
    int ln;
#ifdef SBI_DEV
    int ablate;
#endif

    __device__ __forceinline__ void init(const GemmParams& p, const floatx2* stats, int g, int i)
    {
#pragma unroll
        for (int t = 0; t < kPanelTiles * PW; ++t)
#pragma unroll
            for (int m = 0; m < MB; ++m) acc[t][m] = floatx4{0.f, 0.f, 0.f, 0.f};
        // rows beyond B re-read row B-1: they only feed result columns that are never stored
#pragma unroll
        for (int m = 0; m < MB; ++m) xoff[m] = g * p.xpitch + min(m * 16 + i, p.B - 1);
        goff = g;
        boff = p.kc * 4;
        ln = 0;
#ifdef SBI_DEV
        ablate = p.flags >> 8;
#pragma unroll
        for (int m = 0; m < MB; ++m) xf[m] = half8{0, 0, 0, 0, 0, 0, 0, 0};
#endif
        if constexpr (LN) {
            ln = p.ln;
            if (p.ln) {
#pragma unroll
                for (int m = 0; m < MB; ++m) st[m] = stats[min(m * 16 + i, p.B - 1)];
            }
        }
    }

    // A k-step in two parts, so that the caller can refill each weight tile's registers right after
    // the MFMAs that read them: begin() fetches (and, with LN, normalises) the X operand, tile()
    // multiplies one 16-column tile by it.
    half8 xf[MB];

    __device__ __forceinline__ void begin(const u32x4* xk, const u32x4* ek)
    {
#ifdef SBI_DEV
        if (ablate & 8) return;                                  // no operand read from LDS
#endif
#pragma unroll
        for (int m = 0; m < MB; ++m) xf[m] = __builtin_bit_cast(half8, xk[xoff[m]]);
        if constexpr (LN) {
            if (ln) {
                const half8 gh = __builtin_bit_cast(half8, ek[goff]);
                const half8 bh = __builtin_bit_cast(half8, ek[goff + boff]);
#pragma unroll
                for (int m = 0; m < MB; ++m) xf[m] = ln_apply(xf[m], gh, bh, st[m]);
            }
        }
    }

    __device__ __forceinline__ void tile(int t, u32x4 w)
    {
#ifdef SBI_DEV
        if (ablate & 1) {                                        // no matrix-core work: keep the loaded registers alive only
            acc[t][0][0] += __builtin_bit_cast(float, w[0] ^ w[1] ^ w[2] ^ w[3]);
            return;
        }
#endif
        const half8 wf = __builtin_bit_cast(half8, w);
#pragma unroll
        for (int m = 0; m < MB; ++m)
            acc[t][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf, xf[m], acc[t][m], 0, 0, 0);
    }
};

// One launch may carry several independent GeMMs of the same batch size (the linear layers of
// one transformer layer): their blocks are simply concatenated, so the ramp-up and the tail of
// a launch are paid once per layer instead of once per GeMM.
// LN: the launch may contain problems whose X is layer-normalised (p.ln); the first
// kLnStatsBytes of the dynamic LDS then hold the rows' statistics, which every block computes
// for itself before it starts its weight stream.
template <int MB, int NW, int DEPTH, int PW, bool LN>
__global__ __launch_bounds__(NW * 64) void sbi_mfma_kernel(const GroupParams gp)
{
    constexpr int NT = NW * 64;
    int gi = 0;
    while (gi + 1 < gp.G && (int)blockIdx.x >= gp.first_block[gi + 1]) ++gi;
    const GemmParams& p = gp.g[gi];
    const int bid = (int)blockIdx.x - gp.first_block[gi];
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    u32x4* xs  = reinterpret_cast<u32x4*>(smem_raw + (LN ? kLnStatsBytes : 0));
    floatx2* stats = reinterpret_cast<floatx2*>(smem_raw);
    float* red = reinterpret_cast<float*>(smem_raw);
    __shared__ int s_flag;

    const int tid  = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4;          // k group within a k-step (8 k each)
    const int i = lane & 15;          // column within a tile (A operand) / batch row (B operand)

    if constexpr (LN) {
        if (p.ln) {
            ln_stats<NW>(p, stats, wave, lane);
            __syncthreads();
        }
    }

    const int pgroup = bid / p.S;     // group of PW adjacent panels
    const int split = bid - pgroup * p.S;
    const int panel = pgroup * PW;
    const int npanels = min(PW, p.P - panel);       // the last group of an odd P has one panel
    const int ks0 = split * p.ksps;
    const int ks1 = min(p.KS, ks0 + p.ksps);
    // a missing second panel streams the first one again; its result is dropped
    const int64_t pstride = (npanels > 1) ? (int64_t)p.KS * (kPanelTiles * 64) : 0;

#ifdef SBI_DEV
    if ((p.flags >> 8) & 48) {                                   // development: wave priority by dispatch order
        const int third = (int)(blockIdx.x * 3u / gridDim.x);
        const bool up = ((p.flags >> 8) & 16) != 0;                // 16: later blocks higher, 32: earlier blocks higher
        const int pr = up ? third : 2 - third;
        if (pr == 1) __builtin_amdgcn_s_setprio(1);
        else if (pr == 2) __builtin_amdgcn_s_setprio(3);
    }
#endif
#ifdef SBI_TRACE
    const unsigned long long t_start = wall_clock64();
    unsigned long long tmark[2] = {0ull, 0ull};
#endif
    MfmaOp<MB, PW, LN> op;
    op.init(p, stats, g, i);
    XStage<NT, 4, LN> xst;            // covers NT*64 bytes of X per chunk without a second pass
#ifdef SBI_TRACE
    stream_panel<NW, DEPTH, PW, LN, staging_passes(MB, DEPTH, LN)>(p, xs, xst, op, tid, wave, lane, panel,
                                                                           pstride, ks0, ks1, tmark);
#else
    stream_panel<NW, DEPTH, PW, LN, staging_passes(MB, DEPTH, LN)>(p, xs, xst, op, tid, wave, lane, panel,
                                                                           pstride, ks0, ks1);
#endif
#ifdef SBI_TRACE
    const unsigned long long t_stream = wall_clock64();
    unsigned long long t_sync = 0;
#endif

    // In-block K-split reduction: each wave parks its 64-column x 16-row tile in LDS
    // (the MFMA result holds, per lane, 4 consecutive columns of one batch row).
    // What the epilogues will read (bias, residual) is requested for all passes at once, before the
    // first barrier: one memory latency in the shadow of the wait for the block's last wave,
    // instead of one per pass.
#ifdef SBI_DEV
    if ((p.flags >> 8) & 4) {                                    // no reduction, no epilogue: keep the sums alive only
        if (op.acc[0][0][0] == 1.2345e-30f) p.Y[0] = (_Float16)1.0f;
        return;
    }
#endif
    RowOperands<NW> ops[PW][MB];
#pragma unroll
    for (int q = 0; q < PW; ++q)
#pragma unroll
        for (int m = 0; m < MB; ++m)
            ops[q][m] = request_row_operands<NW>(p, m, min(panel + q, p.P - 1), tid, m == 0, ops[q][0]);
#pragma unroll
    for (int q = 0; q < PW; ++q) {
        if (q < npanels) {
#pragma unroll
            for (int m = 0; m < MB; ++m) {
                __syncthreads();               // X tile / previous pass no longer needed
#ifdef SBI_TRACE
                if (q == 0 && m == 0) t_sync = wall_clock64();
#endif
#pragma unroll
                for (int t = 0; t < kPanelTiles; ++t)
                    *reinterpret_cast<floatx4*>(red + (wave * 16 + i) * kRedPitch + t * kTileN + 4 * g) =
                        op.acc[q * kPanelTiles + t][m];
                __syncthreads();
                reduce_rows<NW>(p, red, m, panel + q, split, tid, ops[q][m]);
            }
            if (p.S > 1) finish_split_k<NT>(p, panel + q, tid, &s_flag);
        }
    }
#ifdef SBI_TRACE
    if (p.trace && tid == 0) {
        unsigned long long* t = p.trace + (size_t)blockIdx.x * 8;
        t[0] = t_start; t[1] = t_stream; t[2] = wall_clock64();
        t[3] = ((unsigned long long)gi << 32) | (unsigned)bid;
        t[4] = t_sync;                 // when the block's last wave finished streaming
        t[5] = tmark[0]; t[6] = tmark[1];
        t[7] = __builtin_amdgcn_s_getreg((4 << 0) | (0 << 6) | (31 << 11)) |                 // HW_ID
               ((unsigned long long)__builtin_amdgcn_s_getreg((20 << 0) | (0 << 6) | (31 << 11)) << 32);   // XCC_ID
    }
#endif
}

// Two-panel blocks for the largest batches, second form: the block's eight waves are two groups of
// four, each group streaming ONE of the two panels (its four waves share that panel's k-steps),
// both reading the same staged X tile.  Against the form above (every wave streams both panels) a
// wave carries half the accumulators, so the ring can be four deep, and the reduction at the end of
// the block is four-way instead of eight-way and runs for both panels side by side: half the LDS
// traffic, half the additions, half the barriers - the part of a block that grows with the batch.
template <int MB, int DEPTH>
__global__ __launch_bounds__(512) void sbi_mfma_wg_kernel(const GroupParams gp)
{
    constexpr int NT = 512, GW = 4;   // threads per block, waves per group
    int gi = 0;
    while (gi + 1 < gp.G && (int)blockIdx.x >= gp.first_block[gi + 1]) ++gi;
    const GemmParams& p = gp.g[gi];
    const int bid = (int)blockIdx.x - gp.first_block[gi];
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    u32x4* xs  = reinterpret_cast<u32x4*>(smem_raw);
    __shared__ int s_flag;

    const int tid  = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave / GW, kwave = wave - grp * GW;
    const int g = lane >> 4;
    const int i = lane & 15;

    const int pgroup = bid / p.S;
    const int split = bid - pgroup * p.S;
    const int panel0 = pgroup * 2;
    const int npanels = min(2, p.P - panel0);
    const int panel = panel0 + min(grp, npanels - 1);   // a missing second panel: its group streams the first again, result dropped
    const int ks0 = split * p.ksps;
    const int ks1 = min(p.KS, ks0 + p.ksps);

    MfmaOp<MB, 1, false> op;
    op.init(p, nullptr, g, i);
    XStage<NT, 4, false> xst;
    stream_panel<GW, DEPTH, 1, false, staging_passes(MB, DEPTH, false, 2)>(p, xs, xst, op, tid, kwave, lane, panel, 0,
                                                                            ks0, ks1);

    float* red = reinterpret_cast<float*>(smem_raw) + grp * (GW * 16 * kRedPitch);
    const int gtid = tid & (GW * 64 - 1);
    RowOperands<GW> ops[MB];
#pragma unroll
    for (int m = 0; m < MB; ++m) ops[m] = request_row_operands<GW>(p, m, panel, gtid, m == 0, ops[0]);
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        __syncthreads();               // X tile / previous pass no longer needed
#pragma unroll
        for (int t = 0; t < kPanelTiles; ++t)
            *reinterpret_cast<floatx4*>(red + (kwave * 16 + i) * kRedPitch + t * kTileN + 4 * g) = op.acc[t][m];
        __syncthreads();
        if (grp < npanels) reduce_rows<GW>(p, red, m, panel, split, gtid, ops[m]);
    }
    if (p.S > 1) {
        for (int q = 0; q < npanels; ++q) finish_split_k<NT>(p, panel0 + q, tid, &s_flag);
    }
}

template <int MB, int DEPTH>
static int launch_wg_one(const GroupParams& gp, size_t lds, hipStream_t st)
{
    if (lds > 64 * 1024) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sbi_mfma_wg_kernel<MB, DEPTH>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return (int)e;
    }
    hipLaunchKernelGGL((sbi_mfma_wg_kernel<MB, DEPTH>), dim3(gp.first_block[gp.G]), dim3(512), lds, st, gp);
    return (int)hipGetLastError();
}

static int launch_wg(const GroupParams& gp, size_t lds, hipStream_t st)
{
    if (!spread_staging_fits(gp, 8, 4, false, 2)) return (int)hipErrorInvalidValue;
    if (lds < 2 * 4 * 16 * kRedPitch * sizeof(float)) return (int)hipErrorInvalidValue;   // two groups' reduction tiles
    switch ((gp.g[0].B + 15) / 16) {
        case 2: return launch_wg_one<2, 4>(gp, lds, st);
        case 3: return launch_wg_one<3, 4>(gp, lds, st);
        case 4: return launch_wg_one<4, 4>(gp, lds, st);
    }
    return (int)hipErrorInvalidValue;
}

template <int MB, int NW, int DEPTH, int PW, bool LN>
static int launch_one(const GroupParams& gp, size_t lds, hipStream_t st)
{
    if (lds > 64 * 1024) {
        // more than the default 64 KiB of dynamic LDS has to be granted to the kernel first
        const hipError_t e = hipFuncSetAttribute(
            reinterpret_cast<const void*>(&sbi_mfma_kernel<MB, NW, DEPTH, PW, LN>),
            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return (int)e;
    }
    hipLaunchKernelGGL((sbi_mfma_kernel<MB, NW, DEPTH, PW, LN>), dim3(gp.first_block[gp.G]), dim3(NW * 64), lds,
                       st, gp);
    return (int)hipGetLastError();
}

template <int NW, int DEPTH, int PW, bool LN>
static int launch_mb(const GroupParams& gp, size_t lds, hipStream_t st)
{
    switch ((gp.g[0].B + 15) / 16) {
        case 1: return launch_one<1, NW, DEPTH, PW, LN>(gp, lds, st);
        case 2: return launch_one<2, NW, DEPTH, PW, LN>(gp, lds, st);
        case 3: return launch_one<3, NW, DEPTH, PW, LN>(gp, lds, st);
        case 4: return launch_one<4, NW, DEPTH, PW, LN>(gp, lds, st);
    }
    return (int)hipErrorInvalidValue;
}

// Layer-norm as a pass of its own, for batches where normalising inside every GeMM block costs more
// than this (above 16 rows): one block per row, mean and biased variance in fp32 (two passes over
// the row, the second and third from cache), the same (x - mean) * rstd * gamma + beta and the same
// single rounding to fp16 as the fused variant (ln_apply).  K % 8 == 0.
struct NormRowsParams {
    const _Float16* X[kMaxGroup];
    _Float16* out[kMaxGroup];
    const _Float16* gamma[kMaxGroup];
    const _Float16* beta[kMaxGroup];
    int K[kMaxGroup];
    float eps[kMaxGroup];
    int B, G;
};

__global__ __launch_bounds__(256) void sbi_layernorm_rows_kernel(const NormRowsParams q)
{
    __shared__ float s_part[4];
    const int g = (int)blockIdx.x / q.B, b = (int)blockIdx.x - g * q.B;
    if (!q.X[g]) return;                               // a problem of the launch without layer-norm
    const int K = q.K[g];
    const int pieces = K / kChunkK;
    const u32x4* row = reinterpret_cast<const u32x4*>(q.X[g] + (int64_t)b * K);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    float s = 0.f;
    for (int c = tid; c < pieces; c += 256) s += piece_sum(row[c]);
    s = wave_sum(s);
    if (lane == 0) s_part[wave] = s;
    __syncthreads();
    const float mean = (s_part[0] + s_part[1] + s_part[2] + s_part[3]) / (float)K;
    __syncthreads();
    float v = 0.f;
    for (int c = tid; c < pieces; c += 256) v += piece_sqdev(row[c], mean);
    v = wave_sum(v);
    if (lane == 0) s_part[wave] = v;
    __syncthreads();
    const float var = (s_part[0] + s_part[1] + s_part[2] + s_part[3]) / (float)K;
    const floatx2 st = {mean, 1.0f / sqrtf(var + q.eps[g])};

    const u32x4* gam = reinterpret_cast<const u32x4*>(q.gamma[g]);
    const u32x4* bet = reinterpret_cast<const u32x4*>(q.beta[g]);
    u32x4* dst = reinterpret_cast<u32x4*>(q.out[g] + (int64_t)b * K);
    for (int c = tid; c < pieces; c += 256) {
        const half8 y = ln_apply(__builtin_bit_cast(half8, row[c]), __builtin_bit_cast(half8, gam[c]),
                                 __builtin_bit_cast(half8, bet[c]), st);
        dst[c] = __builtin_bit_cast(u32x4, y);
    }
}

int launch_layernorm_rows(const GroupParams& gp, hipStream_t st)
{
    NormRowsParams q;
    std::memset(&q, 0, sizeof q);
    q.B = gp.g[0].B; q.G = gp.G;
    bool any = false;
    for (int k = 0; k < gp.G; ++k) {
        const GemmParams& p = gp.g[k];
        if (p.X16 == p.X) continue;                    // nothing to normalise for this problem
        if (p.K % kChunkK != 0) return (int)hipErrorInvalidValue;
        q.X[k] = p.X16; q.out[k] = const_cast<_Float16*>(p.X);
        q.gamma[k] = p.ln_gamma; q.beta[k] = p.ln_beta; q.K[k] = p.K; q.eps[k] = p.ln_eps;
        any = true;
    }
    if (!any) return 0;
    hipLaunchKernelGGL(sbi_layernorm_rows_kernel, dim3(gp.G * q.B), dim3(256), 0, st, q);
    return (int)hipGetLastError();
}

int launch_mfma(const GroupParams& gp, int waves, int depth, int panels, bool layernorm, size_t lds_bytes,
                hipStream_t st)
{
    if (gp.G < 1 || gp.G > kMaxGroup) return (int)hipErrorInvalidValue;
    if (!(panels == 2 && waves == 8 && depth == 4) && !spread_staging_fits(gp, waves, depth, layernorm)) return (int)hipErrorInvalidValue;
    if (layernorm) {                   // layer-norm variants exist for the one-panel shapes the dispatcher uses
        if (panels != 1) return (int)hipErrorInvalidValue;
        if (waves == 4 && depth == 2) return launch_mb<4, 2, 1, true>(gp, lds_bytes, st);
        if (waves == 4 && depth == 4) return launch_mb<4, 4, 1, true>(gp, lds_bytes, st);
        if (waves == 8 && depth == 4) return launch_mb<8, 4, 1, true>(gp, lds_bytes, st);
        return (int)hipErrorInvalidValue;
    }
    if (panels == 1) {
        if (waves == 4 && depth == 2) return launch_mb<4, 2, 1, false>(gp, lds_bytes, st);
        if (waves == 4 && depth == 4) return launch_mb<4, 4, 1, false>(gp, lds_bytes, st);
        if (waves == 4 && depth == 8) return launch_mb<4, 8, 1, false>(gp, lds_bytes, st);
        if (waves == 8 && depth == 2) return launch_mb<8, 2, 1, false>(gp, lds_bytes, st);
        if (waves == 8 && depth == 4) return launch_mb<8, 4, 1, false>(gp, lds_bytes, st);
        if (waves == 8 && depth == 8) return launch_mb<8, 8, 1, false>(gp, lds_bytes, st);
    } else if (panels == 2) {
        if (waves == 8 && depth == 4) return launch_wg(gp, lds_bytes, st);      // two wave groups, one panel each
        if (waves == 4 && depth == 2) return launch_mb<4, 2, 2, false>(gp, lds_bytes, st);
        if (waves == 4 && depth == 4) return launch_mb<4, 4, 2, false>(gp, lds_bytes, st);
        if (waves == 8 && depth == 2) return launch_mb<8, 2, 2, false>(gp, lds_bytes, st);
    }
    return (int)hipErrorInvalidValue;
}

template <int NW, int DEPTH, int PW, bool LN>
static const void* entry_mb(int mb)
{
    switch (mb) {
        case 1: return reinterpret_cast<const void*>(&sbi_mfma_kernel<1, NW, DEPTH, PW, LN>);
        case 2: return reinterpret_cast<const void*>(&sbi_mfma_kernel<2, NW, DEPTH, PW, LN>);
        case 3: return reinterpret_cast<const void*>(&sbi_mfma_kernel<3, NW, DEPTH, PW, LN>);
        case 4: return reinterpret_cast<const void*>(&sbi_mfma_kernel<4, NW, DEPTH, PW, LN>);
    }
    return nullptr;
}

// The kernel launch_mfma would start for this block shape and mb = ceil(B/16) row blocks, for queries
// of its compiled resources (hipFuncGetAttributes); null where launch_mfma has no variant.
const void* mfma_kernel_entry(int mb, int waves, int depth, int panels, bool layernorm)
{
    if (layernorm) {
        if (panels != 1) return nullptr;
        if (waves == 4 && depth == 2) return entry_mb<4, 2, 1, true>(mb);
        if (waves == 4 && depth == 4) return entry_mb<4, 4, 1, true>(mb);
        if (waves == 8 && depth == 4) return entry_mb<8, 4, 1, true>(mb);
        return nullptr;
    }
    if (panels == 1) {
        if (waves == 4 && depth == 2) return entry_mb<4, 2, 1, false>(mb);
        if (waves == 4 && depth == 4) return entry_mb<4, 4, 1, false>(mb);
        if (waves == 4 && depth == 8) return entry_mb<4, 8, 1, false>(mb);
        if (waves == 8 && depth == 2) return entry_mb<8, 2, 1, false>(mb);
        if (waves == 8 && depth == 4) return entry_mb<8, 4, 1, false>(mb);
        if (waves == 8 && depth == 8) return entry_mb<8, 8, 1, false>(mb);
    } else if (panels == 2) {
        if (waves == 8 && depth == 4) {
            switch (mb) {
                case 2: return reinterpret_cast<const void*>(&sbi_mfma_wg_kernel<2, 4>);
                case 3: return reinterpret_cast<const void*>(&sbi_mfma_wg_kernel<3, 4>);
                case 4: return reinterpret_cast<const void*>(&sbi_mfma_wg_kernel<4, 4>);
            }
            return nullptr;
        }
        if (waves == 4 && depth == 2) return entry_mb<4, 2, 2, false>(mb);
        if (waves == 4 && depth == 4) return entry_mb<4, 4, 2, false>(mb);
        if (waves == 8 && depth == 2) return entry_mb<8, 2, 2, false>(mb);
    }
    return nullptr;
}

}  // namespace sbi
