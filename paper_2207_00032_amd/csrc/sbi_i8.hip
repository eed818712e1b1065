// INT8 variant of the small-batch GeMM (paper Sec. III-D, "Support for Different Data Types":
// an INT8 GeMM with the quantize operation fused in front of it and the de-quantisation fused
// into its epilogue; Sec. III-C "Leveraging Full Cache-line" gives INT8 its own wider layout).
//
// Same structure as the fp16 matrix-core kernel - one block per 64-column panel and k-range, the
// weights streamed once through a register ring of 128-bit loads - with three differences:
//   * a k-step is 64 k: a lane's 16 bytes are 16 consecutive k of one column, a 1 KiB tile
//     (16 columns x 64 k) is the A operand of v_mfma_i32_16x16x64_i8, so the same 4 KiB per
//     panel k-step carry twice the k and the weight stream is half as long;
//   * every block first finds the absolute maximum of each of the B rows of X (one pass), then
//     stages X as int8 codes (symmetric, per row; decided in binary32, see i8_stats);
//   * sums are int32 and exact, across waves and across the blocks of a split panel; the
//     de-quantisation acc * (sx[b] * sw[n]) happens once, right before the epilogue.
#include "sbi_block.h"

namespace sbi {

typedef int i32x4 __attribute__((ext_vector_type(4)));

template <int MB, int PW>
struct MfmaI8Op {
    i32x4 acc[kPanelTiles * PW][MB];
    int xoff[MB];

    __device__ __forceinline__ void init(int B, int pitch, int g, int i)
    {
#pragma unroll
        for (int t = 0; t < kPanelTiles * PW; ++t)
#pragma unroll
            for (int m = 0; m < MB; ++m) acc[t][m] = i32x4{0, 0, 0, 0};
#pragma unroll
        for (int m = 0; m < MB; ++m) xoff[m] = g * pitch + min(m * 16 + i, B - 1);
    }

    // A and B operands use the same lane -> k assignment (lane group g: k 16g..16g+15 of the
    // k-step), which is all the contraction needs.
    i32x4 xf[MB];

    __device__ __forceinline__ void begin(const u32x4* xk, const u32x4*)
    {
#pragma unroll
        for (int m = 0; m < MB; ++m) xf[m] = __builtin_bit_cast(i32x4, xk[xoff[m]]);
    }

    __device__ __forceinline__ void tile(int t, u32x4 w)
    {
        const i32x4 wf = __builtin_bit_cast(i32x4, w);
#pragma unroll
        for (int m = 0; m < MB; ++m)
            acc[t][m] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf, xf[m], acc[t][m], 0, 0, 0);
    }
};

// Staging of activation codes that a kernel of their own has already produced (PREQ): the code
// matrix [B,K] int8 is, byte for byte, a [B,K/2] matrix of 16-bit words, and a 64-k step of codes
// is 64 bytes per row exactly like a 32-k step of fp16 - so the fp16 stage does the job on a
// copy of the parameters that says so.
template <int NT, int XU>
struct XStageCodes {
    XStage<NT, XU, false> inner;
    GemmParams q;

    __device__ __forceinline__ void init(const GemmParams& p)
    {
        q = p;
        q.K = p.K / 2;
        q.x_vec = 1;
    }
    __device__ __forceinline__ void request(const GemmParams&, int cb, int cn, int tid, int j = 0) { inner.request(q, cb, cn, tid, j); }
    __device__ __forceinline__ void commit_pass(const GemmParams&, u32x4* xs, int cb, int cn, int tid, int j)
    {
        inner.commit_pass(q, xs, cb, cn, tid, j);
    }
    __device__ __forceinline__ void commit(const GemmParams&, u32x4* xs, int cb, int cn, int tid)
    {
        inner.commit(q, xs, cb, cn, tid);
    }
};

// LDS: [0, kLnStatsBytes) the rows' (inv, scale); behind it the X buffers during the stream and
// the reduction tile afterwards (the scales are still needed then).
// PREQ: p.X points at int8 codes and p.xstats at the rows' (inv, scale) in global memory, both
// written by sbi_quantize_rows_kernel right before this launch (larger batches: quantising
// B rows in every block would cost more than the weight stream).
// PW = 2 (batches above 16, codes from the workspace): a block streams two adjacent panels for the
// same k-steps, as in the fp16 kernel - one staged X tile and one operand read serve 128 columns.
template <int MB, int NW, int DEPTH, int PW, bool PREQ>
__global__ __launch_bounds__(NW * 64) void sbi_i8_kernel(const GroupParams gp)
{
    constexpr int NT = NW * 64;
    int gi = 0;
    while (gi + 1 < gp.G && (int)blockIdx.x >= gp.first_block[gi + 1]) ++gi;
    const GemmParams& p = gp.g[gi];
    const int bid = (int)blockIdx.x - gp.first_block[gi];
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    floatx2* lds_stats = reinterpret_cast<floatx2*>(smem_raw);
    const floatx2* stats = PREQ ? p.xstats : lds_stats;
    u32x4* xs  = reinterpret_cast<u32x4*>(smem_raw + kLnStatsBytes);
    float* red = reinterpret_cast<float*>(smem_raw + kLnStatsBytes);
    __shared__ int s_flag;

    const int tid  = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4;
    const int i = lane & 15;

    if constexpr (!PREQ) {
        i8_stats<NW>(p, lds_stats, wave, lane);
        __syncthreads();
    }

    const int pgroup = bid / p.S;     // group of PW adjacent panels
    const int split = bid - pgroup * p.S;
    const int panel = pgroup * PW;
    const int npanels = min(PW, p.P - panel);       // the last group of an odd P has one panel
    const int ks0 = split * p.ksps;
    const int ks1 = min(p.KS, ks0 + p.ksps);
    // a missing second panel streams the first one again; its result is dropped
    const int64_t pstride = (npanels > 1) ? (int64_t)p.KS * (kPanelTiles * 64) : 0;

    MfmaI8Op<MB, PW> op;
    op.init(p.B, p.xpitch, g, i);
    if constexpr (PREQ) {
        XStageCodes<NT, 4> xst;
        xst.init(p);
        stream_panel<NW, DEPTH, PW, false, staging_passes(MB, DEPTH, false)>(p, xs, xst, op, tid, wave, lane, panel,
                                                                             pstride, ks0, ks1);
    } else {
        XStageI8<NT, 2> xst;       // two 32-byte reads per thread in flight: NT*32 bytes of LDS per pass
        xst.p_stats = lds_stats;
        stream_panel<NW, DEPTH, PW, false>(p, xs, xst, op, tid, wave, lane, panel, pstride, ks0, ks1);
    }

    RowOperands<NW> ops[PW][MB];       // bias / residual of all passes, requested ahead of the first barrier
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
                __syncthreads();               // X buffers / previous pass no longer needed
#pragma unroll
                for (int t = 0; t < kPanelTiles; ++t)
                    *reinterpret_cast<i32x4*>(red + (wave * 16 + i) * kRedPitch + t * kTileN + 4 * g) =
                        op.acc[q * kPanelTiles + t][m];
                __syncthreads();
                reduce_rows<NW, true>(p, red, m, panel + q, split, tid, ops[q][m], stats);
            }
            if (p.S > 1) finish_split_k<NT, true>(p, panel + q, tid, &s_flag, stats);
        }
    }
}

// Two-panel blocks, second form (as sbi_mfma_wg_kernel): eight waves in two groups of four, each group
// streaming one of the two panels against the same staged tile of pre-quantised codes; four-way
// integer reductions, the two panels side by side.
template <int MB, int DEPTH>
__global__ __launch_bounds__(512) void sbi_i8_wg_kernel(const GroupParams gp)
{
    constexpr int NT = 512, GW = 4;
    int gi = 0;
    while (gi + 1 < gp.G && (int)blockIdx.x >= gp.first_block[gi + 1]) ++gi;
    const GemmParams& p = gp.g[gi];
    const int bid = (int)blockIdx.x - gp.first_block[gi];
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    const floatx2* stats = p.xstats;
    u32x4* xs  = reinterpret_cast<u32x4*>(smem_raw + kLnStatsBytes);
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

    MfmaI8Op<MB, 1> op;
    op.init(p.B, p.xpitch, g, i);
    XStageCodes<NT, 4> xst;
    xst.init(p);
    stream_panel<GW, DEPTH, 1, false, staging_passes(MB, DEPTH, false, 2)>(p, xs, xst, op, tid, kwave, lane, panel, 0,
                                                                            ks0, ks1);

    float* red = reinterpret_cast<float*>(smem_raw + kLnStatsBytes) + grp * (GW * 16 * kRedPitch);
    const int gtid = tid & (GW * 64 - 1);
    RowOperands<GW> ops[MB];
#pragma unroll
    for (int m = 0; m < MB; ++m) ops[m] = request_row_operands<GW>(p, m, panel, gtid, m == 0, ops[0]);
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        __syncthreads();
#pragma unroll
        for (int t = 0; t < kPanelTiles; ++t)
            *reinterpret_cast<i32x4*>(red + (kwave * 16 + i) * kRedPitch + t * kTileN + 4 * g) = op.acc[t][m];
        __syncthreads();
        if (grp < npanels) reduce_rows<GW, true>(p, red, m, panel, split, gtid, ops[m], stats);
    }
    if (p.S > 1) {
        for (int q = 0; q < npanels; ++q) finish_split_k<NT, true>(p, panel0 + q, tid, &s_flag, stats);
    }
}

template <int MB, int DEPTH>
static int launch_wg_one(const GroupParams& gp, size_t lds, hipStream_t st)
{
    if (lds > 64 * 1024) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sbi_i8_wg_kernel<MB, DEPTH>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return (int)e;
    }
    hipLaunchKernelGGL((sbi_i8_wg_kernel<MB, DEPTH>), dim3(gp.first_block[gp.G]), dim3(512), lds, st, gp);
    return (int)hipGetLastError();
}

static int launch_wg(const GroupParams& gp, size_t lds, hipStream_t st)
{
    if (lds < kLnStatsBytes + 2 * 4 * 16 * kRedPitch * sizeof(float)) return (int)hipErrorInvalidValue;
    switch ((gp.g[0].B + 15) / 16) {
        case 2: return launch_wg_one<2, 4>(gp, lds, st);
        case 3: return launch_wg_one<3, 4>(gp, lds, st);
        case 4: return launch_wg_one<4, 4>(gp, lds, st);
    }
    return (int)hipErrorInvalidValue;
}

template <int MB, int NW, int DEPTH, int PW, bool PREQ>
static int launch_one(const GroupParams& gp, size_t lds, hipStream_t st)
{
    if (lds > 64 * 1024) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sbi_i8_kernel<MB, NW, DEPTH, PW, PREQ>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return (int)e;
    }
    hipLaunchKernelGGL((sbi_i8_kernel<MB, NW, DEPTH, PW, PREQ>), dim3(gp.first_block[gp.G]), dim3(NW * 64), lds, st, gp);
    return (int)hipGetLastError();
}

template <int NW, int DEPTH, int PW, bool PREQ>
static int launch_mb(const GroupParams& gp, size_t lds, hipStream_t st)
{
    switch ((gp.g[0].B + 15) / 16) {
        case 1: return launch_one<1, NW, DEPTH, PW, PREQ>(gp, lds, st);
        case 2: return launch_one<2, NW, DEPTH, PW, PREQ>(gp, lds, st);
        case 3: return launch_one<3, NW, DEPTH, PW, PREQ>(gp, lds, st);
        case 4: return launch_one<4, NW, DEPTH, PW, PREQ>(gp, lds, st);
    }
    return (int)hipErrorInvalidValue;
}

// Quantises the rows of up to kMaxGroup activation matrices [B,K_g] (one block per row): codes
// to q.codes[g] ([B,K_g] int8), (inv, scale) per row to q.stats[g].  Same decisions as i8_stats /
// quantize16.  K_g % 16 == 0.
struct QuantRowsParams {
    const _Float16* X[kMaxGroup];
    signed char* codes[kMaxGroup];
    floatx2* stats[kMaxGroup];
    const _Float16* gamma[kMaxGroup];     // not null: layer-normalise the row first (see below)
    const _Float16* beta[kMaxGroup];
    float eps[kMaxGroup];
    int K[kMaxGroup];
    int B;
};

// fp64 -> fp16 in ONE rounding step (to nearest, ties to even): the value goes to binary32 rounded to
// odd (truncate, then set the last bit if anything was lost), which keeps enough information for
// the final rounding to the 11-bit significand to be the correct one.
__device__ __forceinline__ _Float16 double_to_half_rn(double d)
{
    float f = __double2float_rz(d);
    if ((double)f != d) f = __builtin_bit_cast(float, __builtin_bit_cast(unsigned int, f) | 1u);
    return (_Float16)f;
}

__device__ __forceinline__ double block_sum_256(double v, double* s_part, int lane, int wave)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    __syncthreads();                       // s_part may still be read from the previous use
    if (lane == 0) s_part[wave] = v;
    __syncthreads();
    return (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
}

// Layer-norm in front of the INT8 GeMM (paper Sec. III-D: the fused regions start with the input
// layer-norm whatever the GeMM's data type).  The normalised fp16 value decides an integer code, so
// it has to be THE fp16 value of the definition, not one that is an ulp off now and then: the row
// statistics and (x - mean) * rstd * gamma + beta are evaluated in fp64 here (a few thousand
// operations per row: nothing next to the weight stream) and rounded once to fp16, after which
// the quantisation is the plain one.  Returns the row's normalised piece c (16 values).
__device__ __forceinline__ void ln_piece16(const _Float16* row, const _Float16* gamma, const _Float16* beta, int c,
                                           double mean, double rstd, u32x4& lo, u32x4& hi)
{
    half8 y[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const half8 x = __builtin_bit_cast(half8, *reinterpret_cast<const u32x4*>(row + c * 16 + h * 8));
        const half8 gm = __builtin_bit_cast(half8, *reinterpret_cast<const u32x4*>(gamma + c * 16 + h * 8));
        const half8 bt = __builtin_bit_cast(half8, *reinterpret_cast<const u32x4*>(beta + c * 16 + h * 8));
#pragma unroll
        for (int e = 0; e < 8; ++e)
            y[h][e] = double_to_half_rn(((double)x[e] - mean) * rstd * (double)gm[e] + (double)bt[e]);
    }
    lo = __builtin_bit_cast(u32x4, y[0]);
    hi = __builtin_bit_cast(u32x4, y[1]);
}

__global__ __launch_bounds__(256) void sbi_quantize_rows_kernel(const QuantRowsParams q)
{
    __shared__ float s_max[4];
    __shared__ double s_part[4];
    const int g = (int)blockIdx.x / q.B, b = (int)blockIdx.x - g * q.B;
    const int K = q.K[g];
    const _Float16* row = q.X[g] + (int64_t)b * K;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pieces = K / 16;
    const _Float16* gamma = q.gamma[g];
    const _Float16* beta = q.beta[g];
    double mean = 0.0, rstd = 0.0;
    if (gamma) {                           // block-uniform
        double s = 0.0;
        for (int c = tid; c < pieces; c += 256) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const half8 x = __builtin_bit_cast(half8, *reinterpret_cast<const u32x4*>(row + c * 16 + h * 8));
#pragma unroll
                for (int e = 0; e < 8; ++e) s += (double)x[e];
            }
        }
        mean = block_sum_256(s, s_part, lane, wave) / (double)K;
        double v = 0.0;
        for (int c = tid; c < pieces; c += 256) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const half8 x = __builtin_bit_cast(half8, *reinterpret_cast<const u32x4*>(row + c * 16 + h * 8));
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const double d = (double)x[e] - mean;
                    v += d * d;
                }
            }
        }
        const double var = block_sum_256(v, s_part, lane, wave) / (double)K;
        rstd = 1.0 / sqrt(var + (double)q.eps[g]);
    }
    float m = 0.f;
    for (int c = tid; c < pieces; c += 256) {
        u32x4 lo, hi;
        if (gamma) {
            ln_piece16(row, gamma, beta, c, mean, rstd, lo, hi);
        } else {
            const u32x4* src = reinterpret_cast<const u32x4*>(row + c * 16);
            lo = src[0];
            hi = src[1];
        }
        const half8 a = __builtin_bit_cast(half8, lo);
        const half8 h = __builtin_bit_cast(half8, hi);
#pragma unroll
        for (int e = 0; e < 8; ++e) m = fmaxf(m, fmaxf(fabsf((float)a[e]), fabsf((float)h[e])));
    }
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) m = fmaxf(m, __shfl_xor(m, s, 64));
    if (lane == 0) s_max[wave] = m;
    __syncthreads();
    const float amax = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
    const float inv = (amax > 0.f) ? 127.0f / amax : 0.f;
    if (tid == 0) q.stats[g][b] = (amax > 0.f) ? floatx2{inv, amax / 127.0f} : floatx2{0.f, 0.f};
    u32x4* dst = reinterpret_cast<u32x4*>(q.codes[g] + (int64_t)b * K);
    for (int c = tid; c < pieces; c += 256) {
        u32x4 lo, hi;
        if (gamma) {                       // the same arithmetic as in the pass above: the same fp16 values
            ln_piece16(row, gamma, beta, c, mean, rstd, lo, hi);
        } else {
            const u32x4* src = reinterpret_cast<const u32x4*>(row + c * 16);
            lo = src[0];
            hi = src[1];
        }
        dst[c] = quantize16(lo, hi, inv);
    }
}

int launch_i8(const GroupParams& gp, int waves, int depth, int panels, bool prequantized, size_t lds_bytes, hipStream_t st)
{
    if (gp.G < 1 || gp.G > kMaxGroup) return (int)hipErrorInvalidValue;
    if (panels == 2 && !(prequantized && waves == 8 && (depth == 2 || depth == 4))) return (int)hipErrorInvalidValue;
    if (panels != 1 && panels != 2) return (int)hipErrorInvalidValue;
    if (prequantized) {
        const bool groups = panels == 2 && depth == 4;      // two wave groups, one panel each
        if (!spread_staging_fits(gp, waves, depth, false, groups ? 2 : 1)) return (int)hipErrorInvalidValue;
        // gp.g[k].X already points at the codes' place in the workspace: fill it from gp.g[k].X16
        QuantRowsParams q;
        for (int k = 0; k < gp.G; ++k) {
            q.X[k] = gp.g[k].X16;
            q.codes[k] = reinterpret_cast<signed char*>(const_cast<_Float16*>(gp.g[k].X));
            q.stats[k] = const_cast<floatx2*>(gp.g[k].xstats);
            q.K[k] = gp.g[k].K;
            q.gamma[k] = gp.g[k].ln ? gp.g[k].ln_gamma : nullptr;       // layer-norm, then quantise
            q.beta[k] = gp.g[k].ln ? gp.g[k].ln_beta : nullptr;
            q.eps[k] = gp.g[k].ln_eps;
        }
        for (int k = gp.G; k < kMaxGroup; ++k) { q.X[k] = nullptr; q.codes[k] = nullptr; q.stats[k] = nullptr; q.gamma[k] = nullptr; q.beta[k] = nullptr; q.eps[k] = 0.f; q.K[k] = 0; }
        q.B = gp.g[0].B;
        hipLaunchKernelGGL(sbi_quantize_rows_kernel, dim3(gp.G * q.B), dim3(256), 0, st, q);
        if (hipGetLastError() != hipSuccess) return (int)hipErrorInvalidValue;
        if (groups) return launch_wg(gp, lds_bytes, st);
        if (panels == 2) return launch_mb<8, 2, 2, true>(gp, lds_bytes, st);
        if (waves == 4 && depth == 2) return launch_mb<4, 2, 1, true>(gp, lds_bytes, st);
        if (waves == 4 && depth == 4) return launch_mb<4, 4, 1, true>(gp, lds_bytes, st);
        if (waves == 8 && depth == 4) return launch_mb<8, 4, 1, true>(gp, lds_bytes, st);
        return (int)hipErrorInvalidValue;
    }
    if (waves == 4 && depth == 2) return launch_mb<4, 2, 1, false>(gp, lds_bytes, st);
    if (waves == 4 && depth == 4) return launch_mb<4, 4, 1, false>(gp, lds_bytes, st);
    if (waves == 8 && depth == 4) return launch_mb<8, 4, 1, false>(gp, lds_bytes, st);
    return (int)hipErrorInvalidValue;
}

template <int NW, int DEPTH, int PW, bool PREQ>
static const void* entry_mb(int mb)
{
    switch (mb) {
        case 1: return reinterpret_cast<const void*>(&sbi_i8_kernel<1, NW, DEPTH, PW, PREQ>);
        case 2: return reinterpret_cast<const void*>(&sbi_i8_kernel<2, NW, DEPTH, PW, PREQ>);
        case 3: return reinterpret_cast<const void*>(&sbi_i8_kernel<3, NW, DEPTH, PW, PREQ>);
        case 4: return reinterpret_cast<const void*>(&sbi_i8_kernel<4, NW, DEPTH, PW, PREQ>);
    }
    return nullptr;
}

// The GeMM kernel launch_i8 would start for this block shape, as mfma_kernel_entry.
const void* i8_kernel_entry(int mb, int waves, int depth, int panels, bool prequantized)
{
    if (prequantized) {
        if (panels == 2 && waves == 8 && depth == 4) {
            switch (mb) {
                case 2: return reinterpret_cast<const void*>(&sbi_i8_wg_kernel<2, 4>);
                case 3: return reinterpret_cast<const void*>(&sbi_i8_wg_kernel<3, 4>);
                case 4: return reinterpret_cast<const void*>(&sbi_i8_wg_kernel<4, 4>);
            }
            return nullptr;
        }
        if (panels == 2) return (waves == 8 && depth == 2) ? entry_mb<8, 2, 2, true>(mb) : nullptr;
        if (waves == 4 && depth == 2) return entry_mb<4, 2, 1, true>(mb);
        if (waves == 4 && depth == 4) return entry_mb<4, 4, 1, true>(mb);
        if (waves == 8 && depth == 4) return entry_mb<8, 4, 1, true>(mb);
        return nullptr;
    }
    if (panels != 1) return nullptr;
    if (waves == 4 && depth == 2) return entry_mb<4, 2, 1, false>(mb);
    if (waves == 4 && depth == 4) return entry_mb<4, 4, 1, false>(mb);
    if (waves == 8 && depth == 4) return entry_mb<8, 4, 1, false>(mb);
    return nullptr;
}

// ---- weight preparation (once, at initialisation) ------------------------------------------
// Pre-layout of int8 codes Wq [K,N] row-major: block (p, ks) writes the 4 KiB of one panel
// k-step; thread (t, g, i) gathers the 16 codes k = ks*64 + 16g .. +15 of column p*64 + 16t + i
// and writes them as one 16-byte piece.  Zero beyond K and N.  Block 0 also writes the header.
__global__ __launch_bounds__(256) void sbi_layout_i8_kernel(const signed char* __restrict__ Wq, int64_t K, int64_t N,
                                                            int64_t KS, int64_t P, unsigned char* __restrict__ out)
{
    const int64_t blk = blockIdx.x;
    const int64_t pn = blk / KS, ks = blk - pn * KS;
    const int tid = threadIdx.x;
    const int t = tid >> 6, lane = tid & 63, g = lane >> 4, i = lane & 15;
    const int64_t n = pn * kPanelN + t * kTileN + i;
    const int64_t k0 = ks * kI8TileK + g * kI8ChunkK;
    unsigned int w[4] = {0u, 0u, 0u, 0u};
    if (n < N) {
#pragma unroll
        for (int e = 0; e < kI8ChunkK; ++e) {
            const int64_t k = k0 + e;
            const unsigned int v = (k < K) ? (unsigned int)(unsigned char)Wq[k * N + n] : 0u;
            w[e >> 2] |= v << (8 * (e & 3));
        }
    }
    u32x4* dst = reinterpret_cast<u32x4*>(out + kHeaderBytes) + (blk * kPanelTiles + t) * 64 + lane;
    *dst = u32x4{w[0], w[1], w[2], w[3]};
    if (blk == 0) {
        constexpr int kHeaderWords = (int)(sizeof(LayoutHeader) / 4);
        if (tid == 0) {
            LayoutHeader h;
            h.magic = kMagic; h.version = kLayoutVersion;
            h.K = K; h.N = N; h.KS = KS; h.P = P;
            h.tile_n = kTileN; h.tile_k = kI8TileK; h.panel_tiles = kPanelTiles; h.chunk_k = kI8ChunkK;
            *reinterpret_cast<LayoutHeader*>(out) = h;
        } else if (tid >= kHeaderWords && tid < kHeaderBytes / 4) {
            reinterpret_cast<uint32_t*>(out)[tid] = 0u;
        }
    }
}

int launch_layout_i8(const void* Wq, int64_t K, int64_t N, void* out, hipStream_t st)
{
    const int64_t KS = ksteps_of_i8(K), P = (N + kPanelN - 1) / kPanelN;
    hipLaunchKernelGGL(sbi_layout_i8_kernel, dim3((unsigned)(KS * P)), dim3(256), 0, st,
                       reinterpret_cast<const signed char*>(Wq), K, N, KS, P, reinterpret_cast<unsigned char*>(out));
    return (int)hipGetLastError();
}

// Symmetric per-column quantisation of W [K,N] fp16 -> codes [K,N] int8 + scales [N] binary32,
// the same decisions as for the activations (amax, inv = 127/amax, rint(w * inv), scale = amax/127).
// One block per 64 columns: thread (r, c) scans rows r, r+4, ... of column c twice.
__global__ __launch_bounds__(256) void sbi_quantize_weights_kernel(const _Float16* __restrict__ W, int64_t K, int64_t N,
                                                                   signed char* __restrict__ Wq, float* __restrict__ scales)
{
    __shared__ float s_max[4][64];
    const int c = threadIdx.x & 63, r = threadIdx.x >> 6;
    const int64_t n = (int64_t)blockIdx.x * 64 + c;
    float m = 0.f;
    if (n < N)
        for (int64_t k = r; k < K; k += 4) m = fmaxf(m, fabsf((float)W[k * N + n]));
    s_max[r][c] = m;
    __syncthreads();
    const float amax = fmaxf(fmaxf(s_max[0][c], s_max[1][c]), fmaxf(s_max[2][c], s_max[3][c]));
    const float inv = (amax > 0.f) ? 127.0f / amax : 0.f;
    if (n < N) {
        if (r == 0) scales[n] = (amax > 0.f) ? amax / 127.0f : 0.f;
        for (int64_t k = r; k < K; k += 4) {
            float q = rintf((float)W[k * N + n] * inv);
            q = fminf(fmaxf(q, -127.0f), 127.0f);
            Wq[k * N + n] = (signed char)(int)q;
        }
    }
}

int launch_quantize_weights(const void* W, int64_t K, int64_t N, void* Wq, void* scales, hipStream_t st)
{
    hipLaunchKernelGGL(sbi_quantize_weights_kernel, dim3((unsigned)((N + 63) / 64)), dim3(256), 0, st,
                       reinterpret_cast<const _Float16*>(W), K, N, reinterpret_cast<signed char*>(Wq),
                       reinterpret_cast<float*>(scales));
    return (int)hipGetLastError();
}

}  // namespace sbi
