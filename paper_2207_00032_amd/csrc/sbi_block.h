// Block-level building blocks shared by the streaming kernels (device code, gfx950):
//   - staging a K-chunk of the small X tile in LDS, in the order the lanes consume it
//   - the in-block K-split reduction through LDS
//   - the cross-block split-K reduction by the last-arriving block (deterministic order)
//   - the fused epilogue (bias, exact-erf GeLU, residual) and the fp16 store
#pragma once
#include "sbi_common.h"

namespace sbi {

// GeLU(v) = v * Phi(v) with the exact-erf definition Phi(v) = (1 + erf(v / sqrt 2)) / 2.
// erfc(|x|) from the rational-times-Gaussian approximation 7.1.26 of Abramowitz & Stegun
// (|error| <= 1.5e-7 in erf): a dozen VALU operations instead of the math library's erff, whose
// ~100 made the epilogue of the large-batch GeLU GeMM (64 x 128 outputs per block) the longest
// part of a block's tail.  Forming Phi from erfc on the negative side keeps the small values of
// the left tail relatively accurate; the error in GeLU is below 1e-7 * |v|, orders of magnitude
// under the fp16 rounding that follows.
__device__ __forceinline__ float gelu_erf(float v)
{
    const float x = fabsf(v) * 0.70710678118654752440f;
    const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * x);
    const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
    const float erfc_x = poly * __builtin_amdgcn_exp2f(-x * x * 1.44269504088896340736f);
    return 0.5f * v * (v < 0.f ? erfc_x : 2.0f - erfc_x);
}

// Final value of one output element from its fp32 sum.
__device__ __forceinline__ float apply_epilogue(const GemmParams& p, float v, int b, int n)
{
    if (p.flags & kEpiBias) v += (float)p.bias[n];
    if (p.flags & kEpiGelu) v = gelu_erf(v);
    if (p.flags & kEpiRes)  v += (float)p.R[(int64_t)b * p.N + n];
    return v;
}

// What the epilogue of the column pair (n, n+1) of row b reads from memory, fetched ahead of the
// sums it will be applied to (so that the reads overlap the reduction instead of following it).
struct EpiOperands {
    float bias0, bias1, res0, res1;
};

__device__ __forceinline__ void load_bias_pair(const GemmParams& p, int n, EpiOperands& e)
{
    if ((p.flags & kEpiBias) && n < p.N) {
        e.bias0 = (float)p.bias[n];
        if (n + 1 < p.N) e.bias1 = (float)p.bias[n + 1];
    }
}

__device__ __forceinline__ void load_residual_pair(const GemmParams& p, int b, int n, EpiOperands& e)
{
    if ((p.flags & kEpiRes) && b < p.B && n < p.N) {
        const _Float16* r = p.R + (int64_t)b * p.N + n;
        e.res0 = (float)r[0];
        if (n + 1 < p.N) e.res1 = (float)r[1];
    }
}

__device__ __forceinline__ EpiOperands load_epilogue_operands(const GemmParams& p, int b, int n)
{
    EpiOperands e = {0.f, 0.f, 0.f, 0.f};
    load_bias_pair(p, n, e);
    load_residual_pair(p, b, n, e);
    return e;
}

__device__ __forceinline__ float apply_epilogue(const GemmParams& p, float v, float bias, float res)
{
    if (p.flags & kEpiBias) v += bias;
    if (p.flags & kEpiGelu) v = gelu_erf(v);
    if (p.flags & kEpiRes)  v += res;
    return v;
}

// Store the column pair (n, n+1) of row b; n is even.  One 4-byte store when both
// columns exist and the row pitch keeps it aligned, 2-byte stores otherwise.
// Epilogue, one rounding to fp16 and store of two adjacent outputs; y0, y1 receive the stored
// (rounded) values, 0 where the column does not exist.
__device__ __forceinline__ void store_pair(const GemmParams& p, int b, int n, float s0, float s1,
                                           const EpiOperands& e, float& y0, float& y1)
{
    y0 = y1 = 0.f;
    if (n >= p.N) return;
    const int64_t off = (int64_t)b * p.N + n;
    const _Float16 h0 = (_Float16)apply_epilogue(p, s0, e.bias0, e.res0);
    y0 = (float)h0;
    if (n + 1 < p.N) {
        const _Float16 h1 = (_Float16)apply_epilogue(p, s1, e.bias1, e.res1);
        y1 = (float)h1;
        if ((p.N & 1) == 0) {
            half2v h = {h0, h1};
            *reinterpret_cast<half2v*>(p.Y + off) = h;
        } else {
            p.Y[off] = h0;
            p.Y[off + 1] = h1;
        }
    } else {
        p.Y[off] = h0;
    }
}

__device__ __forceinline__ void store_pair(const GemmParams& p, int b, int n, float s0, float s1,
                                           float& y0, float& y1)
{
    store_pair(p, b, n, s0, s1, load_epilogue_operands(p, b, n), y0, y1);
}

__device__ __forceinline__ void store_pair(const GemmParams& p, int b, int n, float s0, float s1)
{
    float y0, y1;
    store_pair(p, b, n, s0, s1, y0, y1);
}

// The next layer-norm's share of this epilogue (paper Sec. III-B / III-D: bias, residual and
// the following layer-norm belong to one fused region; a full normalisation needs the whole
// row, which is spread over the panels of different blocks, so what the epilogue can finish is
// each panel's part): the 32 consecutive lanes that have just stored one row's 64 outputs of a
// panel reduce (mean, sum of squared deviations from it) over the stored fp16 values and write
// them to moments_out[b][panel]; the consuming kernel merges the panels of a row exactly
// (ln_stats_from_moments) instead of reading the row again.
__device__ __forceinline__ void emit_moments(const GemmParams& p, int b, int panel, int n, float y0, float y1, int lane)
{
    const int cnt = min(kPanelN, p.N - panel * kPanelN);         // columns of this panel that exist
    float s = y0 + y1;                                            // absent columns were returned as 0
#pragma unroll
    for (int m = 16; m >= 1; m >>= 1) s += __shfl_xor(s, m, 32);  // the other half of the wave may hold another row, or none
    const float mean = s / (float)cnt;
    const float d0 = (n < p.N) ? y0 - mean : 0.f;
    const float d1 = (n + 1 < p.N) ? y1 - mean : 0.f;
    float q = d0 * d0 + d1 * d1;
#pragma unroll
    for (int m = 16; m >= 1; m >>= 1) q += __shfl_xor(q, m, 32);
    if ((lane & 31) == 0) p.moments_out[(int64_t)b * p.P + panel] = floatx2{mean, q};
}

// ---- layer normalisation in front of the GeMM (paper Sec. III-D, regions 1 and 3) ----------
// Every block recomputes the statistics of all B rows of X (the paper does the same: the input
// batch is broadcast to every SM and the operations before the GeMM are repeated there, so no
// kernel boundary is needed).  Wave w takes rows w, w+NW, ...; two passes over the row (mean,
// then the biased variance around it) in fp32, lanes strided over 16-byte pieces, the second
// pass re-reading the row from L2.  stats[b] = (mean, 1/sqrt(var + eps)).
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// Sum of the 8 halfs of a piece, and of their squared distances from `mean`, in fp32.
__device__ __forceinline__ float piece_sum(u32x4 h)
{
    const half8 v = __builtin_bit_cast(half8, h);
    float t = 0.f;
#pragma unroll
    for (int e = 0; e < kChunkK; ++e) t += (float)v[e];
    return t;
}
__device__ __forceinline__ float piece_sqdev(u32x4 h, float mean)
{
    const half8 v = __builtin_bit_cast(half8, h);
    float t = 0.f;
#pragma unroll
    for (int e = 0; e < kChunkK; ++e) {
        const float d = (float)v[e] - mean;
        t += d * d;
    }
    return t;
}

// Row statistics from the per-panel moments the producing GeMM's epilogue left behind
// (emit_moments; panels of 64 features, K % 64 == 0): the exact pairwise merge
//   mean = sum_p n_p mean_p / K,   M2 = sum_p (M2_p + n_p (mean_p - mean)^2),   var = M2 / K.
template <int NW>
__device__ __forceinline__ void ln_stats_from_moments(const GemmParams& p, floatx2* stats, int wave, int lane)
{
    const int P = p.K / kPanelN;
    for (int r = wave; r < p.B; r += NW) {
        const floatx2* m = p.ln_moments + (int64_t)r * P;
        float s = 0.f;
        for (int j = lane; j < P; j += 64) s += m[j][0];
        const float mean = wave_sum(s) / (float)P;
        float q = 0.f;
        for (int j = lane; j < P; j += 64) {
            const floatx2 v = m[j];
            const float d = v[0] - mean;
            q += v[1] + (float)kPanelN * d * d;
        }
        const float var = wave_sum(q) / (float)p.K;
        if (lane == 0) stats[r] = floatx2{mean, 1.0f / sqrtf(var + p.ln_eps)};
    }
}

// R rows per wave at a time (rows r, r + NW, ...), so that their loads share one memory latency.
template <int NW>
__device__ __forceinline__ void ln_stats(const GemmParams& p, floatx2* stats, int wave, int lane)
{
    if (p.ln_moments) {
        ln_stats_from_moments<NW>(p, stats, wave, lane);
        return;
    }
    constexpr int U = 8;                       // 128-bit loads in flight per lane and row: 4096 elements
    constexpr int R = 2;
    const int pieces = p.K / kChunkK;
    const bool resident = pieces <= 64 * U;    // whole rows stay in registers for the second pass
    for (int r0 = wave; r0 < p.B; r0 += R * NW) {
        const _Float16* row[R];
#pragma unroll
        for (int j = 0; j < R; ++j) row[j] = p.X + (int64_t)min(r0 + j * NW, p.B - 1) * p.K;
        u32x4 h[R][U];
        float s[R], q[R], mean[R];
#pragma unroll
        for (int j = 0; j < R; ++j) s[j] = q[j] = 0.f;
        for (int c0 = 0; c0 < pieces; c0 += 64 * U) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = min(c0 + u * 64 + lane, pieces - 1) * kChunkK;
#pragma unroll
                for (int j = 0; j < R; ++j) h[j][u] = *reinterpret_cast<const u32x4*>(row[j] + c);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const bool in = c0 + u * 64 + lane < pieces;
#pragma unroll
                for (int j = 0; j < R; ++j) s[j] += in ? piece_sum(h[j][u]) : 0.f;
            }
        }
#pragma unroll
        for (int j = 0; j < R; ++j) mean[j] = wave_sum(s[j]) / (float)p.K;
        for (int c0 = 0; c0 < pieces; c0 += 64 * U) {
            if (!resident) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int c = min(c0 + u * 64 + lane, pieces - 1) * kChunkK;
#pragma unroll
                    for (int j = 0; j < R; ++j) h[j][u] = *reinterpret_cast<const u32x4*>(row[j] + c);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const bool in = c0 + u * 64 + lane < pieces;
#pragma unroll
                for (int j = 0; j < R; ++j) q[j] += in ? piece_sqdev(h[j][u], mean[j]) : 0.f;
            }
        }
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const float var = wave_sum(q[j]) / (float)p.K;
            if (lane == 0 && r0 + j * NW < p.B) stats[r0 + j * NW] = floatx2{mean[j], 1.0f / sqrtf(var + p.ln_eps)};
        }
    }
}

// y = (x - mean) * rstd * gamma + beta on 8 halfs, computed in fp32, rounded once to fp16.
__device__ __forceinline__ half8 ln_apply(half8 xh, half8 gh, half8 bh, floatx2 st)
{
    half8 y;
#pragma unroll
    for (int e = 0; e < kChunkK; ++e)
        y[e] = (_Float16)(((float)xh[e] - st[0]) * st[1] * (float)gh[e] + (float)bh[e]);
    return y;
}

// Staging of k-steps [cb, cb+cn) of X for all B rows into LDS.  Element order in LDS (16-byte
// units): ((ks - cb)*4 + g)*xpitch + b  holds X[b][ks*32 + g*8 .. +8], zero beyond K.  xpitch is B
// rounded up to an odd number: a wave writes 64 consecutive pieces of one row, i.e. addresses
// xpitch*16 bytes apart, and only an odd pitch spreads those over all LDS banks (an even B >= 8
// would put every lane of the write on the same four banks).
// Two phases so that the global reads can be requested ahead of the weight stream's first
// loads and written to LDS once they arrive: request() issues up to XU unconditional
// 128-bit loads per thread (addresses clamped into the tensor), commit() writes them to LDS
// and handles whatever did not fit (large B) or cannot be read as vectors (K % 8 != 0).
// LN (layer-norm kernel variant) and p.ln set: X is staged raw, and the same k-steps of gamma
// and beta travel along as two further "rows", stored after the X chunk (which always occupies
// p.kc k-steps): gamma piece (ks, g) at p.kc*4*xpitch + (ks - cb)*4 + g, beta p.kc*4 pieces later.
// The normalisation itself happens where the operand is read (see MfmaOp).
template <int NT, int XU, bool LN>
struct XStage {
    u32x4 buf[XU];

    static __device__ __forceinline__ int rows(const GemmParams& p) { return p.B + ((LN && p.ln) ? 2 : 0); }

    // source of piece c of staging row b (rows B and B+1 are gamma and beta)
    static __device__ __forceinline__ const _Float16* src(const GemmParams& p, int b, int k)
    {
        const _Float16* base = p.X + (int64_t)b * p.K;
        if constexpr (LN) {
            base = (b == p.B) ? p.ln_gamma : base;
            base = (b > p.B) ? p.ln_beta : base;
        }
        return base + k;
    }
    static __device__ __forceinline__ int dst(const GemmParams& p, int b, int c)
    {
        int d = c * p.xpitch + b;
        if constexpr (LN) d = (b >= p.B) ? p.kc * 4 * p.xpitch + (b - p.B) * p.kc * 4 + c : d;
        return d;
    }

    // Pass j of a chunk covers pieces [j*NT*XU, (j+1)*NT*XU); the plain request/commit pair is pass 0
    // plus, inside commit, whatever is left.
    __device__ __forceinline__ void request(const GemmParams& p, int cb, int cn, int tid, int j = 0)
    {
        if (!p.x_vec) return;
        const int nc = cn * 4;             // 16-byte pieces per row
        const int items = nc * rows(p);
#pragma unroll
        for (int u = 0; u < XU; ++u) {
            const int idx = min(j * (NT * XU) + tid + u * NT, items - 1);
            const int b = idx / nc;
            const int c = idx - b * nc;
            const int k = min(cb * kTileK + c * kChunkK, p.K - kChunkK);
            buf[u] = *reinterpret_cast<const u32x4*>(src(p, b, k));
        }
    }

    // Writes what request(..., j) fetched (vector-readable X only).
    __device__ __forceinline__ void commit_pass(const GemmParams& p, u32x4* xs, int cb, int cn, int tid, int j)
    {
        const int nc = cn * 4;
        const int items = nc * rows(p);
#pragma unroll
        for (int u = 0; u < XU; ++u) {
            const int idx = j * (NT * XU) + tid + u * NT;
            if (idx < items) {
                const int b = idx / nc;
                const int c = idx - b * nc;
                const bool inside = cb * kTileK + c * kChunkK < p.K;
                xs[dst(p, b, c)] = inside ? buf[u] : u32x4{0u, 0u, 0u, 0u};
            }
        }
    }

    __device__ __forceinline__ void commit(const GemmParams& p, u32x4* xs, int cb, int cn, int tid)
    {
        const int nc = cn * 4;
        const int items = nc * rows(p);
        if (p.x_vec) {
            commit_pass(p, xs, cb, cn, tid, 0);
            // what did not fit in the first pass: further passes of XU pieces per thread, all
            // reads of a pass issued before its LDS writes (one memory latency per pass)
            for (int base = NT * XU; base < items; base += NT * XU) {
                u32x4 v[XU];
#pragma unroll
                for (int u = 0; u < XU; ++u) {
                    const int idx = min(base + tid + u * NT, items - 1);
                    const int b = idx / nc;
                    const int c = idx - b * nc;
                    const int k = min(cb * kTileK + c * kChunkK, p.K - kChunkK);
                    v[u] = *reinterpret_cast<const u32x4*>(src(p, b, k));
                }
#pragma unroll
                for (int u = 0; u < XU; ++u) {
                    const int idx = base + tid + u * NT;
                    if (idx < items) {
                        const int b = idx / nc;
                        const int c = idx - b * nc;
                        const bool inside = cb * kTileK + c * kChunkK < p.K;
                        xs[dst(p, b, c)] = inside ? v[u] : u32x4{0u, 0u, 0u, 0u};
                    }
                }
            }
            return;
        }
        for (int idx = tid; idx < items; idx += NT) {      // K % 8 != 0: element-wise reads (never layer-normed)
            const int b = idx / nc;
            const int c = idx - b * nc;
            const int k = cb * kTileK + c * kChunkK;
            half8 h;
#pragma unroll
            for (int e = 0; e < kChunkK; ++e)
                h[e] = (k + e < p.K) ? p.X[(int64_t)b * p.K + k + e] : (_Float16)0.0f;
            xs[c * p.xpitch + b] = __builtin_bit_cast(u32x4, h);
        }
    }
};

// ---------------------------------------------------------------------------------------
// The weight stream of one block.  The block owns panel `panel` and k-steps [ks0, ks1); its
// NW waves take those k-steps round-robin (wave w: ks0 + w, ks0 + w + NW, ...), so the block
// walks a contiguous run of the laid-out weights.  Each wave keeps DEPTH k-steps (4 x 128-bit
// loads per lane each) in flight in a register ring with static indices: a round consumes
// slot d and refills it in place, d = 0..DEPTH-1, as straight-line code so the load-counter
// waits stay exact.  The ring runs without interruption over the whole range.  All waves of a
// block run the same number of rounds; a step that falls beyond the end of the range re-reads
// the range's last k-step and has its weights replaced by zeros before use, so the loop
// needs no conditional loads (the dispatcher picks splits that leave no such padding for
// the shapes that matter).
// X is staged in LDS in chunks of p.kc k-steps (a multiple of NW*DEPTH, so a round never
// straddles a chunk).  With more than one chunk the LDS holds two buffers: the global reads
// of chunk c+1 are requested when chunk c starts, written to the other buffer when chunk c
// ends, and one barrier separates the chunks - the weight ring is not drained.
// `op.begin(xk, ek)` receives the LDS address of a k-step's X block, `op.tile(t, w)` one of its
// weight tiles; X block: ([4 lane groups][xpitch rows] of 16 bytes).
// ---------------------------------------------------------------------------------------
// One k-step of PW adjacent panels: tiles 0..3 from the first panel, 4..7 from the next one
// (`pstride` 16-byte units further on: the same k-step of the following panel).
template <int PW>
__device__ __forceinline__ void load_step(u32x4 (&slot)[kPanelTiles * PW], const u32x4* src, int64_t pstride)
{
#pragma unroll
    for (int q = 0; q < PW; ++q)
#pragma unroll
        for (int t = 0; t < kPanelTiles; ++t)
            slot[q * kPanelTiles + t] = __builtin_nontemporal_load(src + q * pstride + t * 64);
}

// PW = panels per block (1 or 2): with two panels every wave streams both for the same
// k-steps, so one X operand read from LDS feeds twice as many MFMAs and the X tile is staged
// once for 128 columns - what larger batches need, where X traffic rivals the weight stream.
// LN: the layer-norm kernel variant; with p.ln set every X buffer also carries its k-steps of
// gamma and beta (see XStage) and op.step receives their address as well.
// Stage: how X reaches LDS (XStage for fp16 operands, XStageI8 for int8 codes); both fill
// 64 bytes per batch row and k-step, so the addressing below is the same.
// XP > 1 (batches above 16, where a chunk of X is one round of k-steps and more than one staging
// pass of the block): the passes are not all fetched while the waves wait at the end of the chunk,
// but spread over the round - after every DEPTH/XP steps the pass that has arrived goes to the idle
// buffer and the next one is requested, so each has DEPTH/XP steps of streaming to arrive in.
// staging_passes() gives XP for a kernel shape: the passes the largest batch of its MB needs,
// rounded up to a divisor of DEPTH (1, i.e. everything at the chunk's end, if there are more
// passes than steps, and for MB = 1, where chunks may be longer than a round).
// `wg` = wave groups a block's waves are divided into (each streams its own panel, so a round is
// 1/wg as many k-steps for the same number of staging threads).
__host__ __device__ constexpr int staging_passes(int mb, int depth, bool ln, int wg = 1)
{
    if (mb < 2) return 1;
    const int need = (depth * (16 * mb + (ln ? 2 : 0)) + 64 * wg - 1) / (64 * wg);   // rows * RS * 4 pieces over NT * 4 per pass
    for (int xp = 1; xp <= depth; ++xp)
        if (depth % xp == 0 && xp >= need) return xp;
    return 1;
}

// Host-side check of what spread staging assumes of every problem of a launch: a chunk is exactly
// one round of k-steps and no longer than XP passes of the block.
inline bool spread_staging_fits(const GroupParams& gp, int waves, int depth, bool layernorm, int wg = 1)
{
    const int xp = staging_passes((gp.g[0].B + 15) / 16, depth, layernorm, wg);
    if (xp == 1) return true;
    for (int g = 0; g < gp.G; ++g) {
        const int rows = gp.g[g].B + ((layernorm && gp.g[g].ln) ? 2 : 0);
        if (gp.g[g].kc != waves / wg * depth || gp.g[g].kc * 4 * rows > xp * waves * 64 * 4) return false;
    }
    return true;
}

template <int NW, int DEPTH, int PW, bool LN, int XP = 1, class Stage, class Op>
__device__ __forceinline__ void stream_panel(const GemmParams& p, u32x4* xs, Stage& xst, Op& op, int tid,
                                             int wave, int lane, int panel, int64_t pstride, int ks0, int ks1,
                                             unsigned long long* tmark = nullptr)
{
    static_assert(XP >= 1 && DEPTH % XP == 0, "staging passes are spread evenly over the steps of a round");
    constexpr int RS = NW * DEPTH;                                 // k-steps a block consumes per round
    constexpr int kStepUnits = kPanelTiles * 64;                  // 16-byte units per k-step of a panel
    const int nks = ks1 - ks0;                                     // >= 1
    const int rounds = (nks + RS - 1) / RS;
    const int rpc = p.kc / RS;                                     // rounds per X chunk
    const int nchunks = (rounds + rpc - 1) / rpc;
    const u32x4* wbase = p.Wl + ((int64_t)panel * p.KS + ks0) * kStepUnits + lane;
    const int xblock = 4 * p.xpitch;                               // 16-byte units of X per k-step
    const int eblock = (LN && p.ln) ? 4 : 0;                       // 16-byte units of gamma (and of beta) per k-step
    const int xbuf = p.kc * (xblock + 2 * eblock);                 // 16-byte units per X buffer

    u32x4 ring[DEPTH][kPanelTiles * PW];
#ifdef SBI_DEV
    const bool no_x = (p.flags >> 8) & 2;                          // development: X is not staged at all
    if (!no_x)
#endif
    xst.request(p, ks0, min(nks, p.kc), tid);
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
        load_step<PW>(ring[d], wbase + (int64_t)min(d * NW + wave, nks - 1) * kStepUnits, pstride);
#ifdef SBI_DEV
    if (!no_x) {
#endif
    xst.commit(p, xs, ks0, min(nks, p.kc), tid);
    if (nchunks > 1) xst.request(p, ks0 + p.kc, min(nks - p.kc, p.kc), tid);
    __syncthreads();
#ifdef SBI_DEV
    }
#endif
#ifdef SBI_TRACE
    if (tmark) tmark[0] = wall_clock64();                          // X staged
    bool first_step = true;
#endif

    int t = wave;                                                  // this wave's k-step inside the range
    int c = 0, rc = 0;                                             // X chunk, round inside the chunk
    const u32x4* xc = xs;                                          // xc + t*xblock: X block of step t
    const u32x4* ec = xs + p.kc * xblock;                          // ec + t*eblock: its gamma pieces
    for (int r = 0; r + 1 < rounds; ++r) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            // always inside the range here; every tile's registers are refilled right behind the
            // products that read them, so a slot is out of flight for one tile's products, not a step's
            op.begin(xc + t * xblock, ec + t * eblock);
            const u32x4* src = wbase + (int64_t)min(t + RS, nks - 1) * kStepUnits;
#pragma unroll
            for (int q = 0; q < PW; ++q)
#pragma unroll
                for (int tt = 0; tt < kPanelTiles; ++tt) {
                    op.tile(q * kPanelTiles + tt, ring[d][q * kPanelTiles + tt]);
                    ring[d][q * kPanelTiles + tt] = __builtin_nontemporal_load(src + q * pstride + tt * 64);
                }
            t += NW;
            __builtin_amdgcn_sched_barrier(0);
#ifdef SBI_TRACE
            if (tmark && first_step) { tmark[1] = wall_clock64(); first_step = false; }   // first k-step's weights consumed
#endif
            if constexpr (XP > 1) {
                if ((d + 1) % (DEPTH / XP) == 0 && d + 1 < DEPTH) { // every round ends a chunk: c+1 exists
                    const int j = (d + 1) / (DEPTH / XP) - 1;
                    const int cb = ks0 + (c + 1) * p.kc, cn = min(nks - (c + 1) * p.kc, p.kc);
                    if (p.x_vec) {                                 // (rows that cannot be read as vectors: all at the chunk's end)
                        xst.commit_pass(p, xs + ((c + 1) & 1) * xbuf, cb, cn, tid, j);
                        xst.request(p, cb, cn, tid, j + 1);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        if (XP > 1 || ++rc == rpc) {                               // chunk c is consumed, c+1 exists
            rc = 0;
            ++c;
            u32x4* dst = xs + (c & 1) * xbuf;
            bool staged = false;
            if constexpr (XP > 1) {
                if (p.x_vec) {
                    xst.commit_pass(p, dst, ks0 + c * p.kc, min(nks - c * p.kc, p.kc), tid, XP - 1);
                    staged = true;
                }
            }
            if (!staged) xst.commit(p, dst, ks0 + c * p.kc, min(nks - c * p.kc, p.kc), tid);
            __syncthreads();
            xc = dst - c * p.kc * xblock;
            ec = dst + p.kc * xblock - c * p.kc * eblock;
            if (c + 1 < nchunks) xst.request(p, ks0 + (c + 1) * p.kc, min(nks - (c + 1) * p.kc, p.kc), tid);
        }
    }
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
        if (t >= nks) {                                            // padding step: contributes nothing
#pragma unroll
            for (int q = 0; q < kPanelTiles * PW; ++q) ring[d][q] = u32x4{0u, 0u, 0u, 0u};
        }
        op.begin(xc + min(t, nks - 1) * xblock, ec + min(t, nks - 1) * eblock);
#pragma unroll
        for (int q = 0; q < kPanelTiles * PW; ++q) op.tile(q, ring[d][q]);
        t += NW;
    }
}

// ---- INT8 path (paper Sec. III-D "Support for Different Data Types": INT8 GeMM with the
// quantisation fused in front and the de-quantisation in the epilogue) -----------------------
// Symmetric per-row quantisation of the activations, decided in binary32 exactly as follows:
//   amax = max_k |x_k|,  inv = 127 / amax,  scale = amax / 127   (amax = 0: inv = scale = 0)
//   code = clamp(rint(x * inv), -127, 127)                        (rint: ties to even)
// Every block computes (inv, scale) of all B rows before its weight stream starts (one pass,
// two rows per wave at a time), results in the first kLnStatsBytes of LDS.
template <int NW>
__device__ __forceinline__ void i8_stats(const GemmParams& p, floatx2* stats, int wave, int lane)
{
    constexpr int U = 8;
    const int pieces = p.K / kChunkK;
    for (int r0 = wave; r0 < p.B; r0 += 2 * NW) {
        const bool two = r0 + NW < p.B;
        const _Float16* row0 = p.X + (int64_t)r0 * p.K;
        const _Float16* row1 = p.X + (int64_t)(two ? r0 + NW : r0) * p.K;
        float m0 = 0.f, m1 = 0.f;
        for (int c0 = 0; c0 < pieces; c0 += 64 * U) {
            u32x4 h0[U], h1[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = min(c0 + u * 64 + lane, pieces - 1) * kChunkK;     // a clamped piece is re-read: harmless for a maximum
                h0[u] = *reinterpret_cast<const u32x4*>(row0 + c);
                h1[u] = *reinterpret_cast<const u32x4*>(row1 + c);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const half8 a = __builtin_bit_cast(half8, h0[u]);
                const half8 b = __builtin_bit_cast(half8, h1[u]);
#pragma unroll
                for (int e = 0; e < kChunkK; ++e) {
                    m0 = fmaxf(m0, fabsf((float)a[e]));
                    m1 = fmaxf(m1, fabsf((float)b[e]));
                }
            }
        }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            m0 = fmaxf(m0, __shfl_xor(m0, m, 64));
            m1 = fmaxf(m1, __shfl_xor(m1, m, 64));
        }
        if (lane == 0) {
            stats[r0] = (m0 > 0.f) ? floatx2{127.0f / m0, m0 / 127.0f} : floatx2{0.f, 0.f};
            if (two) stats[r0 + NW] = (m1 > 0.f) ? floatx2{127.0f / m1, m1 / 127.0f} : floatx2{0.f, 0.f};
        }
    }
}

// 16 halfs (two 128-bit pieces) -> 16 int8 codes in one 128-bit piece
__device__ __forceinline__ u32x4 quantize16(u32x4 lo, u32x4 hi, float inv)
{
    const half8 a = __builtin_bit_cast(half8, lo);
    const half8 b = __builtin_bit_cast(half8, hi);
    unsigned int w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const float x = (e < 8) ? (float)a[e & 7] : (float)b[e & 7];
        float r = rintf(x * inv);
        r = fminf(fmaxf(r, -127.0f), 127.0f);
        w[e >> 2] |= ((unsigned int)(int)r & 0xffu) << (8 * (e & 3));
    }
    return u32x4{w[0], w[1], w[2], w[3]};
}

// Staging of k-steps [cb, cb+cn) (64 k each) of X as int8 codes: same LDS order as XStage
// (piece (ks, g) of row b at ((ks - cb)*4 + g)*xpitch + b, here 16 codes = k 16g..16g+15), same
// request/commit split; a piece needs two 128-bit reads of fp16.  Needs K % 16 == 0.
template <int NT, int XU>
struct XStageI8 {
    u32x4 buf[XU][2];

    __device__ __forceinline__ void request(const GemmParams& p, int cb, int cn, int tid)
    {
        const int nc = cn * 4;
        const int items = nc * p.B;
#pragma unroll
        for (int u = 0; u < XU; ++u) {
            const int idx = min(tid + u * NT, items - 1);
            const int b = idx / nc;
            const int c = idx - b * nc;
            const int k = min(cb * 64 + c * 16, p.K - 16);
            const u32x4* src = reinterpret_cast<const u32x4*>(p.X + (int64_t)b * p.K + k);
            buf[u][0] = src[0];
            buf[u][1] = src[1];
        }
    }

    __device__ __forceinline__ void commit(const GemmParams& p, u32x4* xs, int cb, int cn, int tid)
    {
        const int nc = cn * 4;
        const int items = nc * p.B;
#pragma unroll
        for (int u = 0; u < XU; ++u) {
            const int idx = tid + u * NT;
            if (idx < items) {
                const int b = idx / nc;
                const int c = idx - b * nc;
                const bool inside = cb * 64 + c * 16 < p.K;
                const u32x4 q = quantize16(buf[u][0], buf[u][1], p_stats[b][0]);
                xs[c * p.xpitch + b] = inside ? q : u32x4{0u, 0u, 0u, 0u};
            }
        }
        for (int base = NT * XU; base < items; base += NT * XU) {
            u32x4 v[XU][2];
#pragma unroll
            for (int u = 0; u < XU; ++u) {
                const int idx = min(base + tid + u * NT, items - 1);
                const int b = idx / nc;
                const int c = idx - b * nc;
                const int k = min(cb * 64 + c * 16, p.K - 16);
                const u32x4* src = reinterpret_cast<const u32x4*>(p.X + (int64_t)b * p.K + k);
                v[u][0] = src[0];
                v[u][1] = src[1];
            }
#pragma unroll
            for (int u = 0; u < XU; ++u) {
                const int idx = base + tid + u * NT;
                if (idx < items) {
                    const int b = idx / nc;
                    const int c = idx - b * nc;
                    const bool inside = cb * 64 + c * 16 < p.K;
                    const u32x4 q = quantize16(v[u][0], v[u][1], p_stats[b][0]);
                    xs[c * p.xpitch + b] = inside ? q : u32x4{0u, 0u, 0u, 0u};
                }
            }
        }
    }

    const floatx2* p_stats;     // the rows' (inv, scale), set by the kernel before the first commit
};

// A pair of partial sums travels as one 64-bit device-scope access (see finish_split_k).
__device__ __forceinline__ void store_partial(float* dst, float s0, float s1)
{
    const unsigned long long bits = ((unsigned long long)__builtin_bit_cast(unsigned int, s1) << 32) |
                                    (unsigned long long)__builtin_bit_cast(unsigned int, s0);
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(dst), bits, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void load_partial(const float* src, float& s0, float& s1)
{
    const unsigned long long bits = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(src),
                                                      __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s0 = __builtin_bit_cast(float, (unsigned int)(bits & 0xffffffffull));
    s1 = __builtin_bit_cast(float, (unsigned int)(bits >> 32));
}

// After every wave has written its 16-row x 64-column partial tile to `red`
// ([wave][16][kRedPitch] 32-bit values), sum over waves and either finish the rows (S == 1) or
// park them in the workspace for the cross-block reduction.  mb selects rows mb*16..+15.
// I8: the values are int32 sums of code products: added as integers (exactly), de-quantised
// with the row's and the column's scale right before the epilogue; `stats` holds the rows'
// (inv, scale).
__device__ __forceinline__ float dequant(const GemmParams& p, int acc, int b, int n, const floatx2* stats)
{
    return (float)acc * (stats[b][1] * p.sw[min(n, p.N - 1)]);
}

// The outputs reduce_rows will finish in this thread: 16 rows x 32 column pairs over NW*64 threads.
template <int NW>
struct RowOperands {
    static constexpr int kItems = (16 * 32 + NW * 64 - 1) / (NW * 64);
    EpiOperands e[kItems];
};

// Requests the epilogue operands of reduce_rows(…, mb, panel, …) - call it ahead of the barriers
// that reduce_rows has to wait for anyway.  The bias of a thread's column pair is the same for
// every mb of a panel: with `fresh_bias` false it is taken over from `bias_of` instead of loaded.
template <int NW>
__device__ __forceinline__ RowOperands<NW> request_row_operands(const GemmParams& p, int mb, int panel, int tid,
                                                                bool fresh_bias, const RowOperands<NW>& bias_of)
{
    constexpr int NT = NW * 64;
    RowOperands<NW> ops;
#pragma unroll
    for (int j = 0; j < RowOperands<NW>::kItems; ++j) {
        const int item = tid + j * NT;
        const int b = mb * 16 + (item >> 5);
        const int n = panel * kPanelN + (item & 31) * 2;
        EpiOperands e = {0.f, 0.f, 0.f, 0.f};
        if (p.S == 1 && item < 16 * 32) {
            if (fresh_bias) {
                load_bias_pair(p, n, e);
            } else {
                e.bias0 = bias_of.e[j].bias0;
                e.bias1 = bias_of.e[j].bias1;
            }
            load_residual_pair(p, b, n, e);
        }
        ops.e[j] = e;
    }
    return ops;
}

template <int NW, bool I8 = false>
__device__ __forceinline__ void reduce_rows(const GemmParams& p, const float* red, int mb,
                                            int panel, int split, int tid, const RowOperands<NW>& ops,
                                            const floatx2* stats = nullptr)
{
    constexpr int NT = NW * 64;
#pragma unroll
    for (int j = 0; j < RowOperands<NW>::kItems; ++j) {
        const int item = tid + j * NT;
        if (item >= 16 * 32) continue;
        const int bl = item >> 5;
        const int c2 = (item & 31) * 2;
        const int b = mb * 16 + bl;
        if (b >= p.B) continue;
        float s0 = 0.f, s1 = 0.f;
        int i0 = 0, i1 = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const floatx2 v = *reinterpret_cast<const floatx2*>(red + (w * 16 + bl) * kRedPitch + c2);
            if constexpr (I8) {
                const float f0 = v[0], f1 = v[1];        // (a bit cast straight from a vector element picks element 0)
                i0 += __builtin_bit_cast(int, f0);
                i1 += __builtin_bit_cast(int, f1);
            } else {
                s0 += v[0];
                s1 += v[1];
            }
        }
        const int n = panel * kPanelN + c2;
        if (p.S == 1) {
            float y0, y1;
            if constexpr (I8) {
                store_pair(p, b, n, dequant(p, i0, b, n, stats), dequant(p, i1, b, n + 1, stats), ops.e[j], y0, y1);
            } else {
                store_pair(p, b, n, s0, s1, ops.e[j], y0, y1);
                if (p.moments_out) emit_moments(p, b, panel, n, y0, y1, tid);      // tid & 31 == lane & 31
            }
        } else {
            float* dst = p.partials + (((int64_t)panel * p.S + split) * p.B + b) * kPanelN + c2;
            if constexpr (I8) store_partial(dst, __builtin_bit_cast(float, i0), __builtin_bit_cast(float, i1));
            else store_partial(dst, s0, s1);
        }
    }
}

// Cross-block reduction: every block of a panel has parked its partial rows; the block
// that arrives last sums the S slabs in slab order (so the result does not depend on
// which block that is), applies the epilogue and stores.  The counter is left at zero.
//
// Coherence across the chip's eight L2 caches without cache-wide flushes: partial sums are
// written and read with device-scope accesses (they go to, and come from, the memory-side
// coherence point, never a stale or dirty line of one L2).  Order: every wave waits until its own
// partial stores have been acknowledged (wait_stores_acknowledged), the block's barrier collects
// all waves, and only then one thread counts the arrival; the last block issues its loads after
// it has read the full count back (the atomic's return value decides the branch, and a barrier
// separates that branch from the loads).  A device-wide release fence per block would write back
// the whole L2 and serialise the grid (measured: about 0.1 us per block).
template <int NT, bool I8 = false>
__device__ __forceinline__ void finish_split_k(const GemmParams& p, int panel, int tid, int* s_flag,
                                               const floatx2* stats = nullptr)
{
    wait_stores_acknowledged();                               // this wave's partial sums have reached memory
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();                                          // ... and so have every other wave's of the block
    if (tid == 0) {
        const unsigned int old = __hip_atomic_fetch_add(p.counters + panel, 1u, __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT);
        *s_flag = (old == (unsigned int)(p.S - 1));
    }
    __syncthreads();
    if (!*s_flag) return;
    const float* base = p.partials + (int64_t)panel * p.S * p.B * kPanelN;
    const int items = p.B * 32;
    for (int item = tid; item < items; item += NT) {
        const int b = item >> 5;
        const int c2 = (item & 31) * 2;
        const int n = panel * kPanelN + c2;
        const EpiOperands e = load_epilogue_operands(p, b, n);
        float s0 = 0.f, s1 = 0.f;
        int i0 = 0, i1 = 0;
        // the slabs are fetched kSlabBatch at a time (independent loads, one latency per batch) and
        // added in slab order
        constexpr int kSlabBatch = 4;
        for (int sb = 0; sb < p.S; sb += kSlabBatch) {
            float v0[kSlabBatch], v1[kSlabBatch];
#pragma unroll
            for (int u = 0; u < kSlabBatch; ++u)
                load_partial(base + ((int64_t)min(sb + u, p.S - 1) * p.B + b) * kPanelN + c2, v0[u], v1[u]);
#pragma unroll
            for (int u = 0; u < kSlabBatch; ++u) {
                if (sb + u < p.S) {
                    if constexpr (I8) {
                        i0 += __builtin_bit_cast(int, v0[u]);
                        i1 += __builtin_bit_cast(int, v1[u]);
                    } else {
                        s0 += v0[u];
                        s1 += v1[u];
                    }
                }
            }
        }
        float y0, y1;
        if constexpr (I8) {
            store_pair(p, b, n, dequant(p, i0, b, n, stats), dequant(p, i1, b, n + 1, stats), e, y0, y1);
        } else {
            store_pair(p, b, n, s0, s1, e, y0, y1);
            if (p.moments_out) emit_moments(p, b, panel, n, y0, y1, tid);
        }
    }
    if (tid == 0)
        __hip_atomic_store(p.counters + panel, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace sbi
