// C-ABI entry points, host-side argument validation and the batch-size dispatcher.
// Every check here runs on the host before anything is enqueued, so the error paths can be
// exercised without a GPU.
#include "../../include/sbi_gemm.h"
#include "sbi_common.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <atomic>
#include <mutex>
#include <vector>
#if defined(SBI_TRACE) || defined(SBI_DEV)
#include <cstdio>
#include <cstdlib>
#endif

namespace {

using namespace sbi;

constexpr int64_t kMaxDim = int64_t(1) << 22;     // K, N limit: keeps tile counts and grids in 32 bits
constexpr int64_t kMaxLds = 72 * 1024;            // dynamic LDS budget per block (several blocks per CU)
constexpr int64_t kMaxLdsWide = 144 * 1024;       // two-panel blocks of large batches: one block per CU
constexpr int64_t kCounterBytes = (kMaxDim / kPanelN) * 4;   // one arrival counter per possible panel: 256 KiB
constexpr int kStreamMaxBatch = 8;                // vector-ALU kernel instantiations exist for B <= 8
constexpr int kAutoStreamBatch = 0;               // AUTO picks the vector-ALU kernel for B <= this

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

struct Plan {
    int path, nw, depth, S, ksps, kc, grid, block;
    int64_t lds, ws_bytes, counter_bytes;
    int upw, nwaves;          // STREAMK path: units per wavefront, wavefronts
    int pw;                   // MFMA path: panels per block
    bool ln;                  // MFMA path: the kernel variant that can layer-normalise X
    bool i8;                  // the INT8 kernel (64-k steps, int8 X codes in LDS)
    bool prenorm;             // layer-norm requested, batch above kLnFusedMaxBatch: a kernel of its own writes the
                              //   normalised rows to the workspace (xq_bytes) and the plain kernels run on those
    bool preq;                // INT8: activations quantised by a kernel of their own, codes in the workspace
    int64_t xq_bytes;         //   and the workspace bytes those codes and row scales take
};

constexpr int kSkDefaultWaves = 2048;             // wavefronts of a STREAMK launch: 8 per CU
constexpr int64_t kSkMaxUnits = int64_t(1) << 30; // keeps unit indices in 32 bits

// Launch shape of the work-balanced kernel for `units` 4 KiB units in total.
sbi_status plan_streamk(int64_t B, int64_t units, int64_t panels, const sbi_tuning& t, Plan& pl)
{
    if (units > kSkMaxUnits || panels > kCounterBytes / 4) return SBI_ERR_SHAPE;
    int nw = t.waves ? t.waves : 4;
    int depth = t.depth ? t.depth : 4;
    if ((nw != 4 && nw != 8) || (depth != 4 && depth != 8) || t.blocks < 0) return SBI_ERR_TUNING;
    if (nw == 8 && depth == 8 && B > 16) return SBI_ERR_TUNING;      // would not fit the register file
    const int64_t want = t.blocks ? (int64_t)t.blocks * nw : kSkDefaultWaves;
    const int64_t upw = round_up(ceil_div(units, want), kStepGroup);
    const int64_t nwaves = ceil_div(units, upw);
    pl.ln = false; pl.i8 = false; pl.preq = false; pl.prenorm = false; pl.xq_bytes = 0; pl.path = SBI_PATH_STREAMK; pl.nw = nw; pl.depth = depth; pl.S = 0;
    pl.ksps = (int)upw; pl.kc = 0; pl.pw = 1;
    pl.grid = (int)ceil_div(nwaves, nw); pl.block = nw * 64; pl.lds = 0;
    pl.upw = (int)upw; pl.nwaves = (int)nwaves;
    pl.counter_bytes = kCounterBytes;
    pl.ws_bytes = kCounterBytes + nwaves * 2 * B * kPanelN * 4;
    return SBI_OK;
}

sbi_status check_shape(int64_t K, int64_t N)
{
    if (K < 1 || N < 1 || K > kMaxDim || N > kMaxDim) return SBI_ERR_SHAPE;
    return SBI_OK;
}

// Cost, in k-steps of streaming time on the busiest CU, of splitting a panel's K range S ways.
// Measured on MI355X: one block of 8 waves per CU already saturates HBM, every further
// block costs about as much as streaming 20 k-steps (launch, X staging, reduction, arrival),
// and a grid that leaves CUs idle only hurts below about 3/4 occupancy.
double split_cost(int64_t KS, int64_t P, int64_t B, int S, int nw)
{
    const int64_t ksps = ceil_div(KS, S);
    const int64_t blocks = P * S;
    const int64_t rounds = ceil_div(blocks, kNumCU);
    const double block_overhead = 20.0;
    const double busy = (double)std::min<int64_t>(blocks, kNumCU) / kNumCU;     // fraction of CUs with work
    const double starve = busy >= 0.75 ? 1.0 : 0.75 / busy;
    double cost = (double)rounds * ((double)ksps + block_overhead) * starve;
    if (nw == 4) cost *= 1.03;
    if (S > 1) {
        // partial sums: written once and read once, 256 B per batch row per block
        const double bytes = (double)blocks * (double)B * 512.0;
        cost += bytes / kNumCU / 4096.0;
    }
    return cost;
}

sbi_status plan_group(int64_t B, const int64_t* Ks, const int64_t* Ns, int G, Plan* pls, Plan& tot, bool ln,
                      bool i8 = false);

// X staging of a block of `nw` waves that streams `ksps` k-steps, `wd` = waves*depth k-steps per
// round, with at most `cap` bytes of LDS (64 B per batch row per k-step).  One staging pass
// moves 4 pieces of 16 bytes per thread, i.e. nw * 4 KiB; every further pass costs a memory
// latency, so: one buffer if the whole range fits in one pass, else two buffers of `kc` k-steps,
// each within one pass where a round of k-steps allows it.  False if not even one round fits.
// Kernel flavours differ in what sits in LDS: the layer-norm variant keeps the row statistics in
// `front` bytes ahead of the X buffers (reused by the reduction afterwards) and adds gamma and
// beta as two more rows per buffer; the INT8 kernel keeps the rows' scales there through the
// reduction, stores int8 codes (64 k per k-step, still 64 B per row) and stages half as many
// LDS bytes per pass.
enum Flavour { kPlain = 0, kLayerNorm = 1, kInt8 = 2, kInt8Codes = 3 };

// Rows of 16-byte pieces a k-step's lane group occupies in LDS: B rounded up to an odd number, so
// that a wave staging 64 consecutive pieces of one row hits every LDS bank.
inline int64_t x_pitch(int64_t B) { return B | 1; }

// INT8: up to this batch every block quantises the activations itself; above it a kernel of its
// own does it once (measured on MI355X: fused is ahead up to B = 8, behind from B = 16 on).
constexpr int64_t kI8FusedMaxBatch = 8;
// Layer-norm: up to this batch every block normalises what it stages; above it the rows are normalised
// once by a kernel of their own and the plain kernels run on the result.  Measured, fused against
// that pass plus the plain launch: h=1024 layer B = 1 16.3 / 18.4 us; h=4096 layer B = 8 67.3 / 67.9,
// B = 16 70.3 / 69.1, B = 32 104 / 74 us; h=12288 layer (3.6 GB, where the plain launch can use one
// 8-wave block per CU) B = 4 535 / 532, B = 8 561 / 527, B = 16 600 / 534 us.
constexpr int64_t kLnFusedMaxBatch = 8;
constexpr int64_t kLnFusedMaxBatchLarge = 4;     // launches of a gigabyte and more
inline int64_t xn_bytes_of(int64_t B, int64_t K) { return round_up(B * K * 2, 256); }
inline int64_t xq_bytes_of(int64_t B, int64_t K) { return round_up(B * K, 256) + round_up(B * 8, 256); }

// k-steps a block consumes per round of its rings.  (8 waves, depth 4, two panels) is the shape whose
// waves form two groups of four, one panel each: a round is 16 k-steps there.
inline int64_t round_ksteps(int nw, int depth, int pw)
{
    return (pw == 2 && nw == 8 && depth == 4) ? 16 : (int64_t)nw * depth;
}

bool chunking(int64_t B, int64_t ksps, int64_t wd, int nw, int64_t cap, int64_t red_bytes,
              int64_t& kc, int64_t& lds, Flavour fl = kPlain)
{
    const int64_t front = (fl == kPlain) ? 0 : kLnStatsBytes;
    const int64_t rows = x_pitch(B) + (fl == kLayerNorm ? 2 : 0);
    const int64_t pass_bytes = (int64_t)nw * (fl == kInt8 ? 2048 : 4096);
    const int64_t red = (fl == kInt8 || fl == kInt8Codes) ? red_bytes : std::max<int64_t>(red_bytes - front, 0);
    cap -= front;
    const int64_t whole = round_up(ksps, wd);
    bool ok = true;
    if (whole * rows * 64 <= std::min(cap, pass_bytes)) {
        kc = whole;
        lds = std::max(kc * rows * 64, red);
    } else {
        kc = (std::min(cap / 2, pass_bytes) / (rows * 64)) / wd * wd;
        if (kc < wd) kc = (cap / 2 / (rows * 64) >= wd) ? wd : 0;    // a round needs more than one pass
        if (kc >= whole) {                                           // fits in one buffer after all
            kc = whole;
            lds = std::max(kc * rows * 64, red);
            ok = kc * rows * 64 <= cap;
        } else {
            lds = std::max(2 * kc * rows * 64, red);
            ok = kc >= wd;
        }
    }
    lds += front;
    return ok && lds <= cap + front;
}

sbi_status make_plan(int64_t B, int64_t K, int64_t N, const sbi_tuning* tune, Plan& pl)
{
    if (sbi_status s = check_shape(K, N)) return s;
    if (B < 1 || B > SBI_MAX_BATCH) return SBI_ERR_BATCH;
    const int64_t P = ceil_div(N, kPanelN);

    sbi_tuning t = {0, 0, 0, 0, 0, 0, 0, 0};
    if (tune) t = *tune;
    const bool ln = t.layernorm != 0;
    const bool i8 = t.int8 != 0;
    const int64_t KS = i8 ? ksteps_of_i8(K) : ksteps_of(K);
    // INT8 with a layer-norm in front: always from codes (the kernel that quantises the rows normalises them first)
    const bool preq = i8 && (B > kI8FusedMaxBatch || ln);
    const Flavour fl = i8 ? (preq ? kInt8Codes : kInt8) : (ln ? kLayerNorm : kPlain);

    if (t.split_k < 0 || t.blocks < 0 || t.panels < 0 || t.panels > 2) return SBI_ERR_TUNING;
    int path = t.path;
    const bool sk_ok = (K % kChunkK == 0);            // X rows readable as 128-bit pieces
    if (path == SBI_PATH_AUTO) path = (B <= kAutoStreamBatch && !ln && !i8) ? SBI_PATH_STREAM : SBI_PATH_MFMA;
    // layer-norm in front of the GeMM: matrix-core block kernel only, rows read as 128-bit pieces
    if (ln && !i8 && (path != SBI_PATH_MFMA || K % kChunkK != 0 || t.panels == 2)) return SBI_ERR_TUNING;
    // INT8: its own matrix-core kernel, rows read as 32-byte pieces
    if (i8 && (path != SBI_PATH_MFMA || K % kI8ChunkK != 0 || (t.panels == 2 && !preq))) return SBI_ERR_TUNING;
    if (path == SBI_PATH_STREAMK) {
        if (!sk_ok) return SBI_ERR_TUNING;
        return plan_streamk(B, KS * P, P, t, pl);
    }
    if (path != SBI_PATH_STREAM && path != SBI_PATH_MFMA) return SBI_ERR_TUNING;
    if (path == SBI_PATH_STREAM && B > kStreamMaxBatch) return SBI_ERR_TUNING;
    if (path == SBI_PATH_MFMA && t.split_k == 0 && t.waves == 0 && t.depth == 0 && t.panels == 0) {
        Plan one;
        if (sbi_status s = plan_group(B, &K, &N, 1, &one, pl, ln, i8)) return s;
        pl.S = one.S; pl.ksps = one.ksps; pl.kc = one.kc; pl.pw = one.pw;
        return SBI_OK;
    }

    const int pw = (t.panels == 2 && path == SBI_PATH_MFMA) ? 2 : 1;
    if (t.panels == 2 && path != SBI_PATH_MFMA) return SBI_ERR_TUNING;
    if (t.split_k < 0) return SBI_ERR_TUNING;
    // Block shape: what the caller fixed stays; what it left open takes the preferred value first
    // and, if that shape cannot stage its X chunks in LDS at this batch size, smaller ones.
    const int pref_nw = (B <= 32 && KS >= 32) ? 8 : 4;
    const int pref_depth = (B > 32 || pw == 2) ? 2 : 4;
    const int nw_try[3] = {t.waves ? t.waves : pref_nw, 4, 8};
    const int depth_try[3] = {t.depth ? t.depth : pref_depth, 2, 4};
    int nw = 0, depth = 0, S = 0;
    int64_t ksps = 0, PG = 0, kc = 0, lds = 0;
    sbi_status why = SBI_ERR_TUNING;
    bool found = false;
    for (int a = 0; a < (t.waves ? 1 : 3) && !found; ++a)
        for (int b = 0; b < (t.depth ? 1 : 3) && !found; ++b) {
            if ((a > 0 && nw_try[a] == nw_try[0]) || (b > 0 && depth_try[b] == depth_try[0])) continue;
            nw = nw_try[a]; depth = depth_try[b];
            bool depth_ok = depth == 4 || depth == 8 || (depth == 2 && path == SBI_PATH_MFMA);
            if (pw == 2) depth_ok = (nw == 4 && (depth == 2 || depth == 4)) || (nw == 8 && (depth == 2 || (depth == 4 && B > 16)));
            if ((nw != 4 && nw != 8) || !depth_ok) continue;
            if (ln && !i8 && !((nw == 4 && (depth == 2 || depth == 4)) || (nw == 8 && depth == 4))) continue;
            if (i8 && !(pw == 2 ? (nw == 8 && (depth == 2 || depth == 4)) : ((nw == 4 && (depth == 2 || depth == 4)) || (nw == 8 && depth == 4))))
                continue;
            S = t.split_k;
            if (S == 0) {
                const int64_t smax = std::max<int64_t>(1, std::min<int64_t>(KS / nw, 64));
                double best = 0.0;
                for (int s = 1; s <= smax; ++s) {
                    const int64_t k = ceil_div(KS, s);
                    if (ceil_div(KS, k) != s) continue;          // same launch as a smaller s
                    const double c = split_cost(KS, P, B, s, nw);
                    if (S == 0 || c < best) { best = c; S = s; }
                }
            }
            if (S > KS) S = (int)KS;
            ksps = ceil_div(KS, S);
            S = (int)ceil_div(KS, ksps);                             // no empty blocks
            PG = ceil_div(P, pw);                                    // panel groups = blocks per split
            if (PG * S > (int64_t)0x7fffffff) { why = SBI_ERR_SHAPE; continue; }
            found = chunking(B, ksps, round_ksteps(nw, depth, pw), nw, (pw == 2 || ln || i8) ? kMaxLdsWide : kMaxLds,
                             (int64_t)nw * 16 * kRedPitch * 4, kc, lds, fl);
        }
    if (!found) return why;

    pl.ln = ln && !i8; pl.i8 = i8; pl.preq = preq; pl.prenorm = false; pl.xq_bytes = preq ? xq_bytes_of(B, K) : 0;
    pl.path = path; pl.nw = nw; pl.depth = depth; pl.S = S; pl.pw = pw;
    pl.ksps = (int)ksps; pl.kc = (int)kc;
    pl.grid = (int)(PG * S); pl.block = nw * 64;
    pl.lds = lds;
    pl.counter_bytes = (S > 1 || preq) ? kCounterBytes : 0;
    pl.ws_bytes = (S > 1 || preq) ? pl.counter_bytes + (S > 1 ? P * S * B * kPanelN * 4 : 0) + pl.xq_bytes : 0;
    pl.upw = 0; pl.nwaves = 0;
    return SBI_OK;
}

int epilogue_flags(int epi)
{
    switch (epi) {
        case SBI_EPI_NONE: return 0;
        case SBI_EPI_BIAS: return kEpiBias;
        case SBI_EPI_BIAS_GELU: return kEpiBias | kEpiGelu;
        case SBI_EPI_BIAS_RESIDUAL: return kEpiBias | kEpiRes;
        case SBI_EPI_GELU: return kEpiGelu;
        case SBI_EPI_RESIDUAL: return kEpiRes;
    }
    return -1;
}

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// One GeMM of a launch, already validated.
struct GemmArgs {
    const void* Wl; int64_t K, N; const void* X; const void* bias; const void* R; int flags; void* Y;
    const void* gamma; const void* beta; float eps;     // layer-norm of X's rows when gamma != null
    const void* sw;                                     // INT8: per-column weight scales (binary32 [N])
    void* moments_out;                                  // per-panel row moments of Y for a following layer-norm
    const void* ln_moments;                             // such moments of X, for this call's layer-norm
};

// Validation of a layer-norm request in front of a GeMM with K input features.
sbi_status check_layernorm(const void* gamma, const void* beta, float eps, int64_t K)
{
    if (!gamma || !beta) return SBI_ERR_NULL;
    if (K % kChunkK != 0) return SBI_ERR_SHAPE;
    if (!aligned(gamma, 16) || !aligned(beta, 16)) return SBI_ERR_ALIGN;
    if (!(eps >= 0.0f) || !std::isfinite(eps)) return SBI_ERR_EPILOGUE;
    return SBI_OK;
}

// Validation shared by sbi_gemm_ex and sbi_layer_gemms (everything except the workspace).
sbi_status check_gemm_args(const void* W_laid_out, int64_t K, int64_t N, const void* X, int64_t B,
                           const void* bias, const void* residual, int epi, const void* Y, int& flags)
{
    if (!W_laid_out || !X || !Y) return SBI_ERR_NULL;
    if (sbi_status s = check_shape(K, N)) return s;
    if (B < 1 || B > SBI_MAX_BATCH) return SBI_ERR_BATCH;
    flags = epilogue_flags(epi);
    if (flags < 0) return SBI_ERR_EPILOGUE;
    if ((flags & kEpiBias) && !bias) return SBI_ERR_EPILOGUE;
    if ((flags & kEpiRes) && !residual) return SBI_ERR_EPILOGUE;
    const bool x_vec = (K % 8 == 0);
    if (!aligned(W_laid_out, 256) || !aligned(X, x_vec ? 16 : 2) || !aligned(Y, 4)) return SBI_ERR_ALIGN;
    if ((flags & kEpiBias) && !aligned(bias, 2)) return SBI_ERR_ALIGN;
    if ((flags & kEpiRes) && !aligned(residual, 2)) return SBI_ERR_ALIGN;
    const uintptr_t x0 = reinterpret_cast<uintptr_t>(X), x1 = x0 + (uintptr_t)(B * K * 2);
    const uintptr_t y0 = reinterpret_cast<uintptr_t>(Y), y1 = y0 + (uintptr_t)(B * N * 2);
    if (x0 < y1 && y0 < x1) return SBI_ERR_OVERLAP;
    return SBI_OK;
}

// Launch `G` independent GeMMs of batch B as one work-balanced kernel.
sbi_status launch_group(const GemmArgs* a, int G, int64_t B, const Plan& pl, void* workspace, hipStream_t st)
{
    SkParams p;
    std::memset(&p, 0, sizeof p);
    int64_t units = 0, panels = 0;
    for (int g = 0; g < G; ++g) {
        SkProblem& q = p.prob[g];
        q.Wl = reinterpret_cast<const u32x4*>(reinterpret_cast<const unsigned char*>(a[g].Wl) + kHeaderBytes);
        q.X = reinterpret_cast<const _Float16*>(a[g].X);
        q.bias = (a[g].flags & kEpiBias) ? reinterpret_cast<const _Float16*>(a[g].bias) : nullptr;
        q.R = (a[g].flags & kEpiRes) ? reinterpret_cast<const _Float16*>(a[g].R) : nullptr;
        q.Y = reinterpret_cast<_Float16*>(a[g].Y);
        q.K = (int)a[g].K; q.N = (int)a[g].N;
        q.KS = (int)ksteps_of(a[g].K); q.P = (int)ceil_div(a[g].N, kPanelN);
        q.flags = a[g].flags;
        q.unit_base = (int)units; q.panel_base = (int)panels;
        q.fast = (a[g].N % 4 == 0) && aligned(a[g].Y, 8) && (!q.bias || aligned(q.bias, 8)) &&
                 (!q.R || aligned(q.R, 8));
        units += (int64_t)q.KS * q.P;
        panels += q.P;
    }
    p.G = G; p.B = (int)B; p.U = (int)units; p.upw = pl.upw;
    p.counters = reinterpret_cast<unsigned int*>(workspace);
    p.partials = reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(workspace) + pl.counter_bytes);
    return launch_streamk(p, pl.nw, pl.depth, pl.grid, st) == 0 ? SBI_OK : SBI_ERR_HIP;
}

// Block-kernel parameters of one validated GeMM under plan `pl`; its arrival counters start at
// counter index `panel_base` and its partial sums at byte offset `partial_off` of the workspace.
GemmParams fill_params(const GemmArgs& a, int64_t B, const Plan& pl, void* workspace,
                       int64_t panel_base, int64_t partial_off, int64_t xq_off = 0)
{
    GemmParams p;
    p.Wl = reinterpret_cast<const u32x4*>(reinterpret_cast<const unsigned char*>(a.Wl) + kHeaderBytes);
    p.X = reinterpret_cast<const _Float16*>(a.X);
    p.bias = (a.flags & kEpiBias) ? reinterpret_cast<const _Float16*>(a.bias) : nullptr;
    p.R = (a.flags & kEpiRes) ? reinterpret_cast<const _Float16*>(a.R) : nullptr;
    p.Y = reinterpret_cast<_Float16*>(a.Y);
    unsigned char* ws = reinterpret_cast<unsigned char*>(workspace);
    p.counters = (pl.S > 1) ? reinterpret_cast<unsigned int*>(ws) + panel_base : nullptr;
    p.partials = (pl.S > 1) ? reinterpret_cast<float*>(ws + kCounterBytes + partial_off) : nullptr;
    p.B = (int)B; p.K = (int)a.K; p.N = (int)a.N;
    p.KS = (int)(pl.i8 ? ksteps_of_i8(a.K) : ksteps_of(a.K)); p.P = (int)ceil_div(a.N, kPanelN);
    p.S = pl.S; p.ksps = pl.ksps; p.kc = pl.kc; p.xpitch = (int)x_pitch(B);
    p.sw = reinterpret_cast<const float*>(a.sw);
    p.moments_out = reinterpret_cast<floatx2*>(a.moments_out);
    p.ln_moments = reinterpret_cast<const floatx2*>(a.gamma ? a.ln_moments : nullptr);
    p.X16 = p.X;
    p.xstats = nullptr;
    if (pl.preq) {                      // codes and row scales live at byte offset xq_off of the workspace
        p.X = reinterpret_cast<const _Float16*>(ws + xq_off);
        p.xstats = reinterpret_cast<const floatx2*>(ws + xq_off + round_up(B * a.K, 256));
    }
    p.flags = a.flags; p.x_vec = (a.K % 8 == 0) ? 1 : 0;
    // the layer-norm kernel variant reads gamma and beta pieces unconditionally: a problem
    // without layer-norm points them at its X (K readable halfs) and ignores the values
    p.ln = a.gamma ? 1 : 0;
    p.ln_gamma = reinterpret_cast<const _Float16*>(a.gamma ? a.gamma : a.X);
    p.ln_beta = reinterpret_cast<const _Float16*>(a.gamma ? a.beta : a.X);
    p.ln_eps = a.eps;
    if (pl.prenorm && a.gamma) {        // sbi_layernorm_rows_kernel leaves the normalised rows at xq_off of the workspace:
        p.X = reinterpret_cast<const _Float16*>(ws + xq_off);     // the GeMM kernel reads those (X16 keeps the raw rows)
        p.ln = 0;
    }
#ifdef SBI_DEV
    if (const char* e = getenv("SBI_ABLATE")) p.flags |= (int)strtol(e, nullptr, 0) << 8;      // development: switch parts of the kernel off
#endif
#ifdef SBI_TRACE
    p.trace = getenv("SBI_TRACE_PTR") ? reinterpret_cast<unsigned long long*>(strtoull(getenv("SBI_TRACE_PTR"), nullptr, 16)) : nullptr;
#endif
    return p;
}

// Wavefronts per CU that the register file lets the MFMA block kernel keep resident: the vector
// registers the compiled kernel variants allocate (row blocks MB = ceil(B/16), waves, depth; plain
// and layer-norm), in granules of 8, against 512 registers per SIMD lane and 4 SIMDs per CU.
int assumed_vgprs(int mb, int nw, int depth, int pw, bool ln, bool i8, bool preq = false)
{
    // (a 4-wave kernel's figure is its vector registers rounded up to 4 plus its accumulation registers)
    static const int vgpr_i8_w4d2[4] = {108, 180, 200, 220};
    static const int vgpr_i8_w4d4[4] = {168, 188, 222, 232};
    static const int vgpr_i8_w8d4[4] = {138, 154, 164, 190};
    static const int vgpr_i8q_w4d2[4] = {108, 128, 152, 176};   // INT8 from pre-quantised codes
    static const int vgpr_i8q_w4d4[4] = {148, 180, 208, 232};
    static const int vgpr_i8q_w8d4[4] = {133, 156, 198, 226};
    static const int vgpr_i8q_w8d2p2[4] = {149, 183, 219, 252};
    static const int vgpr_i8q_w8d4p2[4] = {151, 151, 180, 212};
    static const int vgpr_w4d2[4] = {108, 128, 152, 176};
    static const int vgpr_w4d4[4] = {148, 176, 216, 248};
    static const int vgpr_w8d4[4] = {134, 158, 201, 225};
    static const int vgpr_w8d2p2[4] = {150, 184, 210, 244};
    static const int vgpr_w8d2[4] = {102, 120, 130, 146};
    static const int vgpr_w8d4p2[4] = {152, 152, 180, 212};     // two wave groups, one panel each (batches above 16)
    static const int vgpr_ln_w4d2[4] = {124, 136, 160, 188};
    static const int vgpr_ln_w4d4[4] = {156, 188, 216, 244};
    static const int vgpr_ln_w8d4[4] = {150, 168, 192, 208};
    const int* tab = (pw == 2) ? (depth == 4 && nw == 8 ? vgpr_w8d4p2 : vgpr_w8d2p2) : (nw == 8) ? (depth == 2 ? vgpr_w8d2 : vgpr_w8d4) : (depth == 2 ? vgpr_w4d2 : vgpr_w4d4);
    if (ln) tab = (nw == 8) ? vgpr_ln_w8d4 : (depth == 2 ? vgpr_ln_w4d2 : vgpr_ln_w4d4);
    if (i8 && preq) tab = (pw == 2) ? (depth == 4 ? vgpr_i8q_w8d4p2 : vgpr_i8q_w8d2p2) : (nw == 8) ? vgpr_i8q_w8d4 : (depth == 2 ? vgpr_i8q_w4d2 : vgpr_i8q_w4d4);
    else if (i8) tab = (nw == 8) ? vgpr_i8_w8d4 : (depth == 2 ? vgpr_i8_w4d2 : vgpr_i8_w4d4);
    return tab[std::min(std::max(mb, 1), 4) - 1];
}

// wavefronts per CU for a kernel of `vgprs` vector registers per lane
int waves_per_cu(int vgprs) { return 4 * std::min(8, 512 / ((vgprs + 7) / 8 * 8)); }

int resident_waves(int mb, int nw, int depth, int pw, bool ln, bool i8, bool preq = false)
{
    return waves_per_cu(assumed_vgprs(mb, nw, depth, pw, ln, i8, preq));
}

// One point of the dispatcher's search space: block shape (waves, depth, panels per block), the
// common block size T in k-steps and the LDS budget the X chunks are cut for.
struct Candidate {
    int nw, depth, pw;
    int64_t T, cap;
    double cost;               // the model's estimate (k-steps of streaming time on the busiest CU)
};

// Launches measured by sbi_layer_tune / sbi_gemm_tune: (batch, shapes, flavour) -> the candidate that
// ran fastest on this machine.  plan_group consults it before the model.  Process-wide, guarded
// by a mutex; g_tuned_version lets the per-thread plan memos notice a new entry.
struct TunedEntry {
    int64_t B, Ks[kMaxGroup], Ns[kMaxGroup];
    int G, flags;
    Candidate c;
};
std::vector<TunedEntry> g_tuned;
std::mutex g_tuned_mutex;
std::atomic<int> g_tuned_version{0};
thread_local const TunedEntry* t_trial = nullptr;     // set by the tuner around its trial launches: this thread's
                                                      //   plans for exactly that problem use the trial's candidate

bool same_problem(const TunedEntry& e, int64_t B, const int64_t* Ks, const int64_t* Ns, int G, int flags)
{
    if (e.B != B || e.G != G || e.flags != flags) return false;
    for (int g = 0; g < G; ++g)
        if (e.Ks[g] != Ks[g] || e.Ns[g] != Ns[g]) return false;
    return true;
}

// Plans for `G` GeMMs that go out as one launch of the block kernel.  A common block size T
// (k-steps) gives all blocks of the launch about the same work; problem g is split
// S_g = ceil(KS_g / T) ways.  Candidates (block shape, LDS budget, T) are ranked by a model of
// the busiest CU: blocks it works through x (stream + per-block overhead), where the blocks a
// CU can hold at once follow from the LDS each block needs for its X chunks and from the
// register file.  Returns per-problem plans plus the launch totals in `tot` (nw, depth, lds,
// grid, ws_bytes).
sbi_status plan_group_search(int64_t B, const int64_t* Ks, const int64_t* Ns, int G, Plan* pls, Plan& tot, bool ln,
                             bool i8, const Candidate* forced = nullptr, std::vector<Candidate>* all = nullptr,
                             Candidate* picked = nullptr);

// The search below is a pure function of its arguments and costs 10-25 us; a serving loop asks
// for the same few launches over and over, so each thread remembers its last results.
sbi_status plan_group(int64_t B, const int64_t* Ks, const int64_t* Ns, int G, Plan* pls, Plan& tot, bool ln, bool i8)
{
    struct Entry {
        int64_t B, Ks[kMaxGroup], Ns[kMaxGroup];
        int G, flags, version;
        Plan pls[kMaxGroup], tot;
        sbi_status status;
        bool used;
    };
    constexpr int kEntries = 16;
    static thread_local Entry memo[kEntries];
    static thread_local int next = 0;
    if (G < 1 || G > kMaxGroup) return SBI_ERR_SHAPE;
#ifdef SBI_DEV
    if (getenv("SBI_PLAN_FORCE")) return plan_group_search(B, Ks, Ns, G, pls, tot, ln, i8);
#endif
    const int flags = (ln ? 1 : 0) | (i8 ? 2 : 0);
    if (t_trial && same_problem(*t_trial, B, Ks, Ns, G, flags))
        return plan_group_search(B, Ks, Ns, G, pls, tot, ln, i8, &t_trial->c);
    const int version = g_tuned_version.load(std::memory_order_acquire);
    for (int e = 0; e < kEntries; ++e) {
        const Entry& m = memo[e];
        if (!m.used || m.B != B || m.G != G || m.flags != flags || m.version != version) continue;
        bool same = true;
        for (int g = 0; g < G; ++g) same = same && m.Ks[g] == Ks[g] && m.Ns[g] == Ns[g];
        if (!same) continue;
        for (int g = 0; g < G; ++g) pls[g] = m.pls[g];
        tot = m.tot;
        return m.status;
    }
    Entry& m = memo[next];
    next = (next + 1) % kEntries;
    m.used = false;
    Candidate tuned;
    bool have_tuned = false;
    if (version > 0) {
        std::lock_guard<std::mutex> lock(g_tuned_mutex);
        for (const TunedEntry& t : g_tuned)
            if (same_problem(t, B, Ks, Ns, G, flags)) { tuned = t.c; have_tuned = true; }
    }
    m.status = plan_group_search(B, Ks, Ns, G, m.pls, m.tot, ln, i8, have_tuned ? &tuned : nullptr);
    m.B = B; m.G = G; m.flags = flags; m.version = version;
    for (int g = 0; g < G; ++g) { m.Ks[g] = Ks[g]; m.Ns[g] = Ns[g]; }
    m.used = true;
    for (int g = 0; g < G; ++g) pls[g] = m.pls[g];
    tot = m.tot;
    return m.status;
}

sbi_status plan_group_search(int64_t B, const int64_t* Ks, const int64_t* Ns, int G, Plan* pls, Plan& tot, bool ln_wanted,
                             bool i8, const Candidate* forced, std::vector<Candidate>* all, Candidate* picked)
{
    if (B < 1 || B > SBI_MAX_BATCH) return SBI_ERR_BATCH;
    for (int g = 0; g < G; ++g)
        if (sbi_status s = check_shape(Ks[g], Ns[g])) return s;
    // layer-norm: inside the GeMM blocks for the smallest batches, as a pass of its own otherwise
    double launch_bytes = 0.0;
    for (int g = 0; g < G; ++g) launch_bytes += 2.0 * (double)Ks[g] * (double)Ns[g];
    const int64_t fused_max = launch_bytes >= 1e9 ? kLnFusedMaxBatchLarge : kLnFusedMaxBatch;
    const bool prenorm = ln_wanted && !i8 && B > fused_max;   // normalise once, then the plain kernels
    const bool ln = ln_wanted && !i8 && !prenorm;              // (INT8: the kernel that quantises the rows normalises them)
    const int mb = (int)ceil_div(B, 16);
    int64_t KS[kMaxGroup], P[kMaxGroup], maxKS = 0, panels = 0;
    for (int g = 0; g < G; ++g) {
        if (sbi_status s = check_shape(Ks[g], Ns[g])) return s;
        KS[g] = i8 ? ksteps_of_i8(Ks[g]) : ksteps_of(Ks[g]); P[g] = ceil_div(Ns[g], kPanelN);
        maxKS = std::max(maxKS, KS[g]); panels += P[g];
    }
    if (panels > kCounterBytes / 4) return SBI_ERR_SHAPE;
    constexpr int64_t kLdsPerCU = 160 * 1024;
    const int64_t lds_caps[4] = {18 * 1024, 36 * 1024, kMaxLds, kMaxLdsWide};   // 9/8 of a power of two: room for the odd pitch
    const bool preq = i8 && (B > kI8FusedMaxBatch || ln_wanted);
    const Flavour fl = i8 ? (preq ? kInt8Codes : kInt8) : (ln ? kLayerNorm : kPlain);
    // (waves, depth, panels per block) candidates; two-panel blocks only pay off for B > 16
    // (ties go to the earlier shape: the measured order at equal modelled cost - the fp16 kernels do
    // best with the shallow ring, the INT8 kernel with the deep one)
    const int shapes_f16[6][3] = {{4, 2, 1}, {8, 4, 1}, {4, 4, 1}, {8, 4, 2}, {8, 2, 2}, {8, 2, 1}};   // (8, 4, 2): two wave groups
    const int shapes_i8[6][3] = {{4, 4, 1}, {8, 4, 1}, {4, 2, 1}, {8, 4, 2}, {8, 2, 2}, {0, 0, 0}};
    const auto& shapes = i8 ? shapes_i8 : shapes_f16;

    int best_nw = 0, best_depth = 0, best_pw = 1;
    int64_t bestT = 0, best_cap = 0;
    double best = 0.0;
    for (const auto& shp : shapes) {
        if (forced && !all) break;                             // nothing to search
        const int nw = shp[0], depth = shp[1], pw = shp[2];
        // 8 waves with the shallow ring, one panel: measured ahead only for grouped launches of up to 16
        // rows (below); no layer-norm variant of it exists
        if (nw == 0 || ((ln || ((mb > 1 || G == 1) && !all)) && nw == 8 && depth == 2 && pw == 1)) continue;
        // INT8 (from pre-quantised codes at these batch sizes): measured ahead only above 32 rows
        if (pw == 2 && (mb < 2 || ln || (i8 && mb < 3))) continue;
        const int64_t wd = round_ksteps(nw, depth, pw);
        const int64_t red_bytes = (int64_t)nw * 16 * kRedPitch * 4;
        for (int64_t cap : lds_caps) {
            // the wide budget belongs to two-panel blocks, and to layer-norm blocks (their statistics
            // take the room that a batch of 64 needs for two X buffers within 64 KiB)
            if ((cap > kMaxLds) != (pw == 2) && !((ln || i8) && cap > kMaxLds)) continue;
            // block sizes worth a look: the ones at which the split of the longest problem changes
            int64_t lastT = 0;
            for (int64_t smax = std::min<int64_t>(ceil_div(maxKS, wd), 64); smax >= 1; --smax) {
                const int64_t T = round_up(ceil_div(maxKS, smax), wd);
                if (T == lastT) continue;
                lastT = T;
                int64_t blocks = 0, work = 0, lds = red_bytes, chunks = 1, longest = 0, nsplit = 0;
                double partial = 0.0;
                bool ok = true, slow_stage = false;   // slow: a chunk needs a second staging pass
                for (int g = 0; g < G && ok; ++g) {
                    const int64_t S = ceil_div(KS[g], T);
                    const int64_t ksps = ceil_div(KS[g], S);
                    int64_t kc = 0, l = 0;
                    ok = chunking(B, ksps, wd, nw, cap, red_bytes, kc, l, fl);
                    if (!ok) break;
                    blocks += ceil_div(P[g], pw) * S;
                    work += ceil_div(P[g], pw) * S * ksps * pw;
                    longest = std::max(longest, ksps * pw);
                    lds = std::max(lds, l);
                    chunks = std::max(chunks, ceil_div(ksps, kc));
                    if (ceil_div(ksps, kc) > 1 && kc * (B + (ln ? 2 : 0)) * 64 > (int64_t)nw * ((i8 && !preq) ? 2048 : 4096)) slow_stage = true;
                    if (S > 1) partial += (double)(P[g] * S) * (double)B * 512.0;
                    if (S > 1) ++nsplit;
                }
                if (!ok) continue;
                const int64_t fit = std::max<int64_t>(1, std::min<int64_t>(kLdsPerCU / lds,
                                                                           resident_waves(mb, nw, depth, pw, ln, i8, preq) / nw));
                // A CU time-slices its share of HBM bandwidth over the blocks it holds, so what counts is
                // how many blocks the busiest CU works through (quantised), each costing its stream plus
                // a start/finish overhead; measured on MI355X (h=4096 layer, 512 MiB single GeMMs):
                //   overhead about 9 k-steps of streaming time per block, 4.5 more when a block has the
                //   CU to itself (nothing hides its ramp-up and epilogue), next to nothing per further
                //   X chunk, about 2 per pass of the layer-norm statistics plus 4 per launch (10 when a
                //   block has its CU to itself);
                //   X staged per block rivals the weight stream once B/(64 pw) exceeds about 0.2, and steeply
                //   so beyond 0.75;
                //   fewer than 24 k-steps in flight per CU no longer cover the memory latency.
                const int64_t per_cu_blocks = ceil_div(blocks, kNumCU);
                const int64_t conc = std::min<int64_t>(fit, per_cu_blocks);              // concurrent blocks on a CU
                const double busy = (double)std::min<int64_t>(blocks, kNumCU) / kNumCU;
                const double x_ratio = (double)B / (64.0 * pw);
                const double stream = (double)work / (double)blocks *
                                      (1.0 + 0.6 * std::max(0.0, x_ratio - 0.2) + 1.4 * std::max(0.0, x_ratio - 0.75));
                double overhead = 9.0 + 0.15 * (double)(chunks - 1) + (conc == 1 ? 4.5 : 0.0);
                // a block of more than 16 rows that has its CU to itself: two staging passes before its first
                // k-step and a reduction of mb (x pw) passes after its last, none of it hidden
                // (h=4096 layer, 64 k-steps x 2 panels per block: 67 / 83 / 96 k-steps at B = 32 / 48 / 64)
                if (conc == 1 && mb >= 2) overhead = 30.0 + 16.0 * mb + 0.15 * (double)(chunks - 1);
                // layer-norm statistics: what a block spends on them is absorbed by the other CUs' streams
                // except at the start of the launch, where every block computes them at once
                const double ln_passes = ln ? (double)(ceil_div(B, 2 * nw) * ceil_div(maxKS, 128)) : 0.0;
                overhead += 2.0 * ln_passes;
                if (i8 && !preq) overhead += (conc == 1 ? 8.0 : 2.0) * (double)(ceil_div(B, 2 * nw) * ceil_div(maxKS, 64));
                // Long single-resident blocks of large batches (384 blocks on 256 CUs): the CUs that hold
                // fewer blocks than the busiest one leave it more of the bandwidth - halfway between the
                // busiest CU's count and the average (h=4096 layer at B = 64: 384 blocks 90 us, 768 blocks 107 us)
                // When a launch holds more blocks than the chip has room for, several to a CU, blocks start as
                // others end and every CU stays busy to the end: what counts then is the average number of
                // blocks per CU, not the busiest CU's (h=4096 layer, B = 1..16: 640 blocks of 8 waves, two
                // resident per CU, 61.4-62.0 us; 768 blocks of 4 waves, all resident, 62.3-64.1 us).
                // (measured for the plain fp16 kernel's 8-wave, depth-2 blocks only; the other shapes keep the
                // busiest CU's count)
                // and for launches in which at most one problem is split: with the h=12288 tensor-parallel slice,
                // whose QKV and FFN1 are both split, the same shape is behind by up to 5 %)
                const bool rolling = !ln && !i8 && nw == 8 && depth == 2 && pw == 1 && nsplit <= 1 && fit >= 2 && blocks > fit * kNumCU;
                if (nw == 8 && depth == 2 && pw == 1 && !rolling && !all) continue;   // this shape was only measured ahead when rolling
                const double eff_blocks = (conc == 1 && mb >= 2)
                    ? 0.5 * ((double)per_cu_blocks + std::max(1.0, (double)blocks / kNumCU))
                    : rolling ? (double)blocks / kNumCU : (double)per_cu_blocks;
                double cost = eff_blocks * (stream + overhead) * (busy >= 0.75 ? 1.0 : 0.75 / busy) +
                              partial / kNumCU / 4096.0 + (conc == 1 ? 10.0 : 4.0) * ln_passes;
                // no launch ends before its longest block, which streams at about a CU's full share when it
                // was dispatched early (same layer: FFN2 in 64 blocks of 512 k-steps next to 128-k-step
                // blocks, 78.9 us)
                if (rolling)
                    cost = std::max(cost, (double)longest * (double)std::max<int64_t>(1, std::min<int64_t>(conc, 2)) * 0.5 *
                                          (busy >= 0.75 ? 1.0 : 0.75 / busy) + overhead + (double)longest * 0.5);
                // several blocks per CU are several weight streams per CU: on launches of gigabytes that
                // costs (h=12288 layer, 3.6 GB: one 8-wave block per CU 523 us, two 540 us, three 4-wave
                // blocks 543 us), on a few hundred megabytes it does not
                const double gbytes = (double)work * 4096.0 / 1e9;
                cost *= 1.0 + 0.045 * std::min((double)(conc - 1), 1.2) * std::min(1.0, std::max(0.0, (gbytes - 0.5) / 2.0));
                // (k-steps in flight on an average CU: a launch of 2.8 blocks per CU leaves some with two)
                // a launch with split panels ends in a chain the stream cannot hide: partial sums out,
                // arrival count, the last block's loads of the slabs, its epilogue (h=4096 QKV, 192
                // panels: unsplit on 192 CUs 18.5 us, split four ways on all of them 19.8 us)
                if (partial > 0.0) cost += 20.0;
                const double inflight = std::min((double)fit, (double)blocks / kNumCU) * nw * depth;
                if (inflight < 24.0) cost *= 1.0 + 0.3 * (24.0 - inflight) / 24.0;
                if (slow_stage) cost *= 1.1;
#ifdef SBI_DEV
                if (getenv("SBI_PLAN_DEBUG"))
                    fprintf(stderr, "plan B=%lld nw=%d depth=%d pw=%d cap=%lld T=%lld blocks=%lld fit=%lld conc=%lld cost=%.1f\n", (long long)B, nw,
                            depth, pw, (long long)cap, (long long)T, (long long)blocks, (long long)fit, (long long)conc, cost);
#endif
                if (all) all->push_back(Candidate{nw, depth, pw, T, cap, cost});
                if (best_nw == 0 || cost < best) {
                    best = cost; best_nw = nw; best_depth = depth; best_pw = pw; bestT = T; best_cap = cap;
                }
            }
        }
    }
#ifdef SBI_DEV
    // development builds: SBI_PLAN_FORCE="waves,depth,panels,T,lds_cap" replaces the search
    if (const char* f = getenv("SBI_PLAN_FORCE")) {
        int a = 0, b = 0, c = 0;
        long long t = 0, cap = 0;
        if (sscanf(f, "%d,%d,%d,%lld,%lld", &a, &b, &c, &t, &cap) == 5) {
            best_nw = a; best_depth = b; best_pw = c; bestT = t; best_cap = cap;
            for (int g = 0; g < G; ++g) {
                const int64_t S = ceil_div(KS[g], bestT), ksps = ceil_div(KS[g], S);
                int64_t kc = 0, l = 0;
                if (!chunking(B, ksps, round_ksteps(a, b, c), a, cap, (int64_t)a * 16 * kRedPitch * 4, kc, l, fl)) return SBI_ERR_TUNING;
            }
        }
    }
#endif
    if (forced) {                       // a measured (or trial) candidate replaces the model's pick
        best_nw = forced->nw; best_depth = forced->depth; best_pw = forced->pw; bestT = forced->T; best_cap = forced->cap;
        for (int g = 0; g < G; ++g) {
            const int64_t S = ceil_div(KS[g], bestT), ksps = ceil_div(KS[g], S);
            int64_t kc = 0, l = 0;
            if (!chunking(B, ksps, round_ksteps(best_nw, best_depth, best_pw), best_nw, best_cap,
                          (int64_t)best_nw * 16 * kRedPitch * 4, kc, l, fl))
                return SBI_ERR_TUNING;
        }
    }
    if (best_nw == 0) return SBI_ERR_SHAPE;
    if (picked) *picked = Candidate{best_nw, best_depth, best_pw, bestT, best_cap, best};
    const int nw = best_nw, depth = best_depth, pw = best_pw;
    const int64_t wd = round_ksteps(nw, depth, pw);
    int64_t grid = 0, partial_bytes = 0, lds = 0;
    bool any_split = false;
    for (int g = 0; g < G; ++g) {
        Plan& pl = pls[g];
        const int64_t S = ceil_div(KS[g], bestT);
        const int64_t ksps = ceil_div(KS[g], S);
        int64_t kc = 0, l = 0;
        chunking(B, ksps, wd, nw, best_cap, (int64_t)nw * 16 * kRedPitch * 4, kc, l, fl);
        pl.path = SBI_PATH_MFMA; pl.nw = nw; pl.depth = depth; pl.pw = pw; pl.ln = ln; pl.i8 = i8; pl.preq = preq; pl.prenorm = prenorm;
        pl.xq_bytes = preq ? xq_bytes_of(B, Ks[g]) : (prenorm ? xn_bytes_of(B, Ks[g]) : 0);
        pl.S = (int)ceil_div(KS[g], ksps); pl.ksps = (int)ksps; pl.kc = (int)kc;
        pl.grid = (int)(ceil_div(P[g], pw) * pl.S); pl.block = nw * 64;
        pl.lds = l;
        pl.counter_bytes = kCounterBytes;
        pl.ws_bytes = (pl.S > 1) ? P[g] * pl.S * B * kPanelN * 4 : 0;     // partial sums only
        pl.upw = 0; pl.nwaves = 0;
        grid += pl.grid; partial_bytes += pl.ws_bytes + pl.xq_bytes; lds = std::max(lds, pl.lds);
        any_split = any_split || pl.S > 1;
    }
    if (grid > (int64_t)0x7fffffff) return SBI_ERR_SHAPE;
    tot = pls[0];
    tot.grid = (int)grid; tot.lds = lds;
    tot.ws_bytes = (any_split || preq || prenorm) ? kCounterBytes + partial_bytes : 0;
    return SBI_OK;
}

// Launch G validated GeMMs as one grouped block-kernel launch (split problems first: their
// cross-block tails then overlap with the streaming of the blocks that start later).
sbi_status launch_block_group(const GemmArgs* a, const Plan* pls, const Plan& tot, int G, int64_t B,
                              void* workspace, hipStream_t st)
{
    int order[kMaxGroup];
    for (int g = 0; g < G; ++g) order[g] = g;
    std::stable_sort(order, order + G, [&](int x, int y) { return pls[x].S > pls[y].S; });
    GroupParams gp;
    std::memset(&gp, 0, sizeof gp);
    gp.G = G;
    int64_t panel_base = 0, partial_off = 0;
    int64_t xq_off = kCounterBytes;                      // codes follow the partial sums of all problems
    for (int g = 0; g < G; ++g) xq_off += pls[g].ws_bytes;
    int first = 0;
    for (int k = 0; k < G; ++k) {
        const int g = order[k];
        gp.g[k] = fill_params(a[g], B, pls[g], workspace, panel_base, partial_off, xq_off);
        xq_off += pls[g].xq_bytes;
        gp.first_block[k] = first;
        first += pls[g].grid;
        panel_base += gp.g[k].P;
        partial_off += pls[g].ws_bytes;
    }
    gp.first_block[G] = first;
    if (tot.ln)                       // statistics, then per X buffer B rows plus gamma and beta
        for (int g = 0; g < G; ++g) {
            const int64_t buffers = pls[g].kc >= pls[g].ksps ? 1 : 2;
            if (tot.lds < kLnStatsBytes + buffers * pls[g].kc * (x_pitch(B) + 2) * 64) return SBI_ERR_TUNING;
        }
    if (tot.i8) {                     // scales through the reduction, then X buffers or the reduction tile
        for (int g = 0; g < G; ++g) {
            const int64_t buffers = pls[g].kc >= pls[g].ksps ? 1 : 2;
            if (tot.lds < kLnStatsBytes + std::max<int64_t>(buffers * pls[g].kc * x_pitch(B) * 64, (int64_t)tot.nw * 16 * kRedPitch * 4))
                return SBI_ERR_TUNING;
        }
        return launch_i8(gp, tot.nw, tot.depth, tot.pw, tot.preq, (size_t)tot.lds, st) == 0 ? SBI_OK : SBI_ERR_HIP;
    }
    if (tot.prenorm && launch_layernorm_rows(gp, st) != 0) return SBI_ERR_HIP;
    return launch_mfma(gp, tot.nw, tot.depth, tot.pw, tot.ln, (size_t)tot.lds, st) == 0 ? SBI_OK : SBI_ERR_HIP;
}

}  // namespace

extern "C" {

size_t sbi_gemm_layout_bytes(int64_t K, int64_t N)
{
    if (check_shape(K, N) != SBI_OK) return 0;
    return (size_t)kHeaderBytes + (size_t)ksteps_of(K) * (size_t)ceil_div(N, kPanelN) * 4096u;
}

size_t sbi_gemm_workspace_bytes(int64_t B, int64_t K, int64_t N)
{
    Plan pl;
    if (make_plan(B, K, N, nullptr, pl) != SBI_OK) return 0;
    return (size_t)pl.ws_bytes;
}

size_t sbi_gemm_ln_workspace_bytes(int64_t B, int64_t K, int64_t N)
{
    const sbi_tuning t = {0, 0, 0, 0, 0, 0, 1, 0};
    Plan pl;
    if (make_plan(B, K, N, &t, pl) != SBI_OK) return 0;
    return (size_t)pl.ws_bytes;
}

sbi_status sbi_gemm_plan(int64_t B, int64_t K, int64_t N, const sbi_tuning* tuning, sbi_plan* plan)
{
    if (!plan) return SBI_ERR_NULL;
    Plan pl;
    if (sbi_status s = make_plan(B, K, N, tuning, pl)) return s;
    plan->path = pl.path; plan->waves = pl.nw; plan->depth = pl.depth; plan->split_k = pl.S;
    plan->ksteps_per_split = pl.ksps; plan->ksteps_per_chunk = pl.kc;
    plan->grid = pl.grid; plan->block = pl.block; plan->panels = pl.pw; plan->reserved = 0;
    plan->lds_bytes = pl.lds; plan->workspace_bytes = pl.ws_bytes;
    return SBI_OK;
}

sbi_status sbi_gemm_layout_weights(const void* W_rowmajor, int64_t K, int64_t N,
                                   void* W_laid_out, size_t laid_out_bytes, void* hip_stream)
{
    if (!W_rowmajor || !W_laid_out) return SBI_ERR_NULL;
    if (sbi_status s = check_shape(K, N)) return s;
    if (!aligned(W_rowmajor, 2) || !aligned(W_laid_out, 256)) return SBI_ERR_ALIGN;
    if (laid_out_bytes < sbi_gemm_layout_bytes(K, N)) return SBI_ERR_LAYOUT_MISMATCH;
    return launch_layout(W_rowmajor, K, N, W_laid_out, (hipStream_t)hip_stream) == 0 ? SBI_OK : SBI_ERR_HIP;
}

sbi_status sbi_gemm_unlayout_weights(const void* W_laid_out, int64_t K, int64_t N,
                                     void* W_rowmajor, void* hip_stream)
{
    if (!W_rowmajor || !W_laid_out) return SBI_ERR_NULL;
    if (sbi_status s = check_shape(K, N)) return s;
    if (!aligned(W_rowmajor, 2) || !aligned(W_laid_out, 256)) return SBI_ERR_ALIGN;
    return launch_unlayout(W_laid_out, K, N, W_rowmajor, (hipStream_t)hip_stream) == 0 ? SBI_OK : SBI_ERR_HIP;
}

static sbi_status layout_check_impl(const void* W_laid_out, int64_t K, int64_t N, void* hip_stream, bool want_i8)
{
    if (!W_laid_out) return SBI_ERR_NULL;
    if (sbi_status s = check_shape(K, N)) return s;
    if (!aligned(W_laid_out, 256)) return SBI_ERR_ALIGN;
    LayoutHeader h;
    std::memset(&h, 0, sizeof h);
    hipStream_t st = (hipStream_t)hip_stream;
    if (hipMemcpyAsync(&h, W_laid_out, sizeof h, hipMemcpyDeviceToHost, st) != hipSuccess) return SBI_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return SBI_ERR_HIP;
    const bool common = h.magic == kMagic && h.version == kLayoutVersion && h.K == K && h.N == N &&
                        h.P == ceil_div(N, kPanelN) && h.tile_n == kTileN && h.panel_tiles == kPanelTiles;
    const bool f16 = common && h.KS == ksteps_of(K) && h.tile_k == kTileK && h.chunk_k == kChunkK;
    const bool i8 = common && h.KS == ksteps_of_i8(K) && h.tile_k == kI8TileK && h.chunk_k == kI8ChunkK;
    return (want_i8 ? i8 : f16) ? SBI_OK : SBI_ERR_LAYOUT_MISMATCH;
}

sbi_status sbi_gemm_layout_check(const void* W_laid_out, int64_t K, int64_t N, void* hip_stream)
{
    return layout_check_impl(W_laid_out, K, N, hip_stream, false);
}

sbi_status sbi_gemm_i8_layout_check(const void* W_laid_out, int64_t K, int64_t N, void* hip_stream)
{
    return layout_check_impl(W_laid_out, K, N, hip_stream, true);
}

static sbi_status gemm_impl(const void* W_laid_out, int64_t K, int64_t N,
                            const void* X, int64_t B, const sbi_layernorm* ln,
                            const void* bias, const void* residual, sbi_epilogue epi,
                            void* Y, void* workspace, size_t workspace_bytes, void* hip_stream,
                            const sbi_tuning* tuning, const void* w_scales = nullptr, bool i8 = false,
                            void* moments_out = nullptr)
{
    int flags = 0;
    if (sbi_status s = check_gemm_args(W_laid_out, K, N, X, B, bias, residual, (int)epi, Y, flags)) return s;
    sbi_tuning t = {0, 0, 0, 0, 0, 0, 0, 0};
    if (tuning) t = *tuning;
    t.layernorm = ln ? 1 : 0;
    t.int8 = i8 ? 1 : 0;
    if (ln) {
        if (sbi_status s = check_layernorm(ln->gamma, ln->beta, ln->eps, K)) return s;
        if (ln->moments && (K % kPanelN != 0)) return SBI_ERR_SHAPE;      // moments come in 64-feature panels
        if (ln->moments && !aligned(ln->moments, 8)) return SBI_ERR_ALIGN;
    }
    if (moments_out && !aligned(moments_out, 8)) return SBI_ERR_ALIGN;
    if (i8 && ln && ln->moments) return SBI_ERR_TUNING;          // the fp64 statistics of the INT8 path read the rows
    if (i8) {
        if (!w_scales) return SBI_ERR_NULL;
        if (K % kI8ChunkK != 0) return SBI_ERR_SHAPE;
        if (!aligned(w_scales, 4)) return SBI_ERR_ALIGN;
    }
    Plan pl;
    if (sbi_status s = make_plan(B, K, N, &t, pl)) return s;
    if (pl.ws_bytes > 0) {
        if (!workspace || workspace_bytes < (size_t)pl.ws_bytes) return SBI_ERR_WORKSPACE;
        if (!aligned(workspace, 256)) return SBI_ERR_ALIGN;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    GemmArgs a = {W_laid_out, K, N, X, bias, residual, flags, Y, nullptr, nullptr, 0.0f, w_scales, moments_out, nullptr};
    if (moments_out && (pl.path != SBI_PATH_MFMA || i8)) return SBI_ERR_TUNING;   // only the fp16 matrix-core kernel emits them
    if (pl.path == SBI_PATH_STREAMK) return launch_group(&a, 1, B, pl, workspace, st);
    if (ln) { a.gamma = ln->gamma; a.beta = ln->beta; a.eps = ln->eps; a.ln_moments = ln->moments; }
    Plan one = pl;
    one.ws_bytes = (pl.S > 1) ? ceil_div(N, kPanelN) * pl.S * B * kPanelN * 4 : 0;      // its partial sums
    if (pl.path == SBI_PATH_MFMA) return launch_block_group(&a, &one, pl, 1, B, workspace, st);
    const GemmParams p = fill_params(a, B, pl, workspace, 0, 0);
    return launch_stream(p, pl.nw, pl.depth, (size_t)pl.lds, st) == 0 ? SBI_OK : SBI_ERR_HIP;
}

sbi_status sbi_gemm_ex(const void* W_laid_out, int64_t K, int64_t N,
                       const void* X, int64_t B,
                       const void* bias, const void* residual, sbi_epilogue epi,
                       void* Y, void* workspace, size_t workspace_bytes, void* hip_stream,
                       const sbi_tuning* tuning)
{
    if (tuning && (tuning->layernorm || tuning->int8)) return SBI_ERR_TUNING;   // those have entry points of their own
    return gemm_impl(W_laid_out, K, N, X, B, nullptr, bias, residual, epi, Y, workspace, workspace_bytes,
                     hip_stream, tuning);
}

sbi_status sbi_gemm(const void* W_laid_out, int64_t K, int64_t N,
                    const void* X, int64_t B,
                    const void* bias, const void* residual, sbi_epilogue epi,
                    void* Y, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return gemm_impl(W_laid_out, K, N, X, B, nullptr, bias, residual, epi, Y, workspace, workspace_bytes,
                     hip_stream, nullptr);
}

}  // extern "C"

// ---- sbi_gemm_static: the workspace of sbi_gemm in device memory the library owns -------------
// `scratch` is this translation unit's name for the array; in host code that name is a stand-in,
// not a device address.  Each GPU holds its own copy at its own address, which scratch_of() asks
// the runtime for once per device and keeps.
namespace {

static __device__ __align__(256) unsigned char scratch[SBI_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];                  // per device: address of its copy of `scratch`, or null
std::mutex g_scratch_mutex;

__global__ __launch_bounds__(256) void sbi_zero_words_kernel(unsigned int* dst, int n)
{
    for (int i = (int)(blockIdx.x * 256 + threadIdx.x); i < n; i += (int)(gridDim.x * 256)) dst[i] = 0u;
}

// Address of the current device's scratch array.  On the first call on a device the arrival
// counters at its start are cleared on `st` (by a kernel, so that the call can sit in a captured
// graph); after that every call leaves them at zero.  Calls no allocating routine.
sbi_status scratch_of(hipStream_t st, void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SBI_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SBI_ERR_HIP;
        hipLaunchKernelGGL(sbi_zero_words_kernel, dim3(64), dim3(256), 0, st,
                           reinterpret_cast<unsigned int*>(ptr), (int)(kCounterBytes / 4));
        if (hipGetLastError() != hipSuccess) return SBI_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SBI_OK;
}

}  // namespace

extern "C" {

sbi_status sbi_gemm_static(const void* W_laid_out, int64_t K, int64_t N,
                           const void* X, int64_t B,
                           const void* bias, const void* residual, sbi_epilogue epi,
                           void* Y, void* hip_stream)
{
    // everything the call can refuse is refused before the device is touched
    int flags = 0;
    if (sbi_status s = check_gemm_args(W_laid_out, K, N, X, B, bias, residual, (int)epi, Y, flags)) return s;
    Plan pl;
    if (sbi_status s = make_plan(B, K, N, nullptr, pl)) return s;
    if (pl.ws_bytes > (int64_t)SBI_STATIC_SCRATCH_BYTES) return SBI_ERR_WORKSPACE;
    void* ws = nullptr;
    if (pl.ws_bytes > 0)
        if (sbi_status s = scratch_of((hipStream_t)hip_stream, &ws)) return s;
    // (the whole array is offered: the launch below plans for itself and checks its need against it)
    return gemm_impl(W_laid_out, K, N, X, B, nullptr, bias, residual, epi, Y, ws, ws ? (size_t)SBI_STATIC_SCRATCH_BYTES : 0,
                     hip_stream, nullptr);
}

sbi_status sbi_gemm_ln(const void* W_laid_out, int64_t K, int64_t N,
                       const void* X, int64_t B, const sbi_layernorm* ln,
                       const void* bias, const void* residual, sbi_epilogue epi,
                       void* Y, void* workspace, size_t workspace_bytes, void* hip_stream,
                       const sbi_tuning* tuning)
{
    if (!ln) return SBI_ERR_NULL;
    if (tuning && tuning->int8) return SBI_ERR_TUNING;
    return gemm_impl(W_laid_out, K, N, X, B, ln, bias, residual, epi, Y, workspace, workspace_bytes,
                     hip_stream, tuning);
}

sbi_status sbi_gemm_moments(const void* W_laid_out, int64_t K, int64_t N,
                            const void* X, int64_t B, const sbi_layernorm* ln,
                            const void* bias, const void* residual, sbi_epilogue epi,
                            void* Y, void* row_moments, void* workspace, size_t workspace_bytes, void* hip_stream,
                            const sbi_tuning* tuning)
{
    if (!row_moments) return SBI_ERR_NULL;
    if (tuning && tuning->int8) return SBI_ERR_TUNING;
    return gemm_impl(W_laid_out, K, N, X, B, ln, bias, residual, epi, Y, workspace, workspace_bytes,
                     hip_stream, tuning, nullptr, false, row_moments);
}

size_t sbi_gemm_i8_layout_bytes(int64_t K, int64_t N)
{
    if (check_shape(K, N) != SBI_OK) return 0;
    return (size_t)kHeaderBytes + (size_t)ksteps_of_i8(K) * (size_t)ceil_div(N, kPanelN) * 4096u;
}

size_t sbi_gemm_i8_workspace_bytes(int64_t B, int64_t K, int64_t N)
{
    const sbi_tuning t = {0, 0, 0, 0, 0, 0, 0, 1};
    Plan pl;
    if (make_plan(B, K, N, &t, pl) != SBI_OK) return 0;
    return (size_t)pl.ws_bytes;
}

sbi_status sbi_gemm_i8_quantize_weights(const void* W_rowmajor, int64_t K, int64_t N,
                                        void* Wq_rowmajor, void* w_scales, void* hip_stream)
{
    if (!W_rowmajor || !Wq_rowmajor || !w_scales) return SBI_ERR_NULL;
    if (sbi_status s = check_shape(K, N)) return s;
    if (!aligned(W_rowmajor, 2) || !aligned(w_scales, 4)) return SBI_ERR_ALIGN;
    return launch_quantize_weights(W_rowmajor, K, N, Wq_rowmajor, w_scales, (hipStream_t)hip_stream) == 0
               ? SBI_OK : SBI_ERR_HIP;
}

sbi_status sbi_gemm_i8_layout_weights(const void* Wq_rowmajor, int64_t K, int64_t N,
                                      void* W_laid_out, size_t laid_out_bytes, void* hip_stream)
{
    if (!Wq_rowmajor || !W_laid_out) return SBI_ERR_NULL;
    if (sbi_status s = check_shape(K, N)) return s;
    if (!aligned(W_laid_out, 256)) return SBI_ERR_ALIGN;
    if (laid_out_bytes < sbi_gemm_i8_layout_bytes(K, N)) return SBI_ERR_LAYOUT_MISMATCH;
    return launch_layout_i8(Wq_rowmajor, K, N, W_laid_out, (hipStream_t)hip_stream) == 0 ? SBI_OK : SBI_ERR_HIP;
}

sbi_status sbi_gemm_i8(const void* W_laid_out, const void* w_scales, int64_t K, int64_t N,
                       const void* X, int64_t B,
                       const void* bias, const void* residual, sbi_epilogue epi,
                       void* Y, void* workspace, size_t workspace_bytes, void* hip_stream,
                       const sbi_tuning* tuning)
{
    if (tuning && tuning->layernorm) return SBI_ERR_TUNING;
    return gemm_impl(W_laid_out, K, N, X, B, nullptr, bias, residual, epi, Y, workspace, workspace_bytes,
                     hip_stream, tuning, w_scales, true);
}

sbi_status sbi_gemm_i8_ln(const void* W_laid_out, const void* w_scales, int64_t K, int64_t N,
                          const void* X, int64_t B, const sbi_layernorm* ln,
                          const void* bias, const void* residual, sbi_epilogue epi,
                          void* Y, void* workspace, size_t workspace_bytes, void* hip_stream,
                          const sbi_tuning* tuning)
{
    if (!ln) return SBI_ERR_NULL;
    return gemm_impl(W_laid_out, K, N, X, B, ln, bias, residual, epi, Y, workspace, workspace_bytes,
                     hip_stream, tuning, w_scales, true);
}

static sbi_status layer_check(const sbi_layer* L, int64_t B)
{
    if (!L) return SBI_ERR_NULL;
    if (!L->Wqkv || !L->Wout || !L->Wffn1 || !L->Wffn2) return SBI_ERR_NULL;
    if (B < 1 || B > SBI_MAX_BATCH) return SBI_ERR_BATCH;
    if (sbi_status s = check_shape(L->h, L->n_qkv)) return s;
    if (sbi_status s = check_shape(L->k_out, L->h)) return s;
    if (sbi_status s = check_shape(L->h, L->n_ffn1)) return s;
    if (sbi_status s = check_shape(L->k_ffn2, L->h)) return s;
    if (L->ln1_gamma || L->ln1_beta)
        if (sbi_status s = check_layernorm(L->ln1_gamma, L->ln1_beta, L->ln_eps, L->h)) return s;
    if (L->ln2_gamma || L->ln2_beta)
        if (sbi_status s = check_layernorm(L->ln2_gamma, L->ln2_beta, L->ln_eps, L->h)) return s;
    if (L->sqkv || L->sout || L->sffn1 || L->sffn2) {            // INT8 layer: all four weight matrices
        if (!L->sqkv || !L->sout || !L->sffn1 || !L->sffn2) return SBI_ERR_NULL;
        if (L->h % kI8ChunkK || L->k_out % kI8ChunkK || L->k_ffn2 % kI8ChunkK) return SBI_ERR_SHAPE;
        if (!aligned(L->sqkv, 4) || !aligned(L->sout, 4) || !aligned(L->sffn1, 4) || !aligned(L->sffn2, 4))
            return SBI_ERR_ALIGN;
    }
    return SBI_OK;
}

static bool layer_is_i8(const sbi_layer* L) { return L->sqkv != nullptr; }

// Plans of a grouped launch over GeMMs [0, count) of the layer.
static sbi_status layer_group_plan(const sbi_layer* L, int64_t B, int count, Plan* pls, Plan& tot)
{
    const int64_t Ks[4] = {L->h, L->k_out, L->h, L->k_ffn2};
    const int64_t Ns[4] = {L->n_qkv, L->h, L->n_ffn1, L->h};
    return plan_group(B, Ks, Ns, count, pls, tot, L->ln1_gamma || L->ln2_gamma, layer_is_i8(L));
}

size_t sbi_layer_workspace_bytes(const sbi_layer* L, int64_t B)
{
    if (layer_check(L, B) != SBI_OK) return 0;
    // a chained FFN2 runs on its own
    size_t m = layer_is_i8(L) ? sbi_gemm_i8_workspace_bytes(B, L->k_ffn2, L->h) : sbi_gemm_workspace_bytes(B, L->k_ffn2, L->h);
    Plan pls[4], tot;
    if (layer_group_plan(L, B, 4, pls, tot) == SBI_OK) m = std::max(m, (size_t)tot.ws_bytes);
    if (layer_group_plan(L, B, 3, pls, tot) == SBI_OK) m = std::max(m, (size_t)tot.ws_bytes);
    return m;
}

sbi_status sbi_layer_plan(const sbi_layer* L, int64_t B, int32_t chained, sbi_plan plans[4], int32_t* total_grid)
{
    if (!plans || !total_grid) return SBI_ERR_NULL;
    if (sbi_status s = layer_check(L, B)) return s;
    const int count = chained ? 3 : 4;
    Plan pls[4], tot;
    if (sbi_status s = layer_group_plan(L, B, count, pls, tot)) return s;
    std::memset(plans, 0, 4 * sizeof(sbi_plan));
    for (int g = 0; g < count; ++g) {
        plans[g].path = pls[g].path; plans[g].waves = tot.nw; plans[g].depth = tot.depth;
        plans[g].split_k = pls[g].S; plans[g].ksteps_per_split = pls[g].ksps;
        plans[g].ksteps_per_chunk = pls[g].kc; plans[g].grid = pls[g].grid; plans[g].block = tot.block;
        plans[g].panels = tot.pw;
        plans[g].lds_bytes = tot.lds; plans[g].workspace_bytes = pls[g].ws_bytes + pls[g].xq_bytes;
    }
    *total_grid = tot.grid;
    return SBI_OK;
}

sbi_status sbi_layer_gemms(const sbi_layer* L, int64_t B,
                           const void* Xqkv, const void* Xout, const void* Xffn1, const void* Xffn2,
                           const void* residual,
                           void* Yqkv, void* Yout, void* Yffn1, void* Yffn2,
                           void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (sbi_status s = layer_check(L, B)) return s;
    if (!Xqkv || !Xout || !Xffn1 || !Yqkv || !Yout || !Yffn1 || !Yffn2) return SBI_ERR_NULL;
    const bool chained = (Xffn2 == nullptr);
    if (chained) {
        if (L->n_ffn1 != L->k_ffn2) return SBI_ERR_SHAPE;
        Xffn2 = Yffn1;
    }
    // what THIS call needs (never more than sbi_layer_workspace_bytes, which covers both forms)
    hipStream_t st = (hipStream_t)hip_stream;
    const int count = chained ? 3 : 4;
    Plan pls[4], tot, last;
    if (sbi_status s = layer_group_plan(L, B, count, pls, tot)) return s;
    size_t need = (size_t)tot.ws_bytes;
    if (chained) {
        const sbi_tuning t8 = {0, 0, 0, 0, 0, 0, 0, 1};
        if (sbi_status s = make_plan(B, L->k_ffn2, L->h, layer_is_i8(L) ? &t8 : nullptr, last)) return s;
        need = std::max(need, (size_t)last.ws_bytes);
    }
    if (workspace_bytes < need || (need > 0 && !workspace)) return SBI_ERR_WORKSPACE;
    if (need > 0 && !aligned(workspace, 256)) return SBI_ERR_ALIGN;

    const sbi_epilogue e0 = L->bqkv ? SBI_EPI_BIAS : SBI_EPI_NONE;
    const sbi_epilogue eo = L->bout ? SBI_EPI_BIAS : SBI_EPI_NONE;
    const sbi_epilogue e1 = L->ffn1_gelu ? (L->bffn1 ? SBI_EPI_BIAS_GELU : SBI_EPI_GELU)
                                         : (L->bffn1 ? SBI_EPI_BIAS : SBI_EPI_NONE);
    const sbi_epilogue e2 = residual ? (L->bffn2 ? SBI_EPI_BIAS_RESIDUAL : SBI_EPI_RESIDUAL)
                                     : (L->bffn2 ? SBI_EPI_BIAS : SBI_EPI_NONE);
    GemmArgs a[4] = {
        {L->Wqkv, L->h, L->n_qkv, Xqkv, L->bqkv, nullptr, 0, Yqkv, L->ln1_gamma, L->ln1_beta, L->ln_eps, L->sqkv},
        {L->Wout, L->k_out, L->h, Xout, L->bout, nullptr, 0, Yout, nullptr, nullptr, 0.0f, L->sout},
        {L->Wffn1, L->h, L->n_ffn1, Xffn1, L->bffn1, nullptr, 0, Yffn1, L->ln2_gamma, L->ln2_beta, L->ln_eps, L->sffn1},
        {L->Wffn2, L->k_ffn2, L->h, Xffn2, L->bffn2, residual, 0, Yffn2, nullptr, nullptr, 0.0f, L->sffn2},
    };
    const sbi_epilogue epis[4] = {e0, eo, e1, e2};
    for (int g = 0; g < 4; ++g)
        if (sbi_status s = check_gemm_args(a[g].Wl, a[g].K, a[g].N, a[g].X, B, a[g].bias, a[g].R,
                                           (int)epis[g], a[g].Y, a[g].flags)) return s;

    // one launch for the independent GeMMs; a chained FFN2 needs FFN1's output and follows
    if (sbi_status s = launch_block_group(a, pls, tot, count, B, workspace, st)) return s;
    if (!chained) return SBI_OK;
    Plan one = last;
    one.ws_bytes = (last.S > 1) ? ceil_div(L->h, kPanelN) * last.S * B * kPanelN * 4 : 0;
    return launch_block_group(&a[3], &one, last, 1, B, workspace, st);
}


}  // extern "C"

// ---- measured plans ---------------------------------------------------------------------------
namespace {

// Average microseconds per call of `n` back-to-back calls of fn() on `st` (fn returns an sbi_status);
// negative if a call or the timing failed.
template <class F>
double time_calls(hipStream_t st, hipEvent_t e0, hipEvent_t e1, int n, F&& fn)
{
    if (hipEventRecord(e0, st) != hipSuccess) return -1.0;
    for (int i = 0; i < n; ++i)
        if (fn(i) != SBI_OK) return -1.0;
    if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) return -1.0;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) return -1.0;
    return (double)ms * 1e3 / n;
}

// Tries the dispatcher's candidates for one problem (those the model puts within 30 % of its best
// estimate, at most 48, distinct plans only) with run(i) = one launch on weight set i, and records
// the fastest.  `ws_limit`: candidates that need a larger workspace are left out.
template <class F>
sbi_status tune_problem(int64_t B, const int64_t* Ks, const int64_t* Ns, int G, bool ln, bool i8, size_t ws_limit,
                        hipStream_t st, int n_sets, sbi_tune_report* report, F&& run)
{
    std::vector<Candidate> all;
    Plan pls[kMaxGroup], tot;
    Candidate model;                    // what the dispatcher picks without measurements: always trial 0
    if (sbi_status s = plan_group_search(B, Ks, Ns, G, pls, tot, ln, i8, nullptr, nullptr, &model)) return s;
    if (sbi_status s = plan_group_search(B, Ks, Ns, G, pls, tot, ln, i8, nullptr, &all)) return s;
    std::stable_sort(all.begin(), all.end(), [](const Candidate& a, const Candidate& b) { return a.cost < b.cost; });
    const double limit = std::min(model.cost, all.empty() ? model.cost : all.front().cost) * 1.3;
    all.insert(all.begin(), model);
    struct Trial { Candidate c; Plan pls[kMaxGroup]; Plan tot; };
    std::vector<Trial> trials;
    for (const Candidate& c : all) {
        if (c.cost > limit || trials.size() >= 48) break;
        Trial t;
        t.c = c;
        if (plan_group_search(B, Ks, Ns, G, t.pls, t.tot, ln, i8, &c) != SBI_OK) continue;
        if ((size_t)t.tot.ws_bytes > ws_limit) continue;
        bool seen = false;
        for (const Trial& o : trials) {
            bool same = o.tot.nw == t.tot.nw && o.tot.depth == t.tot.depth && o.tot.pw == t.tot.pw && o.tot.lds == t.tot.lds;
            for (int g = 0; g < G && same; ++g)
                same = o.pls[g].S == t.pls[g].S && o.pls[g].ksps == t.pls[g].ksps && o.pls[g].kc == t.pls[g].kc;
            seen = seen || same;
        }
        if (!seen) trials.push_back(t);
    }
    if (trials.empty()) return SBI_ERR_WORKSPACE;

    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return SBI_ERR_HIP;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return SBI_ERR_HIP; }
    TunedEntry entry;
    entry.B = B; entry.G = G; entry.flags = (ln ? 1 : 0) | (i8 ? 2 : 0);
    for (int g = 0; g < kMaxGroup; ++g) { entry.Ks[g] = g < G ? Ks[g] : 0; entry.Ns[g] = g < G ? Ns[g] : 0; }
    const int per_run = std::max(6, 2 * n_sets);
    double best_us = -1.0, model_us = -1.0;
    size_t best = 0;
    for (size_t k = 0; k < trials.size(); ++k) {
        entry.c = trials[k].c;
        t_trial = &entry;
        double us = time_calls(st, e0, e1, 3, run) < 0.0 ? -1.0 : 1e30;          // warm-up (code, translations)
        for (int rep = 0; rep < 3 && us >= 0.0; ++rep) {
            const double t = time_calls(st, e0, e1, per_run, run);
            us = t < 0.0 ? -1.0 : std::min(us, t);
        }
        t_trial = nullptr;
        if (us < 0.0) continue;                                                 // this candidate cannot be launched
        if (k == 0) model_us = us;
        if (best_us < 0.0 || us < best_us) { best_us = us; best = k; }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (best_us < 0.0) return SBI_ERR_HIP;
    // a candidate replaces the model's own pick only if it is ahead by more than the run-to-run spread of
    // such measurements (about 1 %): otherwise what looks like a gain is as often a loss in the next run
    if (best != 0 && model_us > 0.0 && best_us > 0.99 * model_us) { best = 0; best_us = model_us; }
    entry.c = trials[best].c;
    {
        std::lock_guard<std::mutex> lock(g_tuned_mutex);
        bool replaced = false;
        for (TunedEntry& t : g_tuned)
            if (same_problem(t, B, Ks, Ns, G, entry.flags)) { t = entry; replaced = true; }
        if (!replaced) g_tuned.push_back(entry);
        g_tuned_version.fetch_add(1, std::memory_order_release);
    }
    if (report) {
        report->candidates = (int32_t)trials.size();
        report->waves = entry.c.nw; report->depth = entry.c.depth; report->panels = entry.c.pw;
        report->block_ksteps = (int32_t)entry.c.T;
        report->us_best = (float)best_us; report->us_model = (float)model_us;
    }
    return SBI_OK;
}

}  // namespace

extern "C" {

sbi_status sbi_layer_tune(const sbi_layer* layers, int32_t n_layers, int64_t B,
                          const void* Xqkv, const void* Xout, const void* Xffn1, const void* Xffn2,
                          const void* residual,
                          void* Yqkv, void* Yout, void* Yffn1, void* Yffn2,
                          void* workspace, size_t workspace_bytes, void* hip_stream, sbi_tune_report* report)
{
    if (!layers || n_layers < 1 || n_layers > 4096) return SBI_ERR_NULL;
    for (int i = 0; i < n_layers; ++i) {
        if (sbi_status s = layer_check(&layers[i], B)) return s;
        const sbi_layer &a = layers[0], &b = layers[i];
        if (a.h != b.h || a.n_qkv != b.n_qkv || a.k_out != b.k_out || a.n_ffn1 != b.n_ffn1 || a.k_ffn2 != b.k_ffn2 ||
            layer_is_i8(&a) != layer_is_i8(&b) || (a.ln1_gamma || a.ln2_gamma) != (b.ln1_gamma || b.ln2_gamma))
            return SBI_ERR_SHAPE;                          // one shape and one flavour per call
    }
    const sbi_layer* L = &layers[0];
    const int count = Xffn2 ? 4 : 3;
    const int64_t Ks[4] = {L->h, L->k_out, L->h, L->k_ffn2};
    const int64_t Ns[4] = {L->n_qkv, L->h, L->n_ffn1, L->h};
    // a first call under the model's plan: reports every argument error before anything is measured
    if (sbi_status s = sbi_layer_gemms(L, B, Xqkv, Xout, Xffn1, Xffn2, residual, Yqkv, Yout, Yffn1, Yffn2, workspace,
                                       workspace_bytes, hip_stream)) return s;
    return tune_problem(B, Ks, Ns, count, L->ln1_gamma || L->ln2_gamma, layer_is_i8(L), workspace_bytes,
                        (hipStream_t)hip_stream, n_layers, report, [&](int i) {
                            return sbi_layer_gemms(&layers[i % n_layers], B, Xqkv, Xout, Xffn1, Xffn2, residual, Yqkv, Yout,
                                                   Yffn1, Yffn2, workspace, workspace_bytes, hip_stream);
                        });
}

sbi_status sbi_gemm_tune(const void* const* W_laid_out, int32_t n_weights, int64_t K, int64_t N,
                         const void* X, int64_t B,
                         const void* bias, const void* residual, sbi_epilogue epi,
                         void* Y, void* workspace, size_t workspace_bytes, void* hip_stream, sbi_tune_report* report)
{
    if (!W_laid_out || n_weights < 1 || n_weights > 4096) return SBI_ERR_NULL;
    for (int i = 0; i < n_weights; ++i)
        if (!W_laid_out[i] || !aligned(W_laid_out[i], 256)) return W_laid_out[i] ? SBI_ERR_ALIGN : SBI_ERR_NULL;
    if (sbi_status s = sbi_gemm(W_laid_out[0], K, N, X, B, bias, residual, epi, Y, workspace, workspace_bytes, hip_stream))
        return s;
    return tune_problem(B, &K, &N, 1, false, false, workspace_bytes, (hipStream_t)hip_stream, n_weights, report, [&](int i) {
        return sbi_gemm(W_laid_out[i % n_weights], K, N, X, B, bias, residual, epi, Y, workspace, workspace_bytes, hip_stream);
    });
}

// Position ranges per (sequence, head) of the attention kernel: one block per CU where the
// context allows it, but no range shorter than 256 cached positions (more, shorter ranges were
// measured slower at every shape: a block's fixed cost is about the time to stream 128 positions).
// A ragged batch (n = its bound + 1) is cut by the same rule: finer cuts were measured no faster
// there either (8 sequences of 256 .. 2048 positions, 32 heads: 37.5 us with one range per sequence
// and head, 38.0 / 38.8 / 39.3 us with two / four / eight).
static int attn_splits(int64_t B, int64_t H, int64_t n)
{
    int64_t target = 256, shortest = 256, cap = 32;
#ifdef SBI_DEV
    if (const char* e = getenv("SBI_ATTN_SPLIT")) {
        long long a, b, c;
        if (sscanf(e, "%lld,%lld,%lld", &a, &b, &c) == 3) { target = a; shortest = b; cap = c; }
    }
#endif
    const int64_t want = ceil_div(target, B * H);
    const int64_t most = std::max<int64_t>(1, n / shortest);
    return (int)std::max<int64_t>(1, std::min<int64_t>(std::min(want, most), std::min<int64_t>(cap, kAttnMaxSplits)));
}

static sbi_status attn_check_dims(int64_t B, int32_t heads, int32_t head_dim, int64_t max_seq)
{
    if (B < 1 || B > SBI_MAX_BATCH) return SBI_ERR_BATCH;
    if (heads < 1 || heads > 1024 || (head_dim != 64 && head_dim != 128) || max_seq < 1 || max_seq > (int64_t(1) << 24))
        return SBI_ERR_SHAPE;
    return SBI_OK;
}

size_t sbi_attn_decode_workspace_bytes(int64_t B, int32_t heads, int32_t head_dim, int64_t max_seq)
{
    if (attn_check_dims(B, heads, head_dim, max_seq) != SBI_OK) return 0;
    const int ns = attn_splits(B, heads, max_seq);
    return ns > 1 ? (size_t)kAttnCounterBytes + (size_t)B * heads * ns * (head_dim + 2) * 4 : 0;
}

// pos_of == NULL: every sequence at `pos`; else pos_of[b], of which `pos` is the bound
static sbi_status attn_decode(const void* qkv, void* k_cache, void* v_cache, int64_t B, int32_t heads, int32_t head_dim,
                              int64_t max_seq, int64_t pos, const int32_t* pos_of, float scale, void* out,
                              void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!qkv || !k_cache || !v_cache || !out) return SBI_ERR_NULL;
    if (sbi_status s = attn_check_dims(B, heads, head_dim, max_seq)) return s;
    if (pos < 0 || pos >= max_seq) return SBI_ERR_SHAPE;
    if (!(scale >= 0.0f) || !std::isfinite(scale)) return SBI_ERR_EPILOGUE;
    if (!aligned(qkv, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16) || !aligned(out, 2)) return SBI_ERR_ALIGN;
    if (scale == 0.0f) scale = 1.0f / std::sqrt((float)head_dim);
    const int ns = attn_splits(B, heads, pos + 1);
    if (ns > 1) {
        const size_t need = (size_t)kAttnCounterBytes + (size_t)B * heads * ns * (head_dim + 2) * 4;
        if (!workspace || workspace_bytes < need) return SBI_ERR_WORKSPACE;
        if (!aligned(workspace, 256)) return SBI_ERR_ALIGN;
    }
    return launch_attn_decode(qkv, k_cache, v_cache, B, heads, head_dim, max_seq, pos, pos_of, scale, out,
                              ns > 1 ? workspace : nullptr, ns, (hipStream_t)hip_stream) == 0 ? SBI_OK : SBI_ERR_HIP;
}

sbi_status sbi_attn_decode(const void* qkv, void* k_cache, void* v_cache, int64_t B, int32_t heads, int32_t head_dim,
                           int64_t max_seq, int64_t pos, float scale, void* out,
                           void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return attn_decode(qkv, k_cache, v_cache, B, heads, head_dim, max_seq, pos, nullptr, scale, out, workspace,
                       workspace_bytes, hip_stream);
}

sbi_status sbi_attn_decode_ragged(const void* qkv, void* k_cache, void* v_cache, int64_t B, int32_t heads,
                                  int32_t head_dim, int64_t max_seq, const int32_t* pos, int64_t pos_bound, float scale,
                                  void* out, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!pos) return SBI_ERR_NULL;
    if (!aligned(pos, 4)) return SBI_ERR_ALIGN;
    return attn_decode(qkv, k_cache, v_cache, B, heads, head_dim, max_seq, pos_bound, pos, scale, out, workspace,
                       workspace_bytes, hip_stream);
}

const char* sbi_status_string(sbi_status s)
{
    switch (s) {
        case SBI_OK: return "ok";
        case SBI_ERR_NULL: return "a required pointer is NULL";
        case SBI_ERR_SHAPE: return "bad shape";
        case SBI_ERR_ALIGN: return "pointer not aligned as documented";
        case SBI_ERR_BATCH: return "batch outside 1..64";
        case SBI_ERR_LAYOUT_MISMATCH: return "laid-out buffer does not match (K, N)";
        case SBI_ERR_WORKSPACE: return "workspace missing or too small";
        case SBI_ERR_EPILOGUE: return "bad epilogue or missing bias/residual";
        case SBI_ERR_HIP: return "HIP runtime error";
        case SBI_ERR_OVERLAP: return "Y overlaps X";
        case SBI_ERR_TUNING: return "unsupported tuning request";
    }
    return "unknown status";
}

sbi_status sbi_kernel_registers(int64_t B, int32_t waves, int32_t depth, int32_t panels, int32_t flavour,
                                int32_t* allocated, int32_t* assumed)
{
    if (!allocated || !assumed) return SBI_ERR_NULL;
    if (B < 1 || B > SBI_MAX_BATCH) return SBI_ERR_BATCH;
    if (flavour < 0 || flavour > 3) return SBI_ERR_TUNING;
    const int mb = (int)((B + 15) / 16);
    const bool ln = flavour == 1, i8 = flavour >= 2, preq = flavour == 3;
    const void* fn = i8 ? sbi::i8_kernel_entry(mb, waves, depth, panels, preq) : sbi::mfma_kernel_entry(mb, waves, depth, panels, ln);
    if (!fn) return SBI_ERR_TUNING;
    hipFuncAttributes attr;
    if (hipFuncGetAttributes(&attr, fn) != hipSuccess) return SBI_ERR_HIP;
    *allocated = attr.numRegs;
    *assumed = assumed_vgprs(mb, waves, depth, panels, ln, i8, preq);
    return SBI_OK;
}

int32_t sbi_version(void) { return 100; }

}  // extern "C"
