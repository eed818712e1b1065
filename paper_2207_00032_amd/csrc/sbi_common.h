// Internal definitions shared by the gfx950 kernels and the C-ABI translation unit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sbi {

// ---- weight layout (one lane = 8 consecutive k of one column = one 128-bit load) ----
constexpr int kChunkK     = 8;                       // halfs per lane per load
constexpr int kTileN      = 16;                      // columns per wavefront tile
constexpr int kTileK      = 32;                      // k per tile ("k-step")
constexpr int kStepGroup  = 8;                       // k-steps per panel are padded to a multiple of this
constexpr int kPanelTiles = 4;                       // tiles per panel
constexpr int kPanelN     = kTileN * kPanelTiles;    // 64 columns
constexpr int kHeaderBytes = 256;
constexpr uint32_t kMagic = 0x47494253u;             // "SBIG"
constexpr uint32_t kLayoutVersion = 2;
constexpr int kNumCU = 256;                          // MI355X

// k-steps per panel of the laid-out buffer (zero padded)
constexpr int64_t ksteps_of(int64_t K) { return ((K + kTileK - 1) / kTileK + kStepGroup - 1) / kStepGroup * kStepGroup; }

struct LayoutHeader {            // lives in the first 256 bytes of a laid-out buffer
    uint32_t magic;
    uint32_t version;
    int64_t  K;
    int64_t  N;
    int64_t  KS;                 // k-steps per panel: ceil(K / 32) rounded up to a multiple of 8
    int64_t  P;                  // ceil(N / 64)
    int32_t  tile_n, tile_k, panel_tiles, chunk_k;
};
static_assert(sizeof(LayoutHeader) <= kHeaderBytes, "header must fit");

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

constexpr int kEpiBias = 1, kEpiGelu = 2, kEpiRes = 4;

// Hand-over of partial results between blocks (split-K, attention position ranges): the producer
// writes them with device-scope stores (write-through, they never sit dirty in one XCD's L2), then
// calls this, then its arrival is counted with a device-scope atomic; the consumer reads them with
// device-scope loads only after it has seen the full count.  What orders "partials visible" before
// "arrival counted" is this wait: on gfx9-family targets loads and stores share one counter
// (vmcnt), and a store leaves it only when the memory system has acknowledged the write.  It is
// the s_waitcnt half of the device-scope release the compiler would emit; the other half, a
// write-back of the whole L2, has nothing to write back here (no ordinary stores are handed over)
// and was measured at twice the kernel time.  The empty statements on either side keep the compiler
// from moving memory accesses across the wait.
__device__ __forceinline__ void wait_stores_acknowledged()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0); expcnt and lgkmcnt fields at their maxima = not waited for
    asm volatile("" ::: "memory");
}

// Pitch (in floats) of one row of the in-block reduction buffer: 64 columns + 4 so that
// the 16 lanes of a group, which write 16-byte pieces of 16 different rows, hit distinct banks.
constexpr int kRedPitch = 68;

struct GemmParams {
    const u32x4*    Wl;        // laid-out weights, past the header
    const _Float16* X;         // [B,K]
    const _Float16* bias;      // [N] or null
    const _Float16* R;         // [B,N] or null
    _Float16*       Y;         // [B,N]
    float*          partials;  // [P][S][B][64] when S > 1
    unsigned int*   counters;  // [P] arrival counters when S > 1
    int B, K, N;
    int KS, P;                 // k-steps, panels
    int S;                     // blocks per panel (split-K factor)
    int ksps;                  // k-steps per block
    int kc;                    // k-steps of X staged per chunk (multiple of waves*depth)
    int xpitch;                // 16-byte pieces between the lane groups of a k-step's X block in LDS: B rounded up to odd
    int flags;                 // kEpi* bits
    int x_vec;                 // 1: X rows are 16-byte aligned and K % 8 == 0
    int ln;                    // 1: layer-normalise the rows of X on their way into LDS
    const _Float16* ln_gamma;  // [K]; in a launch of the layer-norm kernel variant always readable
    const _Float16* ln_beta;   // [K]    (problems with ln == 0 point both at X)
    float ln_eps;
    floatx2* moments_out;      // or null: per row and 64-column panel (mean, sum of squared deviations) of Y
    const floatx2* ln_moments; // or null: such moments of X's rows (64-wide panels), instead of reading the rows
    const float* sw;           // INT8 path: per-column weight scales [N]
    const _Float16* X16;       // INT8 path with activations quantised by a kernel of their own: the fp16 X
    const floatx2* xstats;     //   (X then points at the codes [B,K] int8) and the rows' (inv, scale) [B]
#ifdef SBI_TRACE
    unsigned long long* trace; // development builds: 4 timestamps per block
#endif
};

// ---- grouped launches: up to kMaxGroup independent GeMMs of one batch size per launch ----
constexpr int kMaxGroup = 4;

// Block-decomposed kernel over several problems: blocks [first_block[g], first_block[g+1])
// belong to problem g and are numbered (panel, split) inside it.
struct GroupParams {
    GemmParams g[kMaxGroup];
    int        G;
    int        first_block[kMaxGroup + 1];
};

struct SkProblem {
    const u32x4*    Wl;        // laid-out weights, past the header
    const _Float16* X;         // [B,K], 16-byte aligned, K % 8 == 0
    const _Float16* bias;
    const _Float16* R;
    _Float16*       Y;
    int K, N;
    int KS, P;                 // k-steps per panel (multiple of 8), panels
    int flags;                 // kEpi* bits
    int unit_base;             // index of this problem's first 4 KiB unit in the launch
    int panel_base;            // index of this problem's first panel counter
    int fast;                  // N % 4 == 0 and bias / R / Y 8-byte aligned: 4-wide epilogue
};

struct SkParams {
    SkProblem     prob[kMaxGroup];
    int           G;           // problems in this launch
    int           B;
    int           U;           // total units
    int           upw;         // units per wavefront (multiple of 8)
    float*        partials;    // [wavefronts][2][B][64] fp32
    unsigned int* counters;    // one arrival counter per panel of the launch
};

// launchers implemented in the kernel translation units; return hipError_t as int
int launch_streamk(const SkParams& p, int waves, int depth, int grid, hipStream_t st);
int launch_mfma(const GroupParams& gp, int waves, int depth, int panels, bool layernorm, size_t lds_bytes,
                hipStream_t st);
int launch_i8(const GroupParams& gp, int waves, int depth, int panels, bool prequantized, size_t lds_bytes, hipStream_t st);
// the kernel those two would start (null: no such variant), for queries of its compiled resources
const void* mfma_kernel_entry(int mb, int waves, int depth, int panels, bool layernorm);
const void* i8_kernel_entry(int mb, int waves, int depth, int panels, bool prequantized);
// Normalises the rows of every problem of `gp` whose X16 (raw rows) differs from its X (where the
// GeMM kernel will read the normalised rows), one block per row.
int launch_layernorm_rows(const GroupParams& gp, hipStream_t st);
int launch_layout_i8(const void* Wq, int64_t K, int64_t N, void* out, hipStream_t st);
int launch_quantize_weights(const void* W, int64_t K, int64_t N, void* Wq, void* scales, hipStream_t st);
int launch_attn_decode(const void* qkv, void* Kc, void* Vc, int64_t B, int H, int D, int64_t S, int64_t pos,
                       const int* pos_of, float scale, void* out, void* workspace, int nsplit, hipStream_t st);
constexpr int kAttnMaxSplits = 128;                  // most position ranges one (sequence, head) of the attention kernel is split into
constexpr int kAttnCounterBytes = 256 * 1024;        // arrival counters of the attention kernel's workspace (one per sequence and head)
constexpr int kI8TileK = 64;                         // k per k-step of the int8 layout
constexpr int kI8ChunkK = 16;                        // consecutive k one lane owns (16 bytes)
inline int64_t ksteps_of_i8(int64_t K) { return ((K + kI8TileK - 1) / kI8TileK + kStepGroup - 1) / kStepGroup * kStepGroup; }
constexpr int kLnStatsBytes = 512;                   // LDS in front of the X tile: (mean, 1/std) per batch row
int launch_stream(const GemmParams& p, int waves, int depth, size_t lds_bytes, hipStream_t st);
int launch_layout(const void* W, int64_t K, int64_t N, void* out, hipStream_t st);
int launch_unlayout(const void* Wl, int64_t K, int64_t N, void* out, hipStream_t st);

}  // namespace sbi
