// Vector-ALU streaming kernel for the smallest batches (B <= 8) on gfx950.
//
// Same decomposition and weight stream as the matrix-core kernel: one block per
// (64-column panel, k-range), its wavefronts take the k-steps round-robin, each lane's
// 128-bit load delivers 8 consecutive k of one column.  The products are formed with
// v_dot2_f32_f16 (two fp16 x fp16 products added into an fp32 accumulator), the X operand
// of a lane group is one broadcast 128-bit LDS read per batch row.  A column's K range is
// spread over the four 16-lane groups of a wavefront, so the wave ends with a two-step
// cross-lane reduction (lanes l, l^16, l^32, l^48) before the partial tile goes to LDS:
// the register-level counterpart of the paper's warp-collective reduction (Sec. III-C,
// "Cooperative-Group Reduction").
#include "sbi_block.h"

namespace sbi {

// Per-wave contraction state: lane (g, i) accumulates, for each of the four tiles, column i
// over the k of its lane group g, for BT batch rows.
template <int BT>
struct DotOp {
    float acc[kPanelTiles][BT];
    int xoff;         // the lane group's 16-byte slots inside a k-step's X block

    __device__ __forceinline__ void init(int g, int pitch)
    {
#pragma unroll
        for (int t = 0; t < kPanelTiles; ++t)
#pragma unroll
            for (int b = 0; b < BT; ++b) acc[t][b] = 0.f;
        xoff = g * pitch;
    }

    u32x4 xf[BT];

    __device__ __forceinline__ void begin(const u32x4* xk, const u32x4*)
    {
#pragma unroll
        for (int b = 0; b < BT; ++b) xf[b] = xk[xoff + b];     // same address in all 16 lanes: broadcast
    }

    __device__ __forceinline__ void tile(int t, u32x4 w)
    {
        const unsigned int wq[4] = {w.x, w.y, w.z, w.w};      // k pairs (0,1) (2,3) (4,5) (6,7)
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            const unsigned int xq[4] = {xf[b].x, xf[b].y, xf[b].z, xf[b].w};
            float a = acc[t][b];
            a = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, wq[0]), __builtin_bit_cast(half2v, xq[0]), a, false);
            a = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, wq[1]), __builtin_bit_cast(half2v, xq[1]), a, false);
            a = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, wq[2]), __builtin_bit_cast(half2v, xq[2]), a, false);
            a = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, wq[3]), __builtin_bit_cast(half2v, xq[3]), a, false);
            acc[t][b] = a;
        }
    }
};

template <int BT, int NW, int DEPTH>
__global__ __launch_bounds__(NW * 64) void sbi_stream_kernel(const GemmParams p)
{
    constexpr int NT = NW * 64;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    u32x4* xs  = reinterpret_cast<u32x4*>(smem_raw);
    float* red = reinterpret_cast<float*>(smem_raw);
    __shared__ int s_flag;

    const int tid  = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4;
    const int i = lane & 15;

    const int panel = blockIdx.x / p.S;
    const int split = blockIdx.x - panel * p.S;
    const int ks0 = split * p.ksps;
    const int ks1 = min(p.KS, ks0 + p.ksps);

    DotOp<BT> op;
    op.init(g, p.xpitch);
    XStage<NW * 64, 4, false> xst;
    stream_panel<NW, DEPTH, 1, false>(p, xs, xst, op, tid, wave, lane, panel, 0, ks0, ks1);

    // cross-lane K reduction over the four lane groups, then park the wave's tile in LDS
#pragma unroll
    for (int t = 0; t < kPanelTiles; ++t)
#pragma unroll
        for (int b = 0; b < BT; ++b) {
            float v = op.acc[t][b];
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            op.acc[t][b] = v;
        }
    RowOperands<NW> ops;               // bias / residual, requested ahead of the barriers
    ops = request_row_operands<NW>(p, 0, panel, tid, true, ops);
    __syncthreads();                   // X tile no longer needed
    if (g == 0) {
#pragma unroll
        for (int t = 0; t < kPanelTiles; ++t)
#pragma unroll
            for (int b = 0; b < BT; ++b)
                red[(wave * 16 + b) * kRedPitch + t * kTileN + i] = op.acc[t][b];
    }
    __syncthreads();
    reduce_rows<NW>(p, red, 0, panel, split, tid, ops);

    if (p.S > 1) finish_split_k<NT>(p, panel, tid, &s_flag);
}

template <int BT, int NW, int DEPTH>
static int launch_one(const GemmParams& p, size_t lds, hipStream_t st)
{
    hipLaunchKernelGGL((sbi_stream_kernel<BT, NW, DEPTH>), dim3(p.P * p.S), dim3(NW * 64), lds, st, p);
    return (int)hipGetLastError();
}

template <int NW, int DEPTH>
static int launch_bt(const GemmParams& p, size_t lds, hipStream_t st)
{
    switch (p.B) {
        case 1: return launch_one<1, NW, DEPTH>(p, lds, st);
        case 2: return launch_one<2, NW, DEPTH>(p, lds, st);
        case 3: return launch_one<3, NW, DEPTH>(p, lds, st);
        case 4: return launch_one<4, NW, DEPTH>(p, lds, st);
        case 5: return launch_one<5, NW, DEPTH>(p, lds, st);
        case 6: return launch_one<6, NW, DEPTH>(p, lds, st);
        case 7: return launch_one<7, NW, DEPTH>(p, lds, st);
        case 8: return launch_one<8, NW, DEPTH>(p, lds, st);
    }
    return (int)hipErrorInvalidValue;
}

int launch_stream(const GemmParams& p, int waves, int depth, size_t lds_bytes, hipStream_t st)
{
    if (waves == 4 && depth == 4) return launch_bt<4, 4>(p, lds_bytes, st);
    if (waves == 4 && depth == 8) return launch_bt<4, 8>(p, lds_bytes, st);
    if (waves == 8 && depth == 4) return launch_bt<8, 4>(p, lds_bytes, st);
    if (waves == 8 && depth == 8) return launch_bt<8, 8>(p, lds_bytes, st);
    return (int)hipErrorInvalidValue;
}

}  // namespace sbi
