// One-time weight pre-layout and its inverse (gfx950).
//
// The paper re-tiles W once "during initialization" so that each thread can read several
// consecutive input-dimension elements of a column in one access (Sec. III-C, "Leveraging
// Full Cache-line").  Here the unit is a 32-k x 64-column block of W (4 KiB): it is read
// row-wise, transposed through LDS and written as four 1 KiB wavefront tiles in which
// lane (g*16 + i) owns k = 8g..8g+7 of column i.  Pure permutation with zero padding.
#include "sbi_common.h"

namespace sbi {

constexpr int kLdsPitch = kPanelN + 2;   // halfs per LDS row; odd dword pitch against bank conflicts

__global__ __launch_bounds__(256) void sbi_layout_kernel(const _Float16* __restrict__ W, int64_t K, int64_t N,
                                                         int64_t KS, int64_t P, int w_vec,
                                                         unsigned char* __restrict__ out)
{
    __shared__ _Float16 tile[kTileK][kLdsPitch];
    const int tid = threadIdx.x;
    const int64_t ks = blockIdx.x % KS;
    const int64_t pn = blockIdx.x / KS;

    if (blockIdx.x == 0) {
        // header: the LayoutHeader fields (thread 0), the rest of the 256 bytes zero
        constexpr int kHeaderWords = (int)(sizeof(LayoutHeader) / 4);
        static_assert(sizeof(LayoutHeader) % 4 == 0, "header is written in 32-bit words");
        if (tid == 0) {
            LayoutHeader h;
            h.magic = kMagic; h.version = kLayoutVersion;
            h.K = K; h.N = N; h.KS = KS; h.P = P;
            h.tile_n = kTileN; h.tile_k = kTileK; h.panel_tiles = kPanelTiles; h.chunk_k = kChunkK;
            *reinterpret_cast<LayoutHeader*>(out) = h;
        } else if (tid >= kHeaderWords && tid < kHeaderBytes / 4) {
            reinterpret_cast<uint32_t*>(out)[tid] = 0u;
        }
    }

    // read: 32 rows x 64 columns, thread -> (row, 8-column segment)
    {
        const int r = tid >> 3;
        const int c0 = (tid & 7) * 8;
        const int64_t k = ks * kTileK + r;
        const int64_t n0 = pn * kPanelN + c0;
        if (w_vec && k < K && n0 + 8 <= N) {
            const half8 v = __builtin_bit_cast(half8, *reinterpret_cast<const u32x4*>(W + k * N + n0));
#pragma unroll
            for (int e = 0; e < 8; ++e) tile[r][c0 + e] = v[e];
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int64_t n = n0 + e;
                tile[r][c0 + e] = (k < K && n < N) ? W[k * N + n] : (_Float16)0.0f;
            }
        }
    }
    __syncthreads();
    // write: thread -> (tile t, lane); lane = g*16 + i owns k = 8g..8g+7 of column t*16+i
    {
        const int t = tid >> 6;
        const int lane = tid & 63;
        const int g = lane >> 4;
        const int i = lane & 15;
        half8 v;
#pragma unroll
        for (int e = 0; e < kChunkK; ++e) v[e] = tile[g * kChunkK + e][t * kTileN + i];
        u32x4* dst = reinterpret_cast<u32x4*>(out + kHeaderBytes) +
                     ((pn * KS + ks) * kPanelTiles + t) * 64 + lane;
        *dst = __builtin_bit_cast(u32x4, v);
    }
}

__global__ __launch_bounds__(256) void sbi_unlayout_kernel(const unsigned char* __restrict__ in, int64_t K, int64_t N,
                                                           int64_t KS, _Float16* __restrict__ W)
{
    __shared__ _Float16 tile[kTileK][kLdsPitch];
    const int tid = threadIdx.x;
    const int64_t ks = blockIdx.x % KS;
    const int64_t pn = blockIdx.x / KS;
    {
        const int t = tid >> 6;
        const int lane = tid & 63;
        const int g = lane >> 4;
        const int i = lane & 15;
        const u32x4* src = reinterpret_cast<const u32x4*>(in + kHeaderBytes) +
                           ((pn * KS + ks) * kPanelTiles + t) * 64 + lane;
        const half8 v = __builtin_bit_cast(half8, *src);
#pragma unroll
        for (int e = 0; e < kChunkK; ++e) tile[g * kChunkK + e][t * kTileN + i] = v[e];
    }
    __syncthreads();
    {
        const int r = tid >> 3;
        const int c0 = (tid & 7) * 8;
        const int64_t k = ks * kTileK + r;
        const int64_t n0 = pn * kPanelN + c0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int64_t n = n0 + e;
            if (k < K && n < N) W[k * N + n] = tile[r][c0 + e];
        }
    }
}

int launch_layout(const void* W, int64_t K, int64_t N, void* out, hipStream_t st)
{
    const int64_t KS = ksteps_of(K);
    const int64_t P = (N + kPanelN - 1) / kPanelN;
    const int w_vec = (N % 8 == 0) && ((reinterpret_cast<uintptr_t>(W) & 15) == 0);
    hipLaunchKernelGGL(sbi_layout_kernel, dim3((unsigned)(KS * P)), dim3(256), 0, st,
                       reinterpret_cast<const _Float16*>(W), K, N, KS, P, w_vec,
                       reinterpret_cast<unsigned char*>(out));
    return (int)hipGetLastError();
}

int launch_unlayout(const void* Wl, int64_t K, int64_t N, void* out, hipStream_t st)
{
    const int64_t KS = ksteps_of(K);
    const int64_t P = (N + kPanelN - 1) / kPanelN;
    hipLaunchKernelGGL(sbi_unlayout_kernel, dim3((unsigned)(KS * P)), dim3(256), 0, st,
                       reinterpret_cast<const unsigned char*>(Wl), K, N, KS, reinterpret_cast<_Float16*>(out));
    return (int)hipGetLastError();
}

}  // namespace sbi
