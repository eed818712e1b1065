// Measurement helpers (gfx950): a pure streaming-read kernel with the same access shape as the
// GeMM's weight stream, and a plain copy kernel of known traffic.  The read kernel gives the
// HBM read bandwidth this access pattern can reach at all (the honest ceiling next to the
// 8 TB/s data-sheet figure); the copy kernel is the reference against which hardware
// counters (FETCH_SIZE / WRITE_SIZE) are scaled.
#include "sbi_calib.h"
#include "sbi_common.h"

namespace sbi {

// Block b reads the contiguous run [b*steps, (b+1)*steps) of 4 KiB units; its NW waves take
// the units round-robin and keep DEPTH units (4 x 128-bit loads per lane) in flight each.
template <int NW, int DEPTH, bool NT>
__global__ __launch_bounds__(NW * 64) void sbi_calib_read_kernel(const u32x4* __restrict__ src, int64_t units,
                                                                 int steps, u32x4* __restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t first = (int64_t)blockIdx.x * steps;
    const int cn = (int)min<int64_t>(steps, units - first);
    u32x4 acc = {0u, 0u, 0u, 0u};
    if (cn > 0) {
        const int rounds = (cn + NW * DEPTH - 1) / (NW * DEPTH);
        const u32x4* base = src + first * 256 + lane;
        u32x4 ring[DEPTH][4];
        auto load = [&](u32x4 (&slot)[4], int unit) {
            const u32x4* p = base + (int64_t)min(unit, cn - 1) * 256;
#pragma unroll
            for (int t = 0; t < 4; ++t) slot[t] = NT ? __builtin_nontemporal_load(p + t * 64) : p[t * 64];
        };
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) load(ring[d], d * NW + wave);
        int u = wave;
        for (int r = 0; r + 1 < rounds; ++r) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
#pragma unroll
                for (int t = 0; t < 4; ++t) acc ^= ring[d][t];
                load(ring[d], u + NW * DEPTH);
                u += NW;
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
#pragma unroll
            for (int t = 0; t < 4; ++t) acc ^= ring[d][t];
    }
    // one value per thread keeps the loads alive; written only if the data says so (never for
    // ordinary inputs), so the kernel's traffic is reads only
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) sink[blockIdx.x] = acc;
}

__global__ __launch_bounds__(256) void sbi_calib_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                             int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

template <int NW, int DEPTH>
static int launch_read(const void* src, int64_t units, int steps, void* sink, int blocks, int nt, hipStream_t st)
{
    if (nt)
        hipLaunchKernelGGL((sbi_calib_read_kernel<NW, DEPTH, true>), dim3(blocks), dim3(NW * 64), 0, st,
                           (const u32x4*)src, units, steps, (u32x4*)sink);
    else
        hipLaunchKernelGGL((sbi_calib_read_kernel<NW, DEPTH, false>), dim3(blocks), dim3(NW * 64), 0, st,
                           (const u32x4*)src, units, steps, (u32x4*)sink);
    return (int)hipGetLastError();
}

}  // namespace sbi

extern "C" {

sbi_status sbi_calib_read(const void* src, size_t bytes, void* sink, size_t sink_bytes,
                          int32_t blocks, int32_t waves, int32_t depth, int32_t nontemporal, void* hip_stream)
{
    using namespace sbi;
    if (!src || !sink) return SBI_ERR_NULL;
    if (bytes < 4096 || bytes % 4096 != 0 || blocks < 1) return SBI_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(src) & 255) || (reinterpret_cast<uintptr_t>(sink) & 15)) return SBI_ERR_ALIGN;
    if (sink_bytes < (size_t)blocks * 16) return SBI_ERR_WORKSPACE;
    const int64_t units = (int64_t)(bytes / 4096);
    const int steps = (int)((units + blocks - 1) / blocks);
    hipStream_t st = (hipStream_t)hip_stream;
    int rc = (int)hipErrorInvalidValue;
    if (waves == 4 && depth == 4) rc = launch_read<4, 4>(src, units, steps, sink, blocks, nontemporal, st);
    else if (waves == 4 && depth == 8) rc = launch_read<4, 8>(src, units, steps, sink, blocks, nontemporal, st);
    else if (waves == 8 && depth == 4) rc = launch_read<8, 4>(src, units, steps, sink, blocks, nontemporal, st);
    else if (waves == 8 && depth == 8) rc = launch_read<8, 8>(src, units, steps, sink, blocks, nontemporal, st);
    else if (waves == 16 && depth == 4) rc = launch_read<16, 4>(src, units, steps, sink, blocks, nontemporal, st);
    else return SBI_ERR_TUNING;
    return rc == 0 ? SBI_OK : SBI_ERR_HIP;
}

sbi_status sbi_calib_copy(const void* src, void* dst, size_t bytes, void* hip_stream)
{
    using namespace sbi;
    if (!src || !dst) return SBI_ERR_NULL;
    if (bytes < 16 || bytes % 16 != 0) return SBI_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(src) & 15) || (reinterpret_cast<uintptr_t>(dst) & 15)) return SBI_ERR_ALIGN;
    const int64_t n16 = (int64_t)(bytes / 16);
    const int64_t want = (n16 + 255) / 256;
    const int blocks = (int)(want < (int64_t)kNumCU * 8 ? want : (int64_t)kNumCU * 8);
    hipLaunchKernelGGL(sbi_calib_copy_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream,
                       (const u32x4*)src, (u32x4*)dst, n16);
    return hipGetLastError() == hipSuccess ? SBI_OK : SBI_ERR_HIP;
}

}  // extern "C"
