/*
 * sbi_calib.h - measurement helpers of the MI355X small-batch GeMM library.  Not part of the GeMM
 * path and not part of its public interface (include/sbi_gemm.h): bench.py uses them to find the
 * read bandwidth the weight stream's access pattern can reach at all, and to scale hardware byte
 * counters against a kernel of known traffic.
 */
#ifndef SBI_CALIB_H
#define SBI_CALIB_H

#include "../../include/sbi_gemm.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * sbi_calib_read streams `bytes` (a multiple of 4096, 256-byte aligned, device) from src
 * with the GeMM's own access shape - `blocks` thread blocks of `waves` wavefronts (4, 8 or
 * 16), each wavefront keeping `depth` (4 or 8) 4 KiB units in flight, 128-bit loads,
 * non-temporal if `nontemporal` - and writes nothing in practice (sink, device, >= 16 bytes
 * per block, only keeps the loads alive).  Its bandwidth is the ceiling this access pattern
 * can reach.  sbi_calib_copy copies `bytes` (a multiple of 16; both pointers 16-byte
 * aligned, device) with plain 128-bit loads and stores: a kernel of known HBM traffic
 * against which hardware byte counters are scaled.
 */
sbi_status sbi_calib_read(const void* src, size_t bytes, void* sink, size_t sink_bytes,
                          int32_t blocks, int32_t waves, int32_t depth, int32_t nontemporal, void* hip_stream);
sbi_status sbi_calib_copy(const void* src, void* dst, size_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SBI_CALIB_H */
