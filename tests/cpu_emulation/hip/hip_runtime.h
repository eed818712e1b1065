// Host stand-in for the HIP runtime: lets the kernel sources compile as plain C++ so that
// their addressing can run under AddressSanitizer on the CPU.  One OS thread per GPU thread.
#pragma once
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <algorithm>
#include <pthread.h>

#define __device__
#define __host__
#define __global__
#define __forceinline__ inline __attribute__((always_inline))
#define __launch_bounds__(...)
#define __shared__ static

struct dim3 { unsigned x, y, z; dim3(unsigned a = 1, unsigned b = 1, unsigned c = 1) : x(a), y(b), z(c) {} };
typedef void* hipStream_t;
typedef int hipError_t;
enum { hipSuccess = 0, hipErrorInvalidValue = 1 };
enum { hipFuncAttributeMaxDynamicSharedMemorySize = 8 };
enum { hipMemcpyDeviceToHost = 2 };
inline hipError_t hipGetLastError() { return hipSuccess; }
inline hipError_t hipFuncSetAttribute(const void*, int, int) { return hipSuccess; }
inline hipError_t hipMemcpyAsync(void* d, const void* s, size_t n, int, hipStream_t) { memcpy(d, s, n); return hipSuccess; }
inline hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
// a file-scope device array is an ordinary array here and its "device address" its own
#define __align__(n) __attribute__((aligned(n)))
#define HIP_SYMBOL(x) (x)
inline hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
template <class T> inline hipError_t hipGetSymbolAddress(void** p, T& symbol) { *p = (void*)&symbol; return hipSuccess; }
struct hipFuncAttributes { int numRegs; };
inline hipError_t hipFuncGetAttributes(hipFuncAttributes* a, const void*) { a->numRegs = 0; return hipSuccess; }
typedef int hipEvent_t;
inline hipError_t hipEventCreate(hipEvent_t* e) { *e = 0; return hipSuccess; }
inline hipError_t hipEventDestroy(hipEvent_t) { return hipSuccess; }
inline hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
inline hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
inline hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 1.0f; return hipSuccess; }

namespace emu {
struct Block {
    int nthreads;
    pthread_barrier_t all;
    pthread_barrier_t wave[16];
    pthread_barrier_t half[32];       // 32-lane halves of the waves, for shuffles of width 32
    unsigned char* lds;
    size_t lds_bytes;
    // exchange areas for wave-wide operations
    float shf[16][64];
    _Float16 ma[16][64][8], mb[16][64][8];
};
extern thread_local dim3 t_threadIdx, t_blockIdx, t_blockDim, t_gridDim;
extern thread_local Block* t_block;
void launch(unsigned grid, unsigned block, size_t lds, const std::function<void()>& body);
inline unsigned char* lds() { return t_block->lds; }
}
#define threadIdx emu::t_threadIdx
#define blockIdx emu::t_blockIdx
#define blockDim emu::t_blockDim
#define gridDim emu::t_gridDim

inline void __syncthreads() { pthread_barrier_wait(&emu::t_block->all); }

// width 64: all lanes of the wave take part; width 32: the two halves of a wave are independent
// (one of them may be elsewhere in the program), mask < 32
inline float __shfl_xor(float v, int mask, int width = 64)
{
    emu::Block* b = emu::t_block;
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    pthread_barrier_t* bar = (width == 32) ? &b->half[threadIdx.x >> 5] : &b->wave[w];
    b->shf[w][l] = v;
    pthread_barrier_wait(bar);
    const float r = b->shf[w][l ^ mask];
    pthread_barrier_wait(bar);
    return r;
}
inline int __shfl_xor(int v, int mask, int width = 64)
{
    return __builtin_bit_cast(int, __shfl_xor(__builtin_bit_cast(float, v), mask, width));
}

inline double __shfl_xor(double v, int mask, int width = 64)
{
    unsigned long long bits = __builtin_bit_cast(unsigned long long, v);
    const unsigned int lo = (unsigned int)__shfl_xor((int)(bits & 0xffffffffull), mask, width);
    const unsigned int hi = (unsigned int)__shfl_xor((int)(bits >> 32), mask, width);
    return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}
// binary64 -> binary32 rounded toward zero
inline float __double2float_rz(double d)
{
    float f = (float)d;
    if (f == f && !__builtin_isinf(f) && __builtin_fabs((double)f) > __builtin_fabs(d)) f = __builtin_nextafterf(f, 0.0f);
    return f;
}

typedef _Float16 emu_half8 __attribute__((ext_vector_type(8)));
typedef float emu_floatx4 __attribute__((ext_vector_type(4)));
// D[4*(l/16)+r][l%16] += sum_k A[row][k] * B[k][col];  lane l holds A[l%16][8*(l/16)..+8] and B[8*(l/16)..+8][l%16]
inline emu_floatx4 __builtin_amdgcn_mfma_f32_16x16x32_f16(emu_half8 a, emu_half8 bb, emu_floatx4 c, int, int, int)
{
    emu::Block* b = emu::t_block;
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    for (int e = 0; e < 8; ++e) { b->ma[w][l][e] = a[e]; b->mb[w][l][e] = bb[e]; }
    pthread_barrier_wait(&b->wave[w]);
    const int col = l & 15;
    for (int r = 0; r < 4; ++r) {
        const int row = 4 * (l >> 4) + r;
        float s = c[r];
        for (int kg = 0; kg < 4; ++kg)
            for (int e = 0; e < 8; ++e) s += (float)b->ma[w][kg * 16 + row][e] * (float)b->mb[w][kg * 16 + col][e];
        c[r] = s;
    }
    pthread_barrier_wait(&b->wave[w]);
    return c;
}
typedef int emu_i32x4 __attribute__((ext_vector_type(4)));
// D[4*(l/16)+r][l%16] += sum_k A[row][k] * B[k][col] over 64 int8 k; lane l holds the 16 codes
// k = 16*(l/16)..+15 of A's row l%16 and of B's column l%16 (the kernels rely only on A and B
// using the same lane -> k assignment)
inline emu_i32x4 __builtin_amdgcn_mfma_i32_16x16x64_i8(emu_i32x4 a, emu_i32x4 bb, emu_i32x4 c, int, int, int)
{
    emu::Block* b = emu::t_block;
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    memcpy(b->ma[w][l], &a, 16);
    memcpy(b->mb[w][l], &bb, 16);
    pthread_barrier_wait(&b->wave[w]);
    const int col = l & 15;
    for (int r = 0; r < 4; ++r) {
        const int row = 4 * (l >> 4) + r;
        int s = c[r];
        for (int kg = 0; kg < 4; ++kg) {
            const signed char* pa = reinterpret_cast<const signed char*>(b->ma[w][kg * 16 + row]);
            const signed char* pb = reinterpret_cast<const signed char*>(b->mb[w][kg * 16 + col]);
            for (int e = 0; e < 16; ++e) s += (int)pa[e] * (int)pb[e];
        }
        c[r] = s;
    }
    pthread_barrier_wait(&b->wave[w]);
    return c;
}
inline int __builtin_amdgcn_readfirstlane(int v) { return v; }
inline float __builtin_amdgcn_rcpf(float v) { return 1.0f / v; }
inline float __builtin_amdgcn_exp2f(float v) { return exp2f(v); }
#define __builtin_amdgcn_sched_barrier(x) ((void)0)
#define __builtin_amdgcn_fence(order, scope) __atomic_thread_fence(__ATOMIC_SEQ_CST)
#define __builtin_amdgcn_s_waitcnt(imm) ((void)0)
#define __HIP_MEMORY_SCOPE_AGENT 0
#define __hip_atomic_store(p, v, order, scope) __atomic_store_n(p, v, __ATOMIC_SEQ_CST)
#define __hip_atomic_load(p, order, scope) __atomic_load_n(p, __ATOMIC_SEQ_CST)
#define __hip_atomic_fetch_add(p, v, order, scope) __atomic_fetch_add(p, v, __ATOMIC_SEQ_CST)
inline unsigned long long wall_clock64() { return 0; }
using std::min;
#ifndef INFINITY
#define INFINITY __builtin_inff()
#endif
using std::max;

#define hipLaunchKernelGGL(kernel, grid, block, lds, stream, ...) \
    emu::launch((grid).x, (block).x, (lds), [=]() { kernel(__VA_ARGS__); })
