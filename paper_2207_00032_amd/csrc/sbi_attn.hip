// Single-token attention with a key/value cache (paper Sec. III-D region 2: "transposition plus
// attention" fused into one kernel; Sec. IV: in the token-generation phase the new computation
// depends on one new token and re-uses everything older from the KV cache).
//
// Like the small-batch GeMM it is a streaming kernel: per sequence and head the cached keys and
// values (2 * (pos+1) * d halfs) are read exactly once, with 128-bit loads, and everything else
// happens in registers.  One block per (sequence, head, range of cached positions):
//   * d/8 lanes share one cached position (8 halfs each); a block of NT threads holds NT/(d/8)
//     such lane groups, each walking its own positions with U of them in flight;
//   * a group keeps a running maximum, denominator and its 8-element slice of the weighted value
//     sum (online softmax, base-2 exponentials), so keys and values are consumed as they arrive;
//   * the groups of a block are merged through LDS, the position ranges of a (sequence, head)
//     through the workspace by the last-arriving block (same arrival-counter scheme as the
//     GeMM's split-K), in a fixed order: results do not depend on timing;
//   * the "transposition" - the new token's key and value, which arrive token-major inside the
//     QKV GeMM's output row, go to their head's cache rows - is done by the same kernel, and the
//     new token itself is attended to straight from that row.
#include "sbi_common.h"

namespace sbi {

struct AttnParams {
    const _Float16* qkv;      // [B][3][H][D]
    _Float16* Kc;             // [B][H][S][D]
    _Float16* Vc;
    _Float16* out;            // [B][H*D]
    float* partials;          // [B*H][nsplit][D+2]: unnormalised value sums, then (max, denominator)
    unsigned int* counters;   // [B*H]
    const int* pos_of;        // [B] positions of the new tokens, or NULL: `pos` for every sequence
    int B, H, S, pos, nsplit, per_split;   // pos: the common position, or the bound of pos_of's entries
    float scale_log2;         // scale * log2(e)
};

__device__ __forceinline__ void attn_store(float* dst, float v)
{
    __hip_atomic_store(reinterpret_cast<unsigned int*>(dst), __builtin_bit_cast(unsigned int, v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float attn_load(const float* src)
{
    return __builtin_bit_cast(float, __hip_atomic_load(reinterpret_cast<const unsigned int*>(src), __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT));
}

// D: head dimension; U: positions in flight per lane group; NT: threads per block; AHEAD: a second
// set of U positions is requested while the first is consumed
template <int D, int U, int NT, bool AHEAD>
__global__ __launch_bounds__(NT) void sbi_attn_decode_kernel(const AttnParams p)
{
    constexpr int LPP = D / 8;           // lanes per cached position
    constexpr int NG = NT / LPP;         // lane groups per block
    __shared__ float s_m[NG], s_l[NG];
    __shared__ float s_o[NG][D];
    __shared__ int s_flag;

    const int bh = (int)blockIdx.x / p.nsplit, split = (int)blockIdx.x - bh * p.nsplit;
    const int b = bh / p.H, h = bh - b * p.H;
    const int tid = threadIdx.x, grp = tid / LPP, li = tid - grp * LPP;
    // ragged batch: this sequence's own position, forced into 0 .. p.pos so that no entry can
    // address outside the cache; ranges past a shorter sequence's end come out empty
    const int pos = p.pos_of ? min(max(p.pos_of[b], 0), p.pos) : p.pos;

    const _Float16* qrow = p.qkv + (((int64_t)b * 3 + 0) * p.H + h) * D + li * 8;
    const u32x4 knew = *reinterpret_cast<const u32x4*>(qrow + (int64_t)p.H * D);
    const u32x4 vnew = *reinterpret_cast<const u32x4*>(qrow + (int64_t)2 * p.H * D);
    float qf[8];
    {
        const half8 qh = __builtin_bit_cast(half8, *reinterpret_cast<const u32x4*>(qrow));
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[e] = (float)qh[e] * p.scale_log2;
    }
    const u32x4* K = reinterpret_cast<const u32x4*>(p.Kc + (int64_t)bh * p.S * D) + li;
    const u32x4* V = reinterpret_cast<const u32x4*>(p.Vc + (int64_t)bh * p.S * D) + li;

    // the transposition: the new token's key and value into their head's cache rows
    if (split == 0 && tid < 2 * LPP) {
        _Float16* dst = (tid < LPP ? p.Kc : p.Vc) + ((int64_t)bh * p.S + pos) * D + (tid % LPP) * 8;
        const _Float16* src = p.qkv + (((int64_t)b * 3 + (tid < LPP ? 1 : 2)) * p.H + h) * D + (tid % LPP) * 8;
        *reinterpret_cast<u32x4*>(dst) = *reinterpret_cast<const u32x4*>(src);
    }

    const int n = pos + 1;                                     // positions to attend to; the last one is the new token
    const int j0 = split * p.per_split, j1 = min(n, j0 + p.per_split);
    const int last_cached = max(pos - 1, 0);                   // loads are clamped to rows that exist
    float m = -INFINITY, l = 0.f, o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.f;

    const int iters = j1 > j0 ? (j1 - j0 + NG * U - 1) / (NG * U) : 0;   // the same for every thread of the block
    // AHEAD: two register sets of U positions each; the loads of round it + 1 are issued before
    // round it is consumed.  That is for the ragged batch, whose long sequences' blocks end up
    // alone on the chip and then stream at the rate their own requests in flight allow (8 x 32
    // heads, 256 .. 2048 positions: 37.5 -> 34.5 us; up to 8192: 128 -> 113 us).  A batch of equal
    // lengths keeps every CU busy to the end; there the 36 extra registers only cost resident
    // blocks (8 x 32 heads at 2048 positions: 44.3 -> 46.4 us), so it runs the plain loop.
    // (The products and sums of both loops are written as explicit fused operations: left to the
    // compiler's contraction, the two variants rounded differently.)
    struct Rows { u32x4 k[U], v[U]; };
    auto fetch = [&](Rows& r, int it) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = min(j0 + (it * U + u) * NG + grp, last_cached);
            r.k[u] = __builtin_nontemporal_load(K + (int64_t)j * LPP);
            r.v[u] = __builtin_nontemporal_load(V + (int64_t)j * LPP);
        }
    };
    auto consume = [&](const Rows& r, int it) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + (it * U + u) * NG + grp;
            const bool is_new = (j == pos);
            const half8 kh = __builtin_bit_cast(half8, is_new ? knew : r.k[u]);
            const half8 vh = __builtin_bit_cast(half8, is_new ? vnew : r.v[u]);
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) s = fmaf(qf[e], (float)kh[e], s);
#pragma unroll
            for (int msk = LPP / 2; msk >= 1; msk >>= 1) s += __shfl_xor(s, msk, 64);   // stays inside the lane group
            if (j < j1) {
                const float m_new = fmaxf(m, s);
                const float alpha = exp2f(m - m_new);
                const float w = exp2f(s - m_new);
                l = fmaf(l, alpha, w);
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = fmaf(w, (float)vh[e], o[e] * alpha);
                m = m_new;
            }
        }
    };
    if constexpr (AHEAD) {
        Rows ra, rb;
        if (iters > 0) fetch(ra, 0);
        for (int it = 0; it < iters; it += 2) {
            if (it + 1 < iters) fetch(rb, it + 1);
            consume(ra, it);
            if (it + 1 < iters) {
                if (it + 2 < iters) fetch(ra, it + 2);
                consume(rb, it + 1);
            }
        }
    } else {
        for (int it = 0; it < iters; ++it) {
            u32x4 kk[U], vv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int j = min(j0 + (it * U + u) * NG + grp, last_cached);
                kk[u] = __builtin_nontemporal_load(K + (int64_t)j * LPP);
                vv[u] = __builtin_nontemporal_load(V + (int64_t)j * LPP);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int j = j0 + (it * U + u) * NG + grp;
                const bool is_new = (j == pos);
                const half8 kh = __builtin_bit_cast(half8, is_new ? knew : kk[u]);
                const half8 vh = __builtin_bit_cast(half8, is_new ? vnew : vv[u]);
                float s = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) s = fmaf(qf[e], (float)kh[e], s);
#pragma unroll
                for (int msk = LPP / 2; msk >= 1; msk >>= 1) s += __shfl_xor(s, msk, 64);   // stays inside the lane group
                if (j < j1) {
                    const float m_new = fmaxf(m, s);
                    const float alpha = exp2f(m - m_new);
                    const float w = exp2f(s - m_new);
                    l = fmaf(l, alpha, w);
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] = fmaf(w, (float)vh[e], o[e] * alpha);
                    m = m_new;
                }
            }
        }
    }

    // merge the lane groups of the block
    if (li == 0) { s_m[grp] = m; s_l[grp] = l; }
#pragma unroll
    for (int e = 0; e < 8; ++e) s_o[grp][li * 8 + e] = o[e];
    __syncthreads();
    float M = -INFINITY, Lsum = 0.f, O = 0.f;
    if (tid < D) {
        for (int g = 0; g < NG; ++g) M = fmaxf(M, s_m[g]);
        for (int g = 0; g < NG; ++g) {
            // groups that saw no position count nothing (also when the whole range was empty, M = -inf)
            const float f = s_m[g] == -INFINITY ? 0.f : exp2f(s_m[g] - M);
            Lsum += f * s_l[g];
            O += f * s_o[g][tid];
        }
    }
    if (p.nsplit == 1) {
        if (tid < D) p.out[(int64_t)b * p.H * D + h * D + tid] = (_Float16)(O / Lsum);
        return;
    }

    // merge the position ranges of this (sequence, head): the last-arriving block does it
    float* mine = p.partials + ((int64_t)bh * p.nsplit + split) * (D + 2);
    if (tid < D) attn_store(mine + tid, O);
    if (tid == 0) { attn_store(mine + D, M); attn_store(mine + D + 1, Lsum); }
    wait_stores_acknowledged();                // this wave's partial results have reached memory before the
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();                           // block is counted
    if (tid == 0) {
        const unsigned int old = __hip_atomic_fetch_add(p.counters + bh, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_flag = (old == (unsigned int)(p.nsplit - 1));
    }
    __syncthreads();
    if (!s_flag) return;
    // All loads of the merge are independent of each other: every thread first fetches, then combines
    // (one memory latency per batch of kMergeBatch loads instead of one per position range).
    constexpr int Q = NT / D;                                   // threads per output column
    float* s_f = &s_o[0][0];                                    // [nsplit] factors, then the denominator
    float* s_part = s_f + kAttnMaxSplits + 1;                   // [Q][D] partial column sums
    const float* base = p.partials + (int64_t)bh * p.nsplit * (D + 2);
    float mx = -INFINITY, lx = 0.f;
    if (tid < p.nsplit) {
        mx = attn_load(base + tid * (D + 2) + D);
        lx = attn_load(base + tid * (D + 2) + D + 1);
        s_f[tid] = mx;
    }
    __syncthreads();                                            // also: every thread is done with s_o
    float Mx = -INFINITY;
    for (int s = 0; s < p.nsplit; ++s) Mx = fmaxf(Mx, s_f[s]);
    __syncthreads();
    if (tid < p.nsplit) { s_f[tid] = exp2f(mx - Mx); s_part[tid] = lx; }
    __syncthreads();
    float Ls = 0.f;
    for (int s = 0; s < p.nsplit; ++s) Ls += s_f[s] * s_part[s];   // fixed order, the same in every thread
    __syncthreads();
    const int col = tid % D, q = tid / D;
    float Os = 0.f;
    constexpr int kMergeBatch = 8;
    for (int s0 = q; s0 < p.nsplit; s0 += Q * kMergeBatch) {
        float v[kMergeBatch];
#pragma unroll
        for (int u = 0; u < kMergeBatch; ++u) {
            const int sidx = min(s0 + u * Q, p.nsplit - 1);
            v[u] = attn_load(base + sidx * (D + 2) + col);
        }
#pragma unroll
        for (int u = 0; u < kMergeBatch; ++u)
            if (s0 + u * Q < p.nsplit) Os += s_f[s0 + u * Q] * v[u];
    }
    s_part[q * D + col] = Os;
    __syncthreads();
    if (tid < D) {
        float total = 0.f;
#pragma unroll
        for (int qq = 0; qq < Q; ++qq) total += s_part[qq * D + tid];
        p.out[(int64_t)b * p.H * D + h * D + tid] = (_Float16)(total / Ls);
    }
    if (tid == 0) __hip_atomic_store(p.counters + bh, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

int launch_attn_decode(const void* qkv, void* Kc, void* Vc, int64_t B, int H, int D, int64_t S, int64_t pos,
                       const int* pos_of, float scale, void* out, void* workspace, int nsplit, hipStream_t st)
{
    if (nsplit < 1 || nsplit > kAttnMaxSplits) return (int)hipErrorInvalidValue;
    AttnParams p;
    p.qkv = reinterpret_cast<const _Float16*>(qkv);
    p.Kc = reinterpret_cast<_Float16*>(Kc);
    p.Vc = reinterpret_cast<_Float16*>(Vc);
    p.out = reinterpret_cast<_Float16*>(out);
    p.counters = reinterpret_cast<unsigned int*>(workspace);
    p.partials = workspace ? reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(workspace) + kAttnCounterBytes) : nullptr;
    p.pos_of = pos_of;
    p.B = (int)B; p.H = H; p.S = (int)S; p.pos = (int)pos; p.nsplit = nsplit;
    p.per_split = (int)((pos + 1 + nsplit - 1) / nsplit);
    p.scale_log2 = scale * 1.44269504088896340736f;
    const dim3 grid((unsigned)(B * H * nsplit));
    // 512 threads per block (32 or 64 lane groups) except where there are many short ranges: there
    // the second half of a bigger block would mostly idle (B = 64, 32 heads, 136 positions: 28 us
    // with 256 threads, 31 us with 512; 8 x 32 heads at 2048 positions: 47.8 us against 44.9 us).
    const bool small_blocks = p.per_split <= 192 && (int64_t)B * H * nsplit > 512;
    if (D != 64 && D != 128) return (int)hipErrorInvalidValue;
    const int variant = (D == 128 ? 4 : 0) + (small_blocks ? 2 : 0) + (pos_of ? 1 : 0);
    switch (variant) {
        case 0: hipLaunchKernelGGL((sbi_attn_decode_kernel<64, 4, 512, false>), grid, dim3(512), 0, st, p); break;
        case 1: hipLaunchKernelGGL((sbi_attn_decode_kernel<64, 4, 512, true>), grid, dim3(512), 0, st, p); break;
        case 2: hipLaunchKernelGGL((sbi_attn_decode_kernel<64, 4, 256, false>), grid, dim3(256), 0, st, p); break;
        case 3: hipLaunchKernelGGL((sbi_attn_decode_kernel<64, 4, 256, true>), grid, dim3(256), 0, st, p); break;
        case 4: hipLaunchKernelGGL((sbi_attn_decode_kernel<128, 4, 512, false>), grid, dim3(512), 0, st, p); break;
        case 5: hipLaunchKernelGGL((sbi_attn_decode_kernel<128, 4, 512, true>), grid, dim3(512), 0, st, p); break;
        case 6: hipLaunchKernelGGL((sbi_attn_decode_kernel<128, 4, 256, false>), grid, dim3(256), 0, st, p); break;
        case 7: hipLaunchKernelGGL((sbi_attn_decode_kernel<128, 4, 256, true>), grid, dim3(256), 0, st, p); break;
    }
    return (int)hipGetLastError();
}

}  // namespace sbi
