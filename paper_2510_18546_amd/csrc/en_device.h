// Device-side helpers shared by the HIP translation units of libefficientnav.so
// (gfx950, MI355X, CDNA4, wave64): vector types, wave exchanges and reductions,
// the plan tables' address space and bucket search, and the global -> LDS loader.
//
// Softmax runs in the log2 domain everywhere: scores are scaled by
// log2(e)/sqrt(D) and exponentials are exp2.
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <type_traits>

#include "en_internal.h"

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

#define EN_NEG_INF (-__builtin_inff())

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// A query's rotary pair (k, k + D/2) turned by its position's angle and scaled for the softmax in
// the log2 domain. One definition for every kernel that prepares queries, with the products and
// sums kept as written (no fused multiply-add): the attention kernel and the gather launch then
// produce the same bits.
__device__ __forceinline__ void rope_scale_pair(float x1, float x2, float c, float s, float scale, float &y1, float &y2)
{
#pragma clang fp contract(off)
    y1 = (x1 * c - x2 * s) * scale;
    y2 = (x2 * c + x1 * s) * scale;
}

// Exchange a value with the lane 32 positions away.
__device__ __forceinline__ float xor32(float v)
{
    // v_permlane32_swap exchanges the two halves of the wave in the vector ALU (no LDS crossbar,
    // hence no wait on the LDS counter that the operand prefetches also use)
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    // lanes 0..31 hold (own, partner) in (r[0], r[1]); lanes 32..63 in (r[1], r[0]): pick the partner
    const unsigned lane = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    return __uint_as_float(lane < 32 ? r[1] : r[0]);
}

// ---------------------------------------------------------------------------
// Segment lookup: largest s with bnd[s] <= tok among buckets 0..S (bucket S is
// the new block). Empty buckets are skipped because of the "largest".
// ---------------------------------------------------------------------------
// The plan's tables are read-only for every kernel that takes them from device
// memory. Addressed through the constant address space, their wave-uniform
// reads become scalar loads; as plain global reads they would be vector loads
// whose wait (vmcnt) also waits for every tile load in flight.
typedef const int32_t __attribute__((address_space(4))) *en_table_ptr;
__device__ __forceinline__ en_table_ptr as_table(const int32_t *p)
{
    return (en_table_ptr)(uintptr_t)p;
}

// KV split sp of n_splits takes the 64-key tiles [split_first_tile(sp), split_first_tile(sp + 1))
// of an agent's ntiles. The boundaries are rounded up: when the tiles do not divide evenly it is
// the last splits that get one fewer, and the last split is the one with extra work (the causal
// edge; in a decode step, the step's own keys, written before they can be loaded). Tile t lies in
// split t * n_splits / ntiles. 32-bit arithmetic: n_splits <= 64 and ntiles < 2^25.
__device__ __forceinline__ unsigned split_first_tile(unsigned sp, unsigned ntiles, unsigned n_splits)
{
    return (sp * ntiles + n_splits - 1) / n_splits;
}

template <typename P>
__device__ __forceinline__ int find_bucket(P bnd, int S, int tok)
{
    int lo = 0, hi = S;             // invariant: bnd[lo] <= tok
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (bnd[mid] <= tok)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

// One LDS-DMA load: lane i fetches 16 bytes from sbase + voff and the wave's
// 1024 bytes land at LDS byte address lds_base + IMM + 16*i. Completion is
// tracked by vmcnt; the compiler does not see the LDS write, so every wait is
// explicit.
template <int IMM>
__device__ __forceinline__ void dma16_imm(const void *sbase, uint32_t voff, uint32_t lds_base)
{
    asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_base), "v"(voff), "s"(sbase), "n"(IMM)
                 : "memory", "scc");
}

// The same with a run-time LDS address.
__device__ __forceinline__ void dma16(const void *sbase, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(sbase)
                 : "memory");
}

// The same from a full address per lane (rows that lie anywhere in memory).
template <int IMM>
__device__ __forceinline__ void dma16_addr_imm(unsigned long long addr, uint32_t lds_base)
{
    asm volatile("s_add_u32 m0, %0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_base), "v"(addr), "n"(IMM)
                 : "memory", "scc");
}
__device__ __forceinline__ void dma16_addr(unsigned long long addr, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_addr), "v"(addr)
                 : "memory");
}

__device__ __forceinline__ void wait_all_memory()
{
    __builtin_amdgcn_s_waitcnt(0x0070);      // vmcnt(0) lgkmcnt(0)
}

// The loader writes LDS behind the compiler's back: after a wait or barrier
// that publishes loaded data, no LDS read may be moved up across this point.
__device__ __forceinline__ void lds_data_ready()
{
    asm volatile("" ::: "memory");
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), in order
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>{});
    }
}

__device__ __forceinline__ size_t readlane64(size_t v, int l)
{
    const unsigned lo = __builtin_amdgcn_readlane((int)(unsigned)v, l);
    const unsigned hi = __builtin_amdgcn_readlane((int)(unsigned)(v >> 32), l);
    return ((size_t)hi << 32) | lo;
}

__device__ __forceinline__ float pair_max(float v)
{
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Sum over the 32 lanes of each half of the wave, in every lane of the half: four steps inside the
// rows of 16 lanes in the vector ALU (data-parallel primitives), one exchange between the two rows.
__device__ __forceinline__ float half_sum(float v)
{
    auto dpp = [](float x, auto ctrl) {
        return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), decltype(ctrl)::value, 0xf, 0xf, false));
    };
    v += dpp(v, std::integral_constant<int, 0xB1>{});      // quad_perm [1, 0, 3, 2]
    v += dpp(v, std::integral_constant<int, 0x4E>{});      // quad_perm [2, 3, 0, 1]
    v += dpp(v, std::integral_constant<int, 0x141>{});     // row_half_mirror
    v += dpp(v, std::integral_constant<int, 0x140>{});     // row_mirror
    v += __shfl_xor(v, 16, 64);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        v += __shfl_xor(v, o, 64);
    return v;
}
