// Device code shared by the translation units of the GPU path: element types, bf16
// conversions, the direct global->LDS transfer, MFMA and wait helpers.
#pragma once

#include <cstdio>
#include <cstdlib>
#include <utility>

#include "lpg_internal.h"

namespace lpg {


typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

struct F32 {
    typedef uint32_t raw;
    static constexpr int ES = 4, KV = 4, KF = 8, KB = 32;
};
struct BF16 {
    typedef uint16_t raw;
    static constexpr int ES = 2, KV = 8, KF = 16, KB = 64;
};

// fp32 -> bf16 bit pattern, round to nearest, ties to even; NaN stays NaN.
__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ float bf16_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
// two fp32 -> packed bf16 pair with the hardware converter (round to nearest even); used
// where results are judged by tolerance, the bit-pattern routine above where bytes are
__device__ __forceinline__ uint32_t bf16_pack2(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

template <typename S, typename D>
__device__ __forceinline__ typename D::raw convert_raw(typename S::raw x)
{
    if constexpr (S::ES == D::ES) {
        return x;
    } else if constexpr (S::ES == 4 && D::ES == 2) {
        return (typename D::raw)bf16_rne(__uint_as_float(x));
    } else {
        return (typename D::raw)((uint32_t)x << 16);
    }
}

__device__ __forceinline__ float silu_f(float g) { return g / (1.0f + __expf(-g)); }

// 16 bytes per lane, global -> LDS at lds_addr + lane*16 (lds_addr wave-uniform).  Written
// as inline asm so that the compiler does not serialise later LDS reads of the OTHER stage
// behind this transfer; completion is awaited explicitly (vmcnt) before the stage is read.
__device__ __forceinline__ void lds_dma16(const void *g, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_addr) : "memory", "m0");
}

template <typename IN>
__device__ __forceinline__ void mma_frag(f32x16 &acc, const uint4 &r, const uint4 &l)
{
    if constexpr (IN::ES == 4) {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(r.x), __uint_as_float(l.x), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(r.y), __uint_as_float(l.y), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(r.z), __uint_as_float(l.z), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(r.w), __uint_as_float(l.w), acc, 0, 0, 0);
    } else {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, r),
                                                      __builtin_bit_cast(bf16x8, l), acc, 0, 0, 0);
    }
}

// The same product in J = mma_depth<IN>() separately issued parts (part j of an fp32 fragment is
// its j-th k-pair; a bf16 fragment is one part).
template <typename IN>
__device__ __forceinline__ constexpr int mma_depth() { return IN::ES == 4 ? 4 : 1; }
template <typename IN>
__device__ __forceinline__ void mma_part(f32x16 &acc, const uint4 &r, const uint4 &l, int j)
{
    if constexpr (IN::ES == 4) {
        const uint32_t rj = j == 0 ? r.x : j == 1 ? r.y : j == 2 ? r.z : r.w;
        const uint32_t lj = j == 0 ? l.x : j == 1 ? l.y : j == 2 ? l.z : l.w;
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(rj), __uint_as_float(lj), acc, 0, 0, 0);
    } else {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, r), __builtin_bit_cast(bf16x8, l),
                                                      acc, 0, 0, 0);
    }
}

__device__ __forceinline__ float epi_apply(int epi, float v, float g)
{
    if (epi == LPG_EPI_SILU) return silu_f(v);
    if (epi == LPG_EPI_GATE_SILU) return silu_f(g) * v;
    return v;
}

template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop whose index is a
// constant in every iteration whatever the optimiser's unrolling limits are.  The epilogue
// walks the accumulator tiles with it: one dynamically indexed use would make the whole
// accumulator array live in memory, with a store behind every MFMA of the main loop.
template <int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

struct TileInfo {
    const char *Lp, *Rp;  // first block of the tile's L / R slab at K block 0
    int gl0, gr0;         // first 32-group of the tile in out's free / contraction dimension
    int nlg, nrg;         // groups of the tile that exist in L / R
    int b;                // batch index
};

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int MASK, int N>
__device__ __forceinline__ void sched_group()
{
    if constexpr (N > 0) __builtin_amdgcn_sched_group_barrier(MASK, N, 0);
}

}  // namespace lpg
