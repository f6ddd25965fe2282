// LDS access by byte offset, direct global->LDS transfers and small helpers shared by the GEMM kernels.
#pragma once
#include "svdq_dev.h"

namespace svdq {

template <int V> struct IC { static constexpr int value = V; };

typedef __attribute__((address_space(3))) uint8_t lds_byte;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 lds_read16(uint32_t off) {
    const u32x4 v = *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>((lds_byte*)(uintptr_t)off);
    return uint4{v.x, v.y, v.z, v.w};
}
// volatile variants: stay where the program puts them relative to barriers and scheduling fences
__device__ __forceinline__ uint4 lds_read16_pinned(uint32_t off) {
    const u32x4 v = *reinterpret_cast<const volatile __attribute__((address_space(3))) u32x4*>((lds_byte*)(uintptr_t)off);
    return uint4{v.x, v.y, v.z, v.w};
}
__device__ __forceinline__ uint32_t lds_read2_pinned(uint32_t off) {
    return *reinterpret_cast<const volatile __attribute__((address_space(3))) uint16_t*>((lds_byte*)(uintptr_t)off);
}
__device__ __forceinline__ uint2 lds_read8(uint32_t off) {
    const u32x2 v = *reinterpret_cast<const __attribute__((address_space(3))) u32x2*>((lds_byte*)(uintptr_t)off);
    return uint2{v.x, v.y};
}
__device__ __forceinline__ uint2 lds_read8_pinned(uint32_t off) {
    const u32x2 v = *reinterpret_cast<const volatile __attribute__((address_space(3))) u32x2*>((lds_byte*)(uintptr_t)off);
    return uint2{v.x, v.y};
}
__device__ __forceinline__ uint32_t lds_read4(uint32_t off) {
    return *reinterpret_cast<const __attribute__((address_space(3))) uint32_t*>((lds_byte*)(uintptr_t)off);
}
__device__ __forceinline__ void lds_write8(uint32_t off, uint2 v) {
    const u32x2 t = {v.x, v.y};
    *reinterpret_cast<__attribute__((address_space(3))) u32x2*>((lds_byte*)(uintptr_t)off) = t;
}

// One wave-wide direct global->LDS load: lane l moves 16 bytes from global address sbase + voff(l) to LDS
// byte offset lds_off + 16 l.  sbase and lds_off are wave-uniform (scalar registers), so a transfer costs
// no vector-ALU work.  Written as inline asm so that the compiler does not treat every later LDS read as
// dependent on it; the issuing code waits (vmcnt) and barriers before anyone reads the data.
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff, uint32_t lds_off) {
    const uint64_t a = (uint64_t)(uintptr_t)sbase;
    const uint64_t sa = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32)) << 32) |
                        (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    lds_off = __builtin_amdgcn_readfirstlane(lds_off);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sa), "s"(lds_off) : "memory");
}

// Same for one dword per lane: LDS byte offset lds_off + 4 l.
__device__ __forceinline__ void dma4(const void* sbase, uint32_t voff, uint32_t lds_off) {
    const uint64_t a = (uint64_t)(uintptr_t)sbase;
    const uint64_t sa = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32)) << 32) |
                        (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    lds_off = __builtin_amdgcn_readfirstlane(lds_off);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(voff), "s"(sa), "s"(lds_off) : "memory");
}

// hi | lo << 16 bf16 pieces of v (16 significant bits)
__device__ __forceinline__ uint32_t split_bf16(float v) {
    const uint32_t hi = f_bf16_rne(v);
    const uint32_t lo = f_bf16_rne(v - bits_f(hi << 16));
    return hi | (lo << 16);
}


__device__ __forceinline__ void lds_write8_pinned(uint32_t off, uint2 v) {
    const u32x2 t = {v.x, v.y};
    *reinterpret_cast<volatile __attribute__((address_space(3))) u32x2*>((lds_byte*)(uintptr_t)off) = t;
}

// Epilogue store of one wave's 64-channel x (32 MT)-token output tile as bf16.  In the accumulator layout of the
// 32x32 MFMAs (transposed tile D[n][m]) a lane owns one token and, per register quad, 4 consecutive channels:
// stored directly that is 8-byte pieces scattered over rows, which the memory system handles badly (measured:
// 1.5 TB/s).  Instead the wave transposes its tile through its own LDS region (row stride 144 B) and stores
// 16 bytes per lane, eight lanes per token row: every store instruction writes eight full 128-byte lines.
// `region` must not be in use by anyone else (the callers barrier before the epilogue); only this wave reads
// what it wrote, so no further barrier is needed.  acc(ni, mi, i) returns the finished binary32 value.
constexpr uint32_t YROW = 144;
template <int MT, class AccFn>
__device__ __forceinline__ void store_tile_bf16(AccFn acc, uint32_t region, int lane, uint16_t* __restrict__ yrow0,
                                                int64_t ldy, int64_t rows_left) {
    const int l32 = lane & 31, kh = lane >> 5;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int mi = 0; mi < MT; ++mi)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint2 o = {f2_bf16_rne(acc(ni, mi, 4 * q + 0), acc(ni, mi, 4 * q + 1)),
                                 f2_bf16_rne(acc(ni, mi, 4 * q + 2), acc(ni, mi, 4 * q + 3))};
                lds_write8_pinned(region + (mi * 32 + l32) * YROW + (ni * 32 + 8 * q + 4 * kh) * 2, o);
            }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int rsub = lane >> 3, c16 = lane & 7;
#pragma unroll
    for (int it = 0; it < 4 * MT; ++it) {
        const int row = it * 8 + rsub;
        const uint4 v = lds_read16_pinned(region + row * YROW + c16 * 16);
        if (row < rows_left) *reinterpret_cast<uint4*>(yrow0 + (int64_t)row * ldy + c16 * 8) = v;
    }
}

}  // namespace svdq
