// Helpers shared by the matrix-core attention kernels (gfx950): vector types, direct-to-LDS
// loads with manual vmcnt tracking, uniform-value hints, cross-half max.
#pragma once
#include <atomic>
#include <type_traits>

#include "common.h"

namespace s4c {
namespace mfma {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));   // also the carrier of 8 fp16 elements (16 bytes)
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) unsigned char lds_u8;
typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;

constexpr int kD = 128;
constexpr int kRowB = kD * 2;               // bytes per K/V row

enum TileMode { kPlain = 0, kTail = 1, kTree = 2 };

// One wave-wide direct-to-LDS load: lane i's 16 bytes land at LDS byte address lds_base + 16 i
// (lds_base wave-uniform, passed in M0).  Completion is tracked by vmcnt.  M0 is a register the
// compiler reserves: it loads M0 itself right before any instruction of its own that reads it and
// keeps no value in it across an asm statement, and it refuses M0 in a clobber list (warning
// "reserved register"), so the statement below writes M0 without declaring it.
__device__ __forceinline__ void dma16(const void* g, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_base) : "memory");
}
// Same with a wave-uniform 64-bit base and a 32-bit per-lane byte offset.
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_base) : "memory");
}

// Values that are wave-uniform by construction but that the compiler cannot prove uniform.
__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ const unsigned char* uniform(const unsigned char* p) {
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const unsigned char*)(((uint64_t)hi << 32) | lo);
}

// Wave-uniform read-only 32-bit load through the scalar data path.  The tile loops count their
// direct-to-LDS loads in vmcnt by hand, so a lookup inside them must not be a vector load.
__device__ __forceinline__ int32_t scalar_load_i32(const void* base, uint32_t byte_off) {
    int32_t v;
    asm volatile("s_load_dword %0, %1, %2\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(base), "s"(byte_off) : "memory");
    return v;
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// max(x[l], x[l ^ 32]) in every lane
__device__ __forceinline__ float max_across_halves(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Element-type switch of the matrix-core kernels (F16: IEEE binary16, else bf16).  Fragments are
// 16-byte vectors either way; only the multiply instruction and the two conversions differ.
template <bool F16>
__device__ __forceinline__ f32x16 mma32(const bf16x8& a, const bf16x8& b, const f32x16& c) {
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
template <bool F16>
__device__ __forceinline__ f32x4 mma16(const bf16x8& a, const bf16x8& b, const f32x4& c) {
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
// elements o .. o+7 of an accumulator block, rounded to nearest even
template <bool F16>
__device__ __forceinline__ bf16x8 round8(const f32x16& s, int o) {
    if constexpr (F16) {
        f16x8 r;
#pragma unroll
        for (int e = 0; e < 8; ++e) r[e] = (_Float16)s[o + e];
        return __builtin_bit_cast(bf16x8, r);
    } else {
        bf16x8 r;
#pragma unroll
        for (int e = 0; e < 8; ++e) r[e] = (__bf16)s[o + e];
        return r;
    }
}
template <bool F16>
__device__ __forceinline__ uint32_t round1(float x) {
    if constexpr (F16) return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)x);
    else return (uint32_t)f32_to_bf16(x);
}

}  // namespace mfma

// Raises a kernel's dynamic-LDS limit once per device (the attribute belongs to the device's copy
// of the function).  `done` is a bit per device ordinal; concurrent first calls both set the
// attribute, which is idempotent.
inline hipError_t ensure_dynamic_lds(const void* kernel, int bytes, std::atomic<uint64_t>& done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (dev < 64 && (done.load(std::memory_order_relaxed) & bit)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && dev < 64) done.fetch_or(bit, std::memory_order_relaxed);
    return e;
}
}  // namespace s4c
