// Shared by the kernels that scan logits rows in chunks of 8192 (acceptance statistics,
// candidate-tree construction): a workgroup of 256 threads holds one chunk in registers,
// 32 logits per thread, read once with 16-byte loads.
#pragma once
#include "common.h"

namespace s4c {
namespace rowchunk {

constexpr int kThreads = 256;
constexpr int kPerThread = 32;                       // logits per thread
constexpr int kChunk = kThreads * kPerThread;        // logits per workgroup

struct MaxIdx {
    float v;
    int32_t i;
};

__device__ __forceinline__ MaxIdx better(MaxIdx a, MaxIdx b) {
    // larger value wins; equal values: lower index wins (never depends on reduction order)
    const bool take_b = (b.v > a.v) || (b.v == a.v && b.i < a.i);
    return take_b ? b : a;
}

__device__ __forceinline__ MaxIdx wave_best(MaxIdx x) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        MaxIdx y;
        y.v = __shfl_xor(x.v, off);
        y.i = __shfl_xor(x.i, off);
        x = better(x, y);
    }
    return x;
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
    return x;
}

template <typename T> struct Vec16;   // 16-byte vector of T
template <> struct Vec16<float> { static constexpr int n = 4; };
template <> struct Vec16<bf16_t> { static constexpr int n = 8; };
template <> struct Vec16<f16_t> { static constexpr int n = 8; };

// Thread tid's 32 logits of the chunk [c0, cend) of the row at `base`, as floats: vector j of
// the thread holds the Vec16<T>::n consecutive tokens starting at idx0[j] (ascending in j and
// inside a vector).  Tokens at or beyond cend read as -inf.
template <typename T>
__device__ __forceinline__ void load_chunk(const T* base, int c0, int cend, int tid, float (&x)[kPerThread],
                                           int32_t (&idx0)[kPerThread / Vec16<T>::n]) {
    constexpr int VN = Vec16<T>::n;
    constexpr int NV = kPerThread / VN;
    const bool vec_ok = ((((uintptr_t)base) & 15) == 0);
    if (vec_ok) {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int e0 = c0 + (j * kThreads + tid) * VN;
            idx0[j] = e0;
            if (e0 + VN <= cend) {
                const uint4 raw = *(const uint4*)(base + e0);
                if constexpr (VN == 4) {
                    x[j * VN + 0] = __uint_as_float(raw.x);
                    x[j * VN + 1] = __uint_as_float(raw.y);
                    x[j * VN + 2] = __uint_as_float(raw.z);
                    x[j * VN + 3] = __uint_as_float(raw.w);
                } else {
                    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                    for (int k = 0; k < 4; ++k) unpack2<T>(w[k], x[j * VN + 2 * k], x[j * VN + 2 * k + 1]);
                }
            } else {
#pragma unroll
                for (int k = 0; k < VN; ++k) x[j * VN + k] = (e0 + k < cend) ? to_f32<T>(base[e0 + k]) : -INFINITY;
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int e0 = c0 + (j * kThreads + tid) * VN;
            idx0[j] = e0;
#pragma unroll
            for (int k = 0; k < VN; ++k) x[j * VN + k] = (e0 + k < cend) ? to_f32<T>(base[e0 + k]) : -INFINITY;
        }
    }
}

// this thread's largest logit (lowest token id among equals: the scan ascends, '>' is strict)
template <int VN>
__device__ __forceinline__ MaxIdx thread_best(const float (&x)[kPerThread], const int32_t (&idx0)[kPerThread / VN]) {
    MaxIdx best = {-INFINITY, 0x7FFFFFFF};
#pragma unroll
    for (int j = 0; j < kPerThread / VN; ++j)
#pragma unroll
        for (int k = 0; k < VN; ++k)
            if (x[j * VN + k] > best.v) { best.v = x[j * VN + k]; best.i = idx0[j] + k; }
    return best;
}

}  // namespace rowchunk
}  // namespace s4c
