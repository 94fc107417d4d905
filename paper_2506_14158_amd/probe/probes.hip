// Measurement probes of the benchmark (libs4c_probe.so; see s4c_probe.h): what a plain streaming
// read and a plain back-to-back matrix-core loop reach on the GPU at hand.  The matrix-core rate
// depends on the operand DATA: with random operands the chip lowers its clock under the switching
// power of the multipliers, so the probe offers both a constant and a standard-normal operand
// fill, and both instruction shapes.  Nothing in the verification path calls these.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "s4c_probe.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kProbeThreads = 512;
constexpr int kProbeBlocks = 256;

// every workgroup reads its own contiguous share with 16-byte loads, eight in flight per thread
__global__ __launch_bounds__(256) void probe_stream_read_kernel(const uint4* src, size_t nvec, float* sink) {
    const size_t per = (nvec + gridDim.x - 1) / gridDim.x;
    const size_t lo = (size_t)blockIdx.x * per, hi = (lo + per < nvec) ? lo + per : nvec;
    uint32_t acc = 0;
    size_t i = lo + threadIdx.x;
    for (; i + 7 * 256 < hi; i += 8 * 256) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[i + u * 256];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < hi; i += 256) { const uint4 v = src[i]; acc += v.x ^ v.y ^ v.z ^ v.w; }
    if (acc == 0x12345678u) *sink = 1.f;        // practically never: keeps the loads alive
}

__device__ __forceinline__ uint32_t mix(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// roughly standard normal: four uniforms, centred and scaled
__device__ __forceinline__ float approx_normal(uint32_t s) {
    float u = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) { s = mix(s + 0x9e3779b9u * (i + 1)); u += (s >> 8) * (1.0f / 16777216.0f); }
    return (u - 2.0f) * 1.7320508f;
}

__device__ __forceinline__ void fill_operands(int random_operands, bf16x8 (&a)[8], bf16x8 (&b)[8]) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float x = 0.0625f, y = 0.125f;
            if (random_operands) {
                x = approx_normal(blockIdx.x * 7919u + tid * 131u + t * 17u + e);
                y = approx_normal(blockIdx.x * 104729u + tid * 257u + t * 29u + e + 1000u);
            }
            a[t][e] = (__bf16)x;
            b[t][e] = (__bf16)y;
        }
}

// 32 v_mfma_f32_32x32x16_bf16 per iteration and wave on four independent accumulators
__global__ __launch_bounds__(kProbeThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void probe_mfma32_kernel(int random_operands, int iters, float* sink) {
    bf16x8 a[8], b[8];
    fill_operands(random_operands, a, b);
    f32x16 o[4];
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int j = 0; j < 16; ++j) o[d][j] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int d = 0; d < 4; ++d) o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i + d) & 7], b[i], o[d], 0, 0, 0);
    }
    float acc = 0.f;
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc += o[d][j];
    sink[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = acc;
}

// the same FLOP count from 64 v_mfma_f32_16x16x32_bf16 per iteration on eight accumulators
__global__ __launch_bounds__(kProbeThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void probe_mfma16_kernel(int random_operands, int iters, float* sink) {
    bf16x8 a[8], b[8];
    fill_operands(random_operands, a, b);
    f32x4 o[8];
#pragma unroll
    for (int d = 0; d < 8; ++d)
#pragma unroll
        for (int j = 0; j < 4; ++j) o[d][j] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int d = 0; d < 8; ++d) o[d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[(i + d) & 7], b[i], o[d], 0, 0, 0);
    }
    float acc = 0.f;
#pragma unroll
    for (int d = 0; d < 8; ++d)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc += o[d][j];
    sink[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = acc;
}

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

int s4c_probe_stream_read(const void* buffer, size_t bytes, float* sink, void* hip_stream) {
    if (!buffer || !sink) return -1;
    if (bytes < 16 || (((uintptr_t)buffer) & 15)) return -2;
    hipLaunchKernelGGL(probe_stream_read_kernel, dim3(4096), dim3(256), 0, (hipStream_t)hip_stream, (const uint4*)buffer,
                       bytes / 16, sink);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}

size_t s4c_probe_mfma_sink_bytes(void) { return (size_t)kProbeBlocks * kProbeThreads * sizeof(float); }

int s4c_probe_mfma_bf16(int32_t random_operands, int32_t shape, int32_t iters, float* sink, double* flops,
                        void* hip_stream) {
    if (!sink) return -1;
    if (iters <= 0 || (shape != 0 && shape != 1)) return -2;
    if (flops) *flops = (double)kProbeBlocks * (kProbeThreads / 64) * (double)iters * 32.0 * 32768.0;
    if (shape == 0)
        hipLaunchKernelGGL(probe_mfma32_kernel, dim3(kProbeBlocks), dim3(kProbeThreads), 0, (hipStream_t)hip_stream,
                           random_operands ? 1 : 0, iters, sink);
    else
        hipLaunchKernelGGL(probe_mfma16_kernel, dim3(kProbeBlocks), dim3(kProbeThreads), 0, (hipStream_t)hip_stream,
                           random_operands ? 1 : 0, iters, sink);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}

#pragma GCC visibility pop
}  // extern "C"
