// KV reuse (paper Sec. 3.2, last paragraph): append the accepted path's K/V rows to the cache.
//
// One workgroup per sequence: the path is read from device memory (no host round trip), all
// (path position, KV head) rows are copied with 16-byte accesses, and cache_len is bumped by
// the same workgroup after its copies were issued.  Moves at most max_path * Hkv * D * 2 rows of
// bytes per sequence, so the step is launch-latency bound.
#include "common.h"

namespace s4c {

namespace {

constexpr int kThreads = 1024;
constexpr int kBatch = 4;       // independent 16-byte copies in flight per thread (x2: K and V)

__global__ __launch_bounds__(kThreads) void kv_compact_kernel(CompactArgs a) {
    const int b = blockIdx.x, tid = threadIdx.x;
    const int L = a.accept_len[b];
    const int base = a.cache_len[b];
    const int32_t* pth = a.path + (size_t)b * a.max_path;

    int bad = (L < 0 || L >= a.max_path || base < 0 || (long long)base + L + 1 > a.S_cap);
    if (!bad)
        for (int k = tid; k <= L; k += kThreads) bad |= (pth[k] < 0 || pth[k] >= a.N);
    bad = __syncthreads_or(bad);        // also orders every thread's read of cache_len before the bump

    if (a.dst_index)
        for (int k = tid; k < a.max_path; k += kThreads)
            a.dst_index[(size_t)b * a.max_path + k] = (!bad && k <= L) ? base + k : -1;
    if (tid == 0 && a.status) a.status[b] = bad ? S4C_SEQ_BAD_LEN : 0;
    if (bad) return;

    const int vec_per_row = a.row_bytes / 16;
    const int total = (L + 1) * a.Hkv * vec_per_row;
    for (int e0 = tid; e0 < total; e0 += kThreads * kBatch) {
        uint4 kv[kBatch], vv[kBatch];
        size_t dst[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int e = e0 + u * kThreads;
            if (e < total) {
                const int v = e % vec_per_row;
                const int h = (e / vec_per_row) % a.Hkv;
                const int k = e / (vec_per_row * a.Hkv);
                const size_t src = (((size_t)b * a.N + pth[k]) * a.Hkv + h) * a.row_bytes + (size_t)v * 16;
                dst[u] = (((size_t)b * a.Hkv + h) * a.S_cap + (size_t)(base + k)) * a.row_bytes + (size_t)v * 16;
                kv[u] = *(const uint4*)((const char*)a.k_tree + src);
                vv[u] = *(const uint4*)((const char*)a.v_tree + src);
            }
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            if (e0 + u * kThreads < total) {
                *(uint4*)((char*)a.k_cache + dst[u]) = kv[u];
                *(uint4*)((char*)a.v_cache + dst[u]) = vv[u];
            }
        }
    }
    if (tid == 0) a.cache_len[b] = base + L + 1;
}

}  // namespace

hipError_t launch_compact(const CompactArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(kv_compact_kernel, dim3(a.B), dim3(kThreads), 0, st, a);
    return hipGetLastError();
}

}  // namespace s4c
