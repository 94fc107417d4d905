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
    const int32_t* pth = a.path + (size_t)b * a.max_path;
    // the three loads that everything else depends on go out together (path entries before the
    // accepted length is known; a real path has at most kMaxNodes nodes, longer ones are read in place)
    __shared__ int32_t s_path[kMaxNodes];
    const int L = a.accept_len[b];
    const int base = a.cache_len[b];
    if (tid < kMaxNodes) s_path[tid] = (tid < a.max_path) ? pth[tid] : -1;
    __syncthreads();

    auto node_at = [&](int k) { return k < kMaxNodes ? s_path[k] : pth[k]; };
    int bad = (L < 0 || L >= a.max_path || base < 0 || (long long)base + L + 1 > a.S_cap);
    if (!bad)
        for (int k = tid; k <= L; k += kThreads) {
            bad |= (node_at(k) < 0 || node_at(k) >= a.N);
            if (a.block_table) {                       // the page of every written row must be a page of the pool
                const int id = a.block_table[(size_t)b * a.max_blocks + ((base + k) >> a.page_shift)];
                bad |= (id < 0 || id >= a.num_pages);
            }
        }
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
                const size_t src = (((size_t)b * a.N + node_at(k)) * a.Hkv + h) * a.row_bytes + (size_t)v * 16;
                size_t drow = ((size_t)b * a.Hkv + h) * a.S_cap + (size_t)(base + k);
                if (a.block_table) {
                    const int j = base + k;
                    const size_t id = (size_t)a.block_table[(size_t)b * a.max_blocks + (j >> a.page_shift)];
                    drow = ((id * a.Hkv + h) << a.page_shift) + (size_t)(j & ((1 << a.page_shift) - 1));
                }
                dst[u] = drow * a.row_bytes + (size_t)v * 16;
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

// ---- all layers of a model (and the accepted nodes' feature rows) in one launch -------------
// grid (B, layers [+1]): workgroup (b, y) copies layer y's rows of sequence b; y == layers copies
// the feature rows.  No workgroup writes cache_len here -- all of a sequence's workgroups read it
// in no particular order -- a second one-thread-per-sequence kernel advances it afterwards.
__device__ __forceinline__ int commit_bad(const CommitArgs& a, int b, int tid, int nthreads) {
    const int L = a.accept_len[b];
    const int base = a.cache_len[b];
    const int32_t* pth = a.path + (size_t)b * a.max_path;
    int bad = (L < 0 || L >= a.max_path || base < 0 || (long long)base + L + 1 > a.S_cap);
    if (!bad)
        for (int k = tid; k <= L; k += nthreads) {
            bad |= (pth[k] < 0 || pth[k] >= a.N);
            if (a.block_table) {                       // the page of every written row must be a page of the pool
                const int id = a.block_table[(size_t)b * a.max_blocks + ((base + k) >> a.page_shift)];
                bad |= (id < 0 || id >= a.num_pages);
            }
        }
    return bad;
}

__global__ __launch_bounds__(kThreads) void commit_copy_kernel(CommitArgs a) {
    const int b = blockIdx.x, y = blockIdx.y, tid = threadIdx.x;
    const int bad = __syncthreads_or(commit_bad(a, b, tid, kThreads));
    if (bad) return;
    const int L = a.accept_len[b];
    const int base = a.cache_len[b];
    const int32_t* pth = a.path + (size_t)b * a.max_path;
    if (y == a.layers) {                                   // feature rows -> features_out[b][k]
        const int vpr = a.feature_bytes / 16;
        const int total = (L + 1) * vpr;
        for (int e = tid; e < total; e += kThreads) {
            const int v = e % vpr, k = e / vpr;
            const uint4 x = *(const uint4*)((const char*)a.features + ((size_t)b * a.N + pth[k]) * a.feature_bytes + (size_t)v * 16);
            *(uint4*)((char*)a.features_out + ((size_t)b * a.max_path + k) * a.feature_bytes + (size_t)v * 16) = x;
        }
        return;
    }
    const char* ktl = (const char*)a.k_tree + (size_t)y * a.tree_layer_bytes;
    const char* vtl = (const char*)a.v_tree + (size_t)y * a.tree_layer_bytes;
    char* kcl = (char*)a.k_cache + (size_t)y * a.cache_layer_bytes;
    char* vcl = (char*)a.v_cache + (size_t)y * a.cache_layer_bytes;
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
                size_t drow = ((size_t)b * a.Hkv + h) * a.S_cap + (size_t)(base + k);
                if (a.block_table) {
                    const int j = base + k;
                    const size_t id = (size_t)a.block_table[(size_t)b * a.max_blocks + (j >> a.page_shift)];
                    drow = ((id * a.Hkv + h) << a.page_shift) + (size_t)(j & ((1 << a.page_shift) - 1));
                }
                dst[u] = drow * a.row_bytes + (size_t)v * 16;
                kv[u] = *(const uint4*)(ktl + src);
                vv[u] = *(const uint4*)(vtl + src);
            }
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            if (e0 + u * kThreads < total) {
                *(uint4*)(kcl + dst[u]) = kv[u];
                *(uint4*)(vcl + dst[u]) = vv[u];
            }
        }
    }
}

// one thread per sequence: status, dst_index, and the single advance of cache_len
__global__ void commit_finish_kernel(CommitArgs a) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= a.B) return;
    const int bad = commit_bad(a, b, 0, 1);
    const int L = a.accept_len[b], base = a.cache_len[b];
    if (a.dst_index)
        for (int k = 0; k < a.max_path; ++k) a.dst_index[(size_t)b * a.max_path + k] = (!bad && k <= L) ? base + k : -1;
    if (a.status) a.status[b] = bad ? S4C_SEQ_BAD_LEN : 0;
    if (!bad) a.cache_len[b] = base + L + 1;
}

}  // namespace

hipError_t launch_commit(const CommitArgs& a, hipStream_t st) {
    const bool feats = a.features && a.features_out;
    hipLaunchKernelGGL(commit_copy_kernel, dim3(a.B, a.layers + (feats ? 1 : 0)), dim3(kThreads), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(commit_finish_kernel, dim3((a.B + 255) / 256), dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_compact(const CompactArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(kv_compact_kernel, dim3(a.B), dim3(kThreads), 0, st, a);
    return hipGetLastError();
}

}  // namespace s4c
