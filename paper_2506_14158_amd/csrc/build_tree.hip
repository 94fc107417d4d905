// Candidate-tree construction from the drafter's logits (paper Sec. 3.2: the top-1 continuation
// is drafted first, the next most probable tokens are placed beside it as alternatives).
//
// Kernel 1 (topk_chunk): the HBM-bound part, one workgroup per (row, 8192-logit chunk) of the
// rows that have children.  The chunk is read once into registers; the chunk's nchild[row] largest
// logits are then taken one at a time (block argmax, ties to the lowest token id; only the wave
// that owned the winner rescans its registers), next to the chunk's max and sum of exponentials.
// Kernel 2 (topk_row): one wavefront per row merges the chunks' candidates into the row's top
// nchild tokens and turns their logits into probabilities.
// Kernel 3 (layout): one workgroup per sequence numbers the nodes level by level from the child
// counts (prefix sum), checks that the counts describe a tree of exactly N nodes, and scatters
// parent / token / probability / level of every node.
#include "row_chunk.h"

namespace s4c {

namespace {

using namespace rowchunk;
constexpr int kK = 8;                 // most children per node

template <typename T>
__global__ __launch_bounds__(kThreads) void topk_chunk_kernel(BuildArgs a) {
    constexpr int VN = Vec16<T>::n;
    constexpr int NV = kPerThread / VN;
    const int row = blockIdx.x / a.chunks, ch = blockIdx.x % a.chunks, tid = threadIdx.x;
    const int nc = a.nchild[row];
    if (nc <= 0 || nc > a.kmax) return;                  // leaf (or invalid count: flagged by the layout kernel)
    const int V = a.V;
    const T* base = (const T*)a.logits + (size_t)row * V;
    const int c0 = ch * kChunk;
    const int cend = min(V, c0 + kChunk);

    float x[kPerThread];
    int32_t idx0[NV];
    load_chunk<T>(base, c0, cend, tid, x, idx0);
    MaxIdx best = thread_best<VN>(x, idx0);

    __shared__ float s_v[4];
    __shared__ int32_t s_i[4];
    __shared__ float s_s[4];
    const int wave = tid >> 6, lane = tid & 63;
    const size_t o = (size_t)row * a.chunks + ch;
    for (int r = 0; r < nc; ++r) {                       // a row needs only as many candidates as it has children
        const MaxIdx w = wave_best(best);
        if (lane == 0) { s_v[wave] = w.v; s_i[wave] = w.i; }
        __syncthreads();
        MaxIdx blk = {s_v[0], s_i[0]};
#pragma unroll
        for (int q = 1; q < 4; ++q) blk = better(blk, MaxIdx{s_v[q], s_i[q]});
        if (r == 0) {
            // chunk statistics relative to the chunk maximum (all logits still in place)
            float sum = 0.f;
#pragma unroll
            for (int e = 0; e < kPerThread; ++e) sum += fast_exp2((x[e] - blk.v) * a.inv_temp_log2);   // padding: 0
            sum = wave_sum(sum);
            if (lane == 0) s_s[wave] = sum;
            __syncthreads();
            if (tid == 0) {
                a.ws_max[o] = blk.v;
                a.ws_sum[o] = (s_s[0] + s_s[1]) + (s_s[2] + s_s[3]);
            }
        }
        if (tid == 0) {
            a.ws_topv[o * kK + r] = blk.v;
            a.ws_topi[o * kK + r] = (blk.v == -INFINITY) ? -1 : blk.i;     // chunk exhausted
        }
        // the owner removes the winner and rescans its 32 registers
        if (__any(best.i == blk.i && best.v == blk.v)) {
            if (best.i == blk.i && best.v == blk.v) {
#pragma unroll
                for (int j = 0; j < NV; ++j)
#pragma unroll
                    for (int k = 0; k < VN; ++k)
                        if (idx0[j] + k == blk.i) x[j * VN + k] = -INFINITY;
                best = thread_best<VN>(x, idx0);
            }
        }
        __syncthreads();                                  // s_v / s_i are rewritten by the next round
    }
}

__global__ __launch_bounds__(64) void topk_row_kernel(BuildArgs a) {
    const int row = blockIdx.x, lane = threadIdx.x;
    const int nc = a.nchild[row];
    if (nc <= 0 || nc > a.kmax) return;
    const size_t o = (size_t)row * a.chunks;
    // row maximum and sum of exponentials from the chunk statistics
    float m = -INFINITY;
    for (int c = lane; c < a.chunks; c += 64) m = fmaxf(m, a.ws_max[o + c]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    float S = 0.f;
    for (int c = lane; c < a.chunks; c += 64) S += a.ws_sum[o + c] * fast_exp2((a.ws_max[o + c] - m) * a.inv_temp_log2);
    S = wave_sum(S);
    // merge: nc rounds of "largest remaining candidate"; a lane owns candidates lane, lane+64, ...
    const int ncand = a.chunks * kK;
    const float* cv = a.ws_topv + o * kK;
    const int32_t* ci = a.ws_topi + o * kK;
    MaxIdx prev = {INFINITY, -1};                         // the winner of the previous round
    for (int r = 0; r < nc; ++r) {
        // candidates are distinct tokens, so "remaining" = strictly after the previous winner
        // in the order (value descending, token id ascending)
        MaxIdx best = {-INFINITY, 0x7FFFFFFF};
        for (int c = lane; c < ncand; c += 64) {
            const MaxIdx cand = {cv[c], ci[c]};
            if (c % kK >= nc || cand.i < 0) continue;       // slots beyond nc were not written
            const bool after = (cand.v < prev.v) || (cand.v == prev.v && cand.i > prev.i);
            if (after) best = better(best, cand);
        }
        best = wave_best(best);
        if (lane == 0) {
            const bool found = best.i != 0x7FFFFFFF;
            a.row_tok[(size_t)row * kK + r] = found ? best.i : -1;
            a.row_p[(size_t)row * kK + r] = found ? fast_exp2((best.v - m) * a.inv_temp_log2) / S : 0.f;
        }
        prev = best;
        if (best.i == 0x7FFFFFFF) prev = MaxIdx{-INFINITY, 0x7FFFFFFF};   // nothing left: later rounds find nothing
    }
}

__global__ __launch_bounds__(kMaxNodes) void tree_layout_kernel(BuildArgs a) {
    const int b = blockIdx.x, i = threadIdx.x, N = a.N;
    __shared__ int32_t s_scan[kMaxNodes];
    __shared__ int32_t s_par[kMaxNodes];
    const int nc = (i < N) ? a.nchild[(size_t)b * N + i] : 0;
    int bad = (i < N) && (nc < 0 || nc > a.kmax);
    s_scan[i] = bad ? 0 : nc;
    __syncthreads();
    // inclusive prefix sum of the child counts (Hillis-Steele over 128 entries)
    for (int off = 1; off < kMaxNodes; off <<= 1) {
        const int v = (i >= off) ? s_scan[i - off] : 0;
        __syncthreads();
        s_scan[i] += v;
        __syncthreads();
    }
    const int excl = s_scan[i] - ((i < N && !bad) ? nc : 0);     // children handed out before node i
    if (i >= 1 && i < N && excl < i) bad = 1;                     // node i would be a parent before it exists
    if (i == N - 1 && s_scan[i] != N - 1) bad = 1;                // the counts must describe exactly N nodes
    bad = __syncthreads_or(bad);

    int32_t* par = a.parent + (size_t)b * N;
    int32_t* tok = a.tokens + (size_t)b * N;
    float* pd = a.p_draft + (size_t)b * N;
    if (i < N) s_par[i] = -1;
    __syncthreads();
    if (!bad && i < N) {
        for (int r = 0; r < nc; ++r) s_par[1 + excl + r] = i;
    }
    __syncthreads();
    if (i < N) {
        int32_t t = -1;
        float p = 0.f;
        int lev = 0;
        if (i == 0) {
            t = a.root_token[b];
        } else if (!bad) {
            const int pi = s_par[i];
            const int rank = i - (1 + (s_scan[pi] - a.nchild[(size_t)b * N + pi]));
            t = a.row_tok[((size_t)b * N + pi) * kK + rank];
            p = a.row_p[((size_t)b * N + pi) * kK + rank];
            for (int j = i; j > 0; j = s_par[j]) ++lev;
        }
        par[i] = bad ? -1 : s_par[i];
        tok[i] = t;
        pd[i] = p;
        if (a.level) a.level[(size_t)b * N + i] = lev;
    }
    if (i == 0 && a.status) a.status[b] = bad ? S4C_SEQ_BAD_TREE : 0;
}

}  // namespace

int build_tree_max_children() { return kK; }
int build_tree_chunk_elems() { return kChunk; }

hipError_t launch_build_tree(const BuildArgs& a, hipStream_t st) {
    const dim3 grid1((unsigned)((size_t)a.B * a.N * a.chunks));
    if (a.dtype == S4C_F32) hipLaunchKernelGGL(topk_chunk_kernel<float>, grid1, dim3(kThreads), 0, st, a);
    else if (a.dtype == S4C_F16) hipLaunchKernelGGL(topk_chunk_kernel<f16_t>, grid1, dim3(kThreads), 0, st, a);
    else hipLaunchKernelGGL(topk_chunk_kernel<bf16_t>, grid1, dim3(kThreads), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(topk_row_kernel, dim3((unsigned)(a.B * a.N)), dim3(64), 0, st, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(tree_layout_kernel, dim3(a.B), dim3(kMaxNodes), 0, st, a);
    return hipGetLastError();
}

}  // namespace s4c
