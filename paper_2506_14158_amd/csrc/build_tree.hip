// Candidate-tree construction from the drafter's logits (paper Sec. 3.2: the top-1 continuation
// is drafted first, the next most probable tokens are placed beside it as alternatives).
//
// Kernel 1 (topk_chunk): the HBM-bound part, one workgroup per (row, 8192-logit chunk) of the
// rows that have children; a workgroup walks a segment of consecutive chunks, the next one in
// flight while the current one is searched.  Every wavefront takes the nchild[row] largest of its
// own 2048 logits of the chunk (wavefront maximum, ties to the lowest token id; only the lane that
// owned a winner rescans its registers) and writes them out next to the maximum and the sum of
// exponentials of its part: no barrier, no workgroup-level step.
// Kernel 2 (topk_row): one wavefront per row merges the parts' candidates into the row's top
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
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int N = a.N;
    // workgroup -> (rank k among the sequence's rows that have children, sequence b, segment sg of consecutive
    // chunks), k slowest, so that the workgroups of rows without children are the last of the grid instead of
    // being interleaved
    const int sg = blockIdx.x % a.nseg;
    const int b = (blockIdx.x / a.nseg) % a.B;
    const int k = blockIdx.x / (a.nseg * a.B);
    __shared__ int32_t s_row, s_cnt0;
    const int my_nc = (tid < N) ? a.nchild[(size_t)b * N + tid] : 0;
    const int has = my_nc > 0 && my_nc <= a.kmax;       // (an invalid count is flagged by the layout kernel)
    const unsigned long long mask = __ballot(has);
    if (tid == 0) { s_cnt0 = __popcll(mask); s_row = -1; }
    __syncthreads();
    if (wave < 2 && has) {
        const int rank = __popcll(mask & ((1ull << lane) - 1ull)) + (wave == 1 ? s_cnt0 : 0);
        if (rank == k) s_row = tid;
    }
    __syncthreads();
    if (s_row < 0) return;
    const int row = b * N + s_row;
    const int nc = a.nchild[row];
    const int V = a.V;
    const T* base = (const T*)a.logits + (size_t)row * V;
    const int ch0 = sg * a.seg, ch1 = min(a.chunks, ch0 + a.seg);
    const bool vec_ok = ((((uintptr_t)base) & 15) == 0);

    // whole, aligned chunks are fetched one chunk ahead as raw 16-byte words
    uint4 raw[NV];
    auto whole = [&](int c) { return vec_ok && (c + 1) * kChunk <= V; };
    auto fetch = [&](int c) {
#pragma unroll
        for (int j = 0; j < NV; ++j) raw[j] = *(const uint4*)(base + c * kChunk + (j * kThreads + tid) * VN);
    };
    bool have = ch0 < ch1 && whole(ch0);
    if (have) fetch(ch0);
  for (int ch = ch0; ch < ch1; ++ch) {
    float x[kPerThread];
    int32_t idx0[NV];
    if (have) {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            idx0[j] = ch * kChunk + (j * kThreads + tid) * VN;
            if constexpr (VN == 4) {
                x[j * VN + 0] = __uint_as_float(raw[j].x);
                x[j * VN + 1] = __uint_as_float(raw[j].y);
                x[j * VN + 2] = __uint_as_float(raw[j].z);
                x[j * VN + 3] = __uint_as_float(raw[j].w);
            } else {
                const uint32_t w[4] = {raw[j].x, raw[j].y, raw[j].z, raw[j].w};
#pragma unroll
                for (int q = 0; q < 4; ++q) unpack2<T>(w[q], x[j * VN + 2 * q], x[j * VN + 2 * q + 1]);
            }
        }
    } else {
        load_chunk<T>(base, ch * kChunk, min(V, (ch + 1) * kChunk), tid, x, idx0);
    }
    have = ch + 1 < ch1 && whole(ch + 1);
    if (have) fetch(ch + 1);                           // in flight while this chunk is searched

    // Every wave takes the nc largest of its own 2048 logits (its quarter of the chunk), one at a time, and
    // writes them out itself: the scan has no barrier and no workgroup-level step at all.  The lanes
    // keep only the VALUE of their largest remaining logit; a round is a wavefront maximum of those, after
    // which the lanes that hold that value (nearly always one) look up the lowest token id that attains it
    // in their registers, the lowest of those wins (ties to the lowest token id), and its owner removes it
    // and recomputes its maximum.  The chunk's sum of exponentials is taken per wave against the wave's own
    // maximum.
    auto lane_max = [&]() {
        float m = x[0];
#pragma unroll
        for (int e = 1; e < kPerThread; e += 2) m = __builtin_fmaxf(__builtin_fmaxf(m, x[e]), x[(e + 1) & (kPerThread - 1)]);
        return m;
    };
    float m_t = lane_max();
    const size_t o = ((size_t)row * a.chunks + ch) * 4 + wave;      // this wave's quarter of the chunk
    for (int r = 0; r < nc; ++r) {                       // a row needs only as many candidates as it has children
        float wm = m_t;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) wm = fmaxf(wm, __shfl_xor(wm, off));
        if (r == 0) {
            float sum = 0.f;
            if (wm > -INFINITY) {
#pragma unroll
                for (int e = 0; e < kPerThread; ++e) sum += fast_exp2((x[e] - wm) * a.inv_temp_log2);   // padding: 0
            }
            sum = wave_sum(sum);
            if (lane == 0) { a.ws_max[o] = wm; a.ws_sum[o] = sum; }
        }
        int32_t mine = 0x7FFFFFFF;                       // lowest token id of this lane that attains the wave maximum
        if (m_t == wm && wm > -INFINITY) {
#pragma unroll
            for (int j = NV - 1; j >= 0; --j)
#pragma unroll
                for (int q = VN - 1; q >= 0; --q)
                    if (x[j * VN + q] == wm) mine = idx0[j] + q;
        }
        int32_t win = mine;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) win = min(win, __shfl_xor(win, off));
        if (lane == 0) { a.ws_topv[o * kK + r] = wm; a.ws_topi[o * kK + r] = (win == 0x7FFFFFFF) ? -1 : win; }   // -1: part exhausted
        if (r + 1 < nc && mine == win && win != 0x7FFFFFFF) {          // the owner removes the winner
#pragma unroll
            for (int j = 0; j < NV; ++j)
#pragma unroll
                for (int q = 0; q < VN; ++q)
                    if (idx0[j] + q == win) x[j * VN + q] = -INFINITY;
            m_t = lane_max();
        }
    }
  }
}

__global__ __launch_bounds__(64) void topk_row_kernel(BuildArgs a) {
    const int row = blockIdx.x, lane = threadIdx.x;
    const int nc = a.nchild[row];
    if (nc <= 0 || nc > a.kmax) return;
    const int parts = a.chunks * 4;                          // a wavefront's quarter of a chunk each
    const size_t o = (size_t)row * parts;
    // row maximum and sum of exponentials from the parts' statistics
    float m = -INFINITY;
    for (int c = lane; c < parts; c += 64) m = fmaxf(m, a.ws_max[o + c]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    float S = 0.f;
    for (int c = lane; c < parts; c += 64) {
        const float pm = a.ws_max[o + c];
        if (pm > -INFINITY) S += a.ws_sum[o + c] * fast_exp2((pm - m) * a.inv_temp_log2);        // (a part beyond V is all padding)
    }
    S = wave_sum(S);
    const float* cv = a.ws_topv + o * kK;
    const int32_t* ci = a.ws_topi + o * kK;
    auto emit = [&](int r, MaxIdx best) {
        if (lane == 0) {
            const bool found = best.i != 0x7FFFFFFF;
            a.row_tok[(size_t)row * kK + r] = found ? best.i : -1;
            a.row_p[(size_t)row * kK + r] = found ? fast_exp2((best.v - m) * a.inv_temp_log2) / S : 0.f;
        }
    };
    if (parts <= 64) {
        // Every part's candidates are a descending list of nc entries: lane p keeps part p's list in
        // registers (read once), offers its head in every round, and the lane that wins shifts its list.
        float v[kK];
        int32_t t[kK];
#pragma unroll
        for (int e = 0; e < kK; ++e) {
            const bool there = lane < parts && e < nc;
            v[e] = there ? cv[lane * kK + e] : -INFINITY;
            t[e] = there ? ci[lane * kK + e] : -1;
        }
        for (int r = 0; r < nc; ++r) {
            const MaxIdx head = (t[0] >= 0) ? MaxIdx{v[0], t[0]} : MaxIdx{-INFINITY, 0x7FFFFFFF};
            const MaxIdx best = wave_best(head);
            emit(r, best);
            if (head.i == best.i && best.i != 0x7FFFFFFF) {          // candidates are distinct tokens: one lane matches
#pragma unroll
                for (int e = 0; e + 1 < kK; ++e) { v[e] = v[e + 1]; t[e] = t[e + 1]; }
                v[kK - 1] = -INFINITY;
                t[kK - 1] = -1;
            }
        }
        return;
    }
    // more than 64 parts (rows beyond 131072 logits): nc rounds of "largest remaining candidate" over the lists in
    // memory; a lane owns candidates lane, lane+64, ...
    const int ncand = parts * kK;
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
        emit(r, best);
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
    const dim3 grid1((unsigned)((size_t)a.B * a.N * a.nseg));
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
