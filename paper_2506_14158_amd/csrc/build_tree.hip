// Candidate-tree construction from the drafter's logits (paper Sec. 3.2: the top-1 continuation
// is drafted first, the next most probable tokens are placed beside it as alternatives).
//
// Kernel 1 (topk_chunk): the HBM-bound part, over the rows that have children; a workgroup walks a
// segment of consecutive 8192-logit chunks of one row, the next chunk in flight while the current
// one is searched.  Every wavefront keeps the nchild[row] largest logits of its quarter of the
// segment as a running sorted list (a chunk is only searched where a vote finds something above the
// list's last entry; ties to the lowest token id) and writes the list out at the end, next to the
// maximum and the sum of exponentials of its part: no barrier, no workgroup-level step, no
// cross-lane step per chunk unless the list changes.
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
    float m_e = -INFINITY, s_e = 0.f;                  // this thread's running maximum and sum of exponentials
    float lv[kK];                                      // the wavefront's list (uniform across lanes)
    int32_t li[kK];
#pragma unroll
    for (int e = 0; e < kK; ++e) { lv[e] = (e >= kK - nc) ? -INFINITY : INFINITY; li[e] = -1; }
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

    // this thread's share of the sum of exponentials, relative to its own running maximum (rescaled when that
    // grows): no cross-lane step per chunk
    float m_c = x[0];
#pragma unroll
    for (int e = 1; e < kPerThread; e += 2) m_c = __builtin_fmaxf(__builtin_fmaxf(m_c, x[e]), x[(e + 1) & (kPerThread - 1)]);
    if (m_c > -INFINITY) {
        const float m_new = fmaxf(m_e, m_c);
        float sum = 0.f;
#pragma unroll
        for (int e = 0; e < kPerThread; ++e) sum += fast_exp2((x[e] - m_new) * a.inv_temp_log2);   // padding: 0
        s_e = s_e * fast_exp2((m_e - m_new) * a.inv_temp_log2) + sum;                              // first chunk: 0 * 0
        m_e = m_new;
    }

    // Selection.  The wavefront keeps the nc largest logits it has seen in the segment so far as a sorted list
    // (value descending, token id ascending), the same in every lane.  A chunk can only change the list where a
    // lane holds something larger than the list's last entry, which a vote tells without any cross-lane data
    // movement; after the segment's first chunk most chunks pass with few or no insertions.  An insertion is a
    // wavefront maximum of the lanes' largest remaining logits, a lookup of the lowest token id that attains it
    // (ties to the lowest id), a shift of the list, and the owner retiring the element.
    float m_t = m_c;
    for (int r = 0; r < nc; ++r) {                       // at most nc entries of one chunk can enter
        const float tau = lv[kK - 1];                    // the list's last entry of the nc kept (see the shift below)
        if (!__any(m_t > tau)) break;                    // (an equal later logit has a higher token id: it stays out)
        float wm = m_t;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) wm = fmaxf(wm, __shfl_xor(wm, off));
        int32_t mine = 0x7FFFFFFF;                       // lowest token id of this lane that attains the wave maximum
        if (m_t == wm) {
#pragma unroll
            for (int j = NV - 1; j >= 0; --j)
#pragma unroll
                for (int q = VN - 1; q >= 0; --q)
                    if (x[j * VN + q] == wm) mine = idx0[j] + q;
        }
        int32_t win = mine;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) win = min(win, __shfl_xor(win, off));
        // insert (wm, win): entries are kept in slots kK - nc .. kK - 1, so that the last kept entry sits in
        // slot kK - 1 whatever nc is; everything smaller than the newcomer moves one slot down and the last drops
        // out.  Tokens of later chunks have higher ids, so the newcomer goes behind entries of equal value.
#pragma unroll
        for (int e = kK - 1; e >= 1; --e) {
            const bool moves = lv[e - 1] < wm;           // slot e takes slot e-1's entry
            const bool lands = !moves && lv[e] < wm;     // slot e takes the newcomer
            if (moves) { lv[e] = lv[e - 1]; li[e] = li[e - 1]; }
            else if (lands) { lv[e] = wm; li[e] = win; }
        }
        if (lv[0] < wm) { lv[0] = wm; li[0] = win; }
        if (mine == win) {                               // the owner removes the winner
#pragma unroll
            for (int j = 0; j < NV; ++j)
#pragma unroll
                for (int q = 0; q < VN; ++q)
                    if (idx0[j] + q == win) x[j * VN + q] = -INFINITY;
            m_t = x[0];
#pragma unroll
            for (int e = 1; e < kPerThread; e += 2) m_t = __builtin_fmaxf(__builtin_fmaxf(m_t, x[e]), x[(e + 1) & (kPerThread - 1)]);
        }
    }
  }
    // ---- the wavefront's part of the segment: maximum, sum of exponentials against it, and its list
    float wm = m_e;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) wm = fmaxf(wm, __shfl_xor(wm, off));
    float sum = (m_e > -INFINITY) ? s_e * fast_exp2((m_e - wm) * a.inv_temp_log2) : 0.f;
    sum = wave_sum(sum);
    const size_t o = ((size_t)row * a.nseg + sg) * 4 + wave;
    if (lane == 0) { a.ws_max[o] = wm; a.ws_sum[o] = sum; }
    if (lane < nc) {
        // entry r of the list sits in slot kK - nc + r; a slot that was never filled holds -inf / -1 ("part exhausted")
        float v = -INFINITY;
        int32_t t = -1;
#pragma unroll
        for (int e = 0; e < kK; ++e)
            if (e == kK - nc + lane) { v = lv[e]; t = li[e]; }
        a.ws_topv[o * kK + lane] = v;
        a.ws_topi[o * kK + lane] = t;
    }
}

__global__ __launch_bounds__(64) void topk_row_kernel(BuildArgs a) {
    const int row = blockIdx.x, lane = threadIdx.x;
    const int parts = a.nseg * 4;                            // a wavefront's quarter of a segment of chunks each
    const size_t o = (size_t)row * parts;
    // the child count, this lane's part statistics and (few parts) its whole list are requested together: the
    // kernel is a chain of memory latencies, not of work
    const bool few = parts <= 64, mine = lane < parts;
    const int nc = a.nchild[row];
    const float pm0 = (few && mine) ? a.ws_max[o + lane] : -INFINITY;
    const float ps0 = (few && mine) ? a.ws_sum[o + lane] : 0.f;
    float v[kK];
    int32_t t[kK];
#pragma unroll
    for (int e = 0; e < kK; ++e) {
        v[e] = (few && mine) ? a.ws_topv[(o + lane) * kK + e] : -INFINITY;      // (slots beyond nc hold leftovers: masked below)
        t[e] = (few && mine) ? a.ws_topi[(o + lane) * kK + e] : -1;
    }
    if (nc <= 0 || nc > a.kmax) return;
    // row maximum and sum of exponentials from the parts' statistics
    float m = pm0;
    if (!few)
        for (int c = lane; c < parts; c += 64) m = fmaxf(m, a.ws_max[o + c]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    float S = 0.f;
    if (few) {
        if (pm0 > -INFINITY) S = ps0 * fast_exp2((pm0 - m) * a.inv_temp_log2);
    } else {
        for (int c = lane; c < parts; c += 64) {
            const float pm = a.ws_max[o + c];
            if (pm > -INFINITY) S += a.ws_sum[o + c] * fast_exp2((pm - m) * a.inv_temp_log2);    // (a part beyond V is all padding)
        }
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
    if (few) {
        // Every part's candidates are a descending list of nc entries: lane p keeps part p's list in
        // registers (read once), offers its head in every round, and the lane that wins shifts its list.
#pragma unroll
        for (int e = 0; e < kK; ++e)
            if (e >= nc) { v[e] = -INFINITY; t[e] = -1; }
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
