// Path acceptance (paper Sec. 3.2: per-node test, then the longest accepted path).
//
// Kernel 1 (row_stats): the HBM-bound part (all rows in greedy mode, whose bonus token may come
// from any row; in stochastic mode only the rows of nodes that have children).  Each workgroup reads a segment of consecutive
// 8192-logit chunks of one logits row exactly once with 16-byte loads (the next chunk in flight
// while the current one is reduced in registers), and reduces
//   (max value, lowest index attaining it)   -- argmax, ties to the lowest token id
//   sum exp2((x - segment max) * log2(e)/T)  -- stochastic mode only
// per thread first (no barrier inside the segment), then with wavefront shuffles and across the
// 4 waves through LDS.
// Kernel 2 (path): one workgroup per sequence combines the chunk statistics per row, applies
// the per-node test against the parent's row, ANDs along each node's ancestor chain and picks
// the deepest accepted node (lowest index among equals), writing the path root..node.
#include "row_chunk.h"

namespace s4c {

namespace {

using namespace rowchunk;

template <typename T>
__global__ __launch_bounds__(kThreads) void row_stats_kernel(AcceptArgs a) {
    constexpr int VN = Vec16<T>::n;
    constexpr int NV = kPerThread / VN;               // 16-byte loads per thread and chunk
    const int row = blockIdx.x / a.nseg, sg = blockIdx.x % a.nseg, tid = threadIdx.x;
    const int V = a.V;
    const T* base = (const T*)a.logits + (size_t)row * V;
    const int ch0 = sg * a.seg, ch1 = min(a.chunks, ch0 + a.seg);
    const bool vec_ok = ((((uintptr_t)base) & 15) == 0);
    const bool stochastic = a.mode == S4C_STOCHASTIC;
    if (stochastic) {
        // A leaf's row verifies no node, and the stochastic rule returns no bonus token: not read.
        const int b = row / a.N, node = row % a.N;
        const int has_child = (tid < a.N) && (a.parent[(size_t)b * a.N + tid] == node);
        if (!__syncthreads_or(has_child)) return;
    }

    // per-thread running state over the segment's chunks: argmax (lowest index among equals: the
    // scan ascends and '>' is strict), and a sum of exponentials relative to the thread's own
    // running maximum, rescaled when that grows
    MaxIdx best = {-INFINITY, 0x7FFFFFFF};
    float m_t = -INFINITY, s_t = 0.f;

    // whole, aligned chunks are fetched one chunk ahead as raw 16-byte words
    uint4 raw[NV];
    auto whole = [&](int ch) { return vec_ok && (ch + 1) * kChunk <= V; };
    auto fetch = [&](int ch) {
#pragma unroll
        for (int j = 0; j < NV; ++j) raw[j] = *(const uint4*)(base + ch * kChunk + (j * kThreads + tid) * VN);
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
                    for (int k = 0; k < 4; ++k) unpack2<T>(w[k], x[j * VN + 2 * k], x[j * VN + 2 * k + 1]);
                }
            }
        } else {
            load_chunk<T>(base, ch * kChunk, min(V, (ch + 1) * kChunk), tid, x, idx0);
        }
        have = ch + 1 < ch1 && whole(ch + 1);
        if (have) fetch(ch + 1);                       // in flight while this chunk is reduced

        const MaxIdx cb = thread_best<VN>(x, idx0);
        if (cb.v > best.v) best = cb;
        if (stochastic && cb.v > -INFINITY) {
            const float m_new = fmaxf(m_t, cb.v);
            float sum = 0.f;
#pragma unroll
            for (int e = 0; e < kPerThread; ++e) sum += fast_exp2((x[e] - m_new) * a.inv_temp_log2);   // padding: 0
            s_t = s_t * fast_exp2((m_t - m_new) * a.inv_temp_log2) + sum;                                // first chunk: 0 * 0
            m_t = m_new;
        }
    }

    // ---- combine the 256 threads
    __shared__ float s_v[4];
    __shared__ int32_t s_i[4];
    __shared__ float s_s[4];
    const int wave = tid >> 6, lane = tid & 63;
    const MaxIdx wb = wave_best(best);
    if (lane == 0) { s_v[wave] = wb.v; s_i[wave] = wb.i; }
    __syncthreads();
    MaxIdx blk = {s_v[0], s_i[0]};
#pragma unroll
    for (int w = 1; w < 4; ++w) blk = better(blk, MaxIdx{s_v[w], s_i[w]});
    float sum = 0.f;
    if (stochastic) {
        sum = (m_t > -INFINITY) ? s_t * fast_exp2((m_t - blk.v) * a.inv_temp_log2) : 0.f;
        sum = wave_sum(sum);
        if (lane == 0) s_s[wave] = sum;
        __syncthreads();
        sum = (s_s[0] + s_s[1]) + (s_s[2] + s_s[3]);
    }
    if (tid == 0) {
        const size_t o = (size_t)row * a.nseg + sg;
        a.ws_max[o] = blk.v;
        a.ws_arg[o] = blk.i;
        a.ws_sum[o] = sum;
    }
}

template <typename T>
__global__ __launch_bounds__(kMaxNodes) void path_kernel(AcceptArgs a) {
    const int b = blockIdx.x, i = threadIdx.x;
    const int N = a.N;
    __shared__ int32_t spar[kMaxNodes];
    __shared__ int32_t s_ok[kMaxNodes];
    __shared__ int32_t s_g[kMaxNodes];
    __shared__ int32_t s_best;
    __shared__ int32_t s_tok[kMaxNodes];

    // ---- everything node i needs that does not depend on another load is requested up front (the
    // kernel is a chain of dependent memory latencies, not of work)
    int bad = 0;
    int tok = -1, par_i = -1;
    float u_i = 0.f, pd_i = 0.f;
    if (i < N) {
        const int p = par_i = a.parent[(size_t)b * N + i];
        tok = a.tokens[(size_t)b * N + i];
        if (a.mode == S4C_STOCHASTIC && i > 0) {
            u_i = a.uniforms[(size_t)b * N + i];
            pd_i = a.p_draft[(size_t)b * N + i];
        }
        // tree validation: node 0 is the only root, parents precede children
        spar[i] = p;
        s_tok[i] = tok;
        bad = (i == 0) ? (p != -1) : (p < 0 || p >= i);
    }
    // the target logit of this node's token in its parent's row (needs only parent and token)
    float lx = 0.f;
    if (a.mode == S4C_STOCHASTIC && i > 0 && i < N && !bad && tok >= 0 && tok < a.V)
        lx = to_f32<T>(((const T*)a.logits)[((size_t)b * N + par_i) * a.V + tok]);
    // ---- combine the segment statistics of row i.  In stochastic mode only the rows of nodes with
    // children were scanned; a leaf's slots hold whatever the workspace held, and nothing below reads
    // a leaf's statistics (a node is tested against its PARENT's row; no bonus token in that mode).
    float m = -INFINITY, S = 0.f;
    int32_t g = 0x7FFFFFFF;
    if (i < N) {
        const size_t o = ((size_t)b * N + i) * a.nseg;
        for (int c = 0; c < a.nseg; ++c) {
            const float v = a.ws_max[o + c];
            if (v > m) { m = v; g = a.ws_arg[o + c]; }           // segments ascend: strict '>' keeps lowest index
        }
        if (a.mode == S4C_STOCHASTIC)
            for (int c = 0; c < a.nseg; ++c)
                S += a.ws_sum[o + c] * fast_exp2((a.ws_max[o + c] - m) * a.inv_temp_log2);
        s_g[i] = g;
    }
    if (i == 0) s_best = 0;
    bad = __syncthreads_or(bad);

    __shared__ float s_m[kMaxNodes], s_S[kMaxNodes];
    if (i < N) { s_m[i] = m; s_S[i] = S; }
    __syncthreads();

    int depth = 0;
    if (!bad && i < N) {
        // ---- local test of node i against its parent's row
        int ok = 1;
        if (i > 0) {
            const int p = spar[i];
            if (a.mode == S4C_GREEDY) {
                ok = (tok == s_g[p]);
            } else if (tok < 0 || tok >= a.V) {
                ok = 0;
            } else {
                const float pt = fast_exp2((lx - s_m[p]) * a.inv_temp_log2) / s_S[p];
                const float lhs = u_i * pd_i;
                ok = (lhs < pt);
            }
        }
        s_ok[i] = ok;
    }
    __syncthreads();
    int accepted = 0;
    if (!bad && i < N) {
        accepted = 1;
        for (int j = i; j > 0; j = spar[j]) { accepted &= s_ok[j]; ++depth; }
        if (depth >= a.max_path) bad = 1;
    }
    bad = __syncthreads_or(bad);

    int32_t* pth = a.path + (size_t)b * a.max_path;
    int32_t* atk = a.accepted_tokens + (size_t)b * a.max_path;
    for (int k = i; k < a.max_path; k += kMaxNodes) { pth[k] = (k == 0) ? 0 : -1; atk[k] = -1; }
    if (bad) {
        if (i == 0) {
            a.accept_len[b] = 0;
            a.bonus_token[b] = -1;
            if (a.status) a.status[b] = S4C_SEQ_BAD_TREE;
        }
        return;
    }
    // deepest accepted node, lowest index among equals: maximise depth*256 + (255 - i)
    if (accepted && i < N) atomicMax(&s_best, depth * 256 + (255 - i));
    __syncthreads();
    const int best = 255 - (s_best & 255);
    if (i == best) {
        const int L = depth;
        int node = i;
        for (int k = L; k >= 1; --k) {
            pth[k] = node;
            atk[k - 1] = s_tok[node];
            node = spar[node];
        }
        a.accept_len[b] = L;
        a.bonus_token[b] = (a.mode == S4C_GREEDY) ? s_g[i] : -1;
        if (a.status) a.status[b] = 0;
    }
}

}  // namespace

int accept_chunk_elems() { return kChunk; }

hipError_t launch_accept(const AcceptArgs& a, hipStream_t st) {
    dim3 grid((unsigned)(a.nseg * a.B * a.N)), block(kThreads);
    if (a.dtype == S4C_F32) hipLaunchKernelGGL(row_stats_kernel<float>, grid, block, 0, st, a);
    else if (a.dtype == S4C_F16) hipLaunchKernelGGL(row_stats_kernel<f16_t>, grid, block, 0, st, a);
    else hipLaunchKernelGGL(row_stats_kernel<bf16_t>, grid, block, 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (a.dtype == S4C_F32) hipLaunchKernelGGL(path_kernel<float>, dim3(a.B), dim3(kMaxNodes), 0, st, a);
    else if (a.dtype == S4C_F16) hipLaunchKernelGGL(path_kernel<f16_t>, dim3(a.B), dim3(kMaxNodes), 0, st, a);
    else hipLaunchKernelGGL(path_kernel<bf16_t>, dim3(a.B), dim3(kMaxNodes), 0, st, a);
    return hipGetLastError();
}

}  // namespace s4c
