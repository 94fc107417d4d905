// Path acceptance (paper Sec. 3.2: per-node test, then the longest accepted path) in ONE launch.
//
// Scan (the HBM-bound part).  A workgroup owns a segment of consecutive 8192-logit chunks of one
// logits row and reads it exactly once with 16-byte loads, the next chunk in flight while the
// current one is reduced in registers.  Per thread the hot loop keeps only a running maximum (and,
// in stochastic mode, a sum of exp2 relative to it); the raw words of the chunk that holds the
// thread's maximum are kept aside, and the position of the maximum is looked up in them once, at
// the end of the segment.  The 256 threads are then combined with an order-independent
// (value, lowest index) reduction.  Greedy mode scans every row (the bonus token may come from any
// row); stochastic mode scans only the rows of nodes that have children: workgroup k of a
// sequence takes the k-th such node, found from parent[] in LDS, so the workgroups with nothing
// to do are the last of the grid rather than interleaved with the working ones.
//
// Path step.  Every scanning workgroup publishes its segment statistics as three 8-byte records
// (call nonce in the upper half, the statistic in the lower) with device-coherent stores.  The last
// workgroup of a sequence in grid order is its collector: having finished its own segment (in
// stochastic mode it never has one), it loads everything else the path step needs and then polls
// the records of the sequence until every one carries this call's nonce, combines them per row,
// applies the per-node test against the parent's row, ANDs along each node's ancestor chain and
// writes the deepest accepted node's path (lowest index among equals).  No second launch, no
// read-modify-write atomics (they serialise per address and take microseconds across the chip's
// separate L2s), no cache flush: only the records bypass the non-coherent part of the L2.
// A record needs no initialisation: anything without this call's nonce is "not there yet".  The
// collector overwrites what it consumed with the complement of the nonce, so a captured graph can
// replay the call, nonce and all.  The collector's wait is bounded by wall-clock time; when it runs
// out (which needs a GPU that stops scheduling the sequence's other workgroups) the sequence is
// flagged S4C_SEQ_TIMEOUT and gets the empty result.  Workgroups are dispatched in grid order, so
// by the time a collector starts every other workgroup of its sequence has been given a compute unit.
#include "row_chunk.h"

namespace s4c {

namespace {

using namespace rowchunk;

typedef unsigned long long rec_t;

__device__ __forceinline__ void publish(rec_t* p, uint32_t nonce, uint32_t bits) {
    __hip_atomic_store(p, ((rec_t)nonce << 32) | bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Loads the records of up to four consecutive segments of a row in one burst (the loads are
// independent round trips of a microsecond or two each, so they must not be taken one after the
// other) and repeats until every one carries the nonce or the deadline (100 MHz wall clock) has
// passed; returns whether they all arrived.  bits[3 s + w] = payload of word w of segment s.
__device__ __forceinline__ bool await4(const rec_t* p, int nsegs, int words, uint32_t nonce, long long deadline, uint32_t (&bits)[12]) {
    for (;;) {
        rec_t w[12];
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int q = 0; q < 3; ++q)
                w[3 * s + q] = (s < nsegs && q < words) ? __hip_atomic_load(p + 3 * s + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                                        : ((rec_t)nonce << 32);
        bool all = true;
#pragma unroll
        for (int e = 0; e < 12; ++e) {
            all = all && ((uint32_t)(w[e] >> 32) == nonce);
            bits[e] = (uint32_t)w[e];
        }
        if (all) return true;
        if ((long long)wall_clock64() - deadline >= 0) return false;
        __builtin_amdgcn_s_sleep(8);
    }
}

// The path step for sequence b, run by all kThreads threads of one workgroup (thread i = node i).
template <typename T>
__device__ void path_step(const AcceptArgs& a, int b) {
    const long long deadline = (long long)wall_clock64() + a.wait_ticks;
    const int i = threadIdx.x;
    const int N = a.N;
    __shared__ int32_t spar[kMaxNodes];
    __shared__ int32_t s_ok[kMaxNodes];
    __shared__ int32_t s_g[kMaxNodes];
    __shared__ int32_t s_best;
    __shared__ int32_t s_tok[kMaxNodes];
    __shared__ int32_t s_kids[kMaxNodes];
    __shared__ float s_m[kMaxNodes], s_S[kMaxNodes];

    // ---- everything node i needs that does not depend on another load is requested up front (the
    // step is a chain of dependent memory latencies, not of work)
    int bad = 0;
    int tok = -1, par_i = -1;
    float u_i = 0.f, pd_i = 0.f;
    if (i < kMaxNodes) s_kids[i] = 0;
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
    __syncthreads();
    if (i > 0 && i < N && !bad) s_kids[par_i] = 1;
    if (i == 0) s_best = 0;
    bad = __syncthreads_or(bad);

    // ---- combine the segment statistics of row i.  In stochastic mode only the rows of nodes with
    // children were scanned, and only those are combined (nothing reads a leaf's statistics: a node
    // is tested against its PARENT's row, and that mode has no bonus token).
    float m = -INFINITY, S = 0.f;
    int32_t g = 0x7FFFFFFF;
    int late = 0;
    if (i < N && !bad && (a.mode == S4C_GREEDY || s_kids[i])) {
        rec_t* r = a.rec + ((size_t)b * N + i) * a.nseg * 3;
        const uint32_t spent = ~a.nonce;
        const int words = (a.mode == S4C_STOCHASTIC) ? 3 : 2;
        // pass 1: the row maximum and its token (segments ascend: strict '>' keeps the lowest index);
        // pass 2 (stochastic): the segments' sums of exponentials, rescaled to the row maximum
        for (int c0 = 0; c0 < a.nseg && !late; c0 += 4) {
            uint32_t bits[12];
            if (!await4(r + 3 * c0, min(4, a.nseg - c0), words, a.nonce, deadline, bits)) { late = 1; break; }
#pragma unroll
            for (int s = 0; s < 4; ++s)
                if (c0 + s < a.nseg) {
                    const float v = __uint_as_float(bits[3 * s]);
                    if (v > m) { m = v; g = (int32_t)bits[3 * s + 1]; }
                }
        }
        if (a.mode == S4C_STOCHASTIC)
            for (int c0 = 0; c0 < a.nseg && !late; c0 += 4) {
                uint32_t bits[12];
                if (!await4(r + 3 * c0, min(4, a.nseg - c0), words, a.nonce, deadline, bits)) { late = 1; break; }
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    if (c0 + s < a.nseg)
                        S += __uint_as_float(bits[3 * s + 2]) * fast_exp2((__uint_as_float(bits[3 * s]) - m) * a.inv_temp_log2);
            }
        // consumed: a replay of this very call (same nonce) must not mistake them for its own
        if (!late)
            for (int c = 0; c < 3 * a.nseg; ++c) publish(r + c, spent, 0u);
    }
    late = __syncthreads_or(late);
    if (late) {
        int32_t* pth = a.path + (size_t)b * a.max_path;
        int32_t* atk = a.accepted_tokens + (size_t)b * a.max_path;
        for (int k = i; k < a.max_path; k += kThreads) { pth[k] = (k == 0) ? 0 : -1; atk[k] = -1; }
        if (i == 0) {
            a.accept_len[b] = 0;
            a.bonus_token[b] = -1;
            if (a.status) a.status[b] = S4C_SEQ_TIMEOUT;
        }
        return;
    }
    if (i < N) { s_g[i] = g; s_m[i] = m; s_S[i] = S; }
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
    for (int k = i; k < a.max_path; k += kThreads) { pth[k] = (k == 0) ? 0 : -1; atk[k] = -1; }
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

template <typename T>
__global__ __launch_bounds__(kThreads) void accept_kernel(AcceptArgs a) {
    constexpr int VN = Vec16<T>::n;
    constexpr int NV = kPerThread / VN;               // 16-byte loads per thread and chunk
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // workgroup -> (rank k among the sequence's scanned rows, sequence b, segment sg); k slowest
    const int sg = blockIdx.x % a.nseg;
    const int b = (blockIdx.x / a.nseg) % a.B;
    const int k = blockIdx.x / (a.nseg * a.B);
    const int V = a.V, N = a.N;
    const bool stochastic = a.mode == S4C_STOCHASTIC;

    __shared__ int32_t s_row;
    __shared__ float s_v[4];
    __shared__ int32_t s_i[4];
    __shared__ float s_s[4];

    int row_in_seq = k;                               // greedy: every row is scanned
    if (stochastic) {
        // the k-th node (ascending) that has a child: waves 0 and 1 hold one node per lane
        __shared__ uint32_t s_has[kMaxNodes];
        __shared__ int32_t s_cnt0;
        if (tid < kMaxNodes) s_has[tid] = 0;
        if (tid == 0) s_row = -1;
        __syncthreads();
        if (tid >= 1 && tid < N) {
            const int p = a.parent[(size_t)b * N + tid];
            if (p >= 0 && p < N) s_has[p] = 1;       // a malformed tree is reported by the path step
        }
        __syncthreads();
        const int has = (tid < N) ? (int)s_has[tid] : 0;
        const unsigned long long mask = __ballot(has);
        if (tid == 0) s_cnt0 = __popcll(mask);
        __syncthreads();
        if (wave < 2 && has) {
            const int rank = __popcll(mask & ((1ull << lane) - 1ull)) + (wave == 1 ? s_cnt0 : 0);
            if (rank == k) s_row = tid;
        }
        __syncthreads();
        row_in_seq = s_row;                           // -1: this sequence has fewer than k+1 such nodes
    }

    if (row_in_seq >= 0) {
        const size_t row = (size_t)b * N + row_in_seq;
        const T* base = (const T*)a.logits + row * (size_t)V;
        const int ch0 = sg * a.seg, ch1 = min(a.chunks, ch0 + a.seg);
        const bool vec_ok = ((((uintptr_t)base) & 15) == 0);

        // per-thread running state over the segment: maximum, the 16-byte words and the token offsets of the
        // chunk that holds it, and a sum of exponentials relative to the maximum (rescaled when it grows)
        float m_t = -INFINITY, s_t = 0.f;
        uint4 wbest[NV];
        int32_t ibest[NV];
#pragma unroll
        for (int j = 0; j < NV; ++j) { wbest[j] = make_uint4(0, 0, 0, 0); ibest[j] = 0; }

        auto whole = [&](int ch) { return vec_ok && (ch + 1) * kChunk <= V; };
        auto fetch = [&](uint4 (&raw)[NV], int ch) {
#pragma unroll
            for (int j = 0; j < NV; ++j) raw[j] = *(const uint4*)(base + ch * kChunk + (j * kThreads + tid) * VN);
        };
        auto decode = [&](const uint4 (&raw)[NV], float (&x)[kPerThread]) {
#pragma unroll
            for (int j = 0; j < NV; ++j) {
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
        };
        // whole, aligned chunks are fetched one chunk ahead as raw 16-byte words (kept as they are when the
        // chunk raises the thread's maximum); a ragged or unaligned chunk is loaded element by element
        uint4 raw[NV];
        bool have = ch0 < ch1 && whole(ch0);
        if (have) fetch(raw, ch0);
        for (int ch = ch0; ch < ch1; ++ch) {
            float x[kPerThread];
            int32_t idx0[NV];
            if (have) {
                decode(raw, x);
#pragma unroll
                for (int j = 0; j < NV; ++j) idx0[j] = ch * kChunk + (j * kThreads + tid) * VN;
            } else {
                load_chunk<T>(base, ch * kChunk, min(V, (ch + 1) * kChunk), tid, x, idx0);
            }
            float m_c = x[0];
#pragma unroll
            for (int e = 1; e < kPerThread; e += 2) m_c = __builtin_fmaxf(__builtin_fmaxf(m_c, x[e]), x[(e + 1) & (kPerThread - 1)]);
            const float m_old = m_t;
            if (m_c > m_t) {                               // strict: an equal later chunk never replaces an earlier one
                m_t = m_c;
                if (have) {
#pragma unroll
                    for (int j = 0; j < NV; ++j) wbest[j] = raw[j];
                } else {
#pragma unroll
                    for (int j = 0; j < NV; ++j) {
                        if constexpr (VN == 4) {
                            wbest[j] = make_uint4(__float_as_uint(x[j * 4]), __float_as_uint(x[j * 4 + 1]), __float_as_uint(x[j * 4 + 2]),
                                                  __float_as_uint(x[j * 4 + 3]));
                        } else {
                            uint32_t w[4];
#pragma unroll
                            for (int q = 0; q < 4; ++q) {           // exact: every x is a stored 16-bit value (or -inf)
                                const T lo = from_f32<T>(x[j * VN + 2 * q]), hi = from_f32<T>(x[j * VN + 2 * q + 1]);
                                w[q] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
                            }
                            wbest[j] = make_uint4(w[0], w[1], w[2], w[3]);
                        }
                    }
                }
#pragma unroll
                for (int j = 0; j < NV; ++j) ibest[j] = idx0[j];
            }
            have = ch + 1 < ch1 && whole(ch + 1);
            if (have) fetch(raw, ch + 1);                  // in flight while this chunk's exponentials are summed
            if (stochastic && m_c > -INFINITY) {
                const float ref = m_t * a.inv_temp_log2;   // m_t is max(old maximum, this chunk's) by now
                float sum = 0.f;
#pragma unroll
                for (int e = 0; e < kPerThread; ++e) sum += fast_exp2(fmaf(x[e], a.inv_temp_log2, -ref));   // padding: 0
                s_t = s_t * fast_exp2((m_old - m_t) * a.inv_temp_log2) + sum;                              // first chunk: 0 * 0
            }
        }
        // the thread's argmax: lowest index among its elements equal to its maximum (scan descending,
        // so that the lowest match is written last)
        MaxIdx best = {m_t, 0x7FFFFFFF};
        if (m_t > -INFINITY) {                             // (a thread of a ragged last chunk may hold padding only)
            float xb[kPerThread];
            decode(wbest, xb);
#pragma unroll
            for (int j = NV - 1; j >= 0; --j)
#pragma unroll
                for (int q = VN - 1; q >= 0; --q)
                    if (xb[j * VN + q] == m_t) best.i = ibest[j] + q;
        }

        // ---- combine the 256 threads
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
            rec_t* r = a.rec + (row * a.nseg + sg) * 3;
            publish(r, a.nonce, __float_as_uint(blk.v));
            publish(r + 1, a.nonce, (uint32_t)blk.i);
            publish(r + 2, a.nonce, __float_as_uint(sum));
        }
    }
    // ---- the sequence's last workgroup in grid order collects and runs the path step
    if (k == N - 1 && sg == a.nseg - 1) path_step<T>(a, b);
}

}  // namespace

int accept_chunk_elems() { return kChunk; }

// Segment length: a workgroup streams up to 8 chunks (128 KB of 16-bit logits) of a row, fewer when
// that would leave less than about 1024 workgroups to spread over the chip.  A fixed function of the
// sizes, so the workspace query and the launch agree.
void accept_plan(int B, int N, int V, int* chunks, int* seg, int* nseg) {
    const long long ch = ((long long)V + kChunk - 1) / kChunk;
    const long long units = (long long)B * N * ch;
    long long sg = units / 1024;
    if (sg > 8) sg = 8;
    if (sg > ch) sg = ch;
    if (sg < 1) sg = 1;
    *chunks = (int)ch;
    *seg = (int)sg;
    *nseg = (int)((ch + sg - 1) / sg);
}

hipError_t launch_accept(const AcceptArgs& a, hipStream_t st) {
    static_assert(kThreads >= 2 * 64 && kThreads >= kMaxNodes, "the path step and the row lookup use one thread per node");
    dim3 grid((unsigned)((size_t)a.nseg * a.B * a.N)), block(kThreads);
    if (a.dtype == S4C_F32) hipLaunchKernelGGL(accept_kernel<float>, grid, block, 0, st, a);
    else if (a.dtype == S4C_F16) hipLaunchKernelGGL(accept_kernel<f16_t>, grid, block, 0, st, a);
    else hipLaunchKernelGGL(accept_kernel<bf16_t>, grid, block, 0, st, a);
    return hipGetLastError();
}

}  // namespace s4c
