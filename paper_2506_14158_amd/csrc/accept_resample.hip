// Sibling-sequential acceptance with the correction token (paper Sec. 2, speculative-sampling
// paragraph: accept with probability min(1, p/q), redraw a rejected token from
// norm(max(0, p - q)); Sec. 3.2, second equation: the correction at a fork of the tree).
//
// One 1024-thread workgroup walks one sequence's tree from the root.  The walk is a chain of
// data-dependent decisions, each needing a reduction over the vocabulary, so the parallelism is
// inside a row, not across nodes.  Everything is kept unnormalised so no row is ever rewritten:
//   a_0[v] = exp((l[v] - max l) / T)              S_0 = sum_v a_0[v]        (target row)
//   a_{j+1}[v] = max(0, a_j[v] - S_j q[v])        S_{j+1} = sum_v a_{j+1}[v] (after j+1 rejections)
// so that a_j / S_j is the j-times-corrected distribution.  A child with token x passes iff
// u q[x] < a_j[x] / S_j.  a_j[v] is recomputed from l[v], q[v] and the j scalars S_0..S_{j-1}
// whenever it is needed.  The correction token is the inverse CDF of a_j in token-id order.
// The arithmetic is fp64: the decisions compare sums of 10^5 terms against a uniform number,
// and the work is a few rows per sequence, so accuracy is worth more than VALU rate here.
//
// Vocabulary traversal (all passes): wave w of 16 owns the contiguous blocks
// [w*ipw, (w+1)*ipw) of 512 tokens; in a block lane l owns the 8 tokens 8l..8l+7 (one 16-byte
// load of bf16 logits, two of fp32).
#include "common.h"

namespace s4c {

namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kBlock = 512;            // tokens per (wave, iteration)
constexpr int kMaxBlocks = 4096;       // => V <= 2^21

__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
    return x;
}

__device__ __forceinline__ double wave_incl_scan(double x, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const double y = __shfl_up(x, off);
        if (lane >= off) x += y;
    }
    return x;
}

struct Row {
    const void* lg;       // logits row
    const float* q;       // draft row
    int V;
    bool vec;             // 16-byte loads allowed for both rows
};

// the 8 logits (as float) of tokens base..base+7; tokens >= V read as -inf
template <typename T>
__device__ __forceinline__ void load_logits8(const Row& r, int base, float (&x)[8]) {
    const T* p = (const T*)r.lg;
    if (r.vec && base + 8 <= r.V) {
        if constexpr (sizeof(T) == 2) {
            const uint4 raw = *(const uint4*)(p + base);
            const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                x[2 * k] = __uint_as_float(w[k] << 16);
                x[2 * k + 1] = __uint_as_float(w[k] & 0xFFFF0000u);
            }
        } else {
            const float4 a = *(const float4*)(p + base), b = *(const float4*)(p + base + 4);
            x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
        }
    } else {
#pragma unroll
        for (int k = 0; k < 8; ++k) x[k] = (base + k < r.V) ? to_f32<T>(p[base + k]) : -INFINITY;
    }
}

__device__ __forceinline__ void load_draft8(const Row& r, int base, float (&qv)[8]) {
    if (r.vec && base + 8 <= r.V) {
        const float4 a = *(const float4*)(r.q + base), b = *(const float4*)(r.q + base + 4);
        qv[0] = a.x; qv[1] = a.y; qv[2] = a.z; qv[3] = a.w; qv[4] = b.x; qv[5] = b.y; qv[6] = b.z; qv[7] = b.w;
    } else {
#pragma unroll
        for (int k = 0; k < 8; ++k) qv[k] = (base + k < r.V) ? r.q[base + k] : 0.f;
    }
}

// a_j of one token: the target weight corrected by j rejections
__device__ __forceinline__ double corrected(float l, float qv, float m, double invT, const double* S, int j) {
    double a = exp(((double)l - (double)m) * invT);  // exp(-inf) = 0 for padding
    for (int i = 0; i < j; ++i) a = fmax(0.0, a - S[i] * (double)qv);
    return a;
}

// the 8 weights a_j of a lane's tokens in one block
template <typename T>
__device__ __forceinline__ void weights8(const Row& r, int base, float m, double invT, const double* S, int j,
                                         double (&w)[8]) {
    float x[8], qv[8];
    load_logits8<T>(r, base, x);
    if (j > 0) load_draft8(r, base, qv);
#pragma unroll
    for (int k = 0; k < 8; ++k) w[k] = corrected(x[k], j > 0 ? qv[k] : 0.f, m, invT, S, j);
}

template <typename T>
__global__ __launch_bounds__(kThreads) void accept_resample_kernel(ResampleArgs a) {
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int N = a.N, V = a.V;
    __shared__ int32_t spar[kMaxNodes], stok[kMaxNodes];
    __shared__ double sS[kMaxNodes + 1];          // S_0 .. S_j of the current node
    __shared__ double s_red[kWaves];
    __shared__ float s_redf[kWaves];
    __shared__ double s_blk[kMaxBlocks];          // per-block sums of the sampling pass
    __shared__ int32_t s_pick;

    // ---- tree validation: node 0 is the only root, parents precede children, depth < max_path
    int bad = 0;
    if (tid < N) {
        const int p = a.parent[(size_t)b * N + tid];
        spar[tid] = p;
        stok[tid] = a.tokens[(size_t)b * N + tid];
        bad = (tid == 0) ? (p != -1) : (p < 0 || p >= tid);
    }
    bad = __syncthreads_or(bad);
    if (!bad && tid < N) {
        int depth = 0;
        for (int i = tid; i > 0; i = spar[i]) ++depth;
        bad = depth >= a.max_path;
    }
    bad = __syncthreads_or(bad);

    int32_t* pth = a.path + (size_t)b * a.max_path;
    int32_t* atk = a.accepted_tokens + (size_t)b * a.max_path;
    for (int k = tid; k < a.max_path; k += kThreads) { pth[k] = (k == 0) ? 0 : -1; atk[k] = -1; }
    if (bad) {
        if (tid == 0) {
            a.accept_len[b] = 0;
            a.bonus_token[b] = -1;
            if (a.status) a.status[b] = S4C_SEQ_BAD_TREE;
        }
        return;
    }

    const int nblocks = (V + kBlock - 1) / kBlock;
    const int ipw = (nblocks + kWaves - 1) / kWaves;      // blocks per wave
    const int blk0 = wave * ipw;
    const int blk1 = min(nblocks, blk0 + ipw);
    const double invT = 1.0 / a.temperature;

    Row row;
    row.V = V;
    int cur = 0, L = 0, j = 0;
    float m = 0.f;
    for (;;) {
        row.lg = (const T*)a.logits + ((size_t)b * N + cur) * V;
        row.q = a.draft + ((size_t)b * N + cur) * V;
        row.vec = (((uintptr_t)row.lg | (uintptr_t)row.q) & 15) == 0;

        // ---- row maximum (exact) and S_0
        float mx = -INFINITY;
        for (int blk = blk0; blk < blk1; ++blk) {
            float x[8];
            load_logits8<T>(row, blk * kBlock + lane * 8, x);
#pragma unroll
            for (int k = 0; k < 8; ++k) mx = fmaxf(mx, x[k]);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
        if (lane == 0) s_redf[wave] = mx;
        __syncthreads();
        m = s_redf[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) m = fmaxf(m, s_redf[w]);

        double s = 0.0;
        for (int blk = blk0; blk < blk1; ++blk) {
            double w8[8];
            weights8<T>(row, blk * kBlock + lane * 8, m, invT, sS, 0, w8);
            s += ((w8[0] + w8[1]) + (w8[2] + w8[3])) + ((w8[4] + w8[5]) + (w8[6] + w8[7]));
        }
        s = wave_sum(s);
        if (lane == 0) s_red[wave] = s;
        __syncthreads();
        if (tid == 0) {
            double t = 0.0;
            for (int w = 0; w < kWaves; ++w) t += s_red[w];
            sS[0] = t;
        }
        __syncthreads();
        j = 0;

        // ---- children of cur in increasing node index (every thread takes the same branches)
        int next = -1;
        for (int c = cur + 1; c < N; ++c) {
            if (spar[c] != cur) continue;
            const int x = stok[c];
            if (x < 0 || x >= V) continue;                          // not a token id: rejected, nothing carried
            const float qx = row.q[x];
            const double ax = corrected(to_f32<T>(((const T*)row.lg)[x]), qx, m, invT, sS, j);
            const double lhs = (double)a.uniforms[(size_t)b * N + c] * (double)qx;
            if (lhs < ax / sS[j]) { next = c; break; }
            // rejected: mass of max(0, a_j - S_j q)
            double z = 0.0;
            const double Sj = sS[j];
            for (int blk = blk0; blk < blk1; ++blk) {
                const int base = blk * kBlock + lane * 8;
                float lx[8], qv[8];
                load_logits8<T>(row, base, lx);
                load_draft8(row, base, qv);
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    z += fmax(0.0, corrected(lx[k], qv[k], m, invT, sS, j) - Sj * (double)qv[k]);
            }
            z = wave_sum(z);
            __syncthreads();                                         // s_red free again
            if (lane == 0) s_red[wave] = z;
            __syncthreads();
            double t = 0.0;
            for (int w = 0; w < kWaves; ++w) t += s_red[w];
            if (t > 0.0) {                                           // same value in every thread
                __syncthreads();
                if (tid == 0) sS[j + 1] = t;
                ++j;
                __syncthreads();
            }
        }
        if (next < 0) break;
        ++L;
        if (tid == 0) { pth[L] = next; atk[L - 1] = stok[next]; }
        cur = next;
        __syncthreads();                                             // sS, s_red are rewritten for the next node
    }

    // ---- correction / bonus token: inverse CDF of a_j at u_resample, token-id order
    for (int blk = blk0; blk < blk1; ++blk) {
        double w8[8];
        weights8<T>(row, blk * kBlock + lane * 8, m, invT, sS, j, w8);
        double s = 0.0;
#pragma unroll
        for (int k = 0; k < 8; ++k) s += w8[k];
        s = wave_sum(s);
        if (lane == 0) s_blk[blk] = s;
    }
    if (tid == 0) s_pick = -1;
    __syncthreads();
    // owning block: the first whose inclusive prefix (blocks added in order) exceeds tgt.  Every
    // thread runs the same two loops, so all agree on the block without another exchange.
    double total = 0.0;
    for (int blk = 0; blk < nblocks; ++blk) total += s_blk[blk];
    const double tgt = (double)a.u_resample[b] * total;
    int bsel = -1, blast = 0;
    double bexcl = 0.0, run = 0.0, blexcl = 0.0;
    for (int blk = 0; blk < nblocks; ++blk) {
        const double v = s_blk[blk];
        if (v > 0.0) { blast = blk; blexcl = run; }
        if (bsel < 0 && run + v > tgt) { bsel = blk; bexcl = run; }
        run += v;
    }
    if (bsel < 0) { bsel = blast; bexcl = blexcl; }     // tgt >= total can only come from rounding
    if (wave == bsel / ipw) {
        // owning lane, then owning token
        double w8[8];
        weights8<T>(row, bsel * kBlock + lane * 8, m, invT, sS, j, w8);
        double ls = 0.0;
#pragma unroll
        for (int k = 0; k < 8; ++k) ls += w8[k];
        const double incl = wave_incl_scan(ls, lane);
        const bool hit = (bexcl + incl > tgt) && ls > 0.0;
        const unsigned long long hits = __ballot(hit);
        const unsigned long long pos = __ballot(ls > 0.0);
        int lsel;
        if (hits) lsel = __ffsll((long long)hits) - 1;
        else lsel = 63 - __clzll((long long)(pos ? pos : 1ull));      // rounding: last lane with mass
        if (lane == lsel) {
            double r3 = bexcl + (incl - ls);
            int pick = -1, lastpos = -1;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                r3 += w8[k];
                if (w8[k] > 0.0) lastpos = k;
                if (pick < 0 && r3 > tgt && w8[k] > 0.0) pick = k;
            }
            if (pick < 0) pick = max(lastpos, 0);
            s_pick = bsel * kBlock + lane * 8 + pick;
        }
    }
    __syncthreads();
    if (tid == 0) {
        a.accept_len[b] = L;
        a.bonus_token[b] = s_pick;
        if (a.status) a.status[b] = 0;
    }
}

}  // namespace

int resample_max_vocab() { return kMaxBlocks * kBlock; }

hipError_t launch_accept_resample(const ResampleArgs& a, hipStream_t st) {
    if (a.dtype == S4C_F32) hipLaunchKernelGGL(accept_resample_kernel<float>, dim3(a.B), dim3(kThreads), 0, st, a);
    else hipLaunchKernelGGL(accept_resample_kernel<bf16_t>, dim3(a.B), dim3(kThreads), 0, st, a);
    return hipGetLastError();
}

}  // namespace s4c
