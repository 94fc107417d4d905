// Tree-masked attention, scalar-FMA version (paper Sec. 3.2, Fig. 3).
//
// Used for fp32 data and for 16-bit shapes the MFMA kernels do not take.  One workgroup owns
// a tile of kBM query rows of one (sequence, KV head) and one KV split: it streams key/value
// tiles of kBN rows through LDS, keeps a running max / sum per row (online softmax in log2
// units) and an fp32 output accumulator in registers.  The prefix rows come from the cache;
// the last split then walks the tree rows, where a score is kept only if the key node is the
// query node or one of its ancestors (128-bit ancestor masks built from parent[] in LDS).
// Also holds the merge kernel that combines the KV splits of either attention kernel.
#include "common.h"

namespace s4c {

namespace {

constexpr int kBM = 32;   // query rows per workgroup
constexpr int kBN = 32;   // keys per tile
constexpr int kThreads = 256;

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void tree_attn_generic_kernel(AttnArgs a) {
    __shared__ float Qs[kBM][D + 1];
    __shared__ float Ks[kBN][D + 1];
    __shared__ float Vs[kBN][D];
    __shared__ float Ps[kBM][kBN + 1];
    __shared__ int32_t spar[kMaxNodes];
    __shared__ uint64_t anc_lo[kMaxNodes], anc_hi[kMaxNodes];

    const int tid = threadIdx.x;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int mt = blockIdx.x / a.splits, sp = blockIdx.x % a.splits;
    const int N = a.N, G = a.G, M = a.M;

    const T* q = (const T*)a.q;
    const T* kt = (const T*)a.k_tree;
    const T* vt = (const T*)a.v_tree;
    const T* kc = (const T*)a.k_cache + ((size_t)b * a.Hkv + kvh) * (size_t)a.S_cap * D;
    const T* vc = (const T*)a.v_cache + ((size_t)b * a.Hkv + kvh) * (size_t)a.S_cap * D;

    // ---- validate the sequence (every workgroup does; one of them reports)
    int bad_tree = 0;
    if (tid < N) {
        const int p = a.parent[(size_t)b * N + tid];
        spar[tid] = p;
        bad_tree = (p < -1 || p >= tid);
    }
    bad_tree = __syncthreads_or(bad_tree);
    const int P = a.cache_len[b];
    int bad_len = (P < 0 || P > a.max_cache_len || P > a.S_cap);
    const bool paged = a.block_table != nullptr;
    if (paged) {
        // every page the prefix touches must be a page of the pool
        int bad_page = 0;
        if (!bad_len)
            for (int i = tid; i < ((P + (1 << a.page_shift) - 1) >> a.page_shift); i += kThreads) {
                const int id = a.block_table[(size_t)b * a.max_blocks + i];
                bad_page |= (id < 0 || id >= a.num_pages);
            }
        bad_len |= __syncthreads_or(bad_page);
    }
    if (a.status && tid == 0 && blockIdx.x == 0 && kvh == 0)
        a.status[b] = (bad_tree ? S4C_SEQ_BAD_TREE : 0) | (bad_len ? S4C_SEQ_BAD_LEN : 0);
    const bool bad = bad_tree || bad_len;

    // ---- ancestor-or-self masks (only walked when parent[] is known to be valid)
    if (tid < N && !bad) {
        uint64_t lo = 0, hi = 0;
        for (int j = tid; j >= 0; j = spar[j]) {
            if (j < 64) lo |= 1ull << j; else hi |= 1ull << (j - 64);
        }
        anc_lo[tid] = lo;
        anc_hi[tid] = hi;
    }

    // ---- stage the query tile
    const int row0 = mt * kBM;
    for (int e = tid; e < kBM * D; e += kThreads) {
        const int lr = e / D, d = e % D;
        const int r = row0 + lr;
        float v = 0.f;
        if (r < M) {
            const int node = r / G, g = r % G;
            v = to_f32<T>(q[(((size_t)b * N + node) * a.Hq + (kvh * G + g)) * D + d]);
        }
        Qs[lr][d] = v;
    }
    __syncthreads();

    // thread -> (row, 4 key columns) for scores; (row, D/8 output columns) for the accumulator
    const int lr = tid >> 3, sub = tid & 7;
    const int r = row0 + lr;
    const int node = (r < M) ? r / G : 0;
    uint64_t my_lo = 0, my_hi = 0;
    if (r < M && !bad) { my_lo = anc_lo[node]; my_hi = anc_hi[node]; }

    float m_run = -INFINITY, l_run = 0.f;
    float acc[D / 8];
#pragma unroll
    for (int j = 0; j < D / 8; ++j) acc[j] = 0.f;

    int kb = sp * a.chunk, ke = min(P, (sp + 1) * a.chunk);
    if (bad) { kb = 0; ke = 0; }
    const int n_prefix_tiles = (ke > kb) ? (ke - kb + kBN - 1) / kBN : 0;
    const int n_tree_tiles = (!bad && sp == a.splits - 1) ? (N + kBN - 1) / kBN : 0;

    for (int t = 0; t < n_prefix_tiles + n_tree_tiles; ++t) {
        const bool tree = t >= n_prefix_tiles;
        const int k0 = tree ? (t - n_prefix_tiles) * kBN : kb + t * kBN;
        const int kend = tree ? N : ke;
        // paged cache: the tile's 32 rows lie in one page (pages are powers of two >= 64 rows)
        const T* kcp = kc;
        const T* vcp = vc;
        size_t krow0 = (size_t)k0;
        if (paged && !tree) {
            const int id = a.block_table[(size_t)b * a.max_blocks + (k0 >> a.page_shift)];
            krow0 = (((size_t)id * a.Hkv + kvh) << a.page_shift) + (size_t)(k0 & ((1 << a.page_shift) - 1));
            kcp = (const T*)a.k_cache;
            vcp = (const T*)a.v_cache;
        }
        // ---- load K and V tile
        for (int e = tid; e < kBN * D; e += kThreads) {
            const int c = e / D, d = e % D;
            const int kk = k0 + c;
            float kvv = 0.f, vvv = 0.f;
            if (kk < kend) {
                if (tree) {
                    const size_t off = (((size_t)b * N + kk) * a.Hkv + kvh) * D + d;
                    kvv = to_f32<T>(kt[off]);
                    vvv = to_f32<T>(vt[off]);
                } else {
                    const size_t off = (krow0 + c) * D + d;
                    kvv = to_f32<T>(kcp[off]);
                    vvv = to_f32<T>(vcp[off]);
                }
            }
            Ks[c][d] = kvv;
            Vs[c][d] = vvv;
        }
        __syncthreads();

        // ---- scores for (lr, sub + 8 j)
        float s[4];
        float tmax = -INFINITY;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = sub + 8 * j;
            const int kk = k0 + c;
            float dot = 0.f;
#pragma unroll 8
            for (int d = 0; d < D; ++d) dot = fmaf(Qs[lr][d], Ks[c][d], dot);
            bool vis = (kk < kend) && (r < M);
            if (tree && vis) vis = (kk < 64) ? ((my_lo >> kk) & 1ull) : ((my_hi >> (kk - 64)) & 1ull);
            s[j] = vis ? dot * a.scale_log2 : -INFINITY;
            tmax = fmaxf(tmax, s[j]);
        }
        // row max across the 8 threads of the row
        tmax = fmaxf(tmax, __shfl_xor(tmax, 1));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 2));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 4));
        const float m_new = fmaxf(m_run, tmax);
        float alpha = 1.f, rsum = 0.f;
        if (m_new > -INFINITY) {
            alpha = fast_exp2(m_run - m_new);      // m_run = -inf -> 0
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float p = fast_exp2(s[j] - m_new);   // masked -> 0
                Ps[lr][sub + 8 * j] = p;
                rsum += p;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) Ps[lr][sub + 8 * j] = 0.f;
        }
        rsum += __shfl_xor(rsum, 1);
        rsum += __shfl_xor(rsum, 2);
        rsum += __shfl_xor(rsum, 4);
        l_run = l_run * alpha + rsum;
        m_run = m_new;
        __syncthreads();

        // ---- accumulate: acc[j] covers output column sub + 8 j
#pragma unroll
        for (int j = 0; j < D / 8; ++j) acc[j] *= alpha;
        for (int c = 0; c < kBN; ++c) {
            const float p = Ps[lr][c];
#pragma unroll
            for (int j = 0; j < D / 8; ++j) acc[j] = fmaf(p, Vs[c][sub + 8 * j], acc[j]);
        }
        __syncthreads();
    }

    if (r >= M) return;
    const int g = r % G;
    if (a.splits == 1) {
        const float inv = (l_run > 0.f) ? 1.f / l_run : 0.f;
        T* o = (T*)a.out + (((size_t)b * N + node) * a.Hq + (kvh * G + g)) * D;
#pragma unroll
        for (int j = 0; j < D / 8; ++j) o[sub + 8 * j] = from_f32<T>(acc[j] * inv);
    } else {
        const size_t prow = (((size_t)b * a.Hkv + kvh) * a.splits + sp) * M + r;
        float* o = a.ws_o + prow * D;
#pragma unroll
        for (int j = 0; j < D / 8; ++j) o[sub + 8 * j] = acc[j];
        if (sub == 0) {
            a.ws_ml[prow * 2] = m_run;
            a.ws_ml[prow * 2 + 1] = l_run;
        }
    }
}

// Combine the KV splits: 32 lanes per query row (D = 128: one float4 each; D = 64: float2),
// all splits' loads issued before they are combined, fixed order => deterministic.
template <typename T, int D>
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a) {
    constexpr int kMaxS = 16;                                    // plan_attn never uses more splits
    constexpr int VW = D / 32;                                   // floats per lane
    const int sub = threadIdx.x & 31;
    const size_t row = (size_t)blockIdx.x * 8 + (threadIdx.x >> 5);   // over B*Hkv*M
    const size_t total = (size_t)a.B * a.Hkv * a.M;
    if (row >= total) return;
    const int r = (int)(row % a.M);
    const size_t bh = row / a.M;
    const int kvh = (int)(bh % a.Hkv), b = (int)(bh / a.Hkv);
    const int S = a.splits;
    float ms[kMaxS], ls[kMaxS], v[kMaxS][VW];
#pragma unroll
    for (int s = 0; s < kMaxS; ++s) {
        if (s < S) {
            const size_t prow = (bh * S + s) * a.M + r;
            ms[s] = a.ws_ml[prow * 2];
            ls[s] = a.ws_ml[prow * 2 + 1];
#pragma unroll
            for (int j = 0; j < VW; ++j) v[s][j] = a.ws_o[prow * D + sub * VW + j];
        } else {
            ms[s] = -INFINITY;
            ls[s] = 0.f;
#pragma unroll
            for (int j = 0; j < VW; ++j) v[s][j] = 0.f;
        }
    }
    float m = -INFINITY;
#pragma unroll
    for (int s = 0; s < kMaxS; ++s) m = fmaxf(m, ms[s]);
    float l = 0.f, o[VW];
#pragma unroll
    for (int j = 0; j < VW; ++j) o[j] = 0.f;
#pragma unroll
    for (int s = 0; s < kMaxS; ++s) {
        if (ls[s] > 0.f) {
            const float w = fast_exp2(ms[s] - m);
            l += ls[s] * w;
#pragma unroll
            for (int j = 0; j < VW; ++j) o[j] = fmaf(v[s][j], w, o[j]);
        }
    }
    const float inv = (l > 0.f) ? 1.f / l : 0.f;
    const int node = r / a.G, g = r % a.G;
    T* dst = (T*)a.out + (((size_t)b * a.N + node) * a.Hq + (kvh * a.G + g)) * D + sub * VW;
#pragma unroll
    for (int j = 0; j < VW; ++j) dst[j] = from_f32<T>(o[j] * inv);
}

}  // namespace

hipError_t launch_tree_attn_generic(const AttnArgs& a, int dtype, hipStream_t st) {
    const int mtiles = (a.M + kBM - 1) / kBM;
    dim3 grid(mtiles * a.splits, a.Hkv, a.B), block(kThreads);
    if (dtype == S4C_F32) {
        if (a.D == 64) hipLaunchKernelGGL((tree_attn_generic_kernel<float, 64>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((tree_attn_generic_kernel<float, 128>), grid, block, 0, st, a);
    } else if (dtype == S4C_F16) {
        if (a.D == 64) hipLaunchKernelGGL((tree_attn_generic_kernel<f16_t, 64>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((tree_attn_generic_kernel<f16_t, 128>), grid, block, 0, st, a);
    } else {
        if (a.D == 64) hipLaunchKernelGGL((tree_attn_generic_kernel<bf16_t, 64>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((tree_attn_generic_kernel<bf16_t, 128>), grid, block, 0, st, a);
    }
    return hipGetLastError();
}

hipError_t launch_attn_merge(const AttnArgs& a, int dtype, hipStream_t st) {
    const size_t rows = (size_t)a.B * a.Hkv * a.M;
    dim3 grid((unsigned)((rows + 7) / 8)), block(256);
    if (dtype == S4C_F32) {
        if (a.D == 64) hipLaunchKernelGGL((attn_merge_kernel<float, 64>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((attn_merge_kernel<float, 128>), grid, block, 0, st, a);
    } else if (dtype == S4C_F16) {
        if (a.D == 64) hipLaunchKernelGGL((attn_merge_kernel<f16_t, 64>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((attn_merge_kernel<f16_t, 128>), grid, block, 0, st, a);
    } else {
        if (a.D == 64) hipLaunchKernelGGL((attn_merge_kernel<bf16_t, 64>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((attn_merge_kernel<bf16_t, 128>), grid, block, 0, st, a);
    }
    return hipGetLastError();
}

int generic_rows_per_block() { return kBM; }
int generic_keys_per_tile() { return kBN; }

}  // namespace s4c
