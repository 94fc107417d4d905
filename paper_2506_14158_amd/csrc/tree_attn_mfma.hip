// Tree-masked attention on the CDNA4 matrix cores (paper Sec. 3.2, Fig. 3): bf16 in, fp32
// accumulate, head size 128.
//
// The N tree nodes times the G query heads that share one KV head form a dense tile of
// M = N*G query rows, so both contractions run on v_mfma_f32_32x32x16_bf16.
//   * One workgroup = WR waves; wave w owns 32 query rows.  All waves share the K/V tiles
//     (64 keys) that the workgroup streams HBM -> registers -> LDS, double-buffered, with 16-byte
//     coalesced loads; the next tile's loads are in flight while the current one is consumed.
//   * Scores are computed transposed, S^T = K Q^T (A = K rows from LDS, B = Q^T kept in
//     registers), so every lane owns one query row: the running max / sum and the rescaling of
//     the output accumulator need no cross-lane traffic, and the exponentiated scores already
//     sit in the B-operand layout of the second contraction O^T += V^T P^T.
//   * V^T fragments come from the row-major V tile through the transposing LDS read
//     (ds_read_b64_tr_b16), so V is never transposed in memory.
//   * K rows are padded to 272 B and V rows to 320 B in LDS: conflict-free for the 16-byte row
//     reads of K and for the 4-row x 64-byte transposing reads of V respectively.
//   * Prefix tiles need no mask.  The tree rows follow as extra tiles whose scores are kept only
//     where the key node is the query node or one of its ancestors (128-bit masks built from
//     parent[] in LDS).
//   * With KV splits > 1 the kernel writes unnormalised partials for the merge kernel.
#include "common.h"

namespace s4c {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int kD = 128;
constexpr int kBN = 64;                 // keys per tile
constexpr int kKStr = kD + 8;           // K row stride in LDS (elements): 272 B
constexpr int kVStr = kD + 32;          // V row stride in LDS (elements): 320 B
constexpr int kKBuf = kBN * kKStr;      // elements per K buffer
constexpr int kVBuf = kBN * kVStr;
constexpr int kLdsBytes = 2 * (kKBuf + kVBuf) * 2 + kMaxNodes * 16 + kMaxNodes * 4;

template <int WR>
__global__ __launch_bounds__(WR * 64) void tree_attn_mfma_kernel(AttnArgs a) {
    constexpr int NT = WR * 64;
    constexpr int BM = WR * 32;
    constexpr int CH = (kBN * kD / 8) / NT;      // 16-byte chunks per thread per K (or V) tile
    static_assert(CH >= 1, "tile smaller than the workgroup");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t* Ks = (bf16_t*)smem;                          // [2][kBN][kKStr]
    bf16_t* Vs = Ks + 2 * kKBuf;                         // [2][kBN][kVStr]
    uint32_t* anc = (uint32_t*)(Vs + 2 * kVBuf);         // [kMaxNodes][4]
    int32_t* spar = (int32_t*)(anc + kMaxNodes * 4);     // [kMaxNodes]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int mt = blockIdx.x / a.splits, sp = blockIdx.x % a.splits;
    const int N = a.N, G = a.G, M = a.M;

    // ---- validate the sequence; build ancestor-or-self masks
    int bad_tree = 0;
    if (tid < N) {
        const int p = a.parent[(size_t)b * N + tid];
        spar[tid] = p;
        bad_tree = (p < -1 || p >= tid);
    }
    bad_tree = __syncthreads_or(bad_tree);
    const int P = a.cache_len[b];
    const int bad_len = (P < 0 || P > a.max_cache_len || P > a.S_cap);
    if (a.status && tid == 0 && blockIdx.x == 0 && kvh == 0)
        a.status[b] = (bad_tree ? S4C_SEQ_BAD_TREE : 0) | (bad_len ? S4C_SEQ_BAD_LEN : 0);
    const bool bad = bad_tree || bad_len;
    for (int i = tid; i < N && !bad; i += NT) {
        uint32_t m[4] = {0, 0, 0, 0};
        for (int j = i; j >= 0; j = spar[j]) m[j >> 5] |= 1u << (j & 31);
        anc[i * 4 + 0] = m[0]; anc[i * 4 + 1] = m[1]; anc[i * 4 + 2] = m[2]; anc[i * 4 + 3] = m[3];
    }
    __syncthreads();

    // ---- this lane's query row
    const int g32 = lane >> 5;                    // which half of the wave
    const int rq = mt * BM + wave * 32 + (lane & 31);
    const bool rvalid = rq < M;
    const int node = rvalid ? rq / G : 0;
    const int head = kvh * G + (rvalid ? rq % G : 0);
    uint32_t amask[4] = {0, 0, 0, 0};
    if (rvalid && !bad) {
#pragma unroll
        for (int w = 0; w < 4; ++w) amask[w] = anc[node * 4 + w];
    }

    // Q^T fragments: B operand of step t holds d = 16 t + 8 g32 + (0..7) of row rq
    bf16x8 qf[8];
    {
        const bf16_t* qrow = (const bf16_t*)a.q + (((size_t)b * N + node) * a.Hq + head) * kD + g32 * 8;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (rvalid) raw = *(const uint4*)(qrow + 16 * t);
            qf[t] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    // ---- tiles of this workgroup: prefix range of the split, then (last split) the tree rows
    int kb = sp * a.chunk, ke = min(P, (sp + 1) * a.chunk);
    if (bad || ke < kb) { kb = 0; ke = 0; }
    const int n_pref = (ke - kb + kBN - 1) / kBN;
    const int n_tree = (!bad && sp == a.splits - 1) ? (N + kBN - 1) / kBN : 0;
    const int n_tiles = n_pref + n_tree;

    const bf16_t* kc = (const bf16_t*)a.k_cache + ((size_t)b * a.Hkv + kvh) * (size_t)a.S_cap * kD;
    const bf16_t* vc = (const bf16_t*)a.v_cache + ((size_t)b * a.Hkv + kvh) * (size_t)a.S_cap * kD;
    const bf16_t* kt = (const bf16_t*)a.k_tree + ((size_t)b * N * a.Hkv + kvh) * kD;
    const bf16_t* vt = (const bf16_t*)a.v_tree + ((size_t)b * N * a.Hkv + kvh) * kD;
    const size_t tree_stride = (size_t)a.Hkv * kD;

    uint4 kreg[CH], vreg[CH];
    auto load_tile = [&](int t) {
        const bool tree = t >= n_pref;
        const int k0 = tree ? (t - n_pref) * kBN : kb + t * kBN;
        const int kend = tree ? N : ke;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int chunk = tid + NT * c;
            const int row = chunk >> 4, col = (chunk & 15) * 8;
            const int key = k0 + row;
            uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
            if (key < kend) {
                const size_t off = tree ? (size_t)key * tree_stride + col : (size_t)key * kD + col;
                kv = *(const uint4*)((tree ? kt : kc) + off);
                vv = *(const uint4*)((tree ? vt : vc) + off);
            }
            kreg[c] = kv;
            vreg[c] = vv;
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int chunk = tid + NT * c;
            const int row = chunk >> 4, col = (chunk & 15) * 8;
            *(uint4*)(Ks + buf * kKBuf + row * kKStr + col) = kreg[c];
            *(uint4*)(Vs + buf * kVBuf + row * kVStr + col) = vreg[c];
        }
    };

    // per-lane LDS offsets (elements)
    const int k_lane_off = (lane & 31) * kKStr + g32 * 8;                          // + kblk*32*kKStr + 16 t
    const int i16 = lane & 15, dhalf = (lane >> 4) & 1;
    const int v_lane_off = (4 * g32 + (i16 >> 2)) * kVStr + 16 * dhalf + 4 * (i16 & 3);   // + key0*kVStr + 32 db

    f32x16 o[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int j = 0; j < 16; ++j) o[db][j] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;      // l_run: this lane's half of the keys only

    if (n_tiles > 0) {
        load_tile(0);
        store_tile(0);
    }
    __syncthreads();

    for (int t = 0; t < n_tiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < n_tiles) load_tile(t + 1);

        // ---- S^T = K Q^T for the two 32-key blocks
        f32x16 s[2];
#pragma unroll
        for (int kblk = 0; kblk < 2; ++kblk) {
#pragma unroll
            for (int j = 0; j < 16; ++j) s[kblk][j] = 0.f;
            const bf16_t* kp = Ks + buf * kKBuf + kblk * 32 * kKStr + k_lane_off;
#pragma unroll
            for (int tt = 0; tt < 8; ++tt) {
                const bf16x8 ka = *(const bf16x8*)(kp + 16 * tt);
                s[kblk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[tt], s[kblk], 0, 0, 0);
            }
        }

        // ---- masks: ragged tail of the prefix range / ancestor mask of the tree rows
        const bool tree = t >= n_pref;
        if (tree) {
            const int tt0 = (t - n_pref) * 2;           // 32-key block index of kblk 0
#pragma unroll
            for (int kblk = 0; kblk < 2; ++kblk) {
                const int w = tt0 + kblk;
                const uint32_t word = (w == 0 ? amask[0] : w == 1 ? amask[1] : w == 2 ? amask[2] : amask[3]) >> (4 * g32);
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    if (!((word >> ((j >> 2) * 8 + (j & 3))) & 1u)) s[kblk][j] = -INFINITY;
            }
        } else if (t == n_pref - 1 && (ke - kb) % kBN != 0) {
            const int nvalid = ke - (kb + t * kBN);
#pragma unroll
            for (int kblk = 0; kblk < 2; ++kblk)
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    if (kblk * 32 + (j >> 2) * 8 + 4 * g32 + (j & 3) >= nvalid) s[kblk][j] = -INFINITY;
        }

        // ---- online softmax for this lane's row (log2 units)
        float mx = s[0][0];
#pragma unroll
        for (int kblk = 0; kblk < 2; ++kblk)
#pragma unroll
            for (int j = 0; j < 16; ++j) mx = fmaxf(mx, s[kblk][j]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx * a.scale_log2);
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = fast_exp2(m_run - m_safe);
        float psum = 0.f;
#pragma unroll
        for (int kblk = 0; kblk < 2; ++kblk)
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const float p = fast_exp2(fmaf(s[kblk][j], a.scale_log2, -m_safe));
                s[kblk][j] = p;
                psum += p;
            }
        l_run = l_run * alpha + psum;
        if (__any(m_new > m_run)) {
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int j = 0; j < 16; ++j) o[db][j] *= alpha;
        }
        m_run = m_new;

        // ---- O^T += V^T P^T
#pragma unroll
        for (int kblk = 0; kblk < 2; ++kblk) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                bf16x8 pb;
#pragma unroll
                for (int e = 0; e < 8; ++e) pb[e] = (__bf16)s[kblk][8 * u + e];
                const bf16_t* vp = Vs + buf * kVBuf + (kblk * 32 + 16 * u) * kVStr + v_lane_off;
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp + 32 * db));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp + 8 * kVStr + 32 * db));
                    const s16x8 va = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, va), pb, o[db], 0, 0, 0);
                }
            }
        }

        if (t + 1 < n_tiles) store_tile(buf ^ 1);
        __syncthreads();
    }

    // ---- write this lane's row: d = 32 db + 8 (j/4) + 4 g32 + (j%4)
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (!rvalid) return;
    if (a.splits == 1) {
        const float inv = (l_tot > 0.f) ? 1.f / l_tot : 0.f;
        bf16_t* orow = (bf16_t*)a.out + (((size_t)b * N + node) * a.Hq + head) * kD + 4 * g32;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int jq = 0; jq < 4; ++jq) {
                uint2 pk;
                pk.x = (uint32_t)f32_to_bf16(o[db][4 * jq + 0] * inv) | ((uint32_t)f32_to_bf16(o[db][4 * jq + 1] * inv) << 16);
                pk.y = (uint32_t)f32_to_bf16(o[db][4 * jq + 2] * inv) | ((uint32_t)f32_to_bf16(o[db][4 * jq + 3] * inv) << 16);
                *(uint2*)(orow + 32 * db + 8 * jq) = pk;
            }
    } else {
        const size_t prow = (((size_t)b * a.Hkv + kvh) * a.splits + sp) * M + rq;
        float* orow = a.ws_o + prow * kD + 4 * g32;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int jq = 0; jq < 4; ++jq)
                *(float4*)(orow + 32 * db + 8 * jq) =
                    make_float4(o[db][4 * jq], o[db][4 * jq + 1], o[db][4 * jq + 2], o[db][4 * jq + 3]);
        if (g32 == 0) {
            a.ws_ml[prow * 2] = m_run;
            a.ws_ml[prow * 2 + 1] = l_tot;
        }
    }
}

int pick_wr(int M) { return M <= 32 ? 1 : M <= 64 ? 2 : M <= 128 ? 4 : 8; }

template <int WR>
hipError_t launch(const AttnArgs& a, hipStream_t st) {
    static bool attr_set = false;     // benign race: the attribute call is idempotent
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)tree_attn_mfma_kernel<WR>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int mtiles = (a.M + WR * 32 - 1) / (WR * 32);
    dim3 grid(mtiles * a.splits, a.Hkv, a.B), block(WR * 64);
    hipLaunchKernelGGL((tree_attn_mfma_kernel<WR>), grid, block, kLdsBytes, st, a);
    return hipGetLastError();
}

}  // namespace

bool mfma_path_supported(const s4c_attn_shape& s) { return s.dtype == S4C_BF16 && s.D == kD; }

int mfma_rows_per_block(const s4c_attn_shape& s) { return 32 * pick_wr(s.N * (s.Hq / s.Hkv)); }

hipError_t launch_tree_attn_mfma(const AttnArgs& a, hipStream_t st) {
    switch (pick_wr(a.M)) {
        case 1: return launch<1>(a, st);
        case 2: return launch<2>(a, st);
        case 4: return launch<4>(a, st);
        default: return launch<8>(a, st);
    }
}

}  // namespace s4c
