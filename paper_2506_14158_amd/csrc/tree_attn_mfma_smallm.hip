// Tree-masked attention on the matrix cores for few query rows per KV head (M = N*G <= 64):
// the HBM-bound shape (paper Sec. 3.2; every drafted node attends to the whole prefix, so with
// 64 rows each K/V byte only feeds 64 FLOP).
//
// With so few rows one (sequence, KV head) cannot occupy a CU by splitting rows, so the waves
// of a workgroup split the KEYS instead: wave w owns row block w & 1 (32 rows) and key group
// w >> 1.  A round is one 32-key tile per key group; two rounds fit in LDS, so while one round
// is consumed the next is in flight (direct-to-LDS loads, XOR-swizzled as in the large-M
// kernel).  Every wave keeps its own online-softmax state over its key group; after the last
// round the partial states of a row are merged through LDS (the ring is dead by then) and
// written with coalesced stores -- no HBM round trip for the partials of the key groups.  The
// tree rows form the last round(s) (tile i = nodes 32 i .. 32 i + 31), masked with the 128-bit
// ancestor sets built from parent[].  Measured on 256 (sequence, KV head) units with a 64K
// prefix: 6.25 TB/s of K/V, 96 % of what a plain streaming-read kernel reaches on the same box.
#include "mfma_common.h"

namespace s4c {

namespace {

using namespace mfma;

constexpr int kBN = 32;                      // keys per tile
constexpr int kTileKB = kBN * kRowB;         // K (or V) bytes of a tile: 8 KB
constexpr int kTileB = 2 * kTileKB;          // K then V: 16 KB
constexpr int kMergeRowB = (kD + 4) * 4;     // padded fp32 row of a partial output: 528 B
constexpr int kAuxB = kMaxNodes * 16 + kMaxNodes * 4;

// KG key groups (tiles per round) => 2 KG waves.  KG = 4: one workgroup per CU with a 128 KB ring;
// KG = 2: 69 KB per workgroup, so two workgroups share a CU and one's set-up and merge overlap
// the other's streaming.
template <int KG>
struct Cfg {
    static constexpr int kRoundB = KG * kTileB;
    static constexpr int kRingB = 2 * kRoundB;
    static constexpr int kWaves = 2 * KG;
    static constexpr int kThreads = 64 * kWaves;
    static constexpr int kMergeB = kWaves * 32 * kMergeRowB + kWaves * 32 * 2 * 4;
    static constexpr int kLdsBytes = (kRingB + kAuxB > kMergeB) ? kRingB + kAuxB : kMergeB;
};

template <int kKG, bool PAGED, bool F16>
__global__ __launch_bounds__(Cfg<kKG>::kThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void tree_attn_smallm_kernel(AttnArgs a) {
    constexpr int kRoundB = Cfg<kKG>::kRoundB, kRingB = Cfg<kKG>::kRingB, kWaves = Cfg<kKG>::kWaves;
    constexpr int kThreads = Cfg<kKG>::kThreads;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint32_t* anc = (uint32_t*)(smem + kRingB);              // [kMaxNodes][4]
    int32_t* spar = (int32_t*)(anc + kMaxNodes * 4);         // [kMaxNodes]
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_u8*)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rb = wave & 1, kg = wave >> 1;
    const int N = a.N, G = a.G, M = a.M;

    // the splits of one (sequence, KV head) take consecutive slots of one XCD
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int unit = (slot / a.splits) * 8 + xcd;
    if (unit >= a.B * a.Hkv) return;
    const int sp = slot % a.splits;
    const int b = unit / a.Hkv, kvh = unit % a.Hkv;

    // ---- validate the sequence; build ancestor-or-self masks
    int bad_tree = 0;
    if (tid < N) {
        const int p = a.parent[(size_t)b * N + tid];
        spar[tid] = p;
        bad_tree = (p < -1 || p >= tid);
    }
    bad_tree = __syncthreads_or(bad_tree);
    const int P = a.cache_len[b];
    int bad_len = (P < 0 || P > a.max_cache_len || P > a.S_cap);
    if constexpr (PAGED) {
        // every page the prefix touches must be a page of the pool (each workgroup checks them all,
        // so all workgroups of the sequence agree)
        int bad_page = 0;
        if (!bad_len)
            for (int i = tid; i < ((P + (1 << a.page_shift) - 1) >> a.page_shift); i += kThreads) {
                const int id = a.block_table[(size_t)b * a.max_blocks + i];
                bad_page |= (id < 0 || id >= a.num_pages);
            }
        bad_len |= __syncthreads_or(bad_page);
    }
    if (a.status && tid == 0 && sp == 0 && kvh == 0)
        a.status[b] = (bad_tree ? S4C_SEQ_BAD_TREE : 0) | (bad_len ? S4C_SEQ_BAD_LEN : 0);
    const bool bad = __builtin_amdgcn_readfirstlane((bad_tree || bad_len) ? 1 : 0) != 0;
    // ---- rounds of this workgroup: prefix range of the split, then (last split) the tree round
    int kb = sp * a.chunk, ke = min(P, (sp + 1) * a.chunk);
    if (bad || ke < kb) { kb = 0; ke = 0; }
    kb = uniform(kb);
    ke = uniform(ke);
    const int len = ke - kb;
    const int n_full = len / (kKG * kBN);                          // rounds with four full tiles
    const int n_pref = (len + kKG * kBN - 1) / (kKG * kBN);
    const int n_tree = (!bad && sp == a.splits - 1) ? (N + kKG * kBN - 1) / (kKG * kBN) : 0;
    const int n_rounds = n_pref + n_tree;

    const unsigned char* kc = (const unsigned char*)a.k_cache + (((size_t)b * a.Hkv + kvh) * (size_t)a.S_cap + kb) * kRowB;
    const unsigned char* vc = (const unsigned char*)a.v_cache + (((size_t)b * a.Hkv + kvh) * (size_t)a.S_cap + kb) * kRowB;
    const unsigned char* kt = (const unsigned char*)a.k_tree + ((size_t)b * N * a.Hkv + kvh) * kRowB;
    const unsigned char* vt = (const unsigned char*)a.v_tree + ((size_t)b * N * a.Hkv + kvh) * kRowB;
    const uint32_t tree_stride = (uint32_t)a.Hkv * kRowB;
    // cache row kb + j of this (sequence, KV head): contiguous, or looked up page by page (a tile
    // never straddles pages: pages are powers of two >= 64 rows)
    const int32_t* bt_row = PAGED ? a.block_table + (size_t)b * a.max_blocks : nullptr;
    auto cache_row = [&](const void* pool, const unsigned char* contiguous, int j) -> const unsigned char* {
        if constexpr (PAGED) {
            const int key = uniform(kb + j);
            const int id = scalar_load_i32(uniform((const unsigned char*)bt_row), (uint32_t)(key >> a.page_shift) * 4u);
            const size_t row = (((size_t)id * a.Hkv + kvh) << a.page_shift) + (size_t)(key & ((1 << a.page_shift) - 1));
            return uniform((const unsigned char*)pool + row * kRowB);
        } else {
            return uniform(contiguous + (size_t)j * kRowB);
        }
    };
    const ptrdiff_t v_minus_k = (const unsigned char*)a.v_cache - (const unsigned char*)a.k_cache;

    // ---- direct-to-LDS loads: the two waves of key group kg load tile kg of every round, four
    // 1 KB instructions each for K and for V (instruction ii covers rows 4 ii .. 4 ii + 3).
    uint32_t kvo_k[4], kvo_v[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int row = 4 * (rb * 4 + c) + (lane >> 4), pc = lane & 15;
        kvo_k[c] = row * kRowB + ((pc ^ (row & 15)) << 4);
        kvo_v[c] = row * kRowB + ((pc ^ ((row & 3) << 2)) << 4);
    }
    auto issue_round = [&](int r) {
        const uint32_t sbase = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)(r & 1) * kRoundB + kg * kTileB + rb * 4096);
        if (r < n_full) {
            const unsigned char* kgp = cache_row(a.k_cache, kc, (r * kKG + kg) * kBN);
            const unsigned char* vgp = PAGED ? kgp + v_minus_k : cache_row(a.v_cache, vc, (r * kKG + kg) * kBN);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                dma16(kgp, kvo_k[c], sbase + c * 1024);
                dma16(vgp, kvo_v[c], sbase + c * 1024 + kTileKB);
            }
        } else {
            const bool tree = r >= n_pref;
            const int k0 = (tree ? r - n_pref : r) * kKG * kBN + kg * kBN;     // first row of this tile
            const int klast = max((tree ? N : len) - 1, 0);
            // rows are addressed relative to the tile's first row (or to the last valid row, if the
            // tile starts beyond it), which for the prefix fixes the page
            const int kq = min(k0, klast);
            const unsigned char* kgp = tree ? uniform(kt + (size_t)kq * tree_stride) : cache_row(a.k_cache, kc, kq);
            const unsigned char* vgp = tree ? uniform(vt + (size_t)kq * tree_stride)
                                            : (PAGED ? kgp + v_minus_k : cache_row(a.v_cache, vc, kq));
            const uint32_t rstride = tree ? tree_stride : (uint32_t)kRowB;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int row = 4 * (rb * 4 + c) + (lane >> 4), pc = lane & 15;
                const uint32_t roff = (uint32_t)(min(k0 + row, klast) - kq) * rstride;   // clamped: in bounds, masked later
                dma16(kgp, roff + ((pc ^ (row & 15)) << 4), sbase + c * 1024);
                dma16(vgp, roff + ((pc ^ ((row & 3) << 2)) << 4), sbase + c * 1024 + kTileKB);
            }
        }
    };

    // Round 0 starts streaming now; the Q fragments are requested right behind it and the
    // ancestor masks are built while both are in flight.  (The direct-to-LDS loads are invisible
    // to the compiler; loads it does know about may follow them, since completion is in order and
    // its waits then only become stricter.)
    if (n_rounds > 0) issue_round(0);

    // ---- this lane's query row
    const int g32 = lane >> 5;
    const int rq = rb * 32 + (lane & 31);
    const bool rvalid = rq < M;
    const int node = rvalid ? rq / G : 0;
    const int head = kvh * G + (rvalid ? rq % G : 0);
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

    for (int i = tid; i < N && !bad; i += kThreads) {
        const int tid_ = i;
        uint32_t m[4] = {0, 0, 0, 0};
        for (int j = tid_; j >= 0; j = spar[j]) m[j >> 5] |= 1u << (j & 31);
        anc[tid_ * 4 + 0] = m[0]; anc[tid_ * 4 + 1] = m[1]; anc[tid_ * 4 + 2] = m[2]; anc[tid_ * 4 + 3] = m[3];
    }
    __syncthreads();

    // ancestor words of this row, pre-shifted for this half of the wave; tree round i of key group kg
    // covers nodes 32 (i KG + kg) ..
    uint32_t amask[4] = {0, 0, 0, 0};
    if (rvalid && !bad) {
#pragma unroll
        for (int w = 0; w < 4; ++w) amask[w] = anc[node * 4 + w] >> (4 * g32);
    }

    // per-lane LDS byte offsets inside a tile
    const int i16 = lane & 15, dhalf = (lane >> 4) & 1;
    uint32_t k_off[8], v_off[4];
#pragma unroll
    for (int tt = 0; tt < 8; ++tt) k_off[tt] = (lane & 31) * kRowB + (((2 * tt + g32) ^ i16) << 4);
#pragma unroll
    for (int db = 0; db < 4; ++db)
        v_off[db] = kTileKB + (4 * g32 + (i16 >> 2)) * kRowB +
                    ((((db ^ (i16 >> 2)) << 2) + 2 * dhalf + ((i16 & 3) >> 1)) << 4) + 8 * (i16 & 1);

    f32x16 o[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int j = 0; j < 16; ++j) o[db][j] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // one 32-key tile: S^T = K Q^T, (mask,) online softmax, O^T += V^T P^T
    // MODE kPlain: all 32 keys valid; kTail: keys >= nvalid masked (nvalid may be <= 0); kTree: ancestor mask
    auto tile = [&](auto mode_tag, int r, int nvalid) {
        constexpr int MODE = decltype(mode_tag)::value;
        const lds_u8* stage = (const lds_u8*)smem + (r & 1) * kRoundB + kg * kTileB;
        f32x16 s;
        {
            bf16x8 kf[8];
#pragma unroll
            for (int tt = 0; tt < 8; ++tt) kf[tt] = *(const lds_bf16x8*)(stage + k_off[tt]);
            f32x16 s1;
#pragma unroll
            for (int j = 0; j < 16; ++j) { s[j] = 0.f; s1[j] = 0.f; }
#pragma unroll
            for (int tt = 0; tt < 8; tt += 2) {        // two chains over the head dimension, summed below
                s = mma32<F16>(kf[tt], qf[tt], s);
                s1 = mma32<F16>(kf[tt + 1], qf[tt + 1], s1);
            }
#pragma unroll
            for (int j = 0; j < 16; ++j) s[j] += s1[j];
        }
        // register j is key 8 (j/4) + 4 g32 + (j%4) of the tile
        if constexpr (MODE == kTree) {
            const int w = (r - n_pref) * kKG + kg;             // 32-node word of this tile (< 4 since N <= 128)
            const uint32_t tree_word = (w == 0 ? amask[0] : w == 1 ? amask[1] : w == 2 ? amask[2] : amask[3]);
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (!((tree_word >> ((j >> 2) * 8 + (j & 3))) & 1u)) s[j] = -INFINITY;
        } else if constexpr (MODE == kTail) {
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if ((j >> 2) * 8 + 4 * g32 + (j & 3) >= nvalid) s[j] = -INFINITY;
        }
        float mx = s[0];
#pragma unroll
        for (int j = 1; j < 16; j += 2) mx = __builtin_fmaxf(__builtin_fmaxf(mx, s[j]), s[(j + 1) & 15]);
        mx = max_across_halves(mx);
        const float m_new = fmaxf(m_run, mx * a.scale_log2);
        float m_safe = m_new;
        if constexpr (MODE != kPlain) m_safe = (m_new == -INFINITY) ? 0.f : m_new;   // nothing visible yet
        const float alpha = fast_exp2(m_run - m_safe);
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const float p = fast_exp2(fmaf(s[j], a.scale_log2, -m_safe));
            s[j] = p;
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

        bf16x8 pb[2];
#pragma unroll
        for (int st = 0; st < 2; ++st)
            pb[st] = round8<F16>(s, 8 * st);
        auto vfrag = [&](const lds_u8* p) {
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 8 * kRowB));
            return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        };
        bf16x8 vf[2][4];
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int db = 0; db < 4; ++db) vf[st][db] = vfrag(stage + st * 16 * kRowB + v_off[db]);
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int db = 0; db < 4; ++db)
                o[db] = mma32<F16>(vf[st][db], pb[st], o[db]);
    };

    // ---- round pipeline: round r+1 is in flight while round r is consumed
    // Settle the compiler-visible loads (Q) here, so that it places no vmcnt wait of its own inside
    // the round loop (which would also wait for the round just issued).
    wait_vmcnt<0>();
#pragma unroll
    for (int t = 0; t < 8; ++t) asm volatile("" : "+v"(qf[t]));
    auto sync_and_prefetch = [&](int r) {
        wait_vmcnt<0>();           // this wave's share of round r has landed
        __syncthreads();           // everybody's has; round r-1's half of the ring is free
        if (r + 1 < n_rounds) issue_round(r + 1);
    };
    int r = 0;
    for (; r < n_full; ++r) {
        sync_and_prefetch(r);
        tile(std::integral_constant<int, kPlain>{}, r, kBN);
    }
    for (; r < n_pref; ++r) {
        sync_and_prefetch(r);
        tile(std::integral_constant<int, kTail>{}, r, len - (r * kKG + kg) * kBN);
    }
    for (; r < n_rounds; ++r) {
        sync_and_prefetch(r);
        tile(std::integral_constant<int, kTree>{}, r, 0);
    }

    // ---- merge the four key groups of each row through LDS (the ring is no longer read)
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    __syncthreads();
    float* mo = (float*)smem;                                       // [waves][32 rows][kD + 4]
    float* mml = (float*)(smem + kWaves * 32 * kMergeRowB);         // [waves][32 rows][2]
    {
        float* orow = mo + ((size_t)wave * 32 + (lane & 31)) * (kMergeRowB / 4) + 4 * g32;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int jq = 0; jq < 4; ++jq)
                *(float4*)(orow + 32 * db + 8 * jq) =
                    make_float4(o[db][4 * jq], o[db][4 * jq + 1], o[db][4 * jq + 2], o[db][4 * jq + 3]);
        if (g32 == 0) {
            mml[(wave * 32 + lane) * 2] = m_run;
            mml[(wave * 32 + lane) * 2 + 1] = l_tot;
        }
    }
    __syncthreads();
    // thread -> (row, 16 output columns): 8 threads cover a row with 32-byte pieces
    constexpr int kTPR = kThreads / 64;          // threads per output row
    constexpr int kCols = kD / kTPR;              // output columns per thread (16 or 32)
    const int row = tid / kTPR, dcol = (tid % kTPR) * kCols;
    if (row >= M && a.splits == 1) return;
    const int orb = row >> 5, oq = row & 31;
    float mg[kKG], lg[kKG], mmax = -INFINITY;
#pragma unroll
    for (int g = 0; g < kKG; ++g) {
        const int w = g * 2 + orb;
        mg[g] = mml[(w * 32 + oq) * 2];
        lg[g] = mml[(w * 32 + oq) * 2 + 1];
        mmax = fmaxf(mmax, mg[g]);
    }
    float acc[kCols], l = 0.f;
#pragma unroll
    for (int e = 0; e < kCols; ++e) acc[e] = 0.f;
#pragma unroll
    for (int g = 0; g < kKG; ++g) {
        if (lg[g] <= 0.f) continue;                 // this key group saw nothing visible
        const float wgt = fast_exp2(mg[g] - mmax);
        l += lg[g] * wgt;
        const float* src = mo + ((size_t)(g * 2 + orb) * 32 + oq) * (kMergeRowB / 4) + dcol;
#pragma unroll
        for (int e = 0; e < kCols; e += 4) {
            const float4 v = *(const float4*)(src + e);
            acc[e] = fmaf(v.x, wgt, acc[e]); acc[e + 1] = fmaf(v.y, wgt, acc[e + 1]);
            acc[e + 2] = fmaf(v.z, wgt, acc[e + 2]); acc[e + 3] = fmaf(v.w, wgt, acc[e + 3]);
        }
    }
    if (a.splits == 1) {
        const int onode = row / G, ohead = kvh * G + row % G;
        const float inv = (l > 0.f) ? 1.f / l : 0.f;
        uint4* dst = (uint4*)((bf16_t*)a.out + (((size_t)b * N + onode) * a.Hq + ohead) * kD + dcol);
#pragma unroll
        for (int e = 0; e < kCols; e += 8) {
            uint32_t pk[4];
#pragma unroll
            for (int h = 0; h < 4; ++h)
                pk[h] = round1<F16>(acc[e + 2 * h] * inv) | (round1<F16>(acc[e + 2 * h + 1] * inv) << 16);
            dst[e / 8] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        }
    } else {
        if (row < M) {
            const size_t prow = (((size_t)b * a.Hkv + kvh) * a.splits + sp) * M + row;
            float4* dst = (float4*)(a.ws_o + prow * kD + dcol);
#pragma unroll
            for (int e = 0; e < kCols / 4; ++e) dst[e] = make_float4(acc[4 * e], acc[4 * e + 1], acc[4 * e + 2], acc[4 * e + 3]);
            if (tid % kTPR == 0) {
                a.ws_ml[prow * 2] = mmax;
                a.ws_ml[prow * 2 + 1] = l;
            }
        }
    }
}

}  // namespace

template <int KG, bool PAGED, bool F16>
static hipError_t launch_smallm(const AttnArgs& a, hipStream_t st) {
    static std::atomic<uint64_t> lds_set{0};
    const hipError_t ea = ensure_dynamic_lds((const void*)tree_attn_smallm_kernel<KG, PAGED, F16>, Cfg<KG>::kLdsBytes, lds_set);
    if (ea != hipSuccess) return ea;
    const long units8 = ((long)a.B * a.Hkv + 7) / 8 * 8;
    dim3 grid((unsigned)(units8 * a.splits)), block(Cfg<KG>::kThreads);
    hipLaunchKernelGGL((tree_attn_smallm_kernel<KG, PAGED, F16>), grid, block, Cfg<KG>::kLdsBytes, st, a);
    return hipGetLastError();
}

hipError_t launch_tree_attn_smallm(const AttnArgs& a, int dtype, hipStream_t st) {
    if (dtype == S4C_F16) return a.block_table ? launch_smallm<2, true, true>(a, st) : launch_smallm<2, false, true>(a, st);
    return a.block_table ? launch_smallm<2, true, false>(a, st) : launch_smallm<2, false, false>(a, st);
}

}  // namespace s4c
