// Tree-masked attention on the CDNA4 matrix cores (paper Sec. 3.2, Fig. 3): bf16 or fp16 in, fp32
// accumulate, head size 128.
//
// The N tree nodes times the G query heads that share one KV head form a dense tile of
// M = N*G query rows, so both contractions run on v_mfma_f32_32x32x16_bf16 (_f16 for fp16 data).
//   * One workgroup = WR waves; wave w owns 32 query rows.  All waves share the K/V tiles
//     (64 keys) that the workgroup streams from HBM straight into LDS with
//     global_load_lds_dwordx4 (no staging registers), through a ring of NS tiles: the loads of
//     tile t+NS-1 are issued before tile t is consumed, so several tiles are in flight per CU
//     while the matrix cores work.
//   * Scores are computed transposed, S^T = K Q^T (A = K rows from LDS, B = Q^T kept in
//     registers), so every lane owns one query row: the running max / sum and the rescaling of
//     the output accumulator need no cross-lane traffic (one v_permlane32_swap joins the two
//     halves of a row), and the exponentiated scores already sit in the B-operand layout of the
//     second contraction O^T += V^T P^T.
//   * V^T fragments come from the row-major V tile through the transposing LDS read
//     (ds_read_b64_tr_b16), so V is never transposed in memory.
//   * A direct-to-LDS load writes 1 KB contiguous per wave, so rows cannot be padded; instead the
//     16-byte chunks of a row are XOR-swizzled (K: chunk ^ (row & 15); V: chunk ^ ((row & 3) << 2)),
//     applied on the global-address side of the load.  That makes the 16-byte row reads of K and
//     the 4-row x 64-byte transposing reads of V bank-conflict free.
//   * Full prefix tiles run a mask-free body.  The ragged last prefix tile and the tree rows
//     (extra tiles whose scores are kept only where the key node is the query node or one of its
//     ancestors; 128-bit masks built from parent[] in LDS) run a masked copy of the body.  Rows
//     past the end of a ragged tile are clamped to its last valid row (in bounds, finite).
//   * With KV splits > 1 the kernel writes unnormalised partials for the merge kernel.
#include "mfma_common.h"

namespace s4c {

namespace {

using namespace mfma;

constexpr int kBN = 64;                     // keys per tile
constexpr float kLazyLog2 = 8.0f;           // full tiles rescale only when a row maximum grew by more than 2^8
constexpr int kTileB = kBN * kRowB;         // bytes per K (or V) tile: 16 KB
constexpr int kStageB = 2 * kTileB;         // K then V
constexpr int lds_bytes_for(int ns) { return ns * kStageB + kMaxNodes * 16 + kMaxNodes * 4; }


template <int WR, int NS, int WPE, bool PAGED, bool F16>
__global__ __launch_bounds__(WR * 64) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
void tree_attn_mfma_kernel(AttnArgs a) {
    constexpr int NT = WR * 64;
    constexpr int BM = WR * 32;
    constexpr int CH = (kBN * kD / 8) / NT;      // direct-to-LDS loads per thread per K (or V) tile
    static_assert(CH >= 1, "tile smaller than the workgroup");
    static_assert(NS >= 2 && 2 * CH * (NS - 2) < 64, "too many loads in flight for vmcnt");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint32_t* anc = (uint32_t*)(smem + NS * kStageB);        // [kMaxNodes][4]
    int32_t* spar = (int32_t*)(anc + kMaxNodes * 4);         // [kMaxNodes]
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_u8*)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int N = a.N, G = a.G, M = a.M;

    // Workgroups are handed to the 8 XCDs round-robin by linear id.  The `team` workgroups of
    // one (sequence, KV head) -- its query-row tiles and KV splits -- take consecutive slots of
    // ONE XCD, so the row tiles that stream the same K/V rows share that XCD's L2.
    const int team = a.mtiles * a.splits;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int unit = (slot / team) * 8 + xcd;            // (sequence, KV head) index
    if (unit >= a.B * a.Hkv) return;
    const int member = slot % team;
    const int mt = member / a.splits, sp = member % a.splits;
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
            for (int i = tid; i < ((P + (1 << a.page_shift) - 1) >> a.page_shift); i += NT) {
                const int id = a.block_table[(size_t)b * a.max_blocks + i];
                bad_page |= (id < 0 || id >= a.num_pages);
            }
        bad_len |= __syncthreads_or(bad_page);
    }
    if (a.status && tid == 0 && member == 0 && kvh == 0)
        a.status[b] = (bad_tree ? S4C_SEQ_BAD_TREE : 0) | (bad_len ? S4C_SEQ_BAD_LEN : 0);
    // wave-uniform by construction; tell the compiler so that everything derived from it stays scalar
    const bool bad = __builtin_amdgcn_readfirstlane((bad_tree || bad_len) ? 1 : 0) != 0;
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
    kb = uniform(kb);
    ke = uniform(ke);
    const int n_full = (ke - kb) / kBN;                          // mask-free prefix tiles
    const int n_pref = (ke - kb + kBN - 1) / kBN;
    const int n_tree = (!bad && sp == a.splits - 1) ? (N + kBN - 1) / kBN : 0;
    const int n_tiles = n_pref + n_tree;

    // cache rows kb + j of this (sequence, KV head): contiguous, or looked up page by page (a tile
    // never straddles pages: pages are powers of two >= the tile)
    const unsigned char* kc = (const unsigned char*)a.k_cache + (((size_t)b * a.Hkv + kvh) * (size_t)a.S_cap + kb) * kRowB;
    const unsigned char* vc = (const unsigned char*)a.v_cache + (((size_t)b * a.Hkv + kvh) * (size_t)a.S_cap + kb) * kRowB;
    const int32_t* bt_row = PAGED ? a.block_table + (size_t)b * a.max_blocks : nullptr;
    auto cache_row = [&](const void* pool_or_base, const unsigned char* contiguous, int j) -> const unsigned char* {
        if constexpr (PAGED) {
            const int key = uniform(kb + j);
            const int id = scalar_load_i32(uniform((const unsigned char*)bt_row), (uint32_t)(key >> a.page_shift) * 4u);
            const size_t row = (((size_t)id * a.Hkv + kvh) << a.page_shift) + (size_t)(key & ((1 << a.page_shift) - 1));
            return uniform((const unsigned char*)pool_or_base + row * kRowB);
        } else {
            return uniform(contiguous + (size_t)j * kRowB);
        }
    };
    const unsigned char* kt = (const unsigned char*)a.k_tree + ((size_t)b * N * a.Hkv + kvh) * kRowB;
    const unsigned char* vt = (const unsigned char*)a.v_tree + ((size_t)b * N * a.Hkv + kvh) * kRowB;
    const uint32_t tree_stride = (uint32_t)a.Hkv * kRowB;

    // ---- direct-to-LDS tile loads.  Load c of a wave (instruction ii = wave + WR c of the tile)
    // covers rows 4 ii .. 4 ii + 3: lane -> (row 4 ii + lane/16, physical chunk lane%16) and fetches
    // the logical chunk that the swizzle maps there.  For full prefix tiles the per-lane byte
    // offsets are loop invariants and the tile base advances in scalar registers.
    uint32_t kvo_k[CH], kvo_v[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int row = 4 * (wave + WR * c) + (lane >> 4), pc = lane & 15;
        kvo_k[c] = row * kRowB + ((pc ^ (row & 15)) << 4);
        kvo_v[c] = row * kRowB + ((pc ^ ((row & 3) << 2)) << 4);
    }
    auto issue_tile = [&](int t) {
        const uint32_t sbase = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)(t % NS) * kStageB + wave * 1024);
        if (t < n_full) {
            const unsigned char* kg = cache_row(a.k_cache, kc, t * kBN);
            const unsigned char* vg = PAGED ? kg + ((const unsigned char*)a.v_cache - (const unsigned char*)a.k_cache)
                                            : cache_row(a.v_cache, vc, t * kBN);
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                dma16(kg, kvo_k[c], sbase + WR * c * 1024);
                dma16(vg, kvo_v[c], sbase + WR * c * 1024 + kTileB);
            }
        } else {
            const bool tree = t >= n_pref;
            const int k0 = tree ? (t - n_pref) * kBN : t * kBN;             // relative to kb for the prefix
            const int klast = (tree ? N : ke - kb) - 1;
            // rows are addressed relative to the tile's first row (or the last valid row, if the
            // tile starts beyond it), which for the prefix fixes the page
            const int kq = min(k0, klast);
            const unsigned char* kg = tree ? uniform(kt + (size_t)kq * tree_stride) : cache_row(a.k_cache, kc, kq);
            const unsigned char* vg = tree ? uniform(vt + (size_t)kq * tree_stride)
                                           : (PAGED ? kg + ((const unsigned char*)a.v_cache - (const unsigned char*)a.k_cache)
                                                    : cache_row(a.v_cache, vc, kq));
            const uint32_t rstride = tree ? tree_stride : (uint32_t)kRowB;
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const int row = 4 * (wave + WR * c) + (lane >> 4), pc = lane & 15;
                const uint32_t roff = (uint32_t)(min(k0 + row, klast) - kq) * rstride;
                dma16(kg, roff + ((pc ^ (row & 15)) << 4), sbase + WR * c * 1024);
                dma16(vg, roff + ((pc ^ ((row & 3) << 2)) << 4), sbase + WR * c * 1024 + kTileB);
            }
        }
    };

    // per-lane LDS byte offsets inside a stage
    const int i16 = lane & 15, dhalf = (lane >> 4) & 1;
    uint32_t k_off[8], v_off[4];
#pragma unroll
    for (int tt = 0; tt < 8; ++tt) k_off[tt] = (lane & 31) * kRowB + (((2 * tt + g32) ^ i16) << 4);
#pragma unroll
    for (int db = 0; db < 4; ++db)
        v_off[db] = kTileB + (4 * g32 + (i16 >> 2)) * kRowB +
                    ((((db ^ (i16 >> 2)) << 2) + 2 * dhalf + ((i16 & 3) >> 1)) << 4) + 8 * (i16 & 1);

    f32x16 o[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int j = 0; j < 16; ++j) o[db][j] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;      // l_run: this lane's half of the keys only

    // ---- one tile: scores, (mask,) online softmax, accumulate
    auto tile_body = [&](auto mode_tag, int t) {
        constexpr int MODE = decltype(mode_tag)::value;
        const lds_u8* stage = (const lds_u8*)smem + (t % NS) * kStageB;     // LDS address space throughout

        // S^T = K Q^T for the two 32-key blocks.  The two accumulator chains are interleaved (a
        // dependent MFMA cannot start before its predecessor retires); the K fragments of the
        // second half of the head dimension are requested while the first half is multiplied.
        f32x16 s[2];
        {
            bf16x8 kf[2][4];
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
                kf[0][tt] = *(const lds_bf16x8*)(stage + k_off[tt]);
                kf[1][tt] = *(const lds_bf16x8*)(stage + 32 * kRowB + k_off[tt]);
            }
#pragma unroll
            for (int j = 0; j < 16; ++j) { s[0][j] = 0.f; s[1][j] = 0.f; }
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
                s[0] = mma32<F16>(kf[0][tt], qf[tt], s[0]);
                kf[0][tt] = *(const lds_bf16x8*)(stage + k_off[tt + 4]);
                s[1] = mma32<F16>(kf[1][tt], qf[tt], s[1]);
                kf[1][tt] = *(const lds_bf16x8*)(stage + 32 * kRowB + k_off[tt + 4]);
            }
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
                s[0] = mma32<F16>(kf[0][tt], qf[tt + 4], s[0]);
                s[1] = mma32<F16>(kf[1][tt], qf[tt + 4], s[1]);
            }
            __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);      // 8 LDS reads
#pragma unroll
            for (int tt = 0; tt < 8; ++tt) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // 1 MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // 1 LDS read
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);      // 8 MFMAs
        }

        // key of register j of block kblk, relative to the tile: 32 kblk + 8 (j/4) + 4 g32 + (j%4)
        if constexpr (MODE == kTree) {
            const int w0 = (t - n_pref) * 2;            // 32-node word of block 0
#pragma unroll
            for (int kblk = 0; kblk < 2; ++kblk) {
                const int w = w0 + kblk;
                const uint32_t word = (w == 0 ? amask[0] : w == 1 ? amask[1] : w == 2 ? amask[2] : amask[3]) >> (4 * g32);
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    if (!((word >> ((j >> 2) * 8 + (j & 3))) & 1u)) s[kblk][j] = -INFINITY;
            }
        } else if constexpr (MODE == kTail) {
            const int nvalid = (ke - kb) - t * kBN;
#pragma unroll
            for (int kblk = 0; kblk < 2; ++kblk)
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    if (kblk * 32 + (j >> 2) * 8 + 4 * g32 + (j & 3) >= nvalid) s[kblk][j] = -INFINITY;
        }

        // online softmax for this lane's row (log2 units)
        float mx = fmaxf(s[0][0], s[1][0]);
#pragma unroll
        for (int j = 1; j < 16; ++j) mx = __builtin_fmaxf(__builtin_fmaxf(mx, s[0][j]), s[1][j]);    // v_max3_f32
        mx = max_across_halves(mx);
        float psum = 0.f;
        if constexpr (MODE == kPlain) {
            // Full prefix tiles move the row's reference maximum only when some row of the wave
            // outgrew it by more than 2^kLazyLog2: until then the exponentials are taken against the
            // stale reference (they stay below 2^kLazyLog2, exact in fp32 and in bf16's range), and the
            // 64 multiplications of the output accumulator are skipped.  Sum and accumulator stay
            // consistent with whatever reference is current, which is all the final division (or the
            // merge of KV splits) needs.
            const float mt = mx * a.scale_log2;
            if (__any(mt > m_run + kLazyLog2)) {
                const float m_new = fmaxf(m_run, mt);
                const float alpha = fast_exp2(m_run - m_new);          // first tile: exp2(-inf) = 0
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int j = 0; j < 16; ++j) o[db][j] *= alpha;
                m_run = m_new;
            }
#pragma unroll
            for (int kblk = 0; kblk < 2; ++kblk)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const float p = fast_exp2(fmaf(s[kblk][j], a.scale_log2, -m_run));
                    s[kblk][j] = p;
                    psum += p;
                }
            l_run += psum;
        } else {
            const float m_new = fmaxf(m_run, mx * a.scale_log2);
            float m_safe = m_new;
            if constexpr (MODE == kTree) m_safe = (m_new == -INFINITY) ? 0.f : m_new;   // row with no visible key yet
            const float alpha = fast_exp2(m_run - m_safe);
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
        }

        // O^T += V^T P^T in four steps of 16 keys; the V^T fragments of step i+1 are requested
        // before the MFMAs of step i.
        {
            bf16x8 pb[4];
#pragma unroll
            for (int st = 0; st < 4; ++st)
                pb[st] = round8<F16>(s[st >> 1], 8 * (st & 1));
            auto vfrag = [&](const lds_u8* p) {     // 8 keys x 1 column of V^T: two transposing reads
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 8 * kRowB));
                return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            };
            bf16x8 vf[2][4];
#pragma unroll
            for (int db = 0; db < 4; ++db) vf[0][db] = vfrag(stage + v_off[db]);
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                if (st < 3) {
#pragma unroll
                    for (int db = 0; db < 4; ++db) vf[(st + 1) & 1][db] = vfrag(stage + (st + 1) * 16 * kRowB + v_off[db]);
                }
#pragma unroll
                for (int db = 0; db < 4; ++db)
                    o[db] = mma32<F16>(vf[st & 1][db], pb[st], o[db]);
            }
        }
    };

    // The compiler does not see the direct-to-LDS loads; settle every load it does know about
    // (the Q fragments) here, so that it places no vmcnt wait of its own inside the tile loop.
    wait_vmcnt<0>();
    for (int t = 0; t < NS - 1 && t < n_tiles; ++t) issue_tile(t);

    auto sync_and_prefetch = [&](int t) {
        // tile t has landed once at most NS-2 younger tiles of this wave are outstanding
        if (t + NS - 2 < n_tiles) wait_vmcnt<2 * CH * (NS - 2)>(); else wait_vmcnt<0>();
        __syncthreads();          // every wave's part of tile t is in LDS; stage (t-1) % NS is free
        if (t + NS - 1 < n_tiles) issue_tile(t + NS - 1);
    };
    int t = 0;
    for (; t < n_full; ++t) {
        sync_and_prefetch(t);
        tile_body(std::integral_constant<int, kPlain>{}, t);
    }
    for (; t < n_pref; ++t) {
        sync_and_prefetch(t);
        tile_body(std::integral_constant<int, kTail>{}, t);
    }
    for (; t < n_tiles; ++t) {
        sync_and_prefetch(t);
        tile_body(std::integral_constant<int, kTree>{}, t);
    }

    // ---- write this lane's row: d = 32 db + 8 (j/4) + 4 g32 + (j%4)
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (a.splits == 1) {
        if (!rvalid) return;
        const float inv = (l_tot > 0.f) ? 1.f / l_tot : 0.f;
        bf16_t* orow = (bf16_t*)a.out + (((size_t)b * N + node) * a.Hq + head) * kD + 4 * g32;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int jq = 0; jq < 4; ++jq) {
                uint2 pk;
                pk.x = round1<F16>(o[db][4 * jq + 0] * inv) | (round1<F16>(o[db][4 * jq + 1] * inv) << 16);
                pk.y = round1<F16>(o[db][4 * jq + 2] * inv) | (round1<F16>(o[db][4 * jq + 3] * inv) << 16);
                *(uint2*)(orow + 32 * db + 8 * jq) = pk;
            }
    } else {
        if (rvalid) {
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
}

int pick_wr(int M) { return M <= 128 ? 4 : 8; }

template <int WR, int NS, int WPE, bool PAGED, bool F16>
hipError_t launch(const AttnArgs& a, hipStream_t st) {
    constexpr int kLds = lds_bytes_for(NS);
    static std::atomic<uint64_t> lds_set{0};
    const hipError_t ea = ensure_dynamic_lds((const void*)tree_attn_mfma_kernel<WR, NS, WPE, PAGED, F16>, kLds, lds_set);
    if (ea != hipSuccess) return ea;
    AttnArgs k = a;
    k.mtiles = (a.M + WR * 32 - 1) / (WR * 32);
    const long units8 = ((long)a.B * a.Hkv + 7) / 8 * 8;          // padded to whole XCD rounds
    dim3 grid((unsigned)(units8 * k.mtiles * a.splits)), block(WR * 64);
    hipLaunchKernelGGL((tree_attn_mfma_kernel<WR, NS, WPE, PAGED, F16>), grid, block, kLds, st, k);
    return hipGetLastError();
}

}  // namespace

bool mfma_path_supported(const s4c_attn_shape& s) { return (s.dtype == S4C_BF16 || s.dtype == S4C_F16) && s.D == kD; }

// Few rows: the key-parallel kernel (one 64-row workgroup); otherwise 32 rows per wave.
int mfma_rows_per_block(const s4c_attn_shape& s) {
    const int M = s.N * (s.Hq / s.Hkv);
    return M <= 64 ? 64 : 32 * pick_wr(M);
}

template <bool F16>
static hipError_t launch_by_shape(const AttnArgs& a, hipStream_t st) {
    if (a.block_table) return pick_wr(a.M) == 4 ? launch<4, 4, 1, true, F16>(a, st) : launch<8, 4, 2, true, F16>(a, st);
    return pick_wr(a.M) == 4 ? launch<4, 4, 1, false, F16>(a, st) : launch<8, 4, 2, false, F16>(a, st);
}

hipError_t launch_tree_attn_mfma(const AttnArgs& a, int dtype, hipStream_t st) {
    if (a.M <= 64) return launch_tree_attn_smallm(a, dtype, st);
    return dtype == S4C_F16 ? launch_by_shape<true>(a, st) : launch_by_shape<false>(a, st);
}

}  // namespace s4c
