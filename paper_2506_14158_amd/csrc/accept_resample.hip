// Sibling-sequential acceptance with the correction token (paper Sec. 2, speculative-sampling
// paragraph: accept with probability min(1, p/q), redraw a rejected token from
// norm(max(0, p - q)); Sec. 3.2, second equation: the correction at a fork of the tree).
//
// The walk from the root is a chain of data-dependent decisions, each needing a reduction over
// the vocabulary, so the parallelism is inside a row, not across nodes.  A team of G workgroups
// walks one sequence: every workgroup owns a contiguous slice of the vocabulary, reduces it,
// and the G partial results are exchanged through a per-pass slot array in device memory
// (one relaxed 64-bit atomic store and G polled atomic loads; a slot still holding the
// sentinel has not been written yet).  All G workgroups then add the partials in slot order,
// obtain bit-identical sums and so take the same branches without any other communication.
// The poll is bounded: a workgroup that cannot complete an exchange exits.  Workgroup 0 of the team
// is the only one that writes the sequence's outputs (the owner of the correction token hands it over
// through one more slot), so what the caller sees is either a complete result or, if workgroup 0
// itself gave up anywhere, the flagged empty one -- never a mixture.
//
// Everything is kept unnormalised so no row is ever rewritten:
//   a_0[v] = exp((l[v] - max l) / T)              S_0 = sum_v a_0[v]        (target row)
//   a_{j+1}[v] = max(0, a_j[v] - S_j q[v])        S_{j+1} = sum_v a_{j+1}[v] (after j+1 rejections)
// so that a_j / S_j is the j-times-corrected distribution.  A child with token x passes iff
// u q[x] < a_j[x] / S_j.  a_j[v] is recomputed from l[v], q[v] and the j scalars S_0..S_{j-1}
// whenever it is needed.  The correction token is the inverse CDF of a_j in token-id order.
// The arithmetic is fp64: the decisions compare sums of 10^5 terms against a uniform number,
// and the work is a few rows per sequence, so accuracy is worth more than VALU rate here.
//
// Vocabulary traversal (all passes): blocks of 512 tokens; workgroup g owns blocks
// [g*bpg, (g+1)*bpg), wave w of it the blocks [w*ipw, (w+1)*ipw) of those; in a block lane l owns
// the 8 tokens 8l..8l+7 (one 16-byte load of 16-bit logits, two of fp32).
#include "common.h"

namespace s4c {

namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kBlock = 512;            // tokens per (wave, iteration)
constexpr int kMaxBlocks = 4096;       // => V <= 2^21
constexpr int kMaxTeam = 16;           // workgroups per sequence
constexpr int kTeamBudget = 256;       // teams * team size never exceeds this many workgroups
constexpr uint64_t kEmpty = ~0ull;     // slot not written yet (a NaN pattern no partial result has)
constexpr int kSpinLimit = 1 << 20;    // default number of polls (each followed by a short sleep) before giving up

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

__device__ __forceinline__ double bits_to_f64(uint64_t u) { return __longlong_as_double((long long)u); }
__device__ __forceinline__ uint64_t f64_to_bits(double x) { return (uint64_t)__double_as_longlong(x); }
__device__ __forceinline__ float bits_to_f32(uint64_t u) { return __uint_as_float((uint32_t)u); }

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
            for (int k = 0; k < 4; ++k) unpack2<T>(w[k], x[2 * k], x[2 * k + 1]);
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

// One exchange among the G workgroups of a team.  `slots` are this exchange's 2G words: thread 0
// contributes mineA to slots[g] and (if two) mineB to slots[G + g]; on return gotA[0..G) and
// gotB[0..G) hold everyone's words (the same in all workgroups of the team).  *s_fail is set
// (and stays set) if some word never arrived.
__device__ __forceinline__ void team_exchange(uint64_t* slots, int g, int G, bool two, uint64_t mineA, uint64_t mineB,
                                              uint64_t* gotA, uint64_t* gotB, int* s_fail, int tid, int spin_limit) {
    if (G == 1) {
        if (tid == 0) { gotA[0] = mineA; gotB[0] = mineB; }
        __syncthreads();
        return;
    }
    if (tid == 0) {
        __hip_atomic_store(&slots[g], mineA, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (two) __hip_atomic_store(&slots[G + g], mineB, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (tid < (two ? 2 * G : G)) {
        uint64_t v = __hip_atomic_load(&slots[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (int spin = 0; v == kEmpty && spin < spin_limit; ++spin) {
            __builtin_amdgcn_s_sleep(2);
            v = __hip_atomic_load(&slots[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (tid < G) gotA[tid] = v; else gotB[tid - G] = v;
        if (v == kEmpty) *s_fail = 1;
    }
    __syncthreads();
}

__global__ void fill_slots_kernel(uint64_t* p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        p[i] = kEmpty;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void accept_resample_kernel(ResampleArgs a) {
    const int G = a.team, b = blockIdx.x / G, g = blockIdx.x % G;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int N = a.N, V = a.V;
    __shared__ int32_t spar[kMaxNodes], stok[kMaxNodes];
    __shared__ double sS[kMaxNodes + 1];          // S_0 .. S_j of the current node
    __shared__ double s_red[kWaves];
    __shared__ float s_redf[kWaves];
    __shared__ double s_blk[kMaxBlocks];          // per-block sums of the sampling pass (this slice)
    __shared__ uint64_t s_gotA[kMaxTeam], s_gotB[kMaxTeam];
    __shared__ int s_fail;

    // ---- tree validation: node 0 is the only root, parents precede children, depth < max_path
    int bad = 0;
    if (tid == 0) s_fail = 0;
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
    if (g == 0)
        for (int k = tid; k < a.max_path; k += kThreads) { pth[k] = (k == 0) ? 0 : -1; atk[k] = -1; }
    if (bad) {                                     // every workgroup of the team sees the same tree
        if (g == 0 && tid == 0) {
            a.accept_len[b] = 0;
            a.bonus_token[b] = -1;
            if (a.status) a.status[b] = S4C_SEQ_BAD_TREE;
        }
        return;
    }

    const int nblocks = (V + kBlock - 1) / kBlock;
    const int bpg = (nblocks + G - 1) / G;                 // blocks per workgroup
    const int gblk0 = min(nblocks, g * bpg), gblk1 = min(nblocks, gblk0 + bpg);
    const int ipw = (bpg + kWaves - 1) / kWaves;           // blocks per wave
    const int blk0 = min(gblk1, gblk0 + wave * ipw), blk1 = min(gblk1, blk0 + ipw);
    const double invT = 1.0 / a.temperature;
    if (g == 0 && tid == 0 && a.status) a.status[b] = 0;   // a failed exchange overwrites this later
    uint64_t* slots = a.slots + (size_t)b * a.max_pass * 2 * G;   // [max_pass][2][G]
    int pass = 0;

    // An exchange that cannot complete (or more exchanges than the slot array holds, which a valid
    // tree cannot need): the workgroup leaves; workgroup 0 flags the sequence and empties its outputs
    // on the way out.  The condition is uniform across the workgroup.
#define S4C_TEAM_CHECK()                                                                                   \
    if (s_fail || pass > a.max_pass) {                                                                     \
        if (g == 0) {                                                                                      \
            __syncthreads();   /* thread 0's earlier path entries are ordered before the reset */          \
            for (int k = tid; k < a.max_path; k += kThreads) { pth[k] = (k == 0) ? 0 : -1; atk[k] = -1; }  \
            if (tid == 0) {                                                                                \
                if (a.status) a.status[b] = S4C_SEQ_TIMEOUT;                                               \
                a.accept_len[b] = 0;                                                                       \
                a.bonus_token[b] = -1;                                                                     \
            }                                                                                              \
        }                                                                                                  \
        return;                                                                                            \
    }

    Row row;
    row.V = V;
    int cur = 0, L = 0, j = 0;
    float m = 0.f;
    for (;;) {
        row.lg = (const T*)a.logits + ((size_t)b * N + cur) * V;
        row.q = a.draft + ((size_t)b * N + cur) * V;
        row.vec = (((uintptr_t)row.lg | (uintptr_t)row.q) & 15) == 0;

        // ---- row maximum (exact) and S_0 in ONE pass over the row: every lane keeps a running
        // maximum and a sum relative to it, rescaled when the maximum grows (rare after the
        // first blocks); lanes, waves and workgroups are combined the same way.
        float m_run = -INFINITY;
        double s = 0.0;
        for (int blk = blk0; blk < blk1; ++blk) {
            const int base = blk * kBlock + lane * 8;
            if (base >= V) continue;
            float x[8];
            load_logits8<T>(row, base, x);
            float bm = x[0];
#pragma unroll
            for (int k = 1; k < 8; ++k) bm = fmaxf(bm, x[k]);
            if (bm > m_run) {
                s *= exp(((double)m_run - (double)bm) * invT);     // first block: 0 * exp(-inf) = 0
                m_run = bm;
            }
            double e8[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) e8[k] = exp(((double)x[k] - (double)m_run) * invT);
            s += ((e8[0] + e8[1]) + (e8[2] + e8[3])) + ((e8[4] + e8[5]) + (e8[6] + e8[7]));
        }
        float mw = m_run;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) mw = fmaxf(mw, __shfl_xor(mw, off));
        s = (m_run == -INFINITY) ? 0.0 : s * exp(((double)m_run - (double)mw) * invT);
        s = wave_sum(s);
        if (lane == 0) { s_redf[wave] = mw; s_red[wave] = s; }
        __syncthreads();
        float mg = s_redf[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) mg = fmaxf(mg, s_redf[w]);
        double sg = 0.0;
        if (tid == 0)
            for (int w = 0; w < kWaves; ++w)
                if (s_redf[w] != -INFINITY) sg += s_red[w] * exp(((double)s_redf[w] - (double)mg) * invT);
        // exchange (slice maximum, slice sum relative to it)
        ++pass;
        S4C_TEAM_CHECK();
        team_exchange(slots + (size_t)(pass - 1) * 2 * G, g, G, true, (uint64_t)__float_as_uint(mg), f64_to_bits(sg),
                      s_gotA, s_gotB, &s_fail, tid, a.spin_limit);
        S4C_TEAM_CHECK();
        m = bits_to_f32(s_gotA[0]);
        for (int i = 1; i < G; ++i) m = fmaxf(m, bits_to_f32(s_gotA[i]));
        if (tid == 0) {
            double t = 0.0;
            for (int i = 0; i < G; ++i) {
                const float mi = bits_to_f32(s_gotA[i]);
                if (mi != -INFINITY) t += bits_to_f64(s_gotB[i]) * exp(((double)mi - (double)m) * invT);
            }
            sS[0] = t;
        }
        __syncthreads();
        j = 0;

        // ---- children of cur in increasing node index (every thread of every workgroup of the
        // team takes the same branches)
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
            double zg = 0.0;
            for (int w = 0; w < kWaves; ++w) zg += s_red[w];
            ++pass;
            S4C_TEAM_CHECK();
            team_exchange(slots + (size_t)(pass - 1) * 2 * G, g, G, false, f64_to_bits(zg), 0, s_gotA, s_gotB, &s_fail, tid, a.spin_limit);
            S4C_TEAM_CHECK();
            double t = 0.0;
            for (int i = 0; i < G; ++i) t += bits_to_f64(s_gotA[i]);
            if (t > 0.0) {                                           // same value in every thread
                __syncthreads();
                if (tid == 0) sS[j + 1] = t;
                ++j;
                __syncthreads();
            }
        }
        if (next < 0) break;
        ++L;
        if (g == 0 && tid == 0) { pth[L] = next; atk[L - 1] = stok[next]; }
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
        if (lane == 0) s_blk[blk - gblk0] = s;
    }
    __syncthreads();
    // slice total: this workgroup's blocks added in order
    double slice = 0.0;
    for (int blk = gblk0; blk < gblk1; ++blk) slice += s_blk[blk - gblk0];
    ++pass;
    S4C_TEAM_CHECK();
    team_exchange(slots + (size_t)(pass - 1) * 2 * G, g, G, false, f64_to_bits(slice), 0, s_gotA, s_gotB, &s_fail, tid, a.spin_limit);
    S4C_TEAM_CHECK();
    // owning workgroup: the first whose inclusive prefix (slices added in order) exceeds tgt
    double total = 0.0;
    for (int i = 0; i < G; ++i) total += bits_to_f64(s_gotA[i]);
    const double tgt = (double)a.u_resample[b] * total;
    int gsel = -1, glast = 0;
    double gexcl = 0.0, run = 0.0, glexcl = 0.0;
    for (int i = 0; i < G; ++i) {
        const double v = bits_to_f64(s_gotA[i]);
        if (v > 0.0) { glast = i; glexcl = run; }
        if (gsel < 0 && run + v > tgt) { gsel = i; gexcl = run; }
        run += v;
    }
    if (gsel < 0) { gsel = glast; gexcl = glexcl; }     // tgt >= total can only come from rounding
    if (g != gsel && g != 0) return;
    __shared__ int s_token;
    if (tid == 0) s_token = -1;
    __syncthreads();
    if (g == gsel) {
        // owning block inside the slice, same rule; every thread runs the same loop
        int bsel = -1, blast = gblk0;
        double bexcl = gexcl, r2 = gexcl, blexcl = gexcl;
        for (int blk = gblk0; blk < gblk1; ++blk) {
            const double v = s_blk[blk - gblk0];
            if (v > 0.0) { blast = blk; blexcl = r2; }
            if (bsel < 0 && r2 + v > tgt) { bsel = blk; bexcl = r2; }
            r2 += v;
        }
        if (bsel < 0) { bsel = blast; bexcl = blexcl; }
        if (wave == 0) {
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
                s_token = bsel * kBlock + lane * 8 + pick;
            }
        }
    }
    __syncthreads();
    // ---- the token goes to workgroup 0, which alone writes the outputs of the sequence
    if (gsel != 0) {
        ++pass;
        S4C_TEAM_CHECK();
        uint64_t* slot = slots + (size_t)(pass - 1) * 2 * G;
        if (g == gsel) {
            if (tid == 0) __hip_atomic_store(slot, (uint64_t)(uint32_t)s_token, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        if (tid == 0) {
            uint64_t v = __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            for (int spin = 0; v == kEmpty && spin < a.spin_limit; ++spin) {
                __builtin_amdgcn_s_sleep(2);
                v = __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (v == kEmpty) s_fail = 1; else s_token = (int)(uint32_t)v;
        }
        __syncthreads();
        S4C_TEAM_CHECK();
    }
    if (tid == 0) {
        a.accept_len[b] = L;
        a.bonus_token[b] = s_token;
    }
#undef S4C_TEAM_CHECK
}

}  // namespace

int resample_max_vocab() { return kMaxBlocks * kBlock; }

// Workgroups per sequence: enough blocks per workgroup to keep its waves busy, at most 16, and
// few enough that all teams are resident together (two 8-wave workgroups fit on each of the
// 256 CUs, so 256 workgroups leave a factor two of slack).
int resample_team(int B, int V) {
    const int nblocks = (V + kBlock - 1) / kBlock;
    int G = (nblocks + kWaves - 1) / kWaves;
    if (G > kMaxTeam) G = kMaxTeam;
    while (G > 1 && (long long)B * G > kTeamBudget) G >>= 1;
    return G < 1 ? 1 : G;
}

// exchanges per sequence: one per visited node, one per rejected child, one for the sampling, one
// to hand the token to workgroup 0
int resample_max_pass(int N, int max_path) { return max_path + N + 2; }
int resample_default_spin_limit() { return kSpinLimit; }

size_t resample_slot_words(int B, int N, int V, int max_path) {
    const int G = resample_team(B, V);
    return G == 1 ? 0 : (size_t)B * resample_max_pass(N, max_path) * 2 * G;
}

hipError_t launch_accept_resample(const ResampleArgs& a, hipStream_t st) {
    if (a.team > 1) {
        const size_t n = (size_t)a.B * a.max_pass * 2 * a.team;
        const size_t want = (n + 255) / 256;
        hipLaunchKernelGGL(fill_slots_kernel, dim3((unsigned)(want < 1024 ? want : 1024)), dim3(256), 0, st, a.slots, n);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const dim3 grid((unsigned)(a.B * a.team));
    if (a.dtype == S4C_F32) hipLaunchKernelGGL(accept_resample_kernel<float>, grid, dim3(kThreads), 0, st, a);
    else if (a.dtype == S4C_F16) hipLaunchKernelGGL(accept_resample_kernel<f16_t>, grid, dim3(kThreads), 0, st, a);
    else hipLaunchKernelGGL(accept_resample_kernel<bf16_t>, grid, dim3(kThreads), 0, st, a);
    return hipGetLastError();
}

}  // namespace s4c
