// Input projection of a draft head (paper Eq. 3: h = Linear(concat[e, f])) for FEW tokens (T <= 128):
// the batch-1 operating point of the paper's experiments (Sec. 4.1.2), where a draft tree holds a few
// dozen tokens.  With so few tokens every weight feeds at most 2 T FLOP, far below the chip's
// FLOP-per-byte ridge: the op is a stream over W at the HBM rate, and this kernel is shaped for that.
//
//   * A workgroup owns 128 output features and one slice of the reduction dimension (split-K: the
//     slices are what fills the chip, Hout / 128 tiles alone would not).  There are floor(CUs / tiles)
//     slices, never more workgroups than CUs: every slice writes and re-reads T x Hout partial sums, and
//     a CU with two workgroups would finish last.  The slice is walked in sub-slices: the sub-slice of
//     x = concat[e, f] for ALL tokens is copied into LDS (zero rows up to a multiple of 16 tokens), and
//     between two barriers the workgroup only streams W.  What reaches a CU besides W is the x slice,
//     T / 128 of the W bytes: a workgroup of 64 features measured 10% slower at 60 tokens for that reason.
//   * W never touches LDS: a weight is used by exactly one wavefront, once, for all tokens at a time.
//     out^T = W x^T runs on v_mfma_f32_16x16x32 (A = 16 W rows, B = 16 tokens), and a lane's A fragment
//     is 16 consecutive bytes of a W row, i.e. one global load straight into the operand registers.
//     The reduction index is permuted inside 128-element steps (lane group g takes elements
//     32 g .. 32 g + 31, eight per MFMA) so that the four loads of a step are 64 consecutive bytes per
//     lane and whole 256-byte runs per row; the B fragments are read from LDS with the same permutation.
//     Two steps of loads are in flight per wavefront while a step is multiplied.
//   * 8 wavefronts = 8 blocks of 16 features; the fp32 partial sums of the slice go to the workspace
//     [slices][T][Hout].  A second small kernel adds the slices in order (deterministic), adds the bias
//     and rounds to the storage type.
#include "mfma_common.h"

namespace s4c {

namespace {

using namespace mfma;

constexpr int kBO = 128;                // output features per workgroup: 16 per wavefront
constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kStepK = 128;             // reduction elements per step (4 MFMAs per token block)
constexpr int kMaxT = 128;
#ifndef S4C_DL_STREAM_MAX
#define S4C_DL_STREAM_MAX 512
#endif
constexpr int kLdsX = 128 * 1024;       // LDS for the x sub-slice: a CU holds one workgroup, so it may take most of the 160 KB
constexpr int kPadB = 16;               // row padding: 16 tokens x 16-byte reads hit 16 different bank groups

// reduction elements of x that fit in LDS at a time for this token count: whole steps
__host__ __device__ inline int sub_elems(int Tpad) {
    int n = kLdsX / (Tpad * 2) / kStepK * kStepK;
    return n < kStepK ? kStepK : n;
}

template <bool F16, int TB>            // TB: blocks of 16 tokens (1 .. 8)
__global__ __launch_bounds__(kThreads) void draft_linear_small_kernel(LinearArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int K = 2 * a.H, T = a.T;
    const int tile = blockIdx.x % a.otiles, slice = blockIdx.x / a.otiles;
    const int rowB = a.ksub * 2 + kPadB;                        // bytes per token row in LDS
    const int l16 = lane & 15, g = lane >> 4;
    const int o0 = tile * kBO + wave * 16;                       // this wave: features o0 .. o0+15
    const lds_u8* xl = (const lds_u8*)smem + l16 * rowB + g * 64;

    f32x4 acc[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[tb][j] = 0.f;

    const int kend = min(K, (slice + 1) * a.kslice);
    for (int k0 = slice * a.kslice; k0 < kend; k0 += a.ksub) {
        const int k1 = min(kend, k0 + a.ksub);
        const int klen = k1 - k0;                               // a multiple of 64 (H is a multiple of 32)
        const int s1 = (klen + kStepK - 1) / kStepK;            // steps of 128 reduction elements
        const unsigned char* wrow = (const unsigned char*)a.W + ((size_t)(o0 + l16) * K + k0) * 2 + g * 64;
        // a step's four A fragments: 64 consecutive bytes of this lane's W row; elements past the end of the
        // sub-slice (a last step that is not whole) are never loaded and count as zero
        auto load_step = [&](int s, uint4 (&w)[4]) {
            const int kb = s * kStepK + g * 32;                 // first element of this lane's run, relative to k0
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                w[q] = make_uint4(0, 0, 0, 0);
                if (kb + 8 * q < klen) w[q] = *(const uint4*)(wrow + (size_t)s * (kStepK * 2) + q * 16);
            }
        };
        auto mul_step = [&](int s, const uint4 (&w)[4]) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bf16x8 af = __builtin_bit_cast(bf16x8, w[q]);
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) {
                    const bf16x8 xf = *(const lds_bf16x8*)(xl + tb * 16 * rowB + s * (kStepK * 2) + q * 16);
                    acc[tb] = mma16<F16>(af, xf, acc[tb]);
                }
            }
        };
        // the first two steps of W are requested before x is copied: they need nothing from LDS
        uint4 wa[4], wb[4];
        load_step(0, wa);
        if (1 < s1) load_step(1, wb);

        // ---- x sub-slice -> LDS: [TB*16 tokens][ksub] 16-bit in 16-byte pieces; element k of x is e[k] or f[k-H]
        __syncthreads();                                        // the previous sub-slice is no longer read
        {
            // eight independent 16-byte loads per thread are in flight before the first is stored
            const int pieces = a.ksub / 8, total = TB * 16 * pieces;
            for (int i0 = tid; i0 < total; i0 += kThreads * 8) {
                uint4 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int i = i0 + u * kThreads;
                    const int t = i / pieces, p = i % pieces;
                    const int k = k0 + p * 8;
                    v[u] = make_uint4(0, 0, 0, 0);
                    if (i < total && t < T && k < k1) {
                        const uint16_t* src = (k < a.H) ? (const uint16_t*)a.e + (size_t)t * a.H + k
                                                        : (const uint16_t*)a.f + (size_t)t * a.H + (k - a.H);
                        v[u] = *(const uint4*)src;
                    }
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int i = i0 + u * kThreads;
                    if (i < total) *(uint4*)(smem + (size_t)(i / pieces) * rowB + (i % pieces) * 16) = v[u];
                }
            }
        }
        __syncthreads();

        for (int s = 0; s < s1; s += 2) {
            mul_step(s, wa);
            if (s + 2 < s1) load_step(s + 2, wa);
            if (s + 1 < s1) {
                mul_step(s + 1, wb);
                if (s + 3 < s1) load_step(s + 3, wb);
            }
        }
    }

    // accumulator block: lane holds features o0 + 4 g .. + 3 of token tb*16 + l16
    float* wsp = a.ws + (size_t)slice * T * a.Hout + o0 + 4 * g;
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        const int tok = tb * 16 + l16;
        if (tok < T) *(f32x4*)(wsp + (size_t)tok * a.Hout) = acc[tb];
    }
}

// out[t][o] = round(bias[o] + sum over slices, in slice order); one thread per 4 features of a token
template <bool F16>
__global__ __launch_bounds__(256) void draft_linear_reduce_kernel(LinearArgs a) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t per_row = (size_t)a.Hout / 4;
    if (i >= (size_t)a.T * per_row) return;
    const size_t t = i / per_row, o = (i % per_row) * 4;
    const size_t plane = (size_t)a.T * a.Hout;
    f32x4 s = *(const f32x4*)(a.ws + t * a.Hout + o);
    for (int sl = 1; sl < a.nslices; ++sl) s += *(const f32x4*)(a.ws + sl * plane + t * a.Hout + o);
    if (a.bias) {
        const uint16_t* bp = (const uint16_t*)a.bias + o;
#pragma unroll
        for (int u = 0; u < 4; ++u) s[u] += F16 ? (float)__builtin_bit_cast(_Float16, bp[u]) : bf16_to_f32(bp[u]);
    }
    uint2 pk;
    pk.x = round1<F16>(s[0]) | (round1<F16>(s[1]) << 16);
    pk.y = round1<F16>(s[2]) | (round1<F16>(s[3]) << 16);
    *(uint2*)((uint16_t*)a.out + t * a.Hout + o) = pk;
}

template <bool F16, int TB>
hipError_t launch_small(const LinearArgs& a, hipStream_t st) {
    static std::atomic<uint64_t> lds_set{0};
    const int lds = (TB * 16) * (a.ksub * 2 + kPadB);
    const int bytes = lds;
    const hipError_t ea = ensure_dynamic_lds((const void*)draft_linear_small_kernel<F16, TB>, kLdsX + kMaxT * kPadB, lds_set);
    if (ea != hipSuccess) return ea;
    hipLaunchKernelGGL((draft_linear_small_kernel<F16, TB>), dim3((unsigned)(a.otiles * a.nslices)), dim3(kThreads), bytes, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t n = (size_t)a.T * (a.Hout / 4);
    hipLaunchKernelGGL(draft_linear_reduce_kernel<F16>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, a);
    return hipGetLastError();
}

template <bool F16>
hipError_t launch_small_by_tokens(const LinearArgs& a, hipStream_t st) {
    switch ((a.T + 15) / 16) {
        case 1: return launch_small<F16, 1>(a, st);
        case 2: return launch_small<F16, 2>(a, st);
        case 3: return launch_small<F16, 3>(a, st);
        case 4: return launch_small<F16, 4>(a, st);
        case 5: return launch_small<F16, 5>(a, st);
        case 6: return launch_small<F16, 6>(a, st);
        case 7: return launch_small<F16, 7>(a, st);
        default: return launch_small<F16, 8>(a, st);
    }
}

}  // namespace

int draft_linear_small_max_tokens() { return kMaxT; }
int draft_linear_stream_max_tokens() { return S4C_DL_STREAM_MAX; }

// The split of the reduction dimension for this shape (a fixed function of the sizes and the CU count): as
// many slices as give every CU at most one workgroup, each a whole number of equal sub-slices that fit in LDS.
void draft_linear_small_plan(int T, int H, int Hout, int cus, int* ksub, int* kslice, int* nslices) {
    const int Tpad = (T + 15) / 16 * 16, K = 2 * H, otiles = Hout / kBO;
    const int unit = kStepK;
    int want = cus / otiles;
    if (want < 1) want = 1;
    const int target = ((K + want - 1) / want + unit - 1) / unit * unit;     // slice length that gives `want` slices
    const int cap = sub_elems(Tpad);
    const int subs = (target + cap - 1) / cap;
    *ksub = ((target + subs - 1) / subs + unit - 1) / unit * unit;
    *kslice = subs * *ksub;
    *nslices = (K + *kslice - 1) / *kslice;
}

hipError_t launch_draft_linear_small(const LinearArgs& a, hipStream_t st) {
    LinearArgs k = a;
    k.otiles = a.Hout / kBO;
    return a.dtype == S4C_F16 ? launch_small_by_tokens<true>(k, st) : launch_small_by_tokens<false>(k, st);
}

}  // namespace s4c
