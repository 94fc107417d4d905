// Input projection of a draft head (paper Eq. 3: h = Linear(concat[e, f])) on the CDNA4 matrix
// cores: out[t][o] = bias[o] + sum_k e[t][k] W[o][k] + sum_k f[t][k] W[o][H + k], bf16 in and
// out (fp16 likewise), fp32 accumulate.  The concatenation is never materialised: the K loop walks the first H
// columns of W against e and the last H against f.
//
//   * Both operands have the reduction index contiguous in memory (W is [Hout][2H], e and f are
//     [T][H]), which is what the matrix-core instruction wants for A and for B: a lane's 8 values
//     are 16 consecutive bytes of one row.  The product is formed transposed, D = W x^T (A = W
//     rows, B = token rows), so a lane ends up with 4 consecutive output features of one token
//     and stores them as one 8-byte word.
//   * v_mfma_f32_16x16x32_bf16 rather than the 32x32x16 shape: with random operands the chip is
//     power-limited and the smaller shape sustains a higher clock (measured 7 % faster here); the
//     wave tile keeps the LDS bytes per FLOP the same.
//   * Workgroup tile 256 output features x 256 tokens, K step 32; wave (wo, wt) of 8 owns
//     128 features x 64 tokens = 8 x 4 accumulator blocks of 16 x 16.  W and token tiles stream from HBM /
//     L2 straight into LDS (global_load_lds_dwordx4) through a ring of four 32 KB stages used in
//     pairs: one barrier per two K steps, the next pair in flight while a pair is multiplied.
//     (Four waves with 128 x 128 wave tiles, half the fragment reads per MFMA, measured slower.)
//   * A tile row is 64 bytes (four 16-byte chunks); chunk c of row r sits at chunk
//     c ^ ((r >> 1) & 3), applied on the global-address side of the direct-to-LDS load, so the
//     16-byte fragment reads of 8 consecutive rows fall into 8 different bank groups.
//   * The token tiles of one output-feature tile take consecutive slots of one XCD (workgroup id
//     modulo 8), so the W tile they all read is fetched from HBM once and shared through that L2.
#include "mfma_common.h"

namespace s4c {

namespace {

using namespace mfma;

constexpr int kBO = 256;                   // output features per workgroup
constexpr int kBT = 256;                   // tokens per workgroup
constexpr int kBK = 32;                    // reduction elements per stage
constexpr int kRow = kBK * 2;              // bytes per tile row
constexpr int kHalf = kBO * kRow;          // bytes of the W (or token) part of a stage: 16 KB
constexpr int kStage = 2 * kHalf;
constexpr int kNS = 4;
constexpr int kWaves = 8;
constexpr int kTB = 2;                     // token blocks (of 32) per wave
constexpr int kCH = 16 / kWaves;           // direct-to-LDS loads per wave and half-stage

template <bool F16>
__global__ __launch_bounds__(kWaves * 64) __attribute__((amdgpu_waves_per_eu(2, 2)))
void draft_linear_kernel(LinearArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_u8*)smem;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int team = a.ttiles;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int unit = (slot / team) * 8 + xcd;              // output-feature tile
    if (unit >= a.otiles) return;
    const int o0 = unit * kBO, t0 = (slot % team) * kBT;
    const int H = a.H, T = a.T;
    const size_t wrow = (size_t)2 * H * 2;                 // bytes per W row
    const size_t xrow = (size_t)H * 2;                     // bytes per e / f row

    // ---- direct-to-LDS loads: instruction ii of a half-stage covers rows 16 ii .. 16 ii + 15,
    // lane -> (row 16 ii + lane / 4, physical chunk lane % 4); a wave issues ii = wave, wave + 8
    uint32_t wo_off[kCH], xo_off[kCH];
#pragma unroll
    for (int c = 0; c < kCH; ++c) {
        const int row = 16 * (wave + kWaves * c) + (lane >> 2), pc = lane & 3;
        const int lc = pc ^ ((row >> 1) & 3);
        wo_off[c] = (uint32_t)((size_t)row * wrow) + lc * 16;
        xo_off[c] = (uint32_t)((size_t)min(t0 + row, T - 1) * xrow) + lc * 16;    // rows past T: clamped, never stored
    }
    const unsigned char* wbase = (const unsigned char*)a.W + (size_t)o0 * wrow;
    const int nk = 2 * H / kBK, nk_e = H / kBK;
    auto issue = [&](int kt) {
        const uint32_t sbase = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)(kt % kNS) * kStage + wave * 1024);
        const unsigned char* wg = uniform(wbase + (size_t)kt * kRow);
        const unsigned char* xg = uniform(kt < nk_e ? (const unsigned char*)a.e + (size_t)kt * kRow
                                                    : (const unsigned char*)a.f + (size_t)(kt - nk_e) * kRow);
#pragma unroll
        for (int c = 0; c < kCH; ++c) {
            dma16(wg, wo_off[c], sbase + kWaves * c * 1024);
            dma16(xg, xo_off[c], sbase + kWaves * c * 1024 + kHalf);
        }
    };

    // ---- fragment addresses inside a stage (v_mfma_f32_16x16x32_bf16: a lane supplies row lane % 16,
    // reduction elements 8 (lane / 16) .. + 7, i.e. chunk lane / 16 of the 64-byte row)
    const int wo = wave / (8 / kTB), wt = wave % (8 / kTB), g16 = lane >> 4, l16 = lane & 15;
    uint32_t w_off[8], x_off[2 * kTB];
#pragma unroll
    for (int ob = 0; ob < 8; ++ob) {
        const int row = wo * 128 + ob * 16 + l16;
        w_off[ob] = row * kRow + ((g16 ^ ((row >> 1) & 3)) << 4);
    }
#pragma unroll
    for (int tb = 0; tb < 2 * kTB; ++tb) {
        const int row = wt * (32 * kTB) + tb * 16 + l16;
        x_off[tb] = kHalf + row * kRow + ((g16 ^ ((row >> 1) & 3)) << 4);
    }

    f32x4 acc[8][2 * kTB];
#pragma unroll
    for (int ob = 0; ob < 8; ++ob)
#pragma unroll
        for (int tb = 0; tb < 2 * kTB; ++tb)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[ob][tb][j] = 0.f;

    // Two K steps per barrier: while the pair (kt, kt+1) is multiplied out of two ring stages, the
    // next pair streams into the other two.
    auto compute = [&](int kt) {
        const lds_u8* stage = (const lds_u8*)smem + (kt % kNS) * kStage;
        bf16x8 wf[8], xf[2 * kTB];
#pragma unroll
        for (int ob = 0; ob < 8; ++ob) wf[ob] = *(const lds_bf16x8*)(stage + w_off[ob]);
#pragma unroll
        for (int tb = 0; tb < 2 * kTB; ++tb) xf[tb] = *(const lds_bf16x8*)(stage + x_off[tb]);
#pragma unroll
        for (int ob = 0; ob < 8; ++ob)
#pragma unroll
            for (int tb = 0; tb < 2 * kTB; ++tb)
                acc[ob][tb] = mma16<F16>(wf[ob], xf[tb], acc[ob][tb]);
    };
    issue(0);
    issue(1);                                              // nk is even (nk = 2 H / 32)
    for (int kt = 0; kt < nk; kt += 2) {
        wait_vmcnt<0>();          // this wave's parts of the pair (kt, kt+1) have landed
        __syncthreads();          // everybody's have; the other two stages are free
        if (kt + 2 < nk) { issue(kt + 2); issue(kt + 3); }
        compute(kt);
        compute(kt + 1);
    }

    // ---- epilogue: per block a lane holds features 4 (lane / 16) .. + 3 of token lane % 16
    const uint16_t* bias = (const uint16_t*)a.bias;
    auto elem = [](uint16_t bits) { return F16 ? (float)__builtin_bit_cast(_Float16, bits) : bf16_to_f32(bits); };
#pragma unroll
    for (int tb = 0; tb < 2 * kTB; ++tb) {
        const int tok = t0 + wt * (32 * kTB) + tb * 16 + l16;
        if (tok >= T) continue;
        uint16_t* orow = (uint16_t*)a.out + (size_t)tok * a.Hout + o0 + wo * 128 + 4 * g16;
#pragma unroll
        for (int ob = 0; ob < 8; ++ob) {
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = acc[ob][tb][u];
            if (bias) {
                const uint16_t* bp = bias + o0 + wo * 128 + ob * 16 + 4 * g16;
#pragma unroll
                for (int u = 0; u < 4; ++u) v[u] += elem(bp[u]);
            }
            uint2 pk;
            pk.x = round1<F16>(v[0]) | (round1<F16>(v[1]) << 16);
            pk.y = round1<F16>(v[2]) | (round1<F16>(v[3]) << 16);
            *(uint2*)(orow + ob * 16) = pk;
        }
    }
}

}  // namespace

int draft_linear_tile_out() { return kBO; }
int draft_linear_tile_k() { return kBK; }

template <bool F16>
static hipError_t launch_linear(const LinearArgs& a, hipStream_t st) {
    constexpr int kLds = kNS * kStage;
    static std::atomic<uint64_t> lds_set{0};
    const hipError_t ea = ensure_dynamic_lds((const void*)draft_linear_kernel<F16>, kLds, lds_set);
    if (ea != hipSuccess) return ea;
    LinearArgs k = a;
    k.ttiles = (a.T + kBT - 1) / kBT;
    k.otiles = a.Hout / kBO;
    const long units8 = ((long)k.otiles + 7) / 8 * 8;      // padded to whole XCD rounds
    hipLaunchKernelGGL(draft_linear_kernel<F16>, dim3((unsigned)(units8 * k.ttiles)), dim3(kWaves * 64), kLds, st, k);
    return hipGetLastError();
}

hipError_t launch_draft_linear(const LinearArgs& a, hipStream_t st) {
    return a.dtype == S4C_F16 ? launch_linear<true>(a, st) : launch_linear<false>(a, st);
}

}  // namespace s4c
