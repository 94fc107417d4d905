// Internal declarations shared by the HIP translation units of libs4c (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "s4c.h"

namespace s4c {

constexpr int kMaxNodes = 128;
constexpr float kLog2e = 1.4426950408889634f;

typedef uint16_t bf16_t;   // raw bf16 bits
typedef _Float16 f16_t;    // IEEE binary16

__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x) << 16); }

// round-to-nearest-even; inputs are finite
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename T> __device__ __forceinline__ float to_f32(T x);
template <> __device__ __forceinline__ float to_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t x) { return bf16_to_f32(x); }
template <> __device__ __forceinline__ float to_f32<f16_t>(f16_t x) { return (float)x; }

template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return f32_to_bf16(x); }
template <> __device__ __forceinline__ f16_t from_f32<f16_t>(float x) { return (f16_t)x; }   // round to nearest even

// the two 16-bit elements of a 32-bit word (low half first), as floats
template <typename T> __device__ __forceinline__ void unpack2(uint32_t w, float& lo, float& hi);
template <> __device__ __forceinline__ void unpack2<bf16_t>(uint32_t w, float& lo, float& hi) {
    lo = __uint_as_float(w << 16);
    hi = __uint_as_float(w & 0xFFFF0000u);
}
template <> __device__ __forceinline__ void unpack2<f16_t>(uint32_t w, float& lo, float& hi) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    const h2 v = __builtin_bit_cast(h2, w);
    lo = (float)v[0];
    hi = (float)v[1];
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Arguments of the attention kernels.  Row r of the M = N*G query rows of one (sequence, KV
// head) is node r / G, group head r % G.
struct AttnArgs {
    const void* q;
    const void* k_tree;
    const void* v_tree;
    const void* k_cache;
    const void* v_cache;
    const int32_t* cache_len;
    const int32_t* parent;
    void* out;
    int32_t* status;
    float* ws_o;    // [B][Hkv][splits][M][D]  unnormalised partial outputs
    float* ws_ml;   // [B][Hkv][splits][M][2]  (running max in log2 units, running sum)
    int32_t B, Hq, Hkv, D, N, S_cap, G, M;
    int32_t max_cache_len;
    int32_t splits;   // KV splits; 1 => kernels write `out` directly
    int32_t chunk;    // prefix keys per split (multiple of the key tile)
    int32_t mtiles;   // query-row tiles per (sequence, KV head); set by the launcher
    float scale_log2; // softmax scale * log2(e)
    // paged cache (block_table != null): k_cache / v_cache are pools [num_pages][Hkv][page][D],
    // row j of sequence b is row j & (page-1) of page block_table[b][j >> page_shift]
    const int32_t* block_table;   // [B][max_blocks] or null
    int32_t max_blocks, page_shift, num_pages;
};

// launchers (defined in the kernel translation units); return hipGetLastError()
hipError_t launch_tree_attn_generic(const AttnArgs& a, int dtype, hipStream_t st);
hipError_t launch_tree_attn_mfma(const AttnArgs& a, int dtype, hipStream_t st);      // dtype: S4C_BF16 or S4C_F16
hipError_t launch_tree_attn_smallm(const AttnArgs& a, int dtype, hipStream_t st);   // M <= 64, called by the above
hipError_t launch_attn_merge(const AttnArgs& a, int dtype, hipStream_t st);
bool mfma_path_supported(const s4c_attn_shape& s);
int mfma_rows_per_block(const s4c_attn_shape& s);

struct AcceptArgs {
    const void* logits;
    const int32_t* parent;
    const int32_t* tokens;
    const float* p_draft;
    const float* uniforms;
    int32_t* path;
    int32_t* accept_len;
    int32_t* accepted_tokens;
    int32_t* bonus_token;
    int32_t* status;
    unsigned long long* rec;   // [B*N][nseg][3] (call nonce << 32) | bits of (max, argmax, sum of exponentials)
    uint32_t nonce;    // tells this call's records from whatever the words held before
    long long wait_ticks;   // how long a collector waits for its sequence's records (100 MHz wall clock)
    int32_t B, N, V, chunks, max_path, mode, dtype;
    int32_t seg, nseg; // chunks per workgroup, workgroups per row
    float inv_temp_log2;   // log2(e) / T
};
hipError_t launch_accept(const AcceptArgs& a, hipStream_t st);
int accept_chunk_elems();
void accept_plan(int B, int N, int V, int* chunks, int* seg, int* nseg);

struct ResampleArgs {
    const void* logits;
    const float* draft;        // [B][N][V]
    const int32_t* parent;
    const int32_t* tokens;
    const float* uniforms;     // [B][N]
    const float* u_resample;   // [B]
    int32_t* path;
    int32_t* accept_len;
    int32_t* accepted_tokens;
    int32_t* bonus_token;
    int32_t* status;
    uint64_t* slots;           // [B][max_pass][2][team] exchange words (team > 1)
    int32_t B, N, V, max_path, dtype;
    int32_t team;              // workgroups per sequence
    int32_t max_pass;          // exchanges a sequence may need
    int32_t spin_limit;        // polls before a workgroup gives up on an exchange
    double temperature;
};
hipError_t launch_accept_resample(const ResampleArgs& a, hipStream_t st);
int resample_max_vocab();
int resample_team(int B, int V);
int resample_max_pass(int N, int max_path);
int resample_default_spin_limit();
size_t resample_slot_words(int B, int N, int V, int max_path);

struct CompactArgs {
    const void* k_tree;
    const void* v_tree;
    void* k_cache;
    void* v_cache;
    int32_t* cache_len;
    const int32_t* path;
    const int32_t* accept_len;
    int32_t* dst_index;
    int32_t* status;
    int32_t B, Hkv, N, S_cap, max_path;
    int32_t row_bytes;   // D * element size
    const int32_t* block_table;   // paged cache: [B][max_blocks] (S_cap = max_blocks << page_shift), else null
    int32_t max_blocks, page_shift, num_pages;
};
hipError_t launch_compact(const CompactArgs& a, hipStream_t st);

struct BuildArgs {
    const void* logits;        // draft logits [B][N][V]
    const int32_t* nchild;     // [B][N]
    const int32_t* root_token; // [B]
    int32_t* parent;
    int32_t* tokens;
    float* p_draft;
    int32_t* level;            // nullable
    int32_t* status;           // nullable
    float* ws_max;             // [B*N][chunks]
    float* ws_sum;             // [B*N][chunks]
    float* ws_topv;            // [B*N][chunks][8]
    int32_t* ws_topi;          // [B*N][chunks][8]
    int32_t* row_tok;          // [B*N][8]
    float* row_p;              // [B*N][8]
    int32_t B, N, V, chunks, kmax, dtype;
    int32_t seg, nseg;         // chunks per workgroup of the scan, workgroups per row
    float inv_temp_log2;
};
hipError_t launch_build_tree(const BuildArgs& a, hipStream_t st);
int build_tree_max_children();
int build_tree_chunk_elems();

struct CommitArgs {
    const void* k_tree;        // [layers][B][N][Hkv][D]
    const void* v_tree;
    void* k_cache;             // [layers][B][Hkv][S_cap][D]
    void* v_cache;
    int32_t* cache_len;
    const int32_t* path;
    const int32_t* accept_len;
    const void* features;      // [B][N][feature_bytes] or null
    void* features_out;        // [B][max_path][feature_bytes] or null
    int32_t* dst_index;
    int32_t* status;
    size_t tree_layer_bytes, cache_layer_bytes;
    int32_t B, Hkv, N, S_cap, max_path, layers;
    int32_t row_bytes;         // D * element size
    int32_t feature_bytes;
    // paged pools (block_table != null): k_cache / v_cache are [layers][num_pages][Hkv][page][D], one
    // block table [B][max_blocks] serves every layer; S_cap = max_blocks << page_shift
    const int32_t* block_table;
    int32_t max_blocks, page_shift, num_pages;
};
hipError_t launch_commit(const CommitArgs& a, hipStream_t st);

struct LinearArgs {
    const void* e;       // [T][H] bf16 or fp16
    const void* f;       // [T][H]
    const void* W;       // [Hout][2H]
    const void* bias;    // [Hout] or null
    void* out;           // [T][Hout]
    float* ws;           // few-token path: [nslices][T][Hout] partial sums
    int32_t T, H, Hout, dtype;
    int32_t ttiles, otiles;   // set by the launcher
    int32_t ksub, kslice, nslices;   // few-token path: reduction elements per LDS fill, per workgroup, workgroups per tile
};
hipError_t launch_draft_linear(const LinearArgs& a, hipStream_t st);
hipError_t launch_draft_linear_small(const LinearArgs& a, hipStream_t st);   // T <= draft_linear_small_max_tokens()
int draft_linear_small_max_tokens();      // tokens per launch of the weight-streaming kernel
int draft_linear_stream_max_tokens();     // token count up to which the entry point uses it (in passes)
void draft_linear_small_plan(int T, int H, int Hout, int cus, int* ksub, int* kslice, int* nslices);
int draft_linear_tile_out();
int draft_linear_tile_k();

}  // namespace s4c
