// C ABI of libs4c: argument checks, launch planning, kernel launches.  See include/s4c.h.
#include "common.h"

#include <math.h>
#include <stdlib.h>

#include <atomic>

using namespace s4c;

// Scratch of s4c_accept_path_static: one copy per GPU that loads the library, held until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress; the device address of each
// GPU's copy is looked up once per device (static_scratch) and that pointer is what kernels receive.
static __device__ __align__(256) unsigned char scratch[S4C_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;

// Compute units of the current device (sizes the attention launch plan); the MI355X's 256 when no
// device can be asked (size queries on a host without a GPU).
int device_cus() {
    static std::atomic<int> cached[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n <= 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// Device address of the current GPU's copy of `scratch`.
hipError_t static_scratch(void** out) {
    static std::atomic<void*> addr[kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void* p = addr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        addr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return hipSuccess;
}

bool aligned16(const void* p) { return (((uintptr_t)p) & 15) == 0; }

// A different number for every acceptance call of the process (the records of a workspace tell this
// call's statistics from older contents by it).  Never 0 or ~0: freshly allocated memory is often all
// zeros, which must read as "no record yet", and ~nonce marks a consumed record.
uint32_t next_nonce() {
    static std::atomic<uint32_t> counter{0};
    for (;;) {
        uint32_t x = counter.fetch_add(1, std::memory_order_relaxed) + 0x9E3779B9u;
        x ^= x >> 16; x *= 0x7FEB352Du; x ^= x >> 15; x *= 0x846CA68Bu; x ^= x >> 16;      // a bijection of 32-bit words
        if (x != 0u && x != 0xFFFFFFFFu) return x;
    }
}

bool dtype_ok(int32_t d) { return d == S4C_F32 || d == S4C_BF16 || d == S4C_F16; }

bool shape_ok(const s4c_attn_shape* s, s4c_status* why) {
    if (s->B <= 0 || s->Hq <= 0 || s->Hkv <= 0 || s->D <= 0 || s->N <= 0 || s->S_cap < 0 ||
        s->Hq % s->Hkv != 0) {
        *why = S4C_ERR_SHAPE;
        return false;
    }
    if (s->N > kMaxNodes || (s->D != 64 && s->D != 128) || !dtype_ok(s->dtype) ||
        s->B > 65535 || s->Hkv > 65535) {
        *why = S4C_ERR_UNSUPPORTED;
        return false;
    }
    return true;
}

struct AttnPlan {
    bool mfma;
    int splits;
    int chunk;
    size_t ws_o_bytes, ws_ml_bytes;
};

// Fixed function of (shape, max_cache_len): the same inputs always get the same split count
// and therefore bit-identical results.
AttnPlan plan_attn(const s4c_attn_shape& s, int32_t max_cache_len) {
    AttnPlan p;
    p.mfma = mfma_path_supported(s);
    const int M = s.N * (s.Hq / s.Hkv);
    const int rows = p.mfma ? mfma_rows_per_block(s) : 32;
    const long mtiles = (M + rows - 1) / rows;
    const long units = (long)s.B * s.Hkv * mtiles;
    // Balance unit: the device's CUs (256 on an MI355X) for the matrix-core kernels (HBM- or MFMA-bound: what counts is
    // an equal share of work per CU), four workgroups per CU for the scalar kernel.  Split the prefix so that the launch fills
    // whole rounds of the CUs without paying for more partial results than that needs:
    // cost(s) = rounds * slots / workgroups * (1 + 4 % per extra split), chunks a multiple of 128 keys
    // (32, its key tile, for the scalar kernel, whose launches are latency-bound).
    const long slots = (long)device_cus() * (p.mfma ? 1 : 4);
    const long gran = p.mfma ? 128 : 32;
    // at least 256 keys per split for the matrix-core kernels: below that a split's fixed costs (prologue, partial
    // results, its share of the merge) outweigh what the extra workgroups stream (1024 keys, 32 units: 4 splits
    // measured 7 % faster than 8)
    long max_splits = max_cache_len / (p.mfma ? 256 : 32);
    if (max_splits > 16) max_splits = 16;
    if (max_splits < 1) max_splits = 1;
    long splits = 1;
    double best = 1e30;
    for (long sp = 1; sp <= max_splits; ++sp) {
        const long wgs = units * sp, rounds = (wgs + slots - 1) / slots;
        const double cost = (double)(rounds * slots) / (double)wgs * (1.0 + 0.04 * (double)(sp - 1));
        if (cost < best - 1e-9) { best = cost; splits = sp; }
    }
    long chunk = (max_cache_len + splits - 1) / splits;
    chunk = ((chunk + gran - 1) / gran) * gran;
    if (chunk < gran) chunk = gran;
    splits = (max_cache_len + chunk - 1) / chunk;
    if (splits < 1) splits = 1;
    p.splits = (int)splits;
    p.chunk = (int)chunk;
    if (p.splits == 1) {
        p.ws_o_bytes = p.ws_ml_bytes = 0;
    } else {
        const size_t prow = (size_t)s.B * s.Hkv * p.splits * M;
        p.ws_o_bytes = prow * s.D * sizeof(float);
        p.ws_ml_bytes = ((prow * 2 * sizeof(float) + 255) / 256) * 256;
    }
    return p;
}

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

const char* s4c_strerror(int code) {
    switch (code) {
        case S4C_OK: return "ok";
        case S4C_ERR_NULL: return "a required pointer is NULL";
        case S4C_ERR_SHAPE: return "non-positive or inconsistent sizes";
        case S4C_ERR_UNSUPPORTED: return "unsupported size, dtype or mode (N <= 128, D in {64,128})";
        case S4C_ERR_WORKSPACE: return "workspace missing or too small";
        case S4C_ERR_HIP: return "HIP kernel launch failed";
        case S4C_ERR_STATIC_SCRATCH: return "problem larger than the static scratch of s4c_accept_path_static";
    }
    return "unknown status";
}

size_t s4c_tree_attn_workspace_size(const s4c_attn_shape* shape, int32_t max_cache_len) {
    s4c_status why;
    if (!shape || !shape_ok(shape, &why) || max_cache_len < 0) return 0;
    const AttnPlan p = plan_attn(*shape, max_cache_len);
    return p.ws_o_bytes + p.ws_ml_bytes;
}

int32_t s4c_tree_attn_num_splits(const s4c_attn_shape* shape, int32_t max_cache_len) {
    s4c_status why;
    if (!shape || !shape_ok(shape, &why) || max_cache_len < 0) return 0;
    return plan_attn(*shape, max_cache_len).splits;
}

#pragma GCC visibility pop
}  // extern "C"

namespace {
// log2 of a page size that is a power of two >= 64, else -1
int page_shift_of(int32_t page_size) {
    for (int sh = 6; sh < 31; ++sh)
        if (page_size == (1 << sh)) return sh;
    return -1;
}

s4c_status tree_attn_impl(const s4c_attn_shape* shape, const void* q, const void* k_tree, const void* v_tree,
                          const void* k_cache, const void* v_cache, const int32_t* block_table, int32_t max_blocks,
                          int32_t page_shift, int32_t num_pages, const int32_t* cache_len, const int32_t* parent,
                          int32_t max_cache_len, float scale, void* out, int32_t* status, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
    if (!shape || !q || !k_tree || !v_tree || !cache_len || !parent || !out) return S4C_ERR_NULL;
    s4c_status why;
    if (!shape_ok(shape, &why)) return why;
    if (max_cache_len < 0 || max_cache_len > shape->S_cap) return S4C_ERR_SHAPE;
    if (max_cache_len > 0 && (!k_cache || !v_cache)) return S4C_ERR_NULL;
    if (!aligned16(q) || !aligned16(k_tree) || !aligned16(v_tree) || !aligned16(k_cache) || !aligned16(v_cache) ||
        !aligned16(out))
        return S4C_ERR_SHAPE;
    const AttnPlan p = plan_attn(*shape, max_cache_len);
    const size_t need = p.ws_o_bytes + p.ws_ml_bytes;
    if (need > 0 && (!workspace || workspace_bytes < need || (((uintptr_t)workspace) & 255))) return S4C_ERR_WORKSPACE;

    AttnArgs a;
    a.q = q; a.k_tree = k_tree; a.v_tree = v_tree; a.k_cache = k_cache; a.v_cache = v_cache;
    a.cache_len = cache_len; a.parent = parent; a.out = out; a.status = status;
    a.ws_ml = (float*)workspace;
    a.ws_o = (float*)((char*)workspace + p.ws_ml_bytes);
    a.B = shape->B; a.Hq = shape->Hq; a.Hkv = shape->Hkv; a.D = shape->D; a.N = shape->N;
    a.S_cap = shape->S_cap; a.G = shape->Hq / shape->Hkv; a.M = a.N * a.G;
    a.max_cache_len = max_cache_len; a.splits = p.splits; a.chunk = p.chunk;
    a.scale_log2 = (scale > 0.f ? scale : 1.0f / sqrtf((float)shape->D)) * kLog2e;
    a.block_table = block_table; a.max_blocks = max_blocks; a.page_shift = page_shift; a.num_pages = num_pages;

    hipStream_t st = (hipStream_t)hip_stream;
    // Splits are combined by a second kernel: the kernel boundary is what makes one workgroup's
    // partial results visible to another across the chip's separate L2s at no extra cost.
    hipError_t e = p.mfma ? launch_tree_attn_mfma(a, shape->dtype, st) : launch_tree_attn_generic(a, shape->dtype, st);
    if (e == hipSuccess && p.splits > 1) e = launch_attn_merge(a, shape->dtype, st);
    return e == hipSuccess ? S4C_OK : S4C_ERR_HIP;
}
}  // namespace

extern "C" {
#pragma GCC visibility push(default)

s4c_status s4c_tree_attn(const s4c_attn_shape* shape, const void* q, const void* k_tree,
                         const void* v_tree, const void* k_cache, const void* v_cache,
                         const int32_t* cache_len, const int32_t* parent, int32_t max_cache_len,
                         float scale, void* out, int32_t* status, void* workspace,
                         size_t workspace_bytes, void* hip_stream) {
    return tree_attn_impl(shape, q, k_tree, v_tree, k_cache, v_cache, nullptr, 0, 0, 0, cache_len, parent, max_cache_len,
                          scale, out, status, workspace, workspace_bytes, hip_stream);
}

s4c_status s4c_tree_attn_paged(const s4c_attn_shape* shape, const void* q, const void* k_tree, const void* v_tree,
                               const void* k_pool, const void* v_pool, const int32_t* block_table,
                               int32_t max_blocks, int32_t page_size, int32_t num_pages, const int32_t* cache_len,
                               const int32_t* parent, int32_t max_cache_len, float scale, void* out,
                               int32_t* status, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!shape || !block_table || !k_pool || !v_pool) return S4C_ERR_NULL;
    const int sh = page_shift_of(page_size);
    if (sh < 0) return S4C_ERR_UNSUPPORTED;
    if (max_blocks <= 0 || num_pages <= 0 || (long long)max_blocks * page_size > 0x7FFFFFFFll) return S4C_ERR_SHAPE;
    if (shape->S_cap != max_blocks * page_size) return S4C_ERR_SHAPE;       // the logical capacity of a sequence
    return tree_attn_impl(shape, q, k_tree, v_tree, k_pool, v_pool, block_table, max_blocks, sh, num_pages, cache_len,
                          parent, max_cache_len, scale, out, status, workspace, workspace_bytes, hip_stream);
}

size_t s4c_accept_path_workspace_size(int32_t B, int32_t N, int32_t V) {
    if (B <= 0 || N <= 0 || V <= 0) return 0;
    int chunks, seg, nseg;
    accept_plan(B, N, V, &chunks, &seg, &nseg);
    return (((size_t)B * N * nseg * 3 * sizeof(unsigned long long) + 255) / 256) * 256;   // three records per (row, segment)
}

#pragma GCC visibility pop
}  // extern "C"

namespace {
// checks shared by the two acceptance entry points; everything but the workspace
s4c_status accept_args_ok(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, int32_t mode, float temperature,
                          const void* logits, const int32_t* parent, const int32_t* tokens, const float* p_draft,
                          const float* uniforms, int32_t max_path, int32_t* path, int32_t* accept_len,
                          int32_t* accepted_tokens, int32_t* bonus_token) {
    if (!logits || !parent || !tokens || !path || !accept_len || !accepted_tokens || !bonus_token)
        return S4C_ERR_NULL;
    if (B <= 0 || N <= 0 || V <= 0 || max_path <= 0) return S4C_ERR_SHAPE;
    if (N > kMaxNodes || !dtype_ok(logits_dtype) ||
        (mode != S4C_GREEDY && mode != S4C_STOCHASTIC))
        return S4C_ERR_UNSUPPORTED;
    if (mode == S4C_STOCHASTIC) {
        if (!p_draft || !uniforms) return S4C_ERR_NULL;
        if (!(temperature > 0.f)) return S4C_ERR_SHAPE;
    }
    int chunks, seg, nseg;
    accept_plan(B, N, V, &chunks, &seg, &nseg);
    if ((size_t)B * N * nseg > 0x7FFFFFFFull) return S4C_ERR_UNSUPPORTED;
    return S4C_OK;
}

// `workspace` holds at least s4c_accept_path_workspace_size(B, N, V) bytes, 256-byte aligned
s4c_status accept_launch(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, int32_t mode, float temperature,
                         const void* logits, const int32_t* parent, const int32_t* tokens, const float* p_draft,
                         const float* uniforms, int32_t max_path, int32_t* path, int32_t* accept_len,
                         int32_t* accepted_tokens, int32_t* bonus_token, int32_t* status, void* workspace,
                         void* hip_stream) {
    AcceptArgs a;
    a.logits = logits; a.parent = parent; a.tokens = tokens; a.p_draft = p_draft; a.uniforms = uniforms;
    a.path = path; a.accept_len = accept_len; a.accepted_tokens = accepted_tokens;
    a.bonus_token = bonus_token; a.status = status;
    a.rec = (unsigned long long*)workspace;
    a.nonce = next_nonce();
    // S4C_ACCEPT_WAIT_US (environment, >= 0): how long a sequence's collecting workgroup waits for the
    // statistics of the others before it flags the sequence.  A diagnostic knob: 0 makes a collector that
    // does not find everything at its first look give up, which exercises the flagged path on a healthy GPU.
    long long wait_us = 2000000;
    if (const char* env = getenv("S4C_ACCEPT_WAIT_US")) {
        char* end = nullptr;
        const long long v = strtoll(env, &end, 10);
        if (end != env && v >= 0 && v <= 60000000ll) wait_us = v;
    }
    a.wait_ticks = wait_us * 100;
    a.B = B; a.N = N; a.V = V;
    accept_plan(B, N, V, &a.chunks, &a.seg, &a.nseg);
    a.max_path = max_path; a.mode = mode; a.dtype = logits_dtype;
    a.inv_temp_log2 = kLog2e / (mode == S4C_STOCHASTIC ? temperature : 1.0f);
    return launch_accept(a, (hipStream_t)hip_stream) == hipSuccess ? S4C_OK : S4C_ERR_HIP;
}
}  // namespace

extern "C" {
#pragma GCC visibility push(default)

s4c_status s4c_accept_path(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, int32_t mode,
                           float temperature, const void* logits, const int32_t* parent,
                           const int32_t* tokens, const float* p_draft, const float* uniforms,
                           int32_t max_path, int32_t* path, int32_t* accept_len,
                           int32_t* accepted_tokens, int32_t* bonus_token, int32_t* status,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
    const s4c_status ok = accept_args_ok(B, N, V, logits_dtype, mode, temperature, logits, parent, tokens, p_draft, uniforms,
                                         max_path, path, accept_len, accepted_tokens, bonus_token);
    if (ok != S4C_OK) return ok;
    const size_t need = s4c_accept_path_workspace_size(B, N, V);
    if (!workspace || workspace_bytes < need || (((uintptr_t)workspace) & 255)) return S4C_ERR_WORKSPACE;
    return accept_launch(B, N, V, logits_dtype, mode, temperature, logits, parent, tokens, p_draft, uniforms, max_path, path,
                         accept_len, accepted_tokens, bonus_token, status, workspace, hip_stream);
}

s4c_status s4c_accept_path_static(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, int32_t mode,
                                  float temperature, const void* logits, const int32_t* parent,
                                  const int32_t* tokens, const float* p_draft, const float* uniforms,
                                  int32_t max_path, int32_t* path, int32_t* accept_len,
                                  int32_t* accepted_tokens, int32_t* bonus_token, int32_t* status,
                                  void* hip_stream) {
    const s4c_status ok = accept_args_ok(B, N, V, logits_dtype, mode, temperature, logits, parent, tokens, p_draft, uniforms,
                                         max_path, path, accept_len, accepted_tokens, bonus_token);
    if (ok != S4C_OK) return ok;
    if (s4c_accept_path_workspace_size(B, N, V) > (size_t)S4C_STATIC_SCRATCH_BYTES) return S4C_ERR_STATIC_SCRATCH;
    void* ws = nullptr;
    if (static_scratch(&ws) != hipSuccess) return S4C_ERR_HIP;
    return accept_launch(B, N, V, logits_dtype, mode, temperature, logits, parent, tokens, p_draft, uniforms, max_path, path,
                         accept_len, accepted_tokens, bonus_token, status, ws, hip_stream);
}

size_t s4c_accept_resample_workspace_size(int32_t B, int32_t N, int32_t V, int32_t max_path) {
    if (B <= 0 || N <= 0 || V <= 0 || max_path <= 0 || N > kMaxNodes || V > resample_max_vocab()) return 0;
    return resample_slot_words(B, N, V, max_path) * sizeof(uint64_t);
}

s4c_status s4c_accept_resample(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, float temperature,
                               const void* logits, const float* draft_probs, const int32_t* parent,
                               const int32_t* tokens, const float* uniforms, const float* u_resample,
                               int32_t max_path, int32_t* path, int32_t* accept_len,
                               int32_t* accepted_tokens, int32_t* bonus_token, int32_t* status,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!logits || !draft_probs || !parent || !tokens || !uniforms || !u_resample || !path || !accept_len ||
        !accepted_tokens || !bonus_token)
        return S4C_ERR_NULL;
    if (B <= 0 || N <= 0 || V <= 0 || max_path <= 0 || !(temperature > 0.f)) return S4C_ERR_SHAPE;
    if (N > kMaxNodes || V > resample_max_vocab() || !dtype_ok(logits_dtype))
        return S4C_ERR_UNSUPPORTED;
    const size_t need = s4c_accept_resample_workspace_size(B, N, V, max_path);
    if (need > 0 && (!workspace || workspace_bytes < need || (((uintptr_t)workspace) & 255))) return S4C_ERR_WORKSPACE;
    ResampleArgs a;
    a.logits = logits; a.draft = draft_probs; a.parent = parent; a.tokens = tokens; a.uniforms = uniforms;
    a.u_resample = u_resample; a.path = path; a.accept_len = accept_len; a.accepted_tokens = accepted_tokens;
    a.bonus_token = bonus_token; a.status = status; a.slots = (uint64_t*)workspace;
    a.B = B; a.N = N; a.V = V; a.max_path = max_path; a.dtype = logits_dtype; a.temperature = (double)temperature;
    a.team = resample_team(B, V);
    a.max_pass = resample_max_pass(N, max_path);
    // S4C_RESAMPLE_SPIN_LIMIT (environment, >= 0): polls before a workgroup gives up on an exchange.  A
    // diagnostic knob: 0 makes every exchange between several workgroups fail, which is how the give-up
    // path is exercised without a stuck GPU.
    a.spin_limit = resample_default_spin_limit();
    if (const char* env = getenv("S4C_RESAMPLE_SPIN_LIMIT")) {
        char* end = nullptr;
        const long v = strtol(env, &end, 10);
        if (end != env && v >= 0 && v <= 0x7FFFFFFFl) a.spin_limit = (int32_t)v;
    }
    return launch_accept_resample(a, (hipStream_t)hip_stream) == hipSuccess ? S4C_OK : S4C_ERR_HIP;
}

s4c_status s4c_kv_compact(const s4c_attn_shape* shape, const void* k_tree, const void* v_tree,
                          void* k_cache, void* v_cache, int32_t* cache_len, const int32_t* path,
                          const int32_t* accept_len, int32_t max_path, int32_t* dst_index,
                          int32_t* status, void* hip_stream) {
    if (!shape || !k_tree || !v_tree || !k_cache || !v_cache || !cache_len || !path || !accept_len)
        return S4C_ERR_NULL;
    s4c_attn_shape s = *shape;
    if (s.Hq <= 0) s.Hq = s.Hkv;          // Hq is not used by this call
    if (s.Hkv > 0 && s.Hq % s.Hkv != 0) s.Hq = s.Hkv;
    s4c_status why;
    if (!shape_ok(&s, &why)) return why;
    if (max_path <= 0 || s.S_cap <= 0) return S4C_ERR_SHAPE;

    CompactArgs a;
    a.k_tree = k_tree; a.v_tree = v_tree; a.k_cache = k_cache; a.v_cache = v_cache;
    a.cache_len = cache_len; a.path = path; a.accept_len = accept_len; a.dst_index = dst_index;
    a.status = status; a.B = s.B; a.Hkv = s.Hkv; a.N = s.N; a.S_cap = s.S_cap; a.max_path = max_path;
    a.row_bytes = s.D * (s.dtype == S4C_F32 ? 4 : 2);
    a.block_table = nullptr; a.max_blocks = a.page_shift = a.num_pages = 0;
    return launch_compact(a, (hipStream_t)hip_stream) == hipSuccess ? S4C_OK : S4C_ERR_HIP;
}

s4c_status s4c_kv_compact_paged(const s4c_attn_shape* shape, const void* k_tree, const void* v_tree, void* k_pool,
                                void* v_pool, const int32_t* block_table, int32_t max_blocks, int32_t page_size,
                                int32_t num_pages, int32_t* cache_len, const int32_t* path,
                                const int32_t* accept_len, int32_t max_path, int32_t* dst_index, int32_t* status,
                                void* hip_stream) {
    if (!shape || !k_tree || !v_tree || !k_pool || !v_pool || !block_table || !cache_len || !path || !accept_len)
        return S4C_ERR_NULL;
    const int sh = page_shift_of(page_size);
    if (sh < 0) return S4C_ERR_UNSUPPORTED;
    if (max_blocks <= 0 || num_pages <= 0 || (long long)max_blocks * page_size > 0x7FFFFFFFll) return S4C_ERR_SHAPE;
    s4c_attn_shape s = *shape;
    s.S_cap = max_blocks * page_size;
    if (s.Hq <= 0) s.Hq = s.Hkv;
    if (s.Hkv > 0 && s.Hq % s.Hkv != 0) s.Hq = s.Hkv;
    s4c_status why;
    if (!shape_ok(&s, &why)) return why;
    if (max_path <= 0) return S4C_ERR_SHAPE;
    CompactArgs a;
    a.k_tree = k_tree; a.v_tree = v_tree; a.k_cache = k_pool; a.v_cache = v_pool;
    a.cache_len = cache_len; a.path = path; a.accept_len = accept_len; a.dst_index = dst_index;
    a.status = status; a.B = s.B; a.Hkv = s.Hkv; a.N = s.N; a.S_cap = s.S_cap; a.max_path = max_path;
    a.row_bytes = s.D * (s.dtype == S4C_F32 ? 4 : 2);
    a.block_table = block_table; a.max_blocks = max_blocks; a.page_shift = sh; a.num_pages = num_pages;
    return launch_compact(a, (hipStream_t)hip_stream) == hipSuccess ? S4C_OK : S4C_ERR_HIP;
}

#pragma GCC visibility pop
}  // extern "C"

namespace {
struct BuildLayout { size_t chunks, off_sum, off_topv, off_topi, off_tok, off_p, total; };
BuildLayout build_layout(int32_t B, int32_t N, int32_t V) {
    BuildLayout l;
    l.chunks = ((size_t)V + build_tree_chunk_elems() - 1) / build_tree_chunk_elems();
    const size_t rows = (size_t)B * N, K = (size_t)build_tree_max_children();
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    size_t o = 0;
    const size_t parts = l.chunks * 4;            // every wavefront of the scan reports its quarter of a chunk
    o += up(rows * parts * 4); l.off_sum = o;
    o += up(rows * parts * 4); l.off_topv = o;
    o += up(rows * parts * K * 4); l.off_topi = o;
    o += up(rows * parts * K * 4); l.off_tok = o;
    o += up(rows * K * 4); l.off_p = o;
    o += up(rows * K * 4); l.total = o;
    return l;
}
}  // namespace

extern "C" {
#pragma GCC visibility push(default)

size_t s4c_build_tree_workspace_size(int32_t B, int32_t N, int32_t V) {
    if (B <= 0 || N <= 0 || V <= 0) return 0;
    return build_layout(B, N, V).total;
}

s4c_status s4c_build_tree(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, float temperature,
                          const void* draft_logits, const int32_t* nchild, const int32_t* root_token,
                          int32_t kmax, int32_t* parent, int32_t* tokens, float* p_draft, int32_t* level,
                          int32_t* status, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!draft_logits || !nchild || !root_token || !parent || !tokens || !p_draft) return S4C_ERR_NULL;
    if (B <= 0 || N <= 0 || V <= 0 || kmax <= 0 || !(temperature > 0.f)) return S4C_ERR_SHAPE;
    if (N > kMaxNodes || kmax > build_tree_max_children() || !dtype_ok(logits_dtype))
        return S4C_ERR_UNSUPPORTED;
    const BuildLayout l = build_layout(B, N, V);
    if ((size_t)B * N * l.chunks * 4 * (size_t)build_tree_max_children() > 0x7FFFFFFFull) return S4C_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < l.total || (((uintptr_t)workspace) & 255)) return S4C_ERR_WORKSPACE;
    BuildArgs a;
    a.logits = draft_logits; a.nchild = nchild; a.root_token = root_token; a.parent = parent; a.tokens = tokens;
    a.p_draft = p_draft; a.level = level; a.status = status;
    char* w = (char*)workspace;
    a.ws_max = (float*)w; a.ws_sum = (float*)(w + l.off_sum); a.ws_topv = (float*)(w + l.off_topv);
    a.ws_topi = (int32_t*)(w + l.off_topi); a.row_tok = (int32_t*)(w + l.off_tok); a.row_p = (float*)(w + l.off_p);
    a.B = B; a.N = N; a.V = V; a.chunks = (int32_t)l.chunks; a.kmax = kmax; a.dtype = logits_dtype;
    {   // segments as in the acceptance scan (same chunk size, same sizes of launch)
        int chunks_ = 0;
        accept_plan(B, N, V, &chunks_, &a.seg, &a.nseg);
    }
    a.inv_temp_log2 = kLog2e / temperature;
    return launch_build_tree(a, (hipStream_t)hip_stream) == hipSuccess ? S4C_OK : S4C_ERR_HIP;
}

#pragma GCC visibility pop
}  // extern "C"

namespace {
s4c_status commit_impl(const s4c_attn_shape* shape, int32_t layers, const void* k_tree, const void* v_tree,
                       void* k_cache, void* v_cache, const int32_t* block_table, int32_t max_blocks, int32_t page_shift,
                       int32_t num_pages, int32_t* cache_len, const int32_t* path, const int32_t* accept_len,
                       int32_t max_path, const void* features, int32_t feature_bytes, void* features_out,
                       int32_t* dst_index, int32_t* status, void* hip_stream) {
    if (!shape || !k_tree || !v_tree || !k_cache || !v_cache || !cache_len || !path || !accept_len)
        return S4C_ERR_NULL;
    s4c_attn_shape s = *shape;
    if (block_table) s.S_cap = max_blocks << page_shift;
    if (s.Hq <= 0) s.Hq = s.Hkv;          // Hq is not used by this call
    if (s.Hkv > 0 && s.Hq % s.Hkv != 0) s.Hq = s.Hkv;
    s4c_status why;
    if (!shape_ok(&s, &why)) return why;
    if (max_path <= 0 || s.S_cap <= 0 || layers <= 0 || layers > 65534) return S4C_ERR_SHAPE;
    const bool feats = features || features_out;
    if (feats) {
        if (!features || !features_out) return S4C_ERR_NULL;
        if (feature_bytes <= 0 || feature_bytes % 16 != 0) return S4C_ERR_SHAPE;
        if ((((uintptr_t)features) | ((uintptr_t)features_out)) & 15) return S4C_ERR_SHAPE;
    }
    CommitArgs a;
    a.k_tree = k_tree; a.v_tree = v_tree; a.k_cache = k_cache; a.v_cache = v_cache; a.cache_len = cache_len;
    a.path = path; a.accept_len = accept_len; a.features = features; a.features_out = features_out;
    a.dst_index = dst_index; a.status = status;
    a.B = s.B; a.Hkv = s.Hkv; a.N = s.N; a.S_cap = s.S_cap; a.max_path = max_path; a.layers = layers;
    a.row_bytes = s.D * (s.dtype == S4C_F32 ? 4 : 2);
    a.feature_bytes = feats ? feature_bytes : 0;
    a.tree_layer_bytes = (size_t)s.B * s.N * s.Hkv * a.row_bytes;
    a.cache_layer_bytes = block_table ? (((size_t)num_pages * s.Hkv) << page_shift) * a.row_bytes
                                      : (size_t)s.B * s.Hkv * s.S_cap * a.row_bytes;
    a.block_table = block_table; a.max_blocks = max_blocks; a.page_shift = page_shift; a.num_pages = num_pages;
    return launch_commit(a, (hipStream_t)hip_stream) == hipSuccess ? S4C_OK : S4C_ERR_HIP;
}
}  // namespace

extern "C" {
#pragma GCC visibility push(default)

s4c_status s4c_commit_path(const s4c_attn_shape* shape, int32_t layers, const void* k_tree, const void* v_tree,
                           void* k_cache, void* v_cache, int32_t* cache_len, const int32_t* path,
                           const int32_t* accept_len, int32_t max_path, const void* features,
                           int32_t feature_bytes, void* features_out, int32_t* dst_index, int32_t* status,
                           void* hip_stream) {
    return commit_impl(shape, layers, k_tree, v_tree, k_cache, v_cache, nullptr, 0, 0, 0, cache_len, path, accept_len,
                       max_path, features, feature_bytes, features_out, dst_index, status, hip_stream);
}

s4c_status s4c_commit_path_paged(const s4c_attn_shape* shape, int32_t layers, const void* k_tree, const void* v_tree,
                                 void* k_pool, void* v_pool, const int32_t* block_table, int32_t max_blocks,
                                 int32_t page_size, int32_t num_pages, int32_t* cache_len, const int32_t* path,
                                 const int32_t* accept_len, int32_t max_path, const void* features,
                                 int32_t feature_bytes, void* features_out, int32_t* dst_index, int32_t* status,
                                 void* hip_stream) {
    if (!block_table) return S4C_ERR_NULL;
    const int sh = page_shift_of(page_size);
    if (sh < 0) return S4C_ERR_UNSUPPORTED;
    if (max_blocks <= 0 || num_pages <= 0 || (long long)max_blocks * page_size > 0x7FFFFFFFll) return S4C_ERR_SHAPE;
    return commit_impl(shape, layers, k_tree, v_tree, k_pool, v_pool, block_table, max_blocks, sh, num_pages, cache_len,
                       path, accept_len, max_path, features, feature_bytes, features_out, dst_index, status, hip_stream);
}

size_t s4c_draft_linear_workspace_size(int32_t T, int32_t H, int32_t Hout) {
    if (T <= 0 || H <= 0 || Hout <= 0 || T > draft_linear_stream_max_tokens() || H % draft_linear_tile_k() != 0 ||
        Hout % draft_linear_tile_out() != 0)
        return 0;
    // the largest need of any pass (passes as in s4c_draft_linear: equal sizes, the last one may be shorter)
    const int step = draft_linear_small_max_tokens();
    const int passes = (T + step - 1) / step, per = (T + passes - 1) / passes;
    size_t need = 0;
    for (int t0 = 0; t0 < T; t0 += per) {
        const int Tp = T - t0 < per ? T - t0 : per;
        int ksub, kslice, nslices;
        draft_linear_small_plan(Tp, H, Hout, device_cus(), &ksub, &kslice, &nslices);
        const size_t b = (size_t)nslices * Tp * Hout * sizeof(float);
        if (b > need) need = b;
    }
    return ((need + 255) / 256) * 256;
}

s4c_status s4c_draft_linear(int32_t T, int32_t H, int32_t Hout, int32_t dtype, const void* e, const void* f,
                            const void* W, const void* bias, void* out, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
    if (!e || !f || !W || !out) return S4C_ERR_NULL;
    if (T <= 0 || H <= 0 || Hout <= 0) return S4C_ERR_SHAPE;
    if ((dtype != S4C_BF16 && dtype != S4C_F16) || H % draft_linear_tile_k() != 0 || Hout % draft_linear_tile_out() != 0 ||
        (long long)T * H * 2 >= (1ll << 31) || H > 16384)
        return S4C_ERR_UNSUPPORTED;
    if ((((uintptr_t)e) | ((uintptr_t)f) | ((uintptr_t)W) | ((uintptr_t)out)) & 15) return S4C_ERR_SHAPE;
    LinearArgs a;
    a.e = e; a.f = f; a.W = W; a.bias = bias; a.out = out; a.ws = nullptr; a.T = T; a.H = H; a.Hout = Hout; a.dtype = dtype;
    a.ttiles = a.otiles = 0; a.ksub = a.kslice = a.nslices = 0;
    if (T <= draft_linear_stream_max_tokens()) {
        // few tokens: the weight-streaming kernel with split-K partial sums in the workspace, in passes of at most
        // 128 tokens (each pass streams W once; up to four passes still beat the tiled kernel, which has no split-K
        // and fills few workgroups at these sizes)
        const size_t need = s4c_draft_linear_workspace_size(T, H, Hout);
        if (!workspace || workspace_bytes < need || (((uintptr_t)workspace) & 255)) return S4C_ERR_WORKSPACE;
        const int step = draft_linear_small_max_tokens();
        const int passes = (T + step - 1) / step, per = (T + passes - 1) / passes;      // equal passes
        a.ws = (float*)workspace;
        for (int t0 = 0; t0 < T; t0 += per) {
            LinearArgs p = a;
            p.T = T - t0 < per ? T - t0 : per;
            p.e = (const char*)e + (size_t)t0 * H * 2;
            p.f = (const char*)f + (size_t)t0 * H * 2;
            p.out = (char*)out + (size_t)t0 * Hout * 2;
            draft_linear_small_plan(p.T, H, Hout, device_cus(), &p.ksub, &p.kslice, &p.nslices);
            if (launch_draft_linear_small(p, (hipStream_t)hip_stream) != hipSuccess) return S4C_ERR_HIP;
        }
        return S4C_OK;
    }
    return launch_draft_linear(a, (hipStream_t)hip_stream) == hipSuccess ? S4C_OK : S4C_ERR_HIP;
}

#pragma GCC visibility pop
}  // extern "C"
