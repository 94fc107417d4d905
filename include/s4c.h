/*
 * s4c.h -- C ABI of the MI355X (gfx950) tree-verification library.
 *
 * One verification step of the continuous verification tree (paper Sec. 3.2, Fig. 3):
 *   1. s4c_tree_attn    every drafted node is scored in one pass; a node attends to the shared
 *                       prefix KV cache plus only itself and its ancestors (the tree mask);
 *   2. s4c_accept_path  per-node acceptance (greedy, or the stochastic rule r < min(1, q/p)
 *                       of Sec. 3.2) and the longest accepted root-to-node path;
 *   3. s4c_kv_compact   the accepted path's K/V rows are appended to the cache so the next
 *                       round reuses them (last paragraph of Sec. 3.2).
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller; `shape` structs are HOST
 *     pointers.  The library allocates nothing.  What it keeps between calls is per-GPU set-up
 *     only: which of its kernels already had their dynamic-LDS limit raised, the compute-unit
 *     count it sizes launches by, the address of the fixed scratch of s4c_accept_path_static, and
 *     a counter that gives every acceptance call its own tag.
 *   - Q, K, V, the caches / pools and `out` must be 16-byte aligned (checked: S4C_ERR_SHAPE);
 *     logits rows may have any alignment.  Floating-point inputs must be finite (no NaN, no
 *     infinity): the kernels are compiled without NaN handling, and a non-finite input gives an
 *     unspecified (but in-bounds) result for the sequences that read it.
 *   - Calls only enqueue work on `hip_stream` (a hipStream_t, may be NULL for the default
 *     stream) and never synchronise; they may be chained on one stream
 *     (s4c_accept_path -> s4c_kv_compact reads `path` on the device).
 *   - The return value reports what the host can check (null pointer, shape, unsupported
 *     size, workspace too small, launch failure).  Data-dependent problems (malformed
 *     parent[], cache_len out of range) are reported per sequence in a device `status` word
 *     and the affected sequence gets a defined result, never undefined behaviour.
 *   - Inputs are not modified except k_cache / v_cache / cache_len in s4c_kv_compact.
 *   - Row-major layouts, innermost dimension last.  dtype selects the element type of
 *     Q/K/V/cache/out (and of logits): fp32, or bf16 / fp16 (IEEE binary16, the precision of the
 *     paper's experiments, Sec. 4.1) with fp32 accumulation.
 *   - Limits: 1 <= N <= 128, D in {64, 128}, Hq % Hkv == 0.
 */
#ifndef S4C_H
#define S4C_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    S4C_OK = 0,
    S4C_ERR_NULL = -1,         /* a required pointer is NULL */
    S4C_ERR_SHAPE = -2,        /* non-positive or inconsistent sizes */
    S4C_ERR_UNSUPPORTED = -3,  /* N > 128, D not in {64,128}, unknown dtype or mode */
    S4C_ERR_WORKSPACE = -4,    /* workspace missing or smaller than *_workspace_size() */
    S4C_ERR_HIP = -5,          /* kernel launch failed (hipGetLastError) */
    S4C_ERR_STATIC_SCRATCH = -6 /* s4c_accept_path_static: the problem needs more than S4C_STATIC_SCRATCH_BYTES */
} s4c_status;

typedef enum { S4C_F32 = 0, S4C_BF16 = 1, S4C_F16 = 2 } s4c_dtype;
typedef enum { S4C_GREEDY = 0, S4C_STOCHASTIC = 1 } s4c_accept_mode;

/* bits of the per-sequence device status word */
#define S4C_SEQ_BAD_TREE 1     /* parent[] is not a valid tree / path deeper than max_path */
#define S4C_SEQ_BAD_LEN  2     /* cache_len out of range / accepted rows do not fit S_cap */
#define S4C_SEQ_TIMEOUT  4     /* s4c_accept_path, s4c_accept_resample: the workgroups of a sequence could not
                                  hand their partial results to each other within the waiting limit (a GPU
                                  that stopped scheduling them); accept_len = 0, path = [0], bonus = -1 */

typedef struct {
    int32_t B;       /* sequences */
    int32_t Hq;      /* query heads */
    int32_t Hkv;     /* KV heads; query head h reads KV head h / (Hq/Hkv) */
    int32_t D;       /* head size */
    int32_t N;       /* tree nodes including the root (node 0 = last committed token) */
    int32_t S_cap;   /* row capacity of the KV cache per (sequence, KV head) */
    int32_t dtype;   /* s4c_dtype */
} s4c_attn_shape;

/* Bytes of device workspace s4c_tree_attn needs for this shape when no sequence's cache_len
 * exceeds max_cache_len (0 if the shape is invalid).  May be 0 (single pass, no partials). */
size_t s4c_tree_attn_workspace_size(const s4c_attn_shape* shape, int32_t max_cache_len);

/* Tree-masked attention (Sec. 3.2, Fig. 3 mask matrix).  For sequence b, node i, query head h:
 *   out[b][i][h] = sum_j softmax_j(scale * q[b][i][h] . k_j) v_j
 * over j in { cache rows 0 .. cache_len[b]-1 of KV head h/G } U { tree rows of node i and of
 * its ancestors }.  Accumulation and softmax are fp32.
 *   q, out          [B][N][Hq][D]
 *   k_tree, v_tree  [B][N][Hkv][D]      K/V of the tree nodes (not yet in the cache)
 *   k_cache, v_cache [B][Hkv][S_cap][D]
 *   cache_len       [B]   0 <= cache_len[b] <= min(max_cache_len, S_cap)
 *   parent          [B][N] parent[b][0] = -1 and -1 <= parent[b][i] < i
 *   max_cache_len   host-side upper bound of cache_len[] (sizes the launch)
 *   scale           <= 0 selects 1/sqrt(D)
 *   status          [B] nullable; receives S4C_SEQ_* bits (0 = fine).  A flagged sequence
 *                   gets an all-zero output.
 *   workspace       >= s4c_tree_attn_workspace_size(shape, max_cache_len) bytes, 256-byte
 *                   aligned; contents need not be initialised; may be NULL if that size is 0.
 * Results are deterministic (fixed split count and merge order for a given shape). */
s4c_status s4c_tree_attn(const s4c_attn_shape* shape, const void* q, const void* k_tree,
                         const void* v_tree, const void* k_cache, const void* v_cache,
                         const int32_t* cache_len, const int32_t* parent, int32_t max_cache_len,
                         float scale, void* out, int32_t* status, void* workspace,
                         size_t workspace_bytes, void* hip_stream);

/* s4c_tree_attn over a paged cache (a serving layout; the paper's reuse step does not fix one).
 *   k_pool, v_pool  [num_pages][Hkv][page_size][D]; page_size a power of two >= 64
 *   block_table     [B][max_blocks]: cache row j of sequence b is row j % page_size of page
 *                   block_table[b][j / page_size]; one table serves K and V
 *   shape->S_cap    must equal max_blocks * page_size (the logical capacity of a sequence)
 *   A sequence one of whose pages below cache_len[b] is outside [0, num_pages) is flagged
 *   S4C_SEQ_BAD_LEN and gets an all-zero output.  Everything else as s4c_tree_attn (same
 *   workspace size, same results bit for bit as on the equivalent contiguous cache). */
s4c_status s4c_tree_attn_paged(const s4c_attn_shape* shape, const void* q, const void* k_tree, const void* v_tree,
                               const void* k_pool, const void* v_pool, const int32_t* block_table,
                               int32_t max_blocks, int32_t page_size, int32_t num_pages, const int32_t* cache_len,
                               const int32_t* parent, int32_t max_cache_len, float scale, void* out,
                               int32_t* status, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Bytes of device workspace s4c_accept_path needs (per-row partial statistics).  Its contents need not be
 * initialised and may be anything a previous call left there; two calls that may overlap in time must
 * not share it. */
size_t s4c_accept_path_workspace_size(int32_t B, int32_t N, int32_t V);

/* Acceptance and longest accepted path (Sec. 3.2).
 *   logits  [B][N][V] (logits_dtype); row i is the target model's distribution for the token
 *           that follows node i, i.e. it verifies the children of node i.
 *   parent, tokens [B][N]; node 0 is the unique root (parent -1), 0 <= parent[i] < i.
 *   GREEDY      node i >= 1 passes iff tokens[i] == argmax(logits[parent[i]]), ties in the
 *               argmax resolved to the lowest token id (greedy decoding, Sec. 4.1.2).
 *   STOCHASTIC  node i passes iff uniforms[i] * p_draft[i] < softmax(logits[parent[i]]/T)[tokens[i]]
 *               (the test r < min(1, q(x)/p(x)) of Sec. 3.2 without the division; strict).
 *               p_draft[i] = draft probability of tokens[i] given its parent; uniforms in [0,1);
 *               both [B][N] fp32, entry 0 unused; NULL allowed in greedy mode.  T > 0.
 *   A node is accepted iff it passes and its parent is accepted (the root always is).  The
 *   result is the accepted node of greatest depth, lowest node index among equals.
 *   max_path  row stride of path / accepted_tokens; must exceed the tree's greatest depth.
 *   path            [B][max_path] node ids root..last, -1 padded
 *   accept_len      [B] accepted draft tokens (= path nodes - 1)
 *   accepted_tokens [B][max_path] tokens of path[1..], -1 padded
 *   bonus_token     [B] greedy: argmax of the last path node's row; stochastic: -1
 *   status          [B] nullable; S4C_SEQ_BAD_TREE if parent[] is malformed or a node is deeper
 *                   than max_path-1: then accept_len = 0, path = [0], bonus = -1.  S4C_SEQ_TIMEOUT
 *                   (same result) if the sequence's partial statistics did not all reach its
 *                   collecting workgroup within 2 s -- one launch does the scan and the path step,
 *                   and that wait is bounded so that every kernel ends.  The environment variable
 *                   S4C_ACCEPT_WAIT_US (an integer >= 0, read at every call) replaces the 2 s; 0
 *                   makes a collector that has to wait give up at once, which exercises the
 *                   flagged path on a healthy GPU.
 * Softmax statistics are fp32.  In STOCHASTIC mode the logits rows of leaf nodes are never read (they
 * verify no node and that mode returns no bonus token); in GREEDY mode every row may be read. */
s4c_status s4c_accept_path(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, int32_t mode,
                           float temperature, const void* logits, const int32_t* parent,
                           const int32_t* tokens, const float* p_draft, const float* uniforms,
                           int32_t max_path, int32_t* path, int32_t* accept_len,
                           int32_t* accepted_tokens, int32_t* bonus_token, int32_t* status,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/* s4c_accept_path for callers that cannot allocate device memory or pass a workspace (code under
 * HIP-graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments minus
 * the workspace, same results.  The per-row partial statistics go to a fixed scratch array that
 * lives in the library's device image (S4C_STATIC_SCRATCH_BYTES per GPU, held until the process
 * ends); the call allocates nothing.  Problems with
 * s4c_accept_path_workspace_size(B, N, V) > S4C_STATIC_SCRATCH_BYTES are refused with
 * S4C_ERR_STATIC_SCRATCH (1 MiB covers 43690 row segments of up to 65536 logits; 2048 rows of 128256
 * logits are 4096 segments, 96 KB).  All calls on one GPU share that GPU's array: two calls that may overlap in
 * time on one GPU (different streams) race, calls on one stream do not.  The array's device address
 * is looked up on the first call on each GPU (hipGetSymbolAddress, no allocation); make that first
 * call outside a graph capture. */
#define S4C_STATIC_SCRATCH_BYTES (1 << 20)
s4c_status s4c_accept_path_static(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, int32_t mode,
                                  float temperature, const void* logits, const int32_t* parent,
                                  const int32_t* tokens, const float* p_draft, const float* uniforms,
                                  int32_t max_path, int32_t* path, int32_t* accept_len,
                                  int32_t* accepted_tokens, int32_t* bonus_token, int32_t* status,
                                  void* hip_stream);

/* Sibling-sequential acceptance with the correction token (Sec. 2, speculative-sampling
 * paragraph: accept with probability min(1, p/q), redraw a rejected token from
 * norm(max(0, p - q)); Sec. 3.2, second equation: the correction at a fork of the tree, where
 * the corrected distribution is carried from one rejected sibling to the next).
 *   logits      [B][N][V] (logits_dtype), row i = target distribution after node i
 *   draft_probs [B][N][V] fp32, row i = the distribution the children of node i were proposed
 *               from (rows of leaves are not read)
 *   parent, tokens [B][N] as in s4c_accept_path; uniforms [B][N] fp32 in [0,1), entry 0 unused;
 *   u_resample  [B] fp32 in [0,1)
 *   The walk starts at the root.  At node cur, r = softmax(logits[cur]/T), q = draft_probs[cur].
 *   The children of cur are tried in increasing node index: child c with token x is accepted iff
 *   uniforms[c] * q[x] < r[x] (strict); the walk then moves to c with a fresh r.  After a
 *   rejection r <- norm(max(0, r - q)) (unchanged if that has no mass; a child whose token is
 *   not in [0, V) is skipped with r unchanged).  When no child is accepted (or cur is a leaf) the
 *   walk ends and bonus_token[b] = the lowest v with sum_{w<=v} r[w] > u_resample[b] * sum_w r[w].
 *   With children drawn independently from q the emitted tokens follow the target distribution.
 *   path, accept_len, accepted_tokens, status, max_path: as in s4c_accept_path; bonus_token is
 *   always a token id here (-1 only for a flagged sequence).
 *   workspace  >= s4c_accept_resample_workspace_size(B, N, V, max_path) bytes, 256-byte aligned,
 *              contents need not be initialised; may be NULL if that size is 0.  It carries the
 *              partial sums that the workgroups sharing one sequence exchange, so two calls that
 *              may overlap in time must not share it.
 * Arithmetic is fp64 (row maxima exact).  V <= 2^21.  The kernel polls device memory with a
 * bounded number of tries (S4C_SEQ_TIMEOUT); it needs at most 256 workgroups resident at once.
 * One workgroup per sequence writes all of that sequence's outputs, so a flagged sequence never
 * carries a partial result.  The environment variable S4C_RESAMPLE_SPIN_LIMIT (an integer >= 0,
 * read at every call) replaces the number of tries; 0 makes every exchange between several
 * workgroups give up at once, which exercises the flagged path on a healthy GPU. */
size_t s4c_accept_resample_workspace_size(int32_t B, int32_t N, int32_t V, int32_t max_path);
s4c_status s4c_accept_resample(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, float temperature,
                               const void* logits, const float* draft_probs, const int32_t* parent,
                               const int32_t* tokens, const float* uniforms, const float* u_resample,
                               int32_t max_path, int32_t* path, int32_t* accept_len,
                               int32_t* accepted_tokens, int32_t* bonus_token, int32_t* status,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/* Candidate tree from the drafter's logits (Sec. 3.2: the top-1 continuation is drafted first, the
 * next most probable tokens are placed beside it as alternatives at the same position).
 *   draft_logits [B][N][V] (logits_dtype): row i = the drafter's logits for the token that follows
 *                node i; rows of nodes without children are not read.
 *   nchild       [B][N]: number of children of node i, 0 .. kmax (kmax <= 8).
 *   root_token   [B]: the last committed token (node 0).
 *   Nodes are numbered level by level: the children of node i take the next nchild[i] unused
 *   numbers, in order of decreasing logit (equal logits: lowest token id first), so
 *   parent[i] < i and siblings are contiguous -- the layout s4c_tree_attn / s4c_accept_path expect.
 *   parent  [B][N] (parent[0] = -1)       tokens [B][N] (tokens[0] = root_token[b])
 *   p_draft [B][N] fp32 = softmax(row / T)[token] of the parent's row (entry 0 = 0)
 *   level   [B][N] nullable: depth of every node (root 0)
 *   status  [B] nullable: S4C_SEQ_BAD_TREE if nchild[] does not describe a tree of exactly N nodes
 *           (sum != N-1, an entry outside [0, kmax], or a node that would be a parent before it was
 *           handed out); then parent = -1, tokens = (root, -1, ...), p_draft = 0, level = 0.
 *   A child beyond the V-th token of its row gets token -1 and probability 0.
 *   workspace >= s4c_build_tree_workspace_size(B, N, V) bytes, 256-byte aligned, uninitialised.
 * Probabilities are computed in fp32. */
size_t s4c_build_tree_workspace_size(int32_t B, int32_t N, int32_t V);
s4c_status s4c_build_tree(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, float temperature,
                          const void* draft_logits, const int32_t* nchild, const int32_t* root_token,
                          int32_t kmax, int32_t* parent, int32_t* tokens, float* p_draft, int32_t* level,
                          int32_t* status, void* workspace, size_t workspace_bytes, void* hip_stream);

/* KV reuse (Sec. 3.2, last paragraph): for k = 0 .. accept_len[b], tree row path[b][k] of every
 * KV head is copied to cache row cache_len[b] + k (K and V); then cache_len[b] += accept_len[b]+1.
 * Only shape->B, Hkv, D, N, S_cap, dtype are used.
 *   dst_index [B][max_path] nullable: cache row written for path[k], -1 padded
 *   status    [B] nullable: S4C_SEQ_BAD_LEN if the rows do not fit S_cap or path/accept_len is
 *             malformed; that sequence's cache and cache_len are left untouched. */
s4c_status s4c_kv_compact(const s4c_attn_shape* shape, const void* k_tree, const void* v_tree,
                          void* k_cache, void* v_cache, int32_t* cache_len, const int32_t* path,
                          const int32_t* accept_len, int32_t max_path, int32_t* dst_index,
                          int32_t* status, void* hip_stream);

/* s4c_kv_compact into a paged cache (layout as in s4c_tree_attn_paged; shape->S_cap is ignored, the
 * capacity is max_blocks * page_size).  The pages of rows cache_len[b] .. cache_len[b] + accept_len[b]
 * must already be in the block table; a page id outside [0, num_pages) flags the sequence
 * (S4C_SEQ_BAD_LEN) and leaves it untouched. */
s4c_status s4c_kv_compact_paged(const s4c_attn_shape* shape, const void* k_tree, const void* v_tree, void* k_pool,
                                void* v_pool, const int32_t* block_table, int32_t max_blocks, int32_t page_size,
                                int32_t num_pages, int32_t* cache_len, const int32_t* path,
                                const int32_t* accept_len, int32_t max_path, int32_t* dst_index, int32_t* status,
                                void* hip_stream);

/* The same for every layer of a model in one call, plus the accepted nodes' feature rows (Sec. 3.2,
 * last paragraph: the accepted tokens and their features are kept for the next drafting phase).
 *   k_tree, v_tree   [layers][B][N][Hkv][D]        k_cache, v_cache [layers][B][Hkv][S_cap][D]
 *   cache_len [B] is shared by the layers and advanced once, after all rows were copied.
 *   features      [B][N][feature_bytes] (bytes of any element type; the penultimate-layer
 *                 output of every tree node), nullable together with
 *   features_out  [B][max_path][feature_bytes]: row k receives the feature row of node path[b][k]
 *                 for k = 0 .. accept_len[b]; other rows are left as they were.
 *                 feature_bytes is a positive multiple of 16, both pointers 16-byte aligned.
 *   dst_index, status, max_path: as in s4c_kv_compact; a flagged sequence is untouched in every
 *   layer and in features_out.  1 <= layers <= 65534. */
s4c_status s4c_commit_path(const s4c_attn_shape* shape, int32_t layers, const void* k_tree, const void* v_tree,
                           void* k_cache, void* v_cache, int32_t* cache_len, const int32_t* path,
                           const int32_t* accept_len, int32_t max_path, const void* features,
                           int32_t feature_bytes, void* features_out, int32_t* dst_index, int32_t* status,
                           void* hip_stream);

/* s4c_commit_path into paged pools: k_pool, v_pool [layers][num_pages][Hkv][page_size][D], one block table
 * [B][max_blocks] for every layer (layout and flagging as in s4c_kv_compact_paged; shape->S_cap is
 * ignored).  Everything else as s4c_commit_path. */
s4c_status s4c_commit_path_paged(const s4c_attn_shape* shape, int32_t layers, const void* k_tree, const void* v_tree,
                                 void* k_pool, void* v_pool, const int32_t* block_table, int32_t max_blocks,
                                 int32_t page_size, int32_t num_pages, int32_t* cache_len, const int32_t* path,
                                 const int32_t* accept_len, int32_t max_path, const void* features,
                                 int32_t feature_bytes, void* features_out, int32_t* dst_index, int32_t* status,
                                 void* hip_stream);

/* Input projection of a draft head (Eq. 3: h = Linear(concat[e, f])), the concatenation never formed:
 *   out[t][o] = bias[o] + sum_k e[t][k] W[o][k] + sum_k f[t][k] W[o][H + k]
 *   e, f [T][H]: embedding and feature of every token; W [Hout][2H] (one row per output feature,
 *   the layout of a linear layer's weight); bias [Hout] nullable; out [T][Hout].
 *   dtype S4C_BF16 or S4C_F16 (products and sums in fp32, output rounded to nearest even);
 *   H a multiple of 32 (<= 16384), Hout a multiple of 256, T*H < 2^30; all pointers 16-byte
 *   aligned device pointers.
 *   workspace  >= s4c_draft_linear_workspace_size(T, H, Hout) bytes, 256-byte aligned, contents need
 *              not be initialised; that size is 0 (and the pointer may be NULL) for T > 512.  Up to
 *              512 tokens the op is a stream over W: it runs in passes of at most 128 tokens -- one
 *              pass for a draft tree at batch 1, the operating point of Sec. 4.1.2 -- each split
 *              over the reduction dimension to fill the chip, and the workspace holds the slices'
 *              fp32 partial sums (added in a fixed order: results are deterministic).  S4C_ERR_WORKSPACE
 *              if it is missing, too small or misaligned. */
size_t s4c_draft_linear_workspace_size(int32_t T, int32_t H, int32_t Hout);
s4c_status s4c_draft_linear(int32_t T, int32_t H, int32_t Hout, int32_t dtype, const void* e, const void* f,
                            const void* W, const void* bias, void* out, void* workspace, size_t workspace_bytes,
                            void* hip_stream);

/* Text for a status code (any integer: unknown codes get "unknown status").  Static, never NULL. */
const char* s4c_strerror(int code);

/* Number of KV splits s4c_tree_attn uses for this shape (1 = single pass); for reporting. */
int32_t s4c_tree_attn_num_splits(const s4c_attn_shape* shape, int32_t max_cache_len);

#ifdef __cplusplus
}
#endif
#endif
