/*
 * CPU oracle for the tree-verification step of the continuous verification tree
 * (paper Sec. 3.2, Fig. 3; acceptance rule: the unnumbered equation
 * "r < min(1, q(x)/p(x))" of Sec. 3.2 and the speculative-sampling paragraph of Sec. 2).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, definition-level implementation in
 * double precision.  It shares no code with the HIP library and must never be called from
 * the product path; only tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * Every pointer is a HOST pointer.  dtype: 0 = fp32, 1 = bf16 stored as uint16 bit patterns,
 * 2 = fp16 (IEEE binary16, the precision of the paper's experiments, Sec. 4.1) as uint16 bit patterns.
 * Layouts (row-major, innermost last):
 *   q, out       [B][N][Hq][D]        k_tree, v_tree [B][N][Hkv][D]
 *   k_cache, v_cache [B][Hkv][S_cap][D]   cache_len [B]   parent [B][N]
 *   logits [B][N][V]   tokens, p_draft, uniforms [B][N]
 * Query head h reads KV head h / (Hq/Hkv).
 *
 * Parity pins (tests, CPU only): brute-force per-node sequential causal attention on tiny
 * trees, chain tree == ordinary causal attention (library routine), closed forms (equal
 * keys -> mean of visible values, V == 1 -> output 1, empty prefix root -> V_root),
 * hand-worked acceptance examples, chain == sequential speculative-sampling rule,
 * compaction == appending accepted tokens one at a time; sequential rule with correction:
 * Monte-Carlo check that the emitted tokens follow the target distribution, hand-worked
 * residuals, deterministic-draft and q == p closed forms.  Nothing here is unpinned.
 */
#ifndef S4C_ORACLE_H
#define S4C_ORACLE_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t B, Hq, Hkv, D, N, S_cap, dtype;
} oracle_shape;

/* Decodes n stored elements of the given dtype to double (exposed so the element decoding can be
 * pinned on its own). */
int oracle_decode(int32_t dtype, int32_t n, const void* src, double* dst);

/* status bits written per sequence */
#define ORACLE_BAD_TREE 1
#define ORACLE_BAD_LEN  2

/* Tree-masked attention, Sec. 3.2 / Fig. 3: node i sees cache rows [0, cache_len[b]) and the
 * tree rows of i itself and of its ancestors.  out is double [B][N][Hq][D].  A sequence
 * whose parent[] violates -1 <= parent[i] < i (status bit 1) or whose cache_len is outside
 * [0, S_cap] (bit 2) gets an all-zero output.  scale <= 0 means 1/sqrt(D).  Returns 0. */
int oracle_tree_attn(const oracle_shape* s, const void* q, const void* k_tree, const void* v_tree,
                     const void* k_cache, const void* v_cache, const int32_t* cache_len,
                     const int32_t* parent, double scale, double* out, int32_t* status);

/* Same definition, evaluated only at n sampled (b, node, head) triples; out is [n][D]. */
int oracle_tree_attn_sampled(const oracle_shape* s, const void* q, const void* k_tree,
                             const void* v_tree, const void* k_cache, const void* v_cache,
                             const int32_t* cache_len, const int32_t* parent, double scale,
                             int32_t n, const int32_t* bnh, double* out);

/* Acceptance + longest accepted path (Sec. 3.2).  mode 0 greedy: node i (i >= 1) passes iff
 * tokens[i] equals the lowest-index argmax of logits row parent[i].  mode 1 stochastic: passes
 * iff u[i] * p_draft[i] < softmax(logits[parent[i]] / T)[tokens[i]]  (strict).  A node is
 * accepted iff it passes and its parent is accepted; the root always is.  The result is the
 * accepted node of greatest depth (lowest index among equals) and the path root..node.
 *   path [B][max_path] (-1 padded), accept_len [B] = path nodes - 1,
 *   accepted_tokens [B][max_path] = tokens of path[1..] (-1 padded),
 *   bonus_token [B] = greedy: argmax of the last path node's row; stochastic: -1,
 *   margin [B] (nullable) = min over tested nodes of |u*pd - pt| / max(u*pd, pt)
 *                           (stochastic; +inf in greedy),
 *   status [B] (nullable): bit 1 if parent[0] != -1 or parent[i] not in [0, i) or a path would
 *                          exceed max_path; then accept_len = 0, path = [0], bonus = -1. */
int oracle_accept_path(int32_t B, int32_t N, int32_t V, int32_t dtype, int32_t mode,
                       double temperature, const void* logits, const int32_t* parent,
                       const int32_t* tokens, const float* p_draft, const float* uniforms,
                       int32_t max_path, int32_t* path, int32_t* accept_len,
                       int32_t* accepted_tokens, int32_t* bonus_token, double* margin,
                       int32_t* status);

/* Sibling-sequential acceptance with the correction token (Sec. 2, speculative-sampling
 * paragraph: a rejected token is redrawn from norm(max(0, p - q)); Sec. 3.2, second equation:
 * the correction step at a fork of the tree, which refers to the multi-candidate scheme where
 * the residual is carried from one rejected sibling to the next).
 *   Walk from the root.  At node cur let r = softmax(logits[cur]/T) and q = draft_probs[cur]
 *   (float [B][N][V]: the distribution the children of cur were proposed from).  The children of
 *   cur are tried in increasing node index: child c with token x is accepted iff
 *   uniforms[c] * q[x] < r[x] (strict); then cur = c and the walk continues with a fresh r.
 *   Otherwise r <- norm(max(0, r - q)) (left unchanged if that has no mass, or if x is not a
 *   token id) and the next sibling is tried.  When no child is accepted (or cur is a leaf) the
 *   walk stops and bonus_token = the inverse CDF of r at u_resample[b]: the lowest v with
 *   sum_{w<=v} r[w] > u_resample[b] * sum_w r[w].
 *   path / accept_len / accepted_tokens / status as in oracle_accept_path.
 *   margin_accept [B] (nullable): min over tests of |u q(x) - r(x)| / max(u q(x), r(x));
 *   margin_sample [B] (nullable): distance of u * total to the nearer edge of the chosen
 *                                 token's CDF interval, divided by total. */
int oracle_accept_resample(int32_t B, int32_t N, int32_t V, int32_t dtype, double temperature,
                           const void* logits, const float* draft_probs, const int32_t* parent,
                           const int32_t* tokens, const float* uniforms, const float* u_resample,
                           int32_t max_path, int32_t* path, int32_t* accept_len,
                           int32_t* accepted_tokens, int32_t* bonus_token, double* margin_accept,
                           double* margin_sample, int32_t* status);

/* Row statistics used above, exposed for pins: lowest-index argmax, max, and
 * sum_v exp((l_v - max)/T) in double. */
int oracle_row_stats(int32_t rows, int32_t V, int32_t dtype, double temperature,
                     const void* logits, int32_t* argmax, double* rowmax, double* sumexp);

/* KV reuse (Sec. 3.2, last paragraph): for k = 0..accept_len[b], copy tree row path[b][k] of
 * every KV head into cache row cache_len[b] + k, for K and V; then cache_len[b] += accept_len+1.
 * dst_index [B][max_path] (nullable) receives the cache row written for path[k], -1 padded.
 * A sequence whose rows would not fit S_cap or whose path is malformed is left untouched
 * (status bit 2). */
int oracle_kv_compact(const oracle_shape* s, const void* k_tree, const void* v_tree,
                      void* k_cache, void* v_cache, int32_t* cache_len, const int32_t* path,
                      const int32_t* accept_len, int32_t max_path, int32_t* dst_index,
                      int32_t* status);

/* The same for a whole model in one call (Sec. 3.2, last paragraph: the accepted tokens and
 * their features are kept for the next drafting phase): k_tree, v_tree are [layers][B][N][Hkv][D],
 * k_cache, v_cache [layers][B][Hkv][S_cap][D]; cache_len [B] is shared by the layers and advanced
 * once.  If features (bytes [B][N][feature_bytes]) and features_out ([B][max_path][feature_bytes])
 * are given, features_out[b][k] = features[b][path[b][k]] for k = 0..accept_len[b]; other rows of
 * features_out are left as they were.  A flagged sequence (status bit 2) is untouched everywhere. */
int oracle_commit_path(const oracle_shape* s, int32_t layers, const void* k_tree, const void* v_tree,
                       void* k_cache, void* v_cache, int32_t* cache_len, const int32_t* path,
                       const int32_t* accept_len, int32_t max_path, const void* features,
                       int32_t feature_bytes, void* features_out, int32_t* dst_index, int32_t* status);

/* Candidate tree from the drafter's distributions (Sec. 3.2: the top-1 continuation is drafted
 * first, the next most probable tokens are added beside it as alternatives at the same position).
 *   draft_logits [B][N][V]: row i = drafter's logits for the token after node i (rows of nodes
 *                 without children are not read);  nchild [B][N]: children of node i, 0..kmax.
 *   Nodes are numbered level by level: node i's children take the next nchild[i] unused numbers,
 *   in order of decreasing draft probability (rank 0 = the top-1 token; equal logits: lowest
 *   token id first).  Output: parent [B][N] (parent[0] = -1), tokens [B][N] (tokens[0] =
 *   root_token[b]), p_draft [B][N] float = softmax(row/T)[token] (entry 0 = 0), level [B][N]
 *   (nullable; root 0).  A sequence whose nchild[] does not describe a tree of exactly N nodes
 *   (sum != N-1, an entry outside [0, kmax], or a parent that was never created) gets status bit 1,
 *   parent = -1, tokens = (root, -1, ...), p_draft = 0.  A child beyond the V-th has token -1. */
int oracle_build_tree(int32_t B, int32_t N, int32_t V, int32_t dtype, double temperature,
                      const void* draft_logits, const int32_t* nchild, const int32_t* root_token,
                      int32_t kmax, int32_t* parent, int32_t* tokens, float* p_draft, int32_t* level,
                      int32_t* status);

/* Paged cache (a serving layout; the paper's Sec. 3.2 reuse step does not fix one).  The pool is
 * [num_pages][Hkv][page_size][D]; row j of sequence b lives in page block_table[b][j / page_size]
 * (block_table is [B][max_blocks]) at row j % page_size.  Tree attention over a paged cache is, by
 * definition, tree attention over the contiguous cache that oracle_paged_gather assembles (rows
 * j >= cache_len[b] zero); a sequence whose cache_len exceeds S_cap or max_blocks*page_size, or one
 * of whose needed pages is outside [0, num_pages), gets status bit 2 and an all-zero cache. */
int oracle_paged_gather(const oracle_shape* s, int32_t page_size, int32_t num_pages, int32_t max_blocks,
                        const void* pool, const int32_t* block_table, const int32_t* cache_len, void* cache,
                        int32_t* status);

/* oracle_kv_compact on a paged cache: the accepted rows go to rows cache_len[b] + k of the pages the
 * block table names (they must already be there); same flagging rule as above for those pages. */
int oracle_kv_compact_paged(const oracle_shape* s, int32_t page_size, int32_t num_pages, int32_t max_blocks,
                            const void* k_tree, const void* v_tree, void* k_pool, void* v_pool,
                            const int32_t* block_table, int32_t* cache_len, const int32_t* path,
                            const int32_t* accept_len, int32_t max_path, int32_t* dst_index, int32_t* status);

/* oracle_commit_path into paged pools [layers][num_pages][Hkv][page_size][D]; one block table serves every
 * layer.  Flagging as in oracle_kv_compact_paged; a flagged sequence is untouched everywhere. */
int oracle_commit_path_paged(const oracle_shape* s, int32_t layers, int32_t page_size, int32_t num_pages,
                             int32_t max_blocks, const void* k_tree, const void* v_tree, void* k_pool, void* v_pool,
                             const int32_t* block_table, int32_t* cache_len, const int32_t* path,
                             const int32_t* accept_len, int32_t max_path, const void* features, int32_t feature_bytes,
                             void* features_out, int32_t* dst_index, int32_t* status);

/* Input projection of a draft head (Eq. 3: h = Linear(concat[e, f])): out[t][o] = bias[o] +
 * sum_k e[t][k] W[o][k] + sum_k f[t][k] W[o][H + k], in double.  e, f [T][H]; W [Hout][2H] (one row
 * per output feature, the layout of a linear layer's weight); bias [Hout] nullable; out [T][Hout]. */
int oracle_draft_linear(int32_t T, int32_t H, int32_t Hout, int32_t dtype, const void* e, const void* f,
                        const void* W, const void* bias, double* out);

int oracle_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
