/*
 * CPU oracle (test infrastructure) -- see s4c_oracle.h.  Plain loops, double arithmetic,
 * no blocking or fusion; OpenMP only spreads independent (sequence, head) / row units
 * over the host cores.
 */
#include "s4c_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* IEEE 754 binary16 (1 sign, 5 exponent, 10 fraction bits) -> double, by its definition */
static double half_to_double(uint16_t h) {
    const int sign = (h >> 15) & 1, e = (h >> 10) & 0x1F, frac = h & 0x3FF;
    double v;
    if (e == 0) v = ldexp((double)frac, -24);                       /* zero and subnormals: frac * 2^-24 */
    else if (e == 31) v = frac ? NAN : INFINITY;
    else v = ldexp(1.0 + (double)frac / 1024.0, e - 15);
    return sign ? -v : v;
}

static double load_elem(const void* base, int32_t dtype, size_t idx) {
    if (dtype == 0) return (double)((const float*)base)[idx];
    if (dtype == 2) return half_to_double(((const uint16_t*)base)[idx]);
    uint32_t bits = ((uint32_t)((const uint16_t*)base)[idx]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static size_t elem_size(int32_t dtype) { return dtype == 0 ? 4 : 2; }

/* test hook: decode n stored elements to double */
int oracle_decode(int32_t dtype, int32_t n, const void* src, double* dst) {
    for (int32_t i = 0; i < n; ++i) dst[i] = load_elem(src, dtype, (size_t)i);
    return 0;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* -1 <= parent[i] < i for all i  */
static int forest_ok(const int32_t* parent, int32_t N) {
    for (int32_t i = 0; i < N; ++i)
        if (parent[i] < -1 || parent[i] >= i) return 0;
    return 1;
}

/* One output vector: node i of sequence b, query head h.  Sec. 3.2 / Fig. 3: the visible
 * set is the whole prefix plus the node's own root-to-node path. */
static void attn_one(const oracle_shape* s, const void* q, const void* k_tree, const void* v_tree,
                     const void* k_cache, const void* v_cache, int32_t clen, const int32_t* parent,
                     double scale, int32_t b, int32_t i, int32_t h, double* out) {
    const int32_t D = s->D, N = s->N, Hq = s->Hq, Hkv = s->Hkv;
    const int32_t kvh = h / (Hq / Hkv);
    const size_t qoff = (((size_t)b * N + i) * Hq + h) * D;

    /* visible tree rows: i, parent[i], parent[parent[i]], ... */
    int32_t anc[4096];
    int32_t na = 0;
    for (int32_t j = i; j >= 0; j = parent[j]) anc[na++] = j;

    const int32_t nvis = clen + na;
    double* sc = (double*)malloc(sizeof(double) * (size_t)(nvis > 0 ? nvis : 1));

    for (int32_t t = 0; t < nvis; ++t) {
        size_t koff;
        const void* kb;
        if (t < clen) {
            kb = k_cache;
            koff = (((size_t)b * Hkv + kvh) * s->S_cap + t) * D;
        } else {
            kb = k_tree;
            koff = (((size_t)b * N + anc[t - clen]) * Hkv + kvh) * D;
        }
        double dot = 0.0;
        for (int32_t d = 0; d < D; ++d) dot += load_elem(q, s->dtype, qoff + d) * load_elem(kb, s->dtype, koff + d);
        sc[t] = dot * scale;
    }
    double mx = -INFINITY;
    for (int32_t t = 0; t < nvis; ++t)
        if (sc[t] > mx) mx = sc[t];
    double denom = 0.0;
    for (int32_t t = 0; t < nvis; ++t) {
        sc[t] = exp(sc[t] - mx);
        denom += sc[t];
    }
    for (int32_t d = 0; d < D; ++d) out[d] = 0.0;
    for (int32_t t = 0; t < nvis; ++t) {
        size_t voff;
        const void* vb;
        if (t < clen) {
            vb = v_cache;
            voff = (((size_t)b * Hkv + kvh) * s->S_cap + t) * D;
        } else {
            vb = v_tree;
            voff = (((size_t)b * N + anc[t - clen]) * Hkv + kvh) * D;
        }
        const double w = sc[t] / denom;
        for (int32_t d = 0; d < D; ++d) out[d] += w * load_elem(vb, s->dtype, voff + d);
    }
    free(sc);
}

int oracle_tree_attn(const oracle_shape* s, const void* q, const void* k_tree, const void* v_tree,
                     const void* k_cache, const void* v_cache, const int32_t* cache_len,
                     const int32_t* parent, double scale, double* out, int32_t* status) {
    if (s->N > 4096) return -1;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)s->D);
    const int32_t B = s->B, N = s->N, Hq = s->Hq, D = s->D;
    for (int32_t b = 0; b < B; ++b) {
        int32_t st = 0;
        if (!forest_ok(parent + (size_t)b * N, N)) st |= ORACLE_BAD_TREE;
        if (cache_len[b] < 0 || cache_len[b] > s->S_cap) st |= ORACLE_BAD_LEN;
        if (status) status[b] = st;
        if (st) {
            memset(out + (size_t)b * N * Hq * D, 0, sizeof(double) * (size_t)N * Hq * D);
            continue;
        }
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
        for (int32_t h = 0; h < Hq; ++h)
            for (int32_t i = 0; i < N; ++i)
                attn_one(s, q, k_tree, v_tree, k_cache, v_cache, cache_len[b], parent + (size_t)b * N,
                         scale, b, i, h, out + (((size_t)b * N + i) * Hq + h) * D);
    }
    return 0;
}

int oracle_tree_attn_sampled(const oracle_shape* s, const void* q, const void* k_tree,
                             const void* v_tree, const void* k_cache, const void* v_cache,
                             const int32_t* cache_len, const int32_t* parent, double scale,
                             int32_t n, const int32_t* bnh, double* out) {
    if (s->N > 4096) return -1;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)s->D);
    for (int32_t b = 0; b < s->B; ++b) {
        if (!forest_ok(parent + (size_t)b * s->N, s->N)) return -2;
        if (cache_len[b] < 0 || cache_len[b] > s->S_cap) return -3;
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t t = 0; t < n; ++t) {
        const int32_t b = bnh[3 * t], i = bnh[3 * t + 1], h = bnh[3 * t + 2];
        attn_one(s, q, k_tree, v_tree, k_cache, v_cache, cache_len[b], parent + (size_t)b * s->N,
                 scale, b, i, h, out + (size_t)t * s->D);
    }
    return 0;
}

/* ------------------------------------------------------------------ acceptance */

static void row_stats_one(const void* logits, int32_t dtype, size_t off, int32_t V, double T,
                          int32_t* amax, double* rmax, double* sexp) {
    int32_t g = 0;
    double m = load_elem(logits, dtype, off);
    for (int32_t v = 1; v < V; ++v) {
        const double x = load_elem(logits, dtype, off + v);
        if (x > m) { m = x; g = v; }          /* strict: ties keep the lowest index */
    }
    double sum = 0.0;
    for (int32_t v = 0; v < V; ++v) sum += exp((load_elem(logits, dtype, off + v) - m) / T);
    *amax = g;
    *rmax = m;
    *sexp = sum;
}

int oracle_row_stats(int32_t rows, int32_t V, int32_t dtype, double temperature,
                     const void* logits, int32_t* argmax, double* rowmax, double* sumexp) {
    if (temperature <= 0.0) temperature = 1.0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t r = 0; r < rows; ++r)
        row_stats_one(logits, dtype, (size_t)r * V, V, temperature, &argmax[r], &rowmax[r], &sumexp[r]);
    return 0;
}

int oracle_accept_path(int32_t B, int32_t N, int32_t V, int32_t dtype, int32_t mode,
                       double temperature, const void* logits, const int32_t* parent,
                       const int32_t* tokens, const float* p_draft, const float* uniforms,
                       int32_t max_path, int32_t* path, int32_t* accept_len,
                       int32_t* accepted_tokens, int32_t* bonus_token, double* margin,
                       int32_t* status) {
    if (N < 1 || max_path < 1) return -1;
    if (mode == 1 && temperature <= 0.0) return -1;
    if (mode == 0) temperature = 1.0;
    int32_t* g = (int32_t*)malloc(sizeof(int32_t) * (size_t)B * N);
    double* m = (double*)malloc(sizeof(double) * (size_t)B * N);
    double* S = (double*)malloc(sizeof(double) * (size_t)B * N);
    oracle_row_stats(B * N, V, dtype, temperature, logits, g, m, S);

    for (int32_t b = 0; b < B; ++b) {
        const int32_t* par = parent + (size_t)b * N;
        const int32_t* tok = tokens + (size_t)b * N;
        int32_t* pth = path + (size_t)b * max_path;
        int32_t* atk = accepted_tokens + (size_t)b * max_path;
        for (int32_t k = 0; k < max_path; ++k) { pth[k] = -1; atk[k] = -1; }
        if (margin) margin[b] = INFINITY;

        int32_t* depth = (int32_t*)malloc(sizeof(int32_t) * N);
        char* acc = (char*)malloc(N);
        int bad = (par[0] != -1);
        for (int32_t i = 1; i < N && !bad; ++i)
            if (par[i] < 0 || par[i] >= i) bad = 1;
        if (!bad) {
            depth[0] = 0;
            for (int32_t i = 1; i < N; ++i) {
                depth[i] = depth[par[i]] + 1;
                if (depth[i] >= max_path) bad = 1;
            }
        }
        if (bad) {
            if (status) status[b] = ORACLE_BAD_TREE;
            pth[0] = 0;
            accept_len[b] = 0;
            bonus_token[b] = -1;
            free(depth);
            free(acc);
            continue;
        }
        if (status) status[b] = 0;

        acc[0] = 1;
        for (int32_t i = 1; i < N; ++i) {
            const int32_t p = par[i];
            int ok;
            if (mode == 0) {
                ok = (tok[i] == g[(size_t)b * N + p]);
            } else if (tok[i] < 0 || tok[i] >= V) {
                ok = 0;
            } else {
                const size_t r = (size_t)b * N + p;
                const double lx = load_elem(logits, dtype, r * V + tok[i]);
                const double pt = exp((lx - m[r]) / temperature) / S[r];      /* target prob of the draft token */
                const double lhs = (double)uniforms[(size_t)b * N + i] * (double)p_draft[(size_t)b * N + i];
                ok = (lhs < pt);                                               /* u < pt/pd, strict */
                if (margin) {
                    const double den = lhs > pt ? lhs : pt;
                    const double mg = den > 0.0 ? fabs(lhs - pt) / den : 0.0;
                    if (mg < margin[b]) margin[b] = mg;
                }
            }
            acc[i] = (char)(ok && acc[p]);
        }
        int32_t best = 0;
        for (int32_t i = 1; i < N; ++i)
            if (acc[i] && depth[i] > depth[best]) best = i;     /* strict: lowest index among equal depth */
        const int32_t L = depth[best];
        int32_t node = best;
        for (int32_t k = L; k >= 0; --k) { pth[k] = node; node = par[node]; }
        for (int32_t k = 1; k <= L; ++k) atk[k - 1] = tok[pth[k]];
        accept_len[b] = L;
        bonus_token[b] = (mode == 0) ? g[(size_t)b * N + best] : -1;
        free(depth);
        free(acc);
    }
    free(g);
    free(m);
    free(S);
    return 0;
}

/* ------------------------------------------------------------------ sequential rule + correction token */

/* target distribution of row `off` : r[v] = softmax(logits/T)[v] */
static void target_dist(const void* logits, int32_t dtype, size_t off, int32_t V, double T, double* r) {
    double m = load_elem(logits, dtype, off);
    for (int32_t v = 1; v < V; ++v) {
        const double x = load_elem(logits, dtype, off + v);
        if (x > m) m = x;
    }
    double sum = 0.0;
    for (int32_t v = 0; v < V; ++v) {
        r[v] = exp((load_elem(logits, dtype, off + v) - m) / T);
        sum += r[v];
    }
    for (int32_t v = 0; v < V; ++v) r[v] /= sum;
}

int oracle_accept_resample(int32_t B, int32_t N, int32_t V, int32_t dtype, double temperature,
                           const void* logits, const float* draft_probs, const int32_t* parent,
                           const int32_t* tokens, const float* uniforms, const float* u_resample,
                           int32_t max_path, int32_t* path, int32_t* accept_len,
                           int32_t* accepted_tokens, int32_t* bonus_token, double* margin_accept,
                           double* margin_sample, int32_t* status) {
    if (N < 1 || max_path < 1 || V < 1 || temperature <= 0.0) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t b = 0; b < B; ++b) {
        const int32_t* par = parent + (size_t)b * N;
        const int32_t* tok = tokens + (size_t)b * N;
        int32_t* pth = path + (size_t)b * max_path;
        int32_t* atk = accepted_tokens + (size_t)b * max_path;
        for (int32_t k = 0; k < max_path; ++k) { pth[k] = -1; atk[k] = -1; }
        pth[0] = 0;
        if (margin_accept) margin_accept[b] = INFINITY;
        if (margin_sample) margin_sample[b] = INFINITY;

        int bad = (par[0] != -1);
        for (int32_t i = 1; i < N && !bad; ++i)
            if (par[i] < 0 || par[i] >= i) bad = 1;
        if (!bad) {
            int32_t* depth = (int32_t*)malloc(sizeof(int32_t) * N);
            depth[0] = 0;
            for (int32_t i = 1; i < N; ++i) {
                depth[i] = depth[par[i]] + 1;
                if (depth[i] >= max_path) bad = 1;
            }
            free(depth);
        }
        if (bad) {
            if (status) status[b] = ORACLE_BAD_TREE;
            accept_len[b] = 0;
            bonus_token[b] = -1;
            continue;
        }
        if (status) status[b] = 0;

        double* r = (double*)malloc(sizeof(double) * (size_t)V);   /* the distribution the next token must follow */
        int32_t cur = 0, L = 0;
        for (;;) {
            target_dist(logits, dtype, ((size_t)b * N + cur) * V, V, temperature, r);
            const float* q = draft_probs + ((size_t)b * N + cur) * V;   /* draft distribution at cur */
            int32_t next = -1;
            for (int32_t c = cur + 1; c < N && next < 0; ++c) {
                if (par[c] != cur) continue;
                const int32_t x = tok[c];
                if (x < 0 || x >= V) continue;                 /* not a token: rejected, r unchanged */
                const double lhs = (double)uniforms[(size_t)b * N + c] * (double)q[x];
                const int ok = (lhs < r[x]);                   /* u < r(x)/q(x), strict */
                if (margin_accept) {
                    const double den = lhs > r[x] ? lhs : r[x];
                    const double mg = den > 0.0 ? fabs(lhs - r[x]) / den : 0.0;
                    if (mg < margin_accept[b]) margin_accept[b] = mg;
                }
                if (ok) {
                    next = c;
                } else {
                    /* rejected: r <- norm(max(0, r - q))  (Sec. 2, speculative-sampling paragraph) */
                    double Z = 0.0;
                    for (int32_t v = 0; v < V; ++v) {
                        const double d = r[v] - (double)q[v];
                        Z += d > 0.0 ? d : 0.0;
                    }
                    if (Z > 0.0)
                        for (int32_t v = 0; v < V; ++v) {
                            const double d = r[v] - (double)q[v];
                            r[v] = d > 0.0 ? d / Z : 0.0;
                        }
                }
            }
            if (next < 0) break;
            pth[++L] = next;
            atk[L - 1] = tok[next];
            cur = next;
        }
        /* correction / bonus token: inverse CDF of r in token-id order */
        double total = 0.0;
        for (int32_t v = 0; v < V; ++v) total += r[v];
        const double t = (double)u_resample[b] * total;
        double run = 0.0;
        int32_t pick = -1, last_pos = -1;
        for (int32_t v = 0; v < V; ++v) {
            const double prev = run;
            run += r[v];
            if (r[v] > 0.0) last_pos = v;
            if (run > t) {
                pick = v;
                if (margin_sample) {
                    const double lo = t - prev, hi = run - t;
                    margin_sample[b] = (lo < hi ? lo : hi) / total;
                }
                break;
            }
        }
        if (pick < 0) { pick = last_pos; if (margin_sample) margin_sample[b] = 0.0; }
        accept_len[b] = L;
        bonus_token[b] = pick;
        free(r);
    }
    return 0;
}

/* ------------------------------------------------------------------ compaction */

int oracle_kv_compact(const oracle_shape* s, const void* k_tree, const void* v_tree,
                      void* k_cache, void* v_cache, int32_t* cache_len, const int32_t* path,
                      const int32_t* accept_len, int32_t max_path, int32_t* dst_index,
                      int32_t* status) {
    const size_t es = elem_size(s->dtype);
    const size_t row = (size_t)s->D * es;
    for (int32_t b = 0; b < s->B; ++b) {
        const int32_t L = accept_len[b];
        const int32_t base = cache_len[b];
        const int32_t* pth = path + (size_t)b * max_path;
        if (dst_index)
            for (int32_t k = 0; k < max_path; ++k) dst_index[(size_t)b * max_path + k] = -1;
        int bad = (L < 0 || L >= max_path || base < 0 || (int64_t)base + L + 1 > s->S_cap);
        for (int32_t k = 0; !bad && k <= L; ++k)
            if (pth[k] < 0 || pth[k] >= s->N) bad = 1;
        if (status) status[b] = bad ? ORACLE_BAD_LEN : 0;
        if (bad) continue;
        for (int32_t k = 0; k <= L; ++k) {
            for (int32_t h = 0; h < s->Hkv; ++h) {
                const size_t src = (((size_t)b * s->N + pth[k]) * s->Hkv + h) * row;
                const size_t dst = (((size_t)b * s->Hkv + h) * s->S_cap + (size_t)(base + k)) * row;
                memcpy((char*)k_cache + dst, (const char*)k_tree + src, row);
                memcpy((char*)v_cache + dst, (const char*)v_tree + src, row);
            }
            if (dst_index) dst_index[(size_t)b * max_path + k] = base + k;
        }
        cache_len[b] = base + L + 1;
    }
    return 0;
}

int oracle_commit_path(const oracle_shape* s, int32_t layers, const void* k_tree, const void* v_tree,
                       void* k_cache, void* v_cache, int32_t* cache_len, const int32_t* path,
                       const int32_t* accept_len, int32_t max_path, const void* features,
                       int32_t feature_bytes, void* features_out, int32_t* dst_index, int32_t* status) {
    const size_t es = elem_size(s->dtype);
    const size_t row = (size_t)s->D * es;
    const size_t tree_layer = (size_t)s->B * s->N * s->Hkv * row;
    const size_t cache_layer = (size_t)s->B * s->Hkv * s->S_cap * row;
    for (int32_t b = 0; b < s->B; ++b) {
        const int32_t L = accept_len[b];
        const int32_t base = cache_len[b];
        const int32_t* pth = path + (size_t)b * max_path;
        if (dst_index)
            for (int32_t k = 0; k < max_path; ++k) dst_index[(size_t)b * max_path + k] = -1;
        int bad = (L < 0 || L >= max_path || base < 0 || (int64_t)base + L + 1 > s->S_cap);
        for (int32_t k = 0; !bad && k <= L; ++k)
            if (pth[k] < 0 || pth[k] >= s->N) bad = 1;
        if (status) status[b] = bad ? ORACLE_BAD_LEN : 0;
        if (bad) continue;
        for (int32_t k = 0; k <= L; ++k) {
            for (int32_t l = 0; l < layers; ++l)
                for (int32_t h = 0; h < s->Hkv; ++h) {
                    const size_t src = l * tree_layer + (((size_t)b * s->N + pth[k]) * s->Hkv + h) * row;
                    const size_t dst = l * cache_layer + (((size_t)b * s->Hkv + h) * s->S_cap + (size_t)(base + k)) * row;
                    memcpy((char*)k_cache + dst, (const char*)k_tree + src, row);
                    memcpy((char*)v_cache + dst, (const char*)v_tree + src, row);
                }
            if (features && features_out)
                memcpy((char*)features_out + ((size_t)b * max_path + k) * feature_bytes,
                       (const char*)features + ((size_t)b * s->N + pth[k]) * feature_bytes, (size_t)feature_bytes);
            if (dst_index) dst_index[(size_t)b * max_path + k] = base + k;
        }
        cache_len[b] = base + L + 1;
    }
    return 0;
}

/* ------------------------------------------------------------------ tree construction */

int oracle_build_tree(int32_t B, int32_t N, int32_t V, int32_t dtype, double temperature,
                      const void* draft_logits, const int32_t* nchild, const int32_t* root_token,
                      int32_t kmax, int32_t* parent, int32_t* tokens, float* p_draft, int32_t* level,
                      int32_t* status) {
    if (N < 1 || V < 1 || kmax < 1 || temperature <= 0.0) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t b = 0; b < B; ++b) {
        const int32_t* nc = nchild + (size_t)b * N;
        int32_t* par = parent + (size_t)b * N;
        int32_t* tok = tokens + (size_t)b * N;
        float* pd = p_draft + (size_t)b * N;
        int32_t* lev = level ? level + (size_t)b * N : NULL;
        for (int32_t i = 0; i < N; ++i) { par[i] = -1; tok[i] = -1; pd[i] = 0.f; if (lev) lev[i] = 0; }
        tok[0] = root_token[b];
        /* nodes are numbered level by level: node i's children are the next nchild[i] unused numbers;
         * node i (i >= 1) must itself have been handed out before it can be a parent */
        int bad = 0;
        int64_t cum = 0;
        for (int32_t i = 0; i < N && !bad; ++i) {
            if (i >= 1 && cum < i) bad = 1;
            if (nc[i] < 0 || nc[i] > kmax) bad = 1;
            cum += nc[i] > 0 ? nc[i] : 0;
        }
        if (cum != N - 1) bad = 1;
        if (status) status[b] = bad ? ORACLE_BAD_TREE : 0;
        if (bad) continue;

        char* taken = (char*)malloc((size_t)V);
        int32_t next = 1;
        for (int32_t i = 0; i < N; ++i) {
            const int32_t k = nc[i];
            if (k == 0) continue;
            const size_t off = ((size_t)b * N + i) * V;
            int32_t g;
            double m, S;
            row_stats_one(draft_logits, dtype, off, V, temperature, &g, &m, &S);
            memset(taken, 0, (size_t)V);
            for (int32_t r = 0; r < k; ++r) {
                /* r-th candidate: the largest remaining logit, lowest token id among equals */
                int32_t best = -1;
                double bv = 0.0;
                for (int32_t v = 0; v < V; ++v) {
                    if (taken[v]) continue;
                    const double x = load_elem(draft_logits, dtype, off + v);
                    if (best < 0 || x > bv) { best = v; bv = x; }
                }
                const int32_t c = next++;
                par[c] = i;
                if (lev) lev[c] = lev[i] + 1;
                if (best >= 0) {
                    taken[best] = 1;
                    tok[c] = best;
                    pd[c] = (float)(exp((bv - m) / temperature) / S);
                }
            }
        }
        free(taken);
    }
    return 0;
}

/* ------------------------------------------------------------------ draft-head input projection */

int oracle_draft_linear(int32_t T, int32_t H, int32_t Hout, int32_t dtype, const void* e, const void* f,
                        const void* W, const void* bias, double* out) {
    if (T < 0 || H < 1 || Hout < 1) return -1;
#pragma omp parallel for schedule(static)
    for (int32_t t = 0; t < T; ++t)
        for (int32_t o = 0; o < Hout; ++o) {
            double acc = bias ? load_elem(bias, dtype, (size_t)o) : 0.0;
            const size_t w0 = (size_t)o * 2 * H;
            for (int32_t k = 0; k < H; ++k) acc += load_elem(e, dtype, (size_t)t * H + k) * load_elem(W, dtype, w0 + k);
            for (int32_t k = 0; k < H; ++k) acc += load_elem(f, dtype, (size_t)t * H + k) * load_elem(W, dtype, w0 + H + k);
            out[(size_t)t * Hout + o] = acc;
        }
    return 0;
}

/* ------------------------------------------------------------------ paged cache */

int oracle_paged_gather(const oracle_shape* s, int32_t page_size, int32_t num_pages, int32_t max_blocks,
                        const void* pool, const int32_t* block_table, const int32_t* cache_len, void* cache,
                        int32_t* status) {
    const size_t row = (size_t)s->D * elem_size(s->dtype);
    memset(cache, 0, (size_t)s->B * s->Hkv * s->S_cap * row);
    for (int32_t b = 0; b < s->B; ++b) {
        const int32_t P = cache_len[b];
        int bad = (P < 0 || P > s->S_cap || (int64_t)P > (int64_t)max_blocks * page_size);
        for (int32_t j = 0; !bad && j < P; j += page_size) {
            const int32_t id = block_table[(size_t)b * max_blocks + j / page_size];
            if (id < 0 || id >= num_pages) bad = 1;
        }
        if (status) status[b] = bad ? ORACLE_BAD_LEN : 0;
        if (bad) continue;
        for (int32_t h = 0; h < s->Hkv; ++h)
            for (int32_t j = 0; j < P; ++j) {
                const int32_t id = block_table[(size_t)b * max_blocks + j / page_size];
                const size_t src = (((size_t)id * s->Hkv + h) * page_size + (size_t)(j % page_size)) * row;
                const size_t dst = (((size_t)b * s->Hkv + h) * s->S_cap + (size_t)j) * row;
                memcpy((char*)cache + dst, (const char*)pool + src, row);
            }
    }
    return 0;
}

int oracle_kv_compact_paged(const oracle_shape* s, int32_t page_size, int32_t num_pages, int32_t max_blocks,
                            const void* k_tree, const void* v_tree, void* k_pool, void* v_pool,
                            const int32_t* block_table, int32_t* cache_len, const int32_t* path,
                            const int32_t* accept_len, int32_t max_path, int32_t* dst_index, int32_t* status) {
    const size_t row = (size_t)s->D * elem_size(s->dtype);
    for (int32_t b = 0; b < s->B; ++b) {
        const int32_t L = accept_len[b];
        const int32_t base = cache_len[b];
        const int32_t* pth = path + (size_t)b * max_path;
        if (dst_index)
            for (int32_t k = 0; k < max_path; ++k) dst_index[(size_t)b * max_path + k] = -1;
        int bad = (L < 0 || L >= max_path || base < 0 || (int64_t)base + L + 1 > (int64_t)max_blocks * page_size);
        for (int32_t k = 0; !bad && k <= L; ++k) {
            if (pth[k] < 0 || pth[k] >= s->N) bad = 1;
            const int32_t id = block_table[(size_t)b * max_blocks + (base + k) / page_size];
            if (id < 0 || id >= num_pages) bad = 1;
        }
        if (status) status[b] = bad ? ORACLE_BAD_LEN : 0;
        if (bad) continue;
        for (int32_t k = 0; k <= L; ++k) {
            const int32_t j = base + k;
            const int32_t id = block_table[(size_t)b * max_blocks + j / page_size];
            for (int32_t h = 0; h < s->Hkv; ++h) {
                const size_t src = (((size_t)b * s->N + pth[k]) * s->Hkv + h) * row;
                const size_t dst = (((size_t)id * s->Hkv + h) * page_size + (size_t)(j % page_size)) * row;
                memcpy((char*)k_pool + dst, (const char*)k_tree + src, row);
                memcpy((char*)v_pool + dst, (const char*)v_tree + src, row);
            }
            if (dst_index) dst_index[(size_t)b * max_path + k] = j;
        }
        cache_len[b] = base + L + 1;
    }
    return 0;
}

/* Whole-model commit into paged pools: k_pool, v_pool are [layers][num_pages][Hkv][page_size][D], one
 * block table serves every layer (a sequence's row j sits at the same page slot in all of them). */
int oracle_commit_path_paged(const oracle_shape* s, int32_t layers, int32_t page_size, int32_t num_pages,
                             int32_t max_blocks, const void* k_tree, const void* v_tree, void* k_pool, void* v_pool,
                             const int32_t* block_table, int32_t* cache_len, const int32_t* path,
                             const int32_t* accept_len, int32_t max_path, const void* features, int32_t feature_bytes,
                             void* features_out, int32_t* dst_index, int32_t* status) {
    const size_t row = (size_t)s->D * elem_size(s->dtype);
    const size_t tree_layer = (size_t)s->B * s->N * s->Hkv * row;
    const size_t pool_layer = (size_t)num_pages * s->Hkv * page_size * row;
    for (int32_t b = 0; b < s->B; ++b) {
        const int32_t L = accept_len[b];
        const int32_t base = cache_len[b];
        const int32_t* pth = path + (size_t)b * max_path;
        if (dst_index)
            for (int32_t k = 0; k < max_path; ++k) dst_index[(size_t)b * max_path + k] = -1;
        int bad = (L < 0 || L >= max_path || base < 0 || (int64_t)base + L + 1 > (int64_t)max_blocks * page_size);
        for (int32_t k = 0; !bad && k <= L; ++k) {
            if (pth[k] < 0 || pth[k] >= s->N) bad = 1;
            const int32_t id = block_table[(size_t)b * max_blocks + (base + k) / page_size];
            if (id < 0 || id >= num_pages) bad = 1;
        }
        if (status) status[b] = bad ? ORACLE_BAD_LEN : 0;
        if (bad) continue;
        for (int32_t k = 0; k <= L; ++k) {
            const int32_t j = base + k;
            const int32_t id = block_table[(size_t)b * max_blocks + j / page_size];
            for (int32_t l = 0; l < layers; ++l)
                for (int32_t h = 0; h < s->Hkv; ++h) {
                    const size_t src = l * tree_layer + (((size_t)b * s->N + pth[k]) * s->Hkv + h) * row;
                    const size_t dst = l * pool_layer + (((size_t)id * s->Hkv + h) * page_size + (size_t)(j % page_size)) * row;
                    memcpy((char*)k_pool + dst, (const char*)k_tree + src, row);
                    memcpy((char*)v_pool + dst, (const char*)v_tree + src, row);
                }
            if (features && features_out)
                memcpy((char*)features_out + ((size_t)b * max_path + k) * feature_bytes,
                       (const char*)features + ((size_t)b * s->N + pth[k]) * feature_bytes, (size_t)feature_bytes);
            if (dst_index) dst_index[(size_t)b * max_path + k] = j;
        }
        cache_len[b] = base + L + 1;
    }
    return 0;
}
