/*
 * A verification step driven from plain C through the C ABI of libs4c: no Python, no PyTorch.
 * It is a test of the boundary (include/s4c.h): device memory comes from the HIP runtime, every
 * argument is a pointer or a size.  Expected values are closed forms, worked out here:
 *   - all keys are zero, so every visible key gets the same softmax weight and a node's output
 *     is the MEAN of the value rows it may see (prefix rows and the tree rows of its ancestors
 *     and itself, Sec. 3.2 / Fig. 3);
 *   - greedy acceptance on logits with one planted peak per row;
 *   - compaction appends the accepted path's tree rows, bit for bit.
 * Exit status 0 and a last line "c client ok" mean every check passed.
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "s4c.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %d at %s:%d\n", (int)e_, __FILE__, __LINE__); return 2; } } while (0)
#define CHECK_S4C(x) do { s4c_status s_ = (x); if (s_ != S4C_OK) { printf("s4c error %d (%s) at %s:%d\n", (int)s_, s4c_strerror(s_), __FILE__, __LINE__); return 3; } } while (0)

enum { B = 2, HQ = 4, HKV = 2, D = 128, N = 5, P = 70, S_CAP = 96, V = 1000, MAX_PATH = 4 };
static const int32_t PARENT[N] = {-1, 0, 0, 1, 3};      /* depth 3: 0 - 1 - 3 - 4, and 2 beside 1 */
static const int32_t CACHE_LEN[B] = {P, 33};

/* small integers and halves are exact in every storage type */
static float value_of(int b, int h, int row_kind, int j, int d) { return (float)((j + 3 * row_kind + b) % 7) + 0.5f * (float)((d + h) % 3); }

static uint16_t to_bf16(float x) { uint32_t u; memcpy(&u, &x, 4); return (uint16_t)(u >> 16); }       /* exact for these values */
static float from_bf16(uint16_t h) { uint32_t u = (uint32_t)h << 16; float x; memcpy(&x, &u, 4); return x; }

static void* dev(const void* host, size_t bytes) {
    void* p = NULL;
    if (hipMalloc(&p, bytes) != hipSuccess) return NULL;
    if (host) { if (hipMemcpy(p, host, bytes, hipMemcpyHostToDevice) != hipSuccess) return NULL; }
    else if (hipMemset(p, 0, bytes) != hipSuccess) return NULL;
    return p;
}

static int run(int dtype) {
    const size_t es = dtype == S4C_F32 ? 4 : 2;
    const size_t nq = (size_t)B * N * HQ * D, nt = (size_t)B * N * HKV * D, nc = (size_t)B * HKV * S_CAP * D;
    float* q = malloc(nq * 4); float* vt = malloc(nt * 4); float* vc = malloc(nc * 4);
    for (size_t i = 0; i < nq; ++i) q[i] = (float)((i * 7) % 5) - 2.0f;          /* any finite queries: keys are zero */
    for (int b = 0; b < B; ++b)
        for (int i = 0; i < N; ++i)
            for (int h = 0; h < HKV; ++h)
                for (int d = 0; d < D; ++d) vt[(((size_t)b * N + i) * HKV + h) * D + d] = value_of(b, h, 1, i, d);
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < HKV; ++h)
            for (int j = 0; j < S_CAP; ++j)
                for (int d = 0; d < D; ++d)
                    vc[(((size_t)b * HKV + h) * S_CAP + j) * D + d] = j < CACHE_LEN[b] ? value_of(b, h, 0, j, d) : 99.0f;   /* rows past cache_len must not be read */
    /* storage */
    void* hq = malloc(nq * es); void* hvt = malloc(nt * es); void* hvc = malloc(nc * es);
    if (dtype == S4C_F32) { memcpy(hq, q, nq * 4); memcpy(hvt, vt, nt * 4); memcpy(hvc, vc, nc * 4); }
    else {
        for (size_t i = 0; i < nq; ++i) ((uint16_t*)hq)[i] = to_bf16(q[i]);
        for (size_t i = 0; i < nt; ++i) ((uint16_t*)hvt)[i] = to_bf16(vt[i]);
        for (size_t i = 0; i < nc; ++i) ((uint16_t*)hvc)[i] = to_bf16(vc[i]);
    }
    int32_t par[B * N];
    for (int b = 0; b < B; ++b) memcpy(par + b * N, PARENT, sizeof PARENT);

    s4c_attn_shape sh = {B, HQ, HKV, D, N, S_CAP, dtype};
    void *d_q = dev(hq, nq * es), *d_kt = dev(NULL, nt * es), *d_vt = dev(hvt, nt * es);
    void *d_kc = dev(NULL, nc * es), *d_vc = dev(hvc, nc * es), *d_out = dev(NULL, nq * es);
    int32_t *d_cl = dev(CACHE_LEN, sizeof CACHE_LEN), *d_par = dev(par, sizeof par), *d_st = dev(NULL, B * 4);
    const size_t wsz = s4c_tree_attn_workspace_size(&sh, P);
    void* d_ws = wsz ? dev(NULL, wsz) : NULL;
    if (!d_q || !d_kt || !d_vt || !d_kc || !d_vc || !d_out || !d_cl || !d_par || !d_st || (wsz && !d_ws)) { printf("allocation failed\n"); return 2; }

    CHECK_S4C(s4c_tree_attn(&sh, d_q, d_kt, d_vt, d_kc, d_vc, d_cl, d_par, P, 0.0f, d_out, d_st, d_ws, wsz, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    void* hout = malloc(nq * es);
    int32_t st[B];
    CHECK_HIP(hipMemcpy(hout, d_out, nq * es, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(st, d_st, sizeof st, hipMemcpyDeviceToHost));
    int bad = 0;
    for (int b = 0; b < B; ++b) {
        if (st[b] != 0) { printf("attention status %d for sequence %d\n", st[b], b); return 4; }
        for (int i = 0; i < N; ++i)
            for (int hq_ = 0; hq_ < HQ; ++hq_) {
                const int h = hq_ / (HQ / HKV);
                for (int d = 0; d < D; ++d) {
                    double sum = 0.0; int cnt = 0;
                    for (int j = 0; j < CACHE_LEN[b]; ++j) { sum += value_of(b, h, 0, j, d); ++cnt; }
                    for (int a = i; a >= 0; a = PARENT[a]) { sum += value_of(b, h, 1, a, d); ++cnt; }
                    const double want = sum / cnt;
                    const size_t o = (((size_t)b * N + i) * HQ + hq_) * D + d;
                    const double got = dtype == S4C_F32 ? ((float*)hout)[o] : from_bf16(((uint16_t*)hout)[o]);
                    const double tol = dtype == S4C_F32 ? 1e-5 : ldexp(fabs(want), -8) + 1e-6;     /* one bf16 ulp */
                    if (!(fabs(got - want) <= tol)) { if (bad++ < 5) printf("out[%d][%d][%d][%d] = %g, want %g\n", b, i, hq_, d, got, want); }
                }
            }
    }
    if (bad) { printf("%d attention mismatches\n", bad); return 4; }

    /* greedy acceptance: row r peaks at token (17 r + 3); node 1 and node 3 carry their parent's peak */
    float* lg = calloc((size_t)B * N * V, 4);
    int32_t tok[B * N];
    for (int b = 0; b < B; ++b) {
        for (int r = 0; r < N; ++r) lg[((size_t)b * N + r) * V + (17 * r + 3 + b)] = 10.0f;
        tok[b * N + 0] = 1; tok[b * N + 1] = 17 * 0 + 3 + b; tok[b * N + 2] = 500; tok[b * N + 3] = 17 * 1 + 3 + b; tok[b * N + 4] = 999;
    }
    void* d_lg = dev(lg, (size_t)B * N * V * 4);
    int32_t *d_tok = dev(tok, sizeof tok), *d_path = dev(NULL, B * MAX_PATH * 4), *d_al = dev(NULL, B * 4);
    int32_t *d_at = dev(NULL, B * MAX_PATH * 4), *d_bonus = dev(NULL, B * 4);
    const size_t asz = s4c_accept_path_workspace_size(B, N, V);
    void* d_aws = dev(NULL, asz);
    if (!d_lg || !d_tok || !d_path || !d_al || !d_at || !d_bonus || !d_aws) { printf("allocation failed\n"); return 2; }
    CHECK_S4C(s4c_accept_path(B, N, V, S4C_F32, S4C_GREEDY, 1.0f, d_lg, d_par, d_tok, NULL, NULL, MAX_PATH, d_path, d_al, d_at, d_bonus,
                              d_st, d_aws, asz, NULL));
    /* same stream: compaction reads path / accept_len on the device */
    CHECK_S4C(s4c_kv_compact(&sh, d_kt, d_vt, d_kc, d_vc, d_cl, d_path, d_al, MAX_PATH, NULL, d_st, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    int32_t path[B * MAX_PATH], al[B], bonus[B], cl[B];
    CHECK_HIP(hipMemcpy(path, d_path, sizeof path, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(al, d_al, sizeof al, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(bonus, d_bonus, sizeof bonus, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(cl, d_cl, sizeof cl, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(hvc, d_vc, nc * es, hipMemcpyDeviceToHost));
    for (int b = 0; b < B; ++b) {
        const int32_t want_path[MAX_PATH] = {0, 1, 3, -1};
        if (memcmp(path + b * MAX_PATH, want_path, sizeof want_path) || al[b] != 2 || bonus[b] != 17 * 3 + 3 + b || cl[b] != CACHE_LEN[b] + 3) {
            printf("sequence %d: path %d %d %d %d, accept_len %d, bonus %d, cache_len %d\n", b, path[b * MAX_PATH], path[b * MAX_PATH + 1],
                   path[b * MAX_PATH + 2], path[b * MAX_PATH + 3], al[b], bonus[b], cl[b]);
            return 5;
        }
        for (int k = 0; k < 3; ++k)
            for (int h = 0; h < HKV; ++h) {
                const char* src = (const char*)hvt + ((((size_t)b * N + want_path[k]) * HKV + h) * D) * es;
                const char* dst = (const char*)hvc + ((((size_t)b * HKV + h) * S_CAP + CACHE_LEN[b] + k) * D) * es;
                if (memcmp(src, dst, D * es)) { printf("sequence %d: appended row %d differs\n", b, k); return 5; }
            }
    }
    printf("dtype %d: attention (closed form), greedy path, compaction ok\n", dtype);
    hipFree(d_q); hipFree(d_kt); hipFree(d_vt); hipFree(d_kc); hipFree(d_vc); hipFree(d_out); hipFree(d_cl); hipFree(d_par); hipFree(d_st);
    if (d_ws) hipFree(d_ws);
    hipFree(d_lg); hipFree(d_tok); hipFree(d_path); hipFree(d_al); hipFree(d_at); hipFree(d_bonus); hipFree(d_aws);
    free(q); free(vt); free(vc); free(hq); free(hvt); free(hvc); free(hout); free(lg);
    return 0;
}

int main(void) {
    int n = 0;
    CHECK_HIP(hipGetDeviceCount(&n));
    if (n < 1) { printf("no GPU\n"); return 2; }
    int rc = run(S4C_F32);
    if (rc) return rc;
    rc = run(S4C_BF16);
    if (rc) return rc;
    printf("c client ok\n");
    return 0;
}
