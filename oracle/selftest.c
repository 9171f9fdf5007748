/*
 * selftest.c - drives every entry point of dream_oracle.c once on small inputs held in heap buffers of exactly the
 * documented sizes.  TEST INFRASTRUCTURE ONLY.  Built together with dream_oracle.c as an executable under
 * -fsanitize=address,undefined (`python -m oracle.build --sanitize`), so that an access one element past any
 * argument, a signed overflow or a misaligned access inside the oracle aborts the run.  The values are checked only
 * for being finite and inside their ranges here: what the oracle computes is pinned by the Python tests.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void oracle_set_threads(int n);
int oracle_hw_threads(void);
int oracle_tree_attn(const void *q, const void *k, const void *v, int dtype, int B, int Tq, int Hq, int Hkv, int D,
                     int64_t s_max, const int32_t *prefix_len, int n_tree, const int32_t *parent,
                     const int32_t *q_node, int include_self, double scale, double *out, double *lse);
int oracle_visual_scores(const void *q, const int32_t *q_pos, int n_q, const void *k, int dtype, int B, int Hq,
                         int Hkv, int D, int64_t s_max, int vis_start, int vis_len, double scale, int include_diag,
                         double *scores);
int oracle_keep_count(int vis_len, int keep_num, int keep_den);
int oracle_topk_keep(const double *scores, int B, int vis_start, int vis_len, int keep_num, int keep_den,
                     int32_t *kept);
void oracle_gather_rows(const void *src, int dtype, int B, int64_t n_rows, int64_t row_elems, const int32_t *kept,
                        int k, void *dst);
int oracle_accept_path(const void *logits, int dtype, int B, int T, int V, const int32_t *token,
                       const int32_t *parent, int max_depth, int32_t *node_argmax, int32_t *accept_len,
                       int32_t *accept_path, int32_t *bonus_token);
int oracle_kv_commit(void *cache, int dtype, int B, int Hkv, int64_t s_max, int D, const int32_t *prefix_len, int T,
                     const int32_t *path, int path_stride, const int32_t *accept_len, int32_t *new_len);
int oracle_attention_entropy(const void *q, const int32_t *q_pos, int n_q, const void *k, int dtype, int B, int Hq,
                             int Hkv, int D, int64_t s_max, double scale, double *row_entropy, double *ae);
int oracle_project(const void *x, const void *w, int dtype, int B, int R, int hidden, int H, int D, double *out);

static uint32_t rng_state = 20250519u;
static double uniform01(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return (double)(rng_state >> 8) / 16777216.0;
}

/* n elements of the given dtype (0 = float32, 1 = bf16) with values in [-1, 1) */
static void *random_tensor(size_t n, int dtype)
{
    if (dtype == 0) {
        float *p = (float *)malloc(n * sizeof(float));
        for (size_t i = 0; i < n; i++)
            p[i] = (float)(2.0 * uniform01() - 1.0);
        return p;
    }
    uint16_t *p = (uint16_t *)malloc(n * sizeof(uint16_t));
    for (size_t i = 0; i < n; i++) {
        float f = (float)(2.0 * uniform01() - 1.0);
        uint32_t u;
        memcpy(&u, &f, 4);
        p[i] = (uint16_t)(u >> 16);
    }
    return p;
}

static int all_finite(const double *p, size_t n)
{
    for (size_t i = 0; i < n; i++)
        if (!isfinite(p[i]))
            return 0;
    return 1;
}

#define CHECK(cond)                                                              \
    do {                                                                         \
        if (!(cond)) {                                                           \
            fprintf(stderr, "selftest: %s failed at line %d\n", #cond, __LINE__); \
            return 1;                                                            \
        }                                                                        \
    } while (0)

static int run(int dtype, int threads)
{
    enum { B = 2, T = 9, Hq = 4, Hkv = 2, D = 16, S = 40, V = 37, DEPTH = 3 };
    oracle_set_threads(threads);
    const int32_t parent_one[T] = {-1, 0, 0, 1, 1, 2, 3, 3, 5};
    int32_t *parent = (int32_t *)malloc(sizeof(int32_t) * B * T), *prefix = (int32_t *)malloc(sizeof(int32_t) * B);
    for (int b = 0; b < B; b++)
        memcpy(parent + b * T, parent_one, sizeof parent_one);
    prefix[0] = S - T;   /* the tree rows end exactly at the end of the cache */
    prefix[1] = 0;       /* empty prefix */

    void *q = random_tensor((size_t)B * T * Hq * D, dtype), *k = random_tensor((size_t)B * Hkv * S * D, dtype),
         *v = random_tensor((size_t)B * Hkv * S * D, dtype);
    double *out = (double *)malloc(sizeof(double) * B * T * Hq * D), *lse = (double *)malloc(sizeof(double) * B * Hq * T);
    CHECK(oracle_tree_attn(q, k, v, dtype, B, T, Hq, Hkv, D, S, prefix, T, parent, NULL, 1, 0.25, out, lse) == 0);
    CHECK(all_finite(out, (size_t)B * T * Hq * D) && all_finite(lse, (size_t)B * Hq * T));
    /* strict ancestors, a level of 3 query rows named by q_node */
    int32_t q_node[B * 3] = {3, 4, 5, 6, 7, 8};
    void *q3 = random_tensor((size_t)B * 3 * Hq * D, dtype);
    CHECK(oracle_tree_attn(q3, k, v, dtype, B, 3, Hq, Hkv, D, S, prefix, T, parent, q_node, 0, 0.25, out, NULL) == 0);
    CHECK(all_finite(out, (size_t)B * 3 * Hq * D));

    /* visual scores over all S rows as queries, visual span [3, 3+20), both diagonal readings */
    enum { NQ = S, VS = 3, VL = 20 };
    void *pq = random_tensor((size_t)B * NQ * Hq * D, dtype);
    double *scores = (double *)malloc(sizeof(double) * B * VL);
    for (int diag = 0; diag < 2; diag++) {
        CHECK(oracle_visual_scores(pq, NULL, NQ, k, dtype, B, Hq, Hkv, D, S, VS, VL, 0.25, diag, scores) == 0);
        CHECK(all_finite(scores, (size_t)B * VL));
    }
    const int keep = oracle_keep_count(VL, 1, 4);
    CHECK(keep == 5);
    int32_t *kept = (int32_t *)malloc(sizeof(int32_t) * B * keep);
    CHECK(oracle_topk_keep(scores, B, VS, VL, 1, 4, kept) == keep);
    for (int i = 0; i < B * keep; i++)
        CHECK(kept[i] >= VS && kept[i] < VS + VL);
    void *rows = random_tensor((size_t)B * S * 7, dtype);
    void *gathered = malloc((size_t)B * keep * 7 * (dtype == 0 ? 4 : 2));
    oracle_gather_rows(rows, dtype, B, S, 7, kept, keep, gathered);

    /* attention entropy with explicit positions */
    int32_t *q_pos = (int32_t *)malloc(sizeof(int32_t) * B * 5);
    for (int i = 0; i < B * 5; i++)
        q_pos[i] = (i * 7) % S;
    void *q5 = random_tensor((size_t)B * 5 * Hq * D, dtype);
    double *row_entropy = (double *)malloc(sizeof(double) * B * Hq * 5), ae[B];
    CHECK(oracle_attention_entropy(q5, q_pos, 5, k, dtype, B, Hq, Hkv, D, S, 0.25, row_entropy, ae) == 0);
    CHECK(all_finite(row_entropy, (size_t)B * Hq * 5) && all_finite(ae, B));

    /* greedy acceptance */
    void *logits = random_tensor((size_t)B * T * V, dtype);
    int32_t *token = (int32_t *)malloc(sizeof(int32_t) * B * T);
    for (int i = 0; i < B * T; i++)
        token[i] = (i * 5) % V;
    int32_t node_argmax[B * T], accept_len[B], accept_path[B * (DEPTH + 1)], bonus[B];
    CHECK(oracle_accept_path(logits, dtype, B, T, V, token, parent, DEPTH, node_argmax, accept_len, accept_path, bonus) == 0);
    for (int b = 0; b < B; b++)
        CHECK(accept_len[b] >= 0 && accept_len[b] <= DEPTH && bonus[b] >= 0 && bonus[b] < V && accept_path[b * (DEPTH + 1)] == 0);

    /* KV commit of those paths on the K cache */
    int32_t new_len[B];
    CHECK(oracle_kv_commit(k, dtype, B, Hkv, S, D, prefix, T, accept_path, DEPTH + 1, accept_len, new_len) == 0);
    for (int b = 0; b < B; b++)
        CHECK(new_len[b] == prefix[b] + accept_len[b] + 1);

    /* projections */
    enum { R = 3, HID = 24, H = 2 };
    void *x = random_tensor((size_t)B * R * HID, dtype), *w = random_tensor((size_t)H * D * HID, dtype);
    double *y = (double *)malloc(sizeof(double) * B * R * H * D);
    CHECK(oracle_project(x, w, dtype, B, R, HID, H, D, y) == 0);
    CHECK(all_finite(y, (size_t)B * R * H * D));

    free(parent); free(prefix); free(q); free(k); free(v); free(out); free(lse); free(q3); free(pq); free(scores);
    free(kept); free(rows); free(gathered); free(q_pos); free(q5); free(row_entropy); free(logits); free(token);
    free(x); free(w); free(y);
    return 0;
}

int main(void)
{
    CHECK(oracle_hw_threads() >= 1);
    for (int dtype = 0; dtype < 2; dtype++)
        for (int threads = 1; threads <= 3; threads += 2)
            if (run(dtype, threads))
                return 1;
    printf("oracle selftest ok\n");
    return 0;
}
