/*
 * CPU oracle for the DREAM speculative-decode hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, float64 implementations of the four operations the GPU library provides,
 * written from the paper's definitions.  Nothing here is tuned, blocked or fused, and no
 * source, header, table or helper is shared with the HIP path.  Only the tests, the smoke
 * check and the benchmark's cpu_baseline leg may call into this file; the product never does.
 *
 * What each function follows:
 *   oracle_attn_row / oracle_tree_attn
 *       softmax(Q K^T / sqrt(z)) V  (Section 3.1, Eq. 1) restricted by the draft-tree mask
 *       (Section 3.1, tree-masking paragraph): a tree node sees the whole cached prefix and
 *       its ancestors; in the target's verification pass it also sees itself
 *       (include_self = 1), in the draft's cross-attention only strict ancestors
 *       (include_self = 0; Section 3.1: the key/value set for the next token is the target
 *       features followed by the draft features of the already drafted positions).
 *   oracle_visual_scores
 *       importance of key token j = sum of the attention weights it receives in the
 *       last-layer causal attention matrix (Section 3.3), summed over heads.
 *   oracle_topk_keep / oracle_gather_rows
 *       sort the visual span's scores, keep the top ones according to the keep ratio, record
 *       their indices, subsample the token rows with them (Section 3.3); kept count rounds to
 *       nearest (Section 3: q + round(v / r) draft-side tokens).
 *   oracle_accept_path
 *       greedy (temperature 0) form of the acceptance rule of Section 2.1: a drafted token is
 *       accepted iff it equals the target's arg-max at its parent and its parent is accepted;
 *       everything after the first mismatch on a path is discarded; the target's own token at
 *       the last accepted node is the bonus token (Section 4: up to depth + 1 tokens a round).
 *
 *   oracle_attention_entropy
 *       the token-level attention entropy of a layer, Eq. 2 of Section 3.2: minus the sum of
 *       A log A over each row of the causal attention matrix, averaged over rows and heads.
 *   oracle_project
 *       the linear maps of Eq. 1 (Section 3.1): Q = E W_Q, K = S W_K, V = S W_V, one output row per
 *       input feature row, split into heads.
 *   oracle_kv_commit
 *       what Section 2.1 says happens after verification: the tokens after the first rejection
 *       are discarded and decoding continues from the accepted prefix; with KV caching
 *       (Section 4, setup) that means the cache rows of the accepted root-to-node path become
 *       the next rows of the prefix and every other tree row is dropped.
 *
 * Parity pins (tests/test_oracle_*.py, no GPU needed): chain tree == dense causal attention
 * (library SDPA in float64), Q = 0 closed forms (mean of V rows; harmonic-number column sums),
 * dense-mask brute force, mask-leak detectors, exhaustive subset search for top-k, root-to-leaf
 * path enumeration and planted paths/ties for acceptance; for the commit, hand-written row markers
 * (including a path whose destination rows are other entries' source rows), the no-op chain path and
 * "attention over the committed cache == tree-masked attention of the accepted node"; for the entropy, the closed form log(i+1) of uniform rows, the one-hot limit, and the identity
 * H = LSE - scale q.(attention output with V := K) evaluated through the attention oracle; for the
 * projections, identity and averaging weights, linearity and a float64 library product.  No function
 * here is unpinned.
 *
 * Tensor layouts (C order): q [B,Tq,Hq,D]; k,v [B,Hkv,s_max,D]; logits [B,T,V].
 * dtype: 0 = IEEE float32, 1 = bfloat16 bit patterns (uint16); both are widened exactly to double.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

static double load_as_double(const void *p, int dtype, int64_t i)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)p)[i];
    uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static size_t elem_size(int dtype) { return dtype == ORACLE_F32 ? 4 : 2; }

/* Number of threads the batched entry points use (1 = serial). */
static int g_threads = 1;
void oracle_set_threads(int n) { g_threads = n < 1 ? 1 : n; }
int oracle_get_threads(void) { return g_threads; }
int oracle_hw_threads(void)
{
#ifdef _OPENMP
    return omp_get_num_procs();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------------------------ */
/* Masked attention, one output row.                                                          */
/*   q_row      : element offset of this query's D values inside q                            */
/*   kv_base    : element offset of key row 0 of this (sequence, kv head) inside k and v      */
/*   prefix_len : P, number of prefix rows, all visible                                       */
/*   parent     : this sequence's parent array (parent[0] = -1)                               */
/*   node       : tree node the query belongs to                                              */
/*   include_self : 1 -> node itself and its ancestors visible; 0 -> strict ancestors only    */
/* out[D], *lse (log-sum-exp of the scaled scores).  Empty visible set: out = 0, lse = -inf.  */
/* ------------------------------------------------------------------------------------------ */
void oracle_attn_row(const void *q, const void *k, const void *v, int dtype, int D,
                     int64_t q_row, int64_t kv_base, int prefix_len, const int32_t *parent,
                     int node, int include_self, double scale, double *out, double *lse)
{
    /* visible keys: 0..P-1, then P + a for every visible tree node a */
    int n_anc = 0;
    for (int a = include_self ? node : parent[node]; a >= 0; a = parent[a])
        n_anc++;
    int n_vis = prefix_len + n_anc;
    for (int d = 0; d < D; d++)
        out[d] = 0.0;
    if (n_vis == 0) {
        if (lse)
            *lse = -INFINITY;
        return;
    }
    int64_t *key = (int64_t *)malloc(sizeof(int64_t) * (size_t)n_vis);
    double *s = (double *)malloc(sizeof(double) * (size_t)n_vis);
    for (int j = 0; j < prefix_len; j++)
        key[j] = j;
    int c = prefix_len;
    for (int a = include_self ? node : parent[node]; a >= 0; a = parent[a])
        key[c++] = (int64_t)prefix_len + a;

    double m = -INFINITY;
    for (int j = 0; j < n_vis; j++) {
        double dot = 0.0;
        for (int d = 0; d < D; d++)
            dot += load_as_double(q, dtype, q_row + d) * load_as_double(k, dtype, kv_base + key[j] * D + d);
        s[j] = scale * dot;
        if (s[j] > m)
            m = s[j];
    }
    double denom = 0.0;
    for (int j = 0; j < n_vis; j++) {
        s[j] = exp(s[j] - m);
        denom += s[j];
    }
    for (int j = 0; j < n_vis; j++) {
        double w = s[j] / denom;
        for (int d = 0; d < D; d++)
            out[d] += w * load_as_double(v, dtype, kv_base + key[j] * D + d);
    }
    if (lse)
        *lse = m + log(denom);
    free(key);
    free(s);
}

/* All rows.  q_node[b*Tq + i] names the tree node of query row i (NULL: node i = row i).     */
/* out [B,Tq,Hq,D] double; lse [B,Hq,Tq] double (nullable).                                   */
int oracle_tree_attn(const void *q, const void *k, const void *v, int dtype,
                     int B, int Tq, int Hq, int Hkv, int D, int64_t s_max,
                     const int32_t *prefix_len, int n_tree, const int32_t *parent,
                     const int32_t *q_node, int include_self, double scale,
                     double *out, double *lse)
{
    if (Hkv <= 0 || Hq % Hkv != 0)
        return -1;
    int G = Hq / Hkv;
    int64_t total = (int64_t)B * Hq * Tq;
#pragma omp parallel for schedule(dynamic, 4) num_threads(g_threads)
    for (int64_t w = 0; w < total; w++) {
        int i = (int)(w % Tq);
        int h = (int)((w / Tq) % Hq);
        int b = (int)(w / ((int64_t)Tq * Hq));
        int node = q_node ? q_node[(int64_t)b * Tq + i] : i;
        int64_t q_row = (((int64_t)b * Tq + i) * Hq + h) * D;
        int64_t kv_base = ((int64_t)b * Hkv + h / G) * s_max * D;
        oracle_attn_row(q, k, v, dtype, D, q_row, kv_base, prefix_len[b],
                        parent + (int64_t)b * n_tree, node, include_self, scale,
                        out + q_row, lse ? lse + ((int64_t)b * Hq + h) * Tq + i : NULL);
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------ */
/* Visual-token importance: column sums of the causal attention probabilities (Section 3.3).  */
/* Row r of q sits at position pos = q_pos ? q_pos[b,r] : r and attends keys 0..pos.          */
/* scores[b, j - vis_start] = sum over heads, over rows with pos >= j (pos > j when           */
/* include_diag = 0) of softmax_row(scale q k^T)[j], for j in [vis_start, vis_start+vis_len). */
/* ------------------------------------------------------------------------------------------ */
int oracle_visual_scores(const void *q, const int32_t *q_pos, int n_q, const void *k, int dtype,
                         int B, int Hq, int Hkv, int D, int64_t s_max,
                         int vis_start, int vis_len, double scale, int include_diag,
                         double *scores)
{
    if (Hkv <= 0 || Hq % Hkv != 0)
        return -1;
    int G = Hq / Hkv;
    int64_t nbh = (int64_t)B * Hq;
    double *part = (double *)calloc((size_t)(nbh * (vis_len > 0 ? vis_len : 1)), sizeof(double));
#pragma omp parallel for schedule(dynamic, 1) num_threads(g_threads)
    for (int64_t bh = 0; bh < nbh; bh++) {
        int b = (int)(bh / Hq), h = (int)(bh % Hq);
        int64_t kv_base = ((int64_t)b * Hkv + h / G) * s_max * D;
        double *acc = part + bh * vis_len;
        for (int r = 0; r < n_q; r++) {
            int pos = q_pos ? q_pos[(int64_t)b * n_q + r] : r;
            int n_keys = pos + 1;
            int64_t q_row = (((int64_t)b * n_q + r) * Hq + h) * D;
            double *s = (double *)malloc(sizeof(double) * (size_t)n_keys);
            double m = -INFINITY;
            for (int j = 0; j < n_keys; j++) {
                double dot = 0.0;
                for (int d = 0; d < D; d++)
                    dot += load_as_double(q, dtype, q_row + d) * load_as_double(k, dtype, kv_base + (int64_t)j * D + d);
                s[j] = scale * dot;
                if (s[j] > m)
                    m = s[j];
            }
            double denom = 0.0;
            for (int j = 0; j < n_keys; j++) {
                s[j] = exp(s[j] - m);
                denom += s[j];
            }
            for (int j = vis_start; j < vis_start + vis_len && j < n_keys; j++) {
                if (!include_diag && j == pos)
                    continue;
                acc[j - vis_start] += s[j] / denom;
            }
            free(s);
        }
    }
    for (int b = 0; b < B; b++)
        for (int j = 0; j < vis_len; j++) {
            double t = 0.0;
            for (int h = 0; h < Hq; h++)
                t += part[((int64_t)b * Hq + h) * vis_len + j];
            scores[(int64_t)b * vis_len + j] = t;
        }
    free(part);
    return 0;
}

/* Kept count: v * keep_num / keep_den rounded to nearest, halves up, clamped to [0, v].      */
int oracle_keep_count(int vis_len, int keep_num, int keep_den)
{
    int64_t k = (2 * (int64_t)vis_len * keep_num + keep_den) / (2 * (int64_t)keep_den);
    if (k < 0)
        k = 0;
    if (k > vis_len)
        k = vis_len;
    return (int)k;
}

typedef struct {
    double score;
    int32_t idx;
} scored_t;

static int by_score_desc_then_index(const void *a, const void *b)
{
    const scored_t *x = (const scored_t *)a, *y = (const scored_t *)b;
    if (x->score > y->score)
        return -1;
    if (x->score < y->score)
        return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

static int by_int(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* scores [B, vis_len] -> kept [B, k] absolute positions (vis_start + index), ascending.      */
/* Full sort by (score descending, index ascending); the first k entries are kept.            */
int oracle_topk_keep(const double *scores, int B, int vis_start, int vis_len,
                     int keep_num, int keep_den, int32_t *kept)
{
    int k = oracle_keep_count(vis_len, keep_num, keep_den);
    scored_t *tmp = (scored_t *)malloc(sizeof(scored_t) * (size_t)(vis_len > 0 ? vis_len : 1));
    for (int b = 0; b < B; b++) {
        for (int j = 0; j < vis_len; j++) {
            tmp[j].score = scores[(int64_t)b * vis_len + j];
            tmp[j].idx = j;
        }
        qsort(tmp, (size_t)vis_len, sizeof(scored_t), by_score_desc_then_index);
        for (int t = 0; t < k; t++)
            kept[(int64_t)b * k + t] = vis_start + tmp[t].idx;
        qsort(kept + (int64_t)b * k, (size_t)k, sizeof(int32_t), by_int);
    }
    free(tmp);
    return k;
}

/* dst[b, t, :] = src[b, kept[b, t], :]; rows of row_elems elements of the given dtype.       */
void oracle_gather_rows(const void *src, int dtype, int B, int64_t n_rows, int64_t row_elems,
                        const int32_t *kept, int k, void *dst)
{
    size_t rb = (size_t)row_elems * elem_size(dtype);
    for (int b = 0; b < B; b++)
        for (int t = 0; t < k; t++)
            memcpy((char *)dst + ((size_t)b * k + t) * rb,
                   (const char *)src + ((size_t)b * n_rows + kept[(int64_t)b * k + t]) * rb, rb);
}

/* ------------------------------------------------------------------------------------------ */
/* Greedy acceptance over the verified tree (Section 2.1 rule at temperature 0, Section 4).   */
/* logits [B,T,V]; token,parent [B,T]; outputs node_argmax [B,T], accept_len [B],             */
/* accept_path [B, max_depth+1] (root first, -1 padded), bonus_token [B].                     */
/* Nodes deeper than max_depth are never accepted.                                            */
/* ------------------------------------------------------------------------------------------ */
int oracle_accept_path(const void *logits, int dtype, int B, int T, int V,
                       const int32_t *token, const int32_t *parent, int max_depth,
                       int32_t *node_argmax, int32_t *accept_len, int32_t *accept_path,
                       int32_t *bonus_token)
{
    int64_t rows = (int64_t)B * T;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t r = 0; r < rows; r++) {
        int best = 0;
        double bv = load_as_double(logits, dtype, r * V);
        for (int t = 1; t < V; t++) {
            double x = load_as_double(logits, dtype, r * V + t);
            if (x > bv) { /* strict: the first index of the maximum wins */
                bv = x;
                best = t;
            }
        }
        node_argmax[r] = best;
    }
    int *depth = (int *)malloc(sizeof(int) * (size_t)T);
    char *acc = (char *)malloc((size_t)T);
    for (int b = 0; b < B; b++) {
        const int32_t *par = parent + (int64_t)b * T, *tok = token + (int64_t)b * T;
        const int32_t *am = node_argmax + (int64_t)b * T;
        depth[0] = 0;
        acc[0] = 1;
        int best = 0;
        for (int i = 1; i < T; i++) {
            depth[i] = depth[par[i]] + 1;
            acc[i] = (char)(acc[par[i]] && tok[i] == am[par[i]] && depth[i] <= max_depth);
            if (acc[i] && depth[i] > depth[best])
                best = i; /* strict '>' keeps the lowest node index among equally deep ones */
        }
        accept_len[b] = depth[best];
        int32_t *path = accept_path + (int64_t)b * (max_depth + 1);
        for (int t = 0; t <= max_depth; t++)
            path[t] = -1;
        for (int a = best; a >= 0; a = par[a])
            path[depth[a]] = a;
        bonus_token[b] = am[best];
    }
    free(depth);
    free(acc);
    return 0;
}

/* ------------------------------------------------------------------------------------------ */
/* KV-cache commit after acceptance (Section 2.1; KV caching: Section 4).                     */
/* cache [B,Hkv,s_max,D] of the given dtype, tree rows at [P_b, P_b+T).  For every sequence   */
/* and KV head: new row P_b + j = old row P_b + path[b][j] for j = 0 .. accept_len[b]          */
/* (path[b][0] is the root); every other row keeps its content.  new_len[b] = P_b +           */
/* accept_len[b] + 1.  The old tree rows are copied aside first, so the result is the          */
/* definition itself and does not depend on any order of moves.                                */
/* Returns -1 (cache untouched) if a path entry is outside [0,T) or a length does not fit.     */
/* ------------------------------------------------------------------------------------------ */
int oracle_kv_commit(void *cache, int dtype, int B, int Hkv, int64_t s_max, int D,
                     const int32_t *prefix_len, int T, const int32_t *path, int path_stride,
                     const int32_t *accept_len, int32_t *new_len)
{
    size_t rb = (size_t)D * elem_size(dtype);
    for (int b = 0; b < B; b++) {
        if (accept_len[b] < 0 || accept_len[b] >= path_stride || accept_len[b] >= T)
            return -1;
        if (prefix_len[b] < 0 || (int64_t)prefix_len[b] + T > s_max)
            return -1;
        for (int j = 0; j <= accept_len[b]; j++)
            if (path[(int64_t)b * path_stride + j] < 0 || path[(int64_t)b * path_stride + j] >= T)
                return -1;
    }
    char *old_rows = (char *)malloc(rb * (size_t)T);
    for (int b = 0; b < B; b++) {
        for (int h = 0; h < Hkv; h++) {
            char *tree = (char *)cache + (((size_t)b * Hkv + h) * (size_t)s_max + (size_t)prefix_len[b]) * rb;
            memcpy(old_rows, tree, rb * (size_t)T);
            for (int j = 0; j <= accept_len[b]; j++)
                memcpy(tree + (size_t)j * rb, old_rows + (size_t)path[(int64_t)b * path_stride + j] * rb, rb);
        }
        if (new_len)
            new_len[b] = prefix_len[b] + accept_len[b] + 1;
    }
    free(old_rows);
    return 0;
}

/* ------------------------------------------------------------------------------------------ */
/* Attention entropy, Eq. 2 (Section 3.2).  Row r of q sits at position pos = q_pos ?          */
/* q_pos[b,r] : r and attends keys 0..pos; A = softmax_row(scale q k^T).                       */
/* row_entropy[b,h,r] = - sum_j A_j log A_j (natural log; A_j = 0 contributes 0);              */
/* ae[b] = mean over heads and rows.                                                           */
/* ------------------------------------------------------------------------------------------ */
int oracle_attention_entropy(const void *q, const int32_t *q_pos, int n_q, const void *k, int dtype,
                             int B, int Hq, int Hkv, int D, int64_t s_max, double scale,
                             double *row_entropy, double *ae)
{
    if (Hkv <= 0 || Hq % Hkv != 0)
        return -1;
    int G = Hq / Hkv;
    int64_t nbh = (int64_t)B * Hq;
#pragma omp parallel for schedule(dynamic, 1) num_threads(g_threads)
    for (int64_t bh = 0; bh < nbh; bh++) {
        int b = (int)(bh / Hq), h = (int)(bh % Hq);
        int64_t kv_base = ((int64_t)b * Hkv + h / G) * s_max * D;
        for (int r = 0; r < n_q; r++) {
            int pos = q_pos ? q_pos[(int64_t)b * n_q + r] : r;
            int n_keys = pos + 1;
            int64_t q_row = (((int64_t)b * n_q + r) * Hq + h) * D;
            double *s = (double *)malloc(sizeof(double) * (size_t)n_keys);
            double m = -INFINITY;
            for (int j = 0; j < n_keys; j++) {
                double dot = 0.0;
                for (int d = 0; d < D; d++)
                    dot += load_as_double(q, dtype, q_row + d) * load_as_double(k, dtype, kv_base + (int64_t)j * D + d);
                s[j] = scale * dot;
                if (s[j] > m)
                    m = s[j];
            }
            double denom = 0.0;
            for (int j = 0; j < n_keys; j++)
                denom += exp(s[j] - m);
            double H = 0.0;
            for (int j = 0; j < n_keys; j++) {
                double a = exp(s[j] - m) / denom;
                if (a > 0.0)
                    H -= a * log(a);
            }
            row_entropy[bh * n_q + r] = H;
            free(s);
        }
    }
    for (int b = 0; b < B; b++) {
        double t = 0.0;
        for (int64_t i = 0; i < (int64_t)Hq * n_q; i++)
            t += row_entropy[(int64_t)b * Hq * n_q + i];
        ae[b] = t / ((double)Hq * n_q);
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------ */
/* Projections of Eq. 1 (Section 3.1): y[b,r,h,:] = x[b,r,:] . W[h*D .. h*D+D-1, :]^T          */
/* x [B,R,hidden], w [H*D, hidden] (row n holds the weights of output feature n), both of the   */
/* given dtype; out [B,R,H,D] float64.                                                          */
/* ------------------------------------------------------------------------------------------ */
int oracle_project(const void *x, const void *w, int dtype, int B, int R, int hidden, int H, int D, double *out)
{
    int64_t rows = (int64_t)B * R;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t br = 0; br < rows; br++) {
        for (int n = 0; n < H * D; n++) {
            double acc = 0.0;
            for (int k = 0; k < hidden; k++)
                acc += load_as_double(x, dtype, br * hidden + k) * load_as_double(w, dtype, (int64_t)n * hidden + k);
            out[br * H * D + n] = acc;
        }
    }
    return 0;
}
