// dream_spec_accept: acceptance over the verified tree at a sampling temperature (Section 2.1: a drafted token
// d is accepted with probability min(1, P_target(d) / P_draft(d)); after a rejection the rest is discarded and
// the target's distribution decides the next token; Section 4 evaluates at temperature 1).  For a tree the
// children of the current node are tried in node order; after a rejected child the target distribution becomes
// the positive part of (target - draft), the rejected token leaves the draft distribution, and the next child is
// tried against those; the first accepted child becomes the current node.  With no accepted child the next
// token is drawn from the current target distribution by inverting its cumulative sum in token order.  The
// uniform random numbers are inputs.
//
// Three launches.  softmax_stats_kernel (parallel over rows and 8192-logit chunks) leaves (max, sum of
// exponentials) per chunk for the target row of every node and the draft row of every node with children.
// residual_stats_kernel (same grid) merges them per node and, for nodes with children, leaves the sum of the
// first residual max(p - q, 0) per chunk.  spec_walk_kernel, one workgroup of 1024 threads per sequence, then
// evaluates the test of every node against its parent's untouched distributions in parallel: that is exactly
// the test the walk performs whenever a node is the first child tried, so the walk descends through first
// children by table lookup.  After a first rejection the residual is known through its chunk sums: the second
// child's test is two logit lookups, and a draw needs only the one chunk that holds the drawn point.  Only a
// second rejection at the same node turns the distributions into arrays (one pass over the two logit rows
// writes the second residual and the reduced draft: unnormalised floats in the workspace, L2-resident); later
// siblings are tested against those, one pass per further rejection, and an accepted sibling returns to the
// table walk.  A draw is per-thread contiguous partial sums, a block scan and one thread's rescan.  Every
// reduction has a fixed order, so the result is reproducible.  With at most 12 chunks per row (98304 tokens)
// the second kernel is skipped: the walk merges the statistics itself and sums the first residual of a node only
// when a first child is rejected there, which is cheaper than a launch for short rows.  Roofline: HBM, one read
// of the logit rows (a second read of the rows of nodes with children).
#include "common.h"
#include <type_traits>

using namespace dream;

namespace {

constexpr int NT = 1024;

template <bool BF16>
__device__ __forceinline__ float load_logit(const void *p, int64_t i)
{
    return BF16 ? bf16_bits_to_float(reinterpret_cast<const uint16_t *>(p)[i]) : reinterpret_cast<const float *>(p)[i];
}

// block-wide reductions over 1024 threads (16 waves) in a fixed order; `red` holds 16 floats
__device__ __forceinline__ float block_sum(float v, float *red, int tid)
{
    for (int off = 32; off > 0; off >>= 1)
        v += __shfl_xor(v, off);
    __syncthreads();
    if ((tid & 63) == 0)
        red[tid >> 6] = v;
    __syncthreads();
    float t = 0.0f;
#pragma unroll
    for (int w = 0; w < 16; w++)
        t += red[w];
    return t;
}
__device__ __forceinline__ float block_max(float v, float *red, int tid)
{
    for (int off = 32; off > 0; off >>= 1)
        v = fmaxf(v, __shfl_xor(v, off));
    __syncthreads();
    if ((tid & 63) == 0)
        red[tid >> 6] = v;
    __syncthreads();
    float t = red[0];
#pragma unroll
    for (int w = 1; w < 16; w++)
        t = fmaxf(t, red[w]);
    return t;
}
__device__ __forceinline__ int block_min_int(int v, int *red, int tid)
{
    for (int off = 32; off > 0; off >>= 1)
        v = min(v, __shfl_xor(v, off));
    __syncthreads();
    if ((tid & 63) == 0)
        red[tid >> 6] = v;
    __syncthreads();
    int t = red[0];
#pragma unroll
    for (int w = 1; w < 16; w++)
        t = min(t, red[w]);
    return t;
}

constexpr int STAT_CHUNK = 8192;    // logits per workgroup of the statistics pass

// tokens t .. t+7 of a row (t a multiple of 8); `vec`: the row is 16-byte aligned and holds a multiple of 8 tokens.
// Tokens past the end come back as -inf.
template <bool BF16>
__device__ __forceinline__ void load8(const void *base, int64_t row, int t, int vocab, bool vec, float v[8])
{
    if (vec && t + 8 <= vocab) {
        if (BF16) {
            const uint4 u = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(base) + row + t);
            const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
            for (int j = 0; j < 4; j++) {
                v[2 * j] = __uint_as_float(w[j] << 16);
                v[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
            }
        } else {
            const float4 a = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(base) + row + t);
            const float4 c = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(base) + row + t + 4);
            v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = c.x; v[5] = c.y; v[6] = c.z; v[7] = c.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; j++)
            v[j] = t + j < vocab ? load_logit<BF16>(base, row + t + j) : -INFINITY;
    }
}

// (max, sum of exp(x/temp - max)) of one 8192-logit chunk of one row.  z = 0: target rows; z = 1: draft rows,
// skipped (max = -inf, sum = 0) for nodes without children.
template <bool BF16>
__global__ __launch_bounds__(256) void softmax_stats_kernel(const void *tlogits, const void *dlogits, int n_tree, int vocab,
                                                            int n_chunks, bool vec, const int32_t *parent, float inv_temp,
                                                            float *stat_m, float *stat_s)
{
    const int chunk = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t node_row = blockIdx.y;                      // b * n_tree + node
    const int which = blockIdx.z;
    const int64_t slot = ((int64_t)which * gridDim.y + node_row) * n_chunks + chunk;
    __shared__ float red[4];
    if (which == 1) {
        const int b = (int)(node_row / n_tree), node = (int)(node_row - (int64_t)b * n_tree);
        int kids = 0;
        for (int i = tid; i < n_tree; i += 256)
            kids |= parent[(int64_t)b * n_tree + i] == node;
        if (!__syncthreads_or(kids)) {
            if (tid == 0) {
                stat_m[slot] = -INFINITY;
                stat_s[slot] = 0.0f;
            }
            return;
        }
    }
    const void *base = which ? dlogits : tlogits;
    const int64_t row = node_row * vocab;
    const int begin = chunk * STAT_CHUNK;
    float x[STAT_CHUNK / 256];
    float m = -INFINITY;
#pragma unroll
    for (int r = 0; r < STAT_CHUNK / 2048; r++) {
        load8<BF16>(base, row, begin + (r * 256 + tid) * 8, vocab, vec, x + 8 * r);
#pragma unroll
        for (int j = 0; j < 8; j++) {
            x[8 * r + j] *= inv_temp;
            m = fmaxf(m, x[8 * r + j]);
        }
    }
    for (int off = 32; off > 0; off >>= 1)
        m = fmaxf(m, __shfl_xor(m, off));
    if (lane == 0)
        red[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float sum = 0.0f;
    if (m > -INFINITY) {
#pragma unroll
        for (int j = 0; j < STAT_CHUNK / 256; j++)
            sum += __expf(x[j] - m);                          // exp(-inf) = 0 for the padding
    }
    for (int off = 32; off > 0; off >>= 1)
        sum += __shfl_xor(sum, off);
    __syncthreads();
    if (lane == 0)
        red[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        stat_m[slot] = m;
        stat_s[slot] = (red[0] + red[1]) + (red[2] + red[3]);
    }
}

// (max, sum of exponentials relative to it) of the target row and, if asked, the draft row of a node from their
// chunk statistics.  Every wave does the same: lane c takes chunk c (and c + 64, ... beyond 64 chunks), the
// maximum and then the rescaled sum are reduced with xor shuffles, which is a fixed order.
__device__ __forceinline__ void merge_node_stats(const float *stat_m, const float *stat_s, int64_t node_row, int64_t rows_all,
                                                 int n_chunks, bool with_draft, int lane, float &mt, float &zt, float &md, float &zd)
{
    const float *tm = stat_m + node_row * n_chunks, *ts = stat_s + node_row * n_chunks;
    const float *dm = stat_m + (rows_all + node_row) * n_chunks, *dsum = stat_s + (rows_all + node_row) * n_chunks;
    float m0 = -INFINITY, m1 = -INFINITY;
    for (int c = lane; c < n_chunks; c += 64) {
        m0 = fmaxf(m0, tm[c]);
        if (with_draft)
            m1 = fmaxf(m1, dm[c]);
    }
    for (int off = 32; off > 0; off >>= 1) {
        m0 = fmaxf(m0, __shfl_xor(m0, off));
        m1 = fmaxf(m1, __shfl_xor(m1, off));
    }
    float z0 = 0.0f, z1 = 0.0f;
    for (int c = lane; c < n_chunks; c += 64) {
        const float a = ts[c];
        if (a > 0.0f)
            z0 += a * __expf(tm[c] - m0);
        if (with_draft) {
            const float d = dsum[c];
            if (d > 0.0f)
                z1 += d * __expf(dm[c] - m1);
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        z0 += __shfl_xor(z0, off);
        z1 += __shfl_xor(z1, off);
    }
    mt = m0; zt = z0; md = m1; zd = z1;
}

// The residual max(p - q, 0) of a node after its first rejected child (p, q: the normalised target and draft
// distributions; p itself where the caller says the residual is empty).
__device__ __forceinline__ float residual1(float lt, float ld, float inv_temp, float mt, float md, float ip, float iq)
{
    return fmaxf(__expf(lt * inv_temp - mt) * ip - __expf(ld * inv_temp - md) * iq, 0.0f);
}

// Per node: the merged statistics of its rows (written by the workgroup of chunk 0: the walk reads four
// numbers per node instead of merging again) and, for a node with children, the sum of the first residual over
// each 8192-logit chunk: what the walk needs to test a second child, or to draw after a single rejection,
// without a pass of its own over the vocabulary.
template <bool BF16>
__global__ __launch_bounds__(256) void residual_stats_kernel(const void *tlogits, const void *dlogits, int n_tree, int vocab,
                                                             int n_chunks, bool vec, const int32_t *parent, float inv_temp,
                                                             const float *stat_m, const float *stat_s, float *res_sum,
                                                             float4 *node_stats)
{
    const int chunk = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t node_row = blockIdx.y, rows_all = gridDim.y;
    const int b = (int)(node_row / n_tree), node = (int)(node_row - (int64_t)b * n_tree);
    __shared__ float red[4];
    int kids = 0;
    for (int i = tid; i < n_tree; i += 256)
        kids |= parent[(int64_t)b * n_tree + i] == node;
    const bool has_kids = __syncthreads_or(kids);
    if (!has_kids && chunk > 0) {
        if (tid == 0)
            res_sum[node_row * n_chunks + chunk] = 0.0f;
        return;
    }
    // the logits of this chunk are requested before the statistics they will be scaled with
    const int64_t row = node_row * vocab;
    const int begin = chunk * STAT_CHUNK;
    float tv[STAT_CHUNK / 256], dv[STAT_CHUNK / 256];
    if (has_kids) {
#pragma unroll
        for (int r = 0; r < STAT_CHUNK / 2048; r++) {
            const int t = begin + (r * 256 + tid) * 8;
            load8<BF16>(tlogits, row, t, vocab, vec, tv + 8 * r);
            load8<BF16>(dlogits, row, t, vocab, vec, dv + 8 * r);
        }
    }
    float mt, zt, md, zd;
    merge_node_stats(stat_m, stat_s, node_row, rows_all, n_chunks, has_kids, lane, mt, zt, md, zd);
    if (chunk == 0 && tid == 0)
        node_stats[node_row] = float4{mt, zt, md, zd};
    if (!has_kids) {
        if (tid == 0)
            res_sum[node_row * n_chunks] = 0.0f;
        return;
    }
    const float ip = 1.0f / zt, iq = zd > 0.0f ? 1.0f / zd : 0.0f;
    float sum = 0.0f;
#pragma unroll
    for (int r = 0; r < STAT_CHUNK / 2048; r++) {
        const int t = begin + (r * 256 + tid) * 8;
#pragma unroll
        for (int j = 0; j < 8; j++)
            if (t + j < vocab)
                sum += residual1(tv[8 * r + j], dv[8 * r + j], inv_temp, mt, md, ip, iq);
    }
    for (int off = 32; off > 0; off >>= 1)
        sum += __shfl_xor(sum, off);
    if (lane == 0)
        red[wave] = sum;
    __syncthreads();
    if (tid == 0)
        res_sum[node_row * n_chunks + chunk] = (red[0] + red[1]) + (red[2] + red[3]);
}

// LAZY (at most LAZY_CHUNKS chunks per row): residual_stats_kernel has not run; the walk merges the chunk
// statistics of every node itself and sums the first residual over the chunks of a node only when a first child
// is rejected there: one pass of the workgroup over two short rows is cheaper than a launch.
constexpr int LAZY_CHUNKS = 12;

template <bool BF16, bool LAZY>
__global__ __launch_bounds__(NT) void spec_walk_kernel(const void *tlogits, const void *dlogits, int n_tree, int vocab, int n_chunks,
                                                       bool vec, const int32_t *token, const int32_t *parent, const float *u_accept,
                                                       const float *u_bonus, int max_depth, float inv_temp, const float *stat_m,
                                                       const float *stat_s, const float *res_sum, const float4 *node_stats, float *work,
                                                       int32_t *accept_len, int32_t *accept_path, int32_t *bonus_token)
{
    __shared__ int32_t s_par[DREAM_MAX_TREE_ACCEPT];
    __shared__ int32_t s_tok[DREAM_MAX_TREE_ACCEPT];
    __shared__ int32_t s_first[DREAM_MAX_TREE_ACCEPT];     // first child of a node, or INT_MAX
    __shared__ float s_mt[DREAM_MAX_TREE_ACCEPT], s_zt[DREAM_MAX_TREE_ACCEPT];   // target row: max, sum
    __shared__ float s_md[DREAM_MAX_TREE_ACCEPT], s_zd[DREAM_MAX_TREE_ACCEPT];   // draft row
    __shared__ float s_qx[DREAM_MAX_TREE_ACCEPT];          // unnormalised draft mass of a node's token at its parent
    __shared__ uint8_t s_ok[DREAM_MAX_TREE_ACCEPT];        // the node passes its test when it is the first child tried
    __shared__ float s_redf[16];
    __shared__ int s_redi[16];
    __shared__ float s_scan[16];
    constexpr int NONE = 0x7fffffff;
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t bt = (int64_t)b * n_tree;
    for (int i = tid; i < n_tree; i += NT) {
        const int par = parent[bt + i];
        s_par[i] = par < i ? par : -1;
        s_tok[i] = min(max(token[bt + i], 0), vocab - 1);   // device metadata is trusted but kept inside the row
        s_first[i] = NONE;
        if (LAZY) {
            const int64_t rows_all = (int64_t)gridDim.x * n_tree;
            const float *tm = stat_m + (bt + i) * n_chunks, *ts = stat_s + (bt + i) * n_chunks;
            const float *dm = stat_m + (rows_all + bt + i) * n_chunks, *dsum = stat_s + (rows_all + bt + i) * n_chunks;
            // one row at a time: a workgroup of 1024 threads has 128 registers per thread
            float mt = -INFINITY, md = -INFINITY, zt = 0.0f, zd = 0.0f;
            {
                float am[LAZY_CHUNKS], as[LAZY_CHUNKS];
#pragma unroll
                for (int u = 0; u < LAZY_CHUNKS; u++) {
                    am[u] = u < n_chunks ? tm[u] : -INFINITY;
                    as[u] = u < n_chunks ? ts[u] : 0.0f;
                }
#pragma unroll
                for (int u = 0; u < LAZY_CHUNKS; u++)
                    mt = fmaxf(mt, am[u]);
#pragma unroll
                for (int u = 0; u < LAZY_CHUNKS; u++)
                    if (u < n_chunks && as[u] > 0.0f)
                        zt += as[u] * __expf(am[u] - mt);
            }
            {
                float bm[LAZY_CHUNKS], bs[LAZY_CHUNKS];
#pragma unroll
                for (int u = 0; u < LAZY_CHUNKS; u++) {
                    bm[u] = u < n_chunks ? dm[u] : -INFINITY;
                    bs[u] = u < n_chunks ? dsum[u] : 0.0f;
                }
#pragma unroll
                for (int u = 0; u < LAZY_CHUNKS; u++)
                    md = fmaxf(md, bm[u]);
#pragma unroll
                for (int u = 0; u < LAZY_CHUNKS; u++)
                    if (u < n_chunks && bs[u] > 0.0f)
                        zd += bs[u] * __expf(bm[u] - md);
            }
            s_mt[i] = mt; s_zt[i] = zt; s_md[i] = md; s_zd[i] = zd;
        } else {
            const float4 ns = node_stats[bt + i];
            s_mt[i] = ns.x; s_zt[i] = ns.y; s_md[i] = ns.z; s_zd[i] = ns.w;
        }
    }
    float *P = work + (int64_t)b * 3 * vocab, *Q = P + vocab, *R = Q + vocab;
    int32_t *path = accept_path + (int64_t)b * (max_depth + 1);
    if (tid <= max_depth)
        path[tid] = tid == 0 ? 0 : -1;
    __syncthreads();
    for (int i = tid; i < n_tree; i += NT) {
        const int p = s_par[i];
        if (i > 0 && p >= 0) {
            atomicMin(&s_first[p], i);
            const int x = s_tok[i];
            const float px = __expf(load_logit<BF16>(tlogits, (bt + p) * vocab + x) * inv_temp - s_mt[p]);
            const float qx = __expf(load_logit<BF16>(dlogits, (bt + p) * vocab + x) * inv_temp - s_md[p]);
            const float ratio = qx > 0.0f ? (px / s_zt[p]) / (qx / s_zd[p]) : (px > 0.0f ? INFINITY : 0.0f);
            s_qx[i] = qx;
            s_ok[i] = u_accept[bt + i] < fminf(1.0f, ratio);
        }
    }
    __syncthreads();

    // Inverse-CDF draw over the values val(t) of tokens [r0, r1) (r0 a multiple of 8), read through
    // `fetch8(t, v)` (8 tokens from t, zeros past r1): `before` is the mass below r0 and `target` the point to
    // invert.  Contiguous tokens per thread, block scan, the owning thread rescans.  Without an owner (rounding
    // left the target at or above the sum) the last token with mass in the range is taken.
    auto draw = [&](int r0, int r1, float mass_before, float total, auto fetch8) {   // total < 0: the sum of the range itself
        const int cpt = (((r1 - r0) + NT - 1) / NT + 7) & ~7;
        const int t0 = min(r0 + tid * cpt, r1), t1 = min(t0 + cpt, r1);
        float local = 0.0f;
        for (int t = t0; t < t1; t += 8) {
            float v[8];
            fetch8(t, v);
#pragma unroll
            for (int j = 0; j < 8; j++)
                local += v[j];
        }
        float inc = local;   // inclusive scan of the per-thread sums: inside a wave by shuffles, wave totals through LDS
        for (int off = 1; off < 64; off <<= 1) {
            const float o = __shfl_up(inc, off);
            if (lane >= off)
                inc += o;
        }
        __syncthreads();
        if (lane == 63)
            s_scan[wave] = inc;
        __syncthreads();
        float base = mass_before, scanned = 0.0f;
#pragma unroll
        for (int w = 0; w < 16; w++) {
            if (w < wave)
                base += s_scan[w];
            scanned += s_scan[w];
        }
        const float target = u_bonus[b] * (total < 0.0f ? scanned : total);
        const float before = base + inc - local;        // mass of all tokens below t0
        int owner = (before + local > target && t1 > t0) ? tid : NONE;
        owner = block_min_int(owner, s_redi, tid);
        if (owner == NONE) {
            int last = -1;
            for (int t = t0; t < t1; t += 8) {
                float v[8];
                fetch8(t, v);
#pragma unroll
                for (int j = 0; j < 8; j++)
                    if (v[j] > 0.0f)
                        last = t + j;
            }
            last = -block_min_int(-last, s_redi, tid);
            if (tid == 0)
                bonus_token[b] = last >= 0 ? last : min(r0, vocab - 1);
        } else if (tid == owner) {
            float run = before;
            int pick = t1 - 1;
            bool found = false;
            for (int t = t0; t < t1 && !found; t += 8) {
                float v[8];
                fetch8(t, v);
#pragma unroll
                for (int j = 0; j < 8; j++) {
                    run += v[j];
                    if (!found && run > target && t + j < t1) {
                        pick = t + j;
                        found = true;
                    }
                }
            }
            bonus_token[b] = pick;
        }
    };
    // The same draw when the mass of every 8192-token chunk is known (`chunk_mass(c)`): the chunk that holds the
    // target is found from those sums, in chunk order, and only that chunk is read.  The sums are staged in LDS
    // (one thread per chunk); beyond MAX_CHUNKS chunks the whole range is scanned instead.
    constexpr int MAX_CHUNKS = 64;
    __shared__ float s_cm[MAX_CHUNKS];
    auto draw_by_chunks = [&](auto chunk_mass, auto fetch8) {
        __syncthreads();
        if (tid < min(n_chunks, MAX_CHUNKS))
            s_cm[tid] = chunk_mass(tid);
        __syncthreads();
        if (n_chunks > MAX_CHUNKS) {
            float total = 0.0f;
            for (int c = 0; c < n_chunks; c++)
                total += chunk_mass(c);
            draw(0, vocab, 0.0f, total, fetch8);
            return;
        }
        float total = 0.0f;
        for (int c = 0; c < n_chunks; c++)
            total += s_cm[c];
        const float target = u_bonus[b] * total;
        int pick = -1, last_mass = 0;
        float before = 0.0f, before_last = 0.0f, run = 0.0f;
        for (int c = 0; c < n_chunks; c++) {
            const float mc = s_cm[c];
            if (mc > 0.0f) {
                last_mass = c;
                before_last = run;
            }
            if (pick < 0 && run + mc > target) {
                pick = c;
                before = run;
            }
            run += mc;
        }
        if (pick < 0) {           // rounding left the target at or above the total: the last chunk with mass
            pick = last_mass;
            before = before_last;
        }
        draw(pick * STAT_CHUNK, min((pick + 1) * STAT_CHUNK, vocab), before, total, fetch8);
    };

    int cur = 0, depth = 0;
    for (;;) {
        // ---- descend through first children whose (precomputed) test passes
        int first = depth < max_depth ? s_first[cur] : NONE;
        while (first != NONE && s_ok[first]) {
            cur = first;
            depth++;
            if (tid == 0)
                path[depth] = cur;
            first = depth < max_depth ? s_first[cur] : NONE;
        }
        const int64_t row = (bt + cur) * vocab;
        const float mt = s_mt[cur], md = s_md[cur];
        if (first == NONE) {
            // ---- no child to try: draw from the node's own target distribution, straight from the logits
            const float *cm = stat_m + (bt + cur) * n_chunks, *cs = stat_s + (bt + cur) * n_chunks;
            draw_by_chunks([&](int c) { const float sc = cs[c]; return sc > 0.0f ? sc * __expf(cm[c] - mt) : 0.0f; },
                           [&](int t, float v[8]) {
                               load8<BF16>(tlogits, row, t, vocab, vec, v);
#pragma unroll
                               for (int j = 0; j < 8; j++)
                                   v[j] = t + j < vocab ? __expf(v[j] * inv_temp - mt) : 0.0f;
                           });
            break;
        }
        // ---- the first child was rejected.  The residual target max(p - q, 0) is known through its chunk sums;
        // the draft loses the rejected token.
        const float ip = 1.0f / s_zt[cur], iq = s_zd[cur] > 0.0f ? 1.0f / s_zd[cur] : 0.0f;
        __shared__ float s_res[LAZY_CHUNKS];
        __shared__ float s_wres[NT / 64][LAZY_CHUNKS];
        if (LAZY) {
            // chunk sums of the first residual of this node: iteration k of the workgroup covers chunk k exactly
            for (int k = 0; k < n_chunks; k++) {
                float tv[8], dv[8], part = 0.0f;
                const int t = k * STAT_CHUNK + tid * 8;
                load8<BF16>(tlogits, row, t, vocab, vec, tv);
                load8<BF16>(dlogits, row, t, vocab, vec, dv);
#pragma unroll
                for (int j = 0; j < 8; j++)
                    if (t + j < vocab)
                        part += residual1(tv[j], dv[j], inv_temp, mt, md, ip, iq);
                for (int off = 32; off > 0; off >>= 1)
                    part += __shfl_xor(part, off);
                if (lane == 0)
                    s_wres[wave][k] = part;
            }
            __syncthreads();
            if (tid < n_chunks) {
                float t = 0.0f;
#pragma unroll
                for (int w = 0; w < NT / 64; w++)
                    t += s_wres[w][tid];
                s_res[tid] = t;
            }
            __syncthreads();
        }
        const float *rs = LAZY ? s_res : res_sum + (bt + cur) * n_chunks;
        float Z1 = 0.0f;
        for (int c0 = 0; c0 < n_chunks; c0 += 16) {   // chunk order, 16 loads in flight
            float a[16];
#pragma unroll
            for (int u = 0; u < 16; u++)
                a[u] = rs[min(c0 + u, n_chunks - 1)];
#pragma unroll
            for (int u = 0; u < 16; u++)
                if (c0 + u < n_chunks)
                    Z1 += a[u];
        }
        const bool empty1 = !(Z1 > 0.0f);   // target == draft: the residual is empty and the target stays as it is
        const int x1 = s_tok[first];
        const float W1 = fmaxf(1.0f - s_qx[first] * iq, 0.0f);
        // first residual of token t, and the draft after the first rejection (both normalised by Z1 resp. W1 later)
        auto r1_of = [&](float lt, float ld) { return empty1 ? __expf(lt * inv_temp - mt) * ip : residual1(lt, ld, inv_temp, mt, md, ip, iq); };
        const float Zr1 = empty1 ? 1.0f : Z1;

        int child = NONE;
        for (int i = tid; i < n_tree; i += NT)
            if (i > first && s_par[i] == cur)
                child = min(child, i);
        child = block_min_int(child, s_redi, tid);
        if (child == NONE) {
            // ---- the only child was rejected: draw from the first residual, one chunk read
            if (empty1) {
                const float *cm = stat_m + (bt + cur) * n_chunks, *cs = stat_s + (bt + cur) * n_chunks;
                draw_by_chunks([&](int c) { const float sc = cs[c]; return sc > 0.0f ? sc * __expf(cm[c] - mt) : 0.0f; },
                               [&](int t, float v[8]) {
                                   load8<BF16>(tlogits, row, t, vocab, vec, v);
#pragma unroll
                                   for (int j = 0; j < 8; j++)
                                       v[j] = t + j < vocab ? __expf(v[j] * inv_temp - mt) : 0.0f;
                               });
            } else {
                draw_by_chunks([&](int c) { return rs[c]; },
                               [&](int t, float v[8]) {
                                   float dv[8];
                                   load8<BF16>(tlogits, row, t, vocab, vec, v);
                                   load8<BF16>(dlogits, row, t, vocab, vec, dv);
#pragma unroll
                                   for (int j = 0; j < 8; j++)
                                       v[j] = t + j < vocab ? residual1(v[j], dv[j], inv_temp, mt, md, ip, iq) : 0.0f;
                               });
            }
            break;
        }
        // ---- second child: tested against the first residual and the reduced draft, two logit lookups
        int accepted = -1;
        {
            const int x2 = s_tok[child];
            const float lt = load_logit<BF16>(tlogits, row + x2), ld = load_logit<BF16>(dlogits, row + x2);
            const float px = r1_of(lt, ld);
            const float qx = x2 == x1 ? 0.0f : __expf(ld * inv_temp - md) * iq;
            const float ratio = qx > 0.0f ? (px / Zr1) / (qx / W1) : (px > 0.0f ? INFINITY : 0.0f);
            if (u_accept[bt + child] < fminf(1.0f, ratio))
                accepted = child;
        }
        if (accepted < 0) {
            // ---- second rejection: from here the distributions live as arrays.  One pass writes the second
            // residual R2 = max(r1/Z1 - q1/W1, 0) and the reduced draft q1 (normalised probabilities).
            const float iz1 = 1.0f / Zr1, iw1 = W1 > 0.0f ? 1.0f / W1 : 0.0f;
            float s = 0.0f;
            for (int t = tid * 8; t < vocab; t += NT * 8) {
                float tv[8], dv[8], r[8];
                load8<BF16>(tlogits, row, t, vocab, vec, tv);
                load8<BF16>(dlogits, row, t, vocab, vec, dv);
#pragma unroll
                for (int j = 0; j < 8; j++) {
                    const float r1 = r1_of(tv[j], dv[j]);
                    dv[j] = t + j == x1 ? 0.0f : __expf(dv[j] * inv_temp - md) * iq;
                    tv[j] = r1;
                    r[j] = t + j < vocab ? fmaxf(r1 * iz1 - dv[j] * iw1, 0.0f) : 0.0f;
                    s += r[j];
                }
                if (vec) {
                    *reinterpret_cast<float4 *>(R + t) = float4{r[0], r[1], r[2], r[3]};
                    *reinterpret_cast<float4 *>(R + t + 4) = float4{r[4], r[5], r[6], r[7]};
                    *reinterpret_cast<float4 *>(Q + t) = float4{dv[0], dv[1], dv[2], dv[3]};
                    *reinterpret_cast<float4 *>(Q + t + 4) = float4{dv[4], dv[5], dv[6], dv[7]};
                    *reinterpret_cast<float4 *>(P + t) = float4{tv[0], tv[1], tv[2], tv[3]};
                    *reinterpret_cast<float4 *>(P + t + 4) = float4{tv[4], tv[5], tv[6], tv[7]};
                } else {
#pragma unroll
                    for (int j = 0; j < 8; j++)
                        if (t + j < vocab) {
                            R[t + j] = r[j];
                            Q[t + j] = dv[j];
                            P[t + j] = tv[j];
                        }
                }
            }
            s = block_sum(s, s_redf, tid);
            float Zp = Zr1, Zq = W1;       // P holds r1 (sum Z1), Q the reduced draft (sum W1)
            if (s > 0.0f) {                // otherwise the second residual is empty and the target stays r1
                float *tmp = P;
                P = R;
                R = tmp;
                Zp = s;
            }
            __syncthreads();               // the arrays are complete before anybody reads or clears an entry
            {
                const int x2 = s_tok[child];
                const float q2 = Q[x2];
                __syncthreads();
                if (tid == 0)
                    Q[x2] = 0.0f;
                Zq = fmaxf(Zq - q2, 0.0f);
            }
            // ---- later siblings, one pass per further rejection
            for (;;) {
                int next = NONE;
                for (int i = tid; i < n_tree; i += NT)
                    if (i > child && s_par[i] == cur)
                        next = min(next, i);
                child = block_min_int(next, s_redi, tid);   // (its barriers also publish the cleared entry and the new P)
                if (child == NONE)
                    break;
                const int x = s_tok[child];
                const float px = P[x], qx = Q[x];
                const float ratio = qx > 0.0f ? (px / Zp) / (qx / Zq) : (px > 0.0f ? INFINITY : 0.0f);
                if (u_accept[bt + child] < fminf(1.0f, ratio)) {
                    accepted = child;
                    break;
                }
                const float ip2 = 1.0f / Zp, iq2 = Zq > 0.0f ? 1.0f / Zq : 0.0f;
                float s2 = 0.0f;
                if (vec) {
                    for (int t = tid * 4; t < vocab; t += NT * 4) {
                        const float4 pv = *reinterpret_cast<const float4 *>(P + t), qv = *reinterpret_cast<const float4 *>(Q + t);
                        const float4 r = {fmaxf(pv.x * ip2 - qv.x * iq2, 0.0f), fmaxf(pv.y * ip2 - qv.y * iq2, 0.0f),
                                          fmaxf(pv.z * ip2 - qv.z * iq2, 0.0f), fmaxf(pv.w * ip2 - qv.w * iq2, 0.0f)};
                        *reinterpret_cast<float4 *>(R + t) = r;
                        s2 += (r.x + r.y) + (r.z + r.w);
                    }
                } else {
                    for (int t = tid; t < vocab; t += NT) {
                        const float r = fmaxf(P[t] * ip2 - Q[t] * iq2, 0.0f);
                        R[t] = r;
                        s2 += r;
                    }
                }
                s2 = block_sum(s2, s_redf, tid);
                if (s2 > 0.0f) {
                    float *tmp = P;
                    P = R;
                    R = tmp;
                    Zp = s2;
                }
                __syncthreads();   // everybody has read Q[x] before it is cleared
                if (tid == 0)
                    Q[x] = 0.0f;
                Zq = fmaxf(Zq - qx, 0.0f);
            }
            if (accepted < 0) {
                // ---- every child rejected: draw from the residual array
                const float *Pc = P;
                draw(0, vocab, 0.0f, -1.0f, [&](int t, float v[8]) {
                    if (vec && t + 8 <= vocab) {
                        const float4 a = *reinterpret_cast<const float4 *>(Pc + t), c4 = *reinterpret_cast<const float4 *>(Pc + t + 4);
                        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = c4.x; v[5] = c4.y; v[6] = c4.z; v[7] = c4.w;
                    } else {
#pragma unroll
                        for (int j = 0; j < 8; j++)
                            v[j] = t + j < vocab ? Pc[t + j] : 0.0f;
                    }
                });
                break;
            }
        }
        cur = accepted;
        depth++;
        if (tid == 0)
            path[depth] = cur;
        __syncthreads();   // the arrays may be rewritten at a deeper node: finish reading them first
    }
    if (tid == 0)
        accept_len[b] = depth;
}

}  // namespace

extern "C" {

size_t dream_spec_accept_workspace(int32_t batch, int32_t n_tree, int32_t vocab)
{
    if (batch < 1 || n_tree < 1 || vocab < 1)
        return DREAM_WORKSPACE_MIN_BYTES;
    const size_t stats = align_up((size_t)2 * batch * n_tree * ceil_div(vocab, STAT_CHUNK) * sizeof(float), 256);
    return DREAM_WORKSPACE_MIN_BYTES + align_up((size_t)batch * 3 * vocab * sizeof(float), 256) + 3 * stats + align_up((size_t)batch * n_tree * 4 * sizeof(float), 256);
}

int dream_spec_accept(const void *target_logits, const void *draft_logits, int32_t logits_dtype, int32_t batch, int32_t n_tree,
                      int32_t vocab, const int32_t *token, const int32_t *parent, const float *u_accept, const float *u_bonus,
                      int32_t max_depth, float temperature, int32_t *accept_len, int32_t *accept_path, int32_t *bonus_token,
                      void *workspace, size_t workspace_bytes, void *stream)
{
    const char *who = "dream_spec_accept";
    if (!target_logits || !draft_logits || !token || !parent || !u_accept || !u_bonus || !accept_len || !accept_path || !bonus_token)
        return fail(DREAM_ERR_INVALID_ARG, "%s: NULL argument", who);
    if (logits_dtype != DREAM_F32 && logits_dtype != DREAM_BF16)
        return fail(DREAM_ERR_INVALID_ARG, "%s: unknown logits dtype %d", who, logits_dtype);
    if (batch < 1 || batch > 65535 || vocab < 1 || max_depth < 0 || max_depth >= NT)
        return fail(DREAM_ERR_INVALID_ARG, "%s: batch in [1, 65535], vocab positive and 0 <= max_depth < %d required", who, NT);
    if (n_tree < 1 || n_tree > DREAM_MAX_TREE_ACCEPT)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: n_tree %d outside [1, %d]", who, n_tree, DREAM_MAX_TREE_ACCEPT);
    if ((int64_t)batch * n_tree > 65535)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: batch * n_tree = %lld exceeds 65535 rows", who, (long long)batch * n_tree);
    if (!(temperature > 0.0f))
        return fail(DREAM_ERR_INVALID_ARG, "%s: temperature must be positive (use dream_accept_path for the greedy rule)", who);
    const size_t need = dream_spec_accept_workspace(batch, n_tree, vocab);
    if (!workspace || workspace_bytes < need)
        return fail(DREAM_ERR_WORKSPACE, "%s: workspace of %zu bytes, %zu needed", who, workspace_bytes, need);
    const int n_chunks = ceil_div(vocab, STAT_CHUNK);
    const size_t stats = align_up((size_t)2 * batch * n_tree * n_chunks * sizeof(float), 256);
    char *wsb = static_cast<char *>(workspace) + DREAM_WORKSPACE_MIN_BYTES;
    float *work = reinterpret_cast<float *>(wsb);
    float *stat_m = reinterpret_cast<float *>(wsb + align_up((size_t)batch * 3 * vocab * sizeof(float), 256));
    float *stat_s = reinterpret_cast<float *>(reinterpret_cast<char *>(stat_m) + stats);
    float *res_sum = reinterpret_cast<float *>(reinterpret_cast<char *>(stat_s) + stats);   // [B * n_tree, n_chunks]
    float4 *node_stats = reinterpret_cast<float4 *>(reinterpret_cast<char *>(res_sum) + stats);   // [B * n_tree]
    const int esz = logits_dtype == DREAM_BF16 ? 2 : 4;
    const bool vec = vocab % 8 == 0 &&
                     ((reinterpret_cast<uintptr_t>(target_logits) | reinterpret_cast<uintptr_t>(draft_logits) |
                       reinterpret_cast<uintptr_t>(workspace)) & 15) == 0 && ((size_t)vocab * esz) % 16 == 0;
    const float inv_temp = 1.0f / temperature;
    hipStream_t st = as_stream(stream);
    const dim3 sgrid(n_chunks, batch * n_tree, 2);
    const bool lazy = n_chunks <= LAZY_CHUNKS;
    auto launch_all = [&](auto bf16) {
        constexpr bool BF = decltype(bf16)::value;
        hipLaunchKernelGGL(softmax_stats_kernel<BF>, sgrid, dim3(256), 0, st, target_logits, draft_logits, n_tree, vocab, n_chunks, vec,
                           parent, inv_temp, stat_m, stat_s);
        if (lazy) {
            hipLaunchKernelGGL((spec_walk_kernel<BF, true>), dim3(batch), dim3(NT), 0, st, target_logits, draft_logits, n_tree, vocab, n_chunks,
                               vec, token, parent, u_accept, u_bonus, max_depth, inv_temp, stat_m, stat_s, nullptr, nullptr, work, accept_len,
                               accept_path, bonus_token);
        } else {
            hipLaunchKernelGGL(residual_stats_kernel<BF>, dim3(n_chunks, batch * n_tree), dim3(256), 0, st, target_logits, draft_logits, n_tree,
                               vocab, n_chunks, vec, parent, inv_temp, stat_m, stat_s, res_sum, node_stats);
            hipLaunchKernelGGL((spec_walk_kernel<BF, false>), dim3(batch), dim3(NT), 0, st, target_logits, draft_logits, n_tree, vocab, n_chunks,
                               vec, token, parent, u_accept, u_bonus, max_depth, inv_temp, stat_m, stat_s, res_sum, node_stats, work,
                               accept_len, accept_path, bonus_token);
        }
    };
    if (logits_dtype == DREAM_BF16)
        launch_all(std::true_type{});
    else
        launch_all(std::false_type{});
    return check_launch("spec_accept kernels");
}

}  // extern "C"
