// Tree-masked attention kernels for gfx950: dream_tree_verify_attn and dream_draft_xattn.
//
// Both calls compute softmax(q k^T * scale) v (Section 3.1, Eq. 1) over the keys a tree node may
// see: the whole cached prefix plus its ancestors in the draft tree (Section 3.1, tree-masking
// paragraph); verification includes the node itself, the draft's cross-attention does not.
//
// bf16 path (attn_bf16_kernel): one workgroup per (key-range split, group of query heads that
// share a KV head, sequence).  K and V tiles of BN keys are staged through LDS once and shared
// by every query row of the tree and every query head of the GQA group; each of the 4 waves owns
// NQT 16-row query tiles.  Scores are formed transposed, S^T = K Q^T, with
// v_mfma_f32_16x16x32_bf16, so a lane owns one query column: the online-softmax state is a
// per-lane scalar and the fp32 score registers are, after conversion to bf16, already the B operand
// of the second contraction O^T += V^T P^T.  The A operand of that contraction (V transposed) is
// fetched with the LDS transpose read ds_read_b64_tr_b16.  Key ranges are split across workgroups
// when B * heads alone cannot fill 256 CUs; partial (max, sum, O) triples are merged in a fixed
// order by attn_combine_kernel, so results do not depend on scheduling.
//
// fp32 path (attn_f32_kernel): plain vector-ALU kernel, one workgroup per (query row, head,
// sequence), used for float32 tensors (the small correctness configuration).
#include "common.h"
#include <math.h>

using namespace dream;

namespace {

struct AttnArgs {
    const void *q, *k, *v;
    const int32_t *prefix_len, *parent, *q_node;
    const uint64_t *tree_mask;
    void *out;
    float *lse;
    float *part_o;   // [B, head chunks, splits, rows_per_wg, D] un-normalised partial outputs
    float *part_ml;  // [B, head chunks, splits, rows_per_wg, 2] running max (log2 units) and sum
    int32_t n_q_heads, n_kv_heads, group;
    int32_t n_q, n_tree, include_self;
    int32_t tiles_per_head;  // 16-row query tiles per head
    int32_t heads_per_wg;    // query heads handled by one workgroup (divides group)
    int64_t s_max;
    float scale, scale_log2;
};

__device__ __forceinline__ uint64_t visible_nodes(const AttnArgs &a, int b, int node, const int32_t *lds_parent)
{
    if (a.tree_mask)
        return a.tree_mask[(int64_t)b * a.n_tree + node];
    uint64_t m = a.include_self ? (1ull << node) : 0ull;
    for (int p = lds_parent[node]; p >= 0; p = lds_parent[p])
        m |= 1ull << p;
    return m;
}

template <int D, int NQT, int BN>
struct TileGeom {
    static constexpr int KSTR = D + 8;    // K row stride in LDS (elements): 16-byte pad -> b128 reads hit all banks
    static constexpr int VSTR = D + 16;   // V row stride in LDS (elements): 4 consecutive rows land 8 banks apart
    static constexpr int KTILE = BN * KSTR;
    static constexpr int VTILE = BN * VSTR;
    static constexpr int CH = BN * D / 8 / 256;   // 16-byte chunks per thread per tensor per tile
    static constexpr size_t LDS_BYTES = (size_t)(2 * KTILE + 2 * VTILE) * 2 + DREAM_MAX_TREE * sizeof(int32_t);
    static constexpr int ROWS_PER_WG = 64 * NQT;
};

template <int D, int NQT, int BN>
__global__ __launch_bounds__(256) void attn_bf16_kernel(AttnArgs a)
{
    using G = TileGeom<D, NQT, BN>;
    constexpr int KSTR = G::KSTR, VSTR = G::VSTR, CH = G::CH;
    constexpr int NDT = D / 16;   // 16-wide output column tiles
    constexpr int NKS = D / 32;   // 32-deep contraction steps of q.k
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    uint16_t *ldsK = reinterpret_cast<uint16_t *>(smem_raw);
    uint16_t *ldsV = ldsK + 2 * G::KTILE;
    int32_t *lds_parent = reinterpret_cast<int32_t *>(ldsV + 2 * G::VTILE);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int split = blockIdx.x, nsplit = gridDim.x, hc = blockIdx.y, b = blockIdx.z;
    const int hq0 = hc * a.heads_per_wg;
    const int kvh = hq0 / a.group;
    const int P = a.prefix_len[b];
    const int kv_len = P + a.n_tree;
    const int tiles_total = (kv_len + BN - 1) / BN;
    const int tps = (tiles_total + nsplit - 1) / nsplit;
    const int t_begin = split * tps;
    const int t_end = min(t_begin + tps, tiles_total);

    const uint16_t *kbase = reinterpret_cast<const uint16_t *>(a.k) + ((int64_t)b * a.n_kv_heads + kvh) * a.s_max * D;
    const uint16_t *vbase = reinterpret_cast<const uint16_t *>(a.v) + ((int64_t)b * a.n_kv_heads + kvh) * a.s_max * D;

    if (!a.tree_mask && tid < a.n_tree)
        lds_parent[tid] = a.parent[(int64_t)b * a.n_tree + tid];

    // register staging of one K/V tile
    uint4 kreg[CH], vreg[CH];
    auto load_tile = [&](int t) {
#pragma unroll
        for (int i = 0; i < CH; i++) {
            int chunk = i * 256 + tid;
            int row = chunk / (D / 8), col = chunk % (D / 8);
            int key = t * BN + row;
            if (key < kv_len) {
                kreg[i] = *reinterpret_cast<const uint4 *>(kbase + (int64_t)key * D + col * 8);
                vreg[i] = *reinterpret_cast<const uint4 *>(vbase + (int64_t)key * D + col * 8);
            } else {
                kreg[i] = make_uint4(0, 0, 0, 0);
                vreg[i] = make_uint4(0, 0, 0, 0);
            }
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < CH; i++) {
            int chunk = i * 256 + tid;
            int row = chunk / (D / 8), col = chunk % (D / 8);
            *reinterpret_cast<uint4 *>(ldsK + buf * G::KTILE + row * KSTR + col * 8) = kreg[i];
            *reinterpret_cast<uint4 *>(ldsV + buf * G::VTILE + row * VSTR + col * 8) = vreg[i];
        }
    };
    if (t_begin < t_end)
        load_tile(t_begin);

    __syncthreads();   // parents staged

    // per query tile: which (head, row) this lane's column is, its mask, its Q fragments
    bf16x8 qf[NQT][NKS];
    uint64_t qmask[NQT];
    int q_row[NQT], q_head[NQT];
#pragma unroll
    for (int qt = 0; qt < NQT; qt++) {
        int t = wave * NQT + qt;
        int hh = t / a.tiles_per_head, nt = t % a.tiles_per_head;
        int row = nt * 16 + c;
        bool valid = hh < a.heads_per_wg && row < a.n_q;
        q_row[qt] = valid ? row : -1;
        q_head[qt] = hq0 + hh;
        qmask[qt] = 0;
        if (valid) {
            int node = a.q_node ? a.q_node[(int64_t)b * a.n_q + row] : row;
            qmask[qt] = visible_nodes(a, b, node, lds_parent);
            const uint16_t *qp = reinterpret_cast<const uint16_t *>(a.q) +
                                 (((int64_t)b * a.n_q + row) * a.n_q_heads + q_head[qt]) * D + g * 8;
#pragma unroll
            for (int ks = 0; ks < NKS; ks++)
                qf[qt][ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 32);
        } else {
#pragma unroll
            for (int ks = 0; ks < NKS; ks++)
#pragma unroll
                for (int i = 0; i < 8; i++)
                    qf[qt][ks][i] = (__bf16)0.0f;
        }
    }

    f32x4 oacc[NQT][NDT];
    float m_run[NQT], l_run[NQT];
#pragma unroll
    for (int qt = 0; qt < NQT; qt++) {
        m_run[qt] = -INFINITY;
        l_run[qt] = 0.0f;
#pragma unroll
        for (int dt = 0; dt < NDT; dt++)
            oacc[qt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    int buf = 0;
    for (int t = t_begin; t < t_end; t++) {
        store_tile(buf);
        __syncthreads();
        if (t + 1 < t_end)
            load_tile(t + 1);
        const uint16_t *tk = ldsK + buf * G::KTILE;
        const uint16_t *tv = ldsV + buf * G::VTILE;
        const int key0 = t * BN;
        const bool needs_mask = key0 + BN > P;   // tile touches tree rows or the ragged end

#pragma unroll 1
        for (int s = 0; s < BN / 32; s++) {
            // ---- S^T = K Q^T for 32 keys x (16 * NQT) query columns
            f32x4 sacc[2][NQT];
#pragma unroll
            for (int qt = 0; qt < NQT; qt++) {
                sacc[0][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
                sacc[1][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int ks = 0; ks < NKS; ks++) {
                bf16x8 kf0 = *reinterpret_cast<const bf16x8 *>(tk + (s * 32 + c) * KSTR + ks * 32 + g * 8);
                bf16x8 kf1 = *reinterpret_cast<const bf16x8 *>(tk + (s * 32 + 16 + c) * KSTR + ks * 32 + g * 8);
#pragma unroll
                for (int qt = 0; qt < NQT; qt++) {
                    sacc[0][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf0, qf[qt][ks], sacc[0][qt], 0, 0, 0);
                    sacc[1][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf1, qf[qt][ks], sacc[1][qt], 0, 0, 0);
                }
            }
            // ---- online softmax; lane owns query column c, key rows g*4+r of both 16-key tiles
            bf16x8 pf[NQT];
#pragma unroll
            for (int qt = 0; qt < NQT; qt++) {
                float sv[8];
                float mx = -INFINITY;
#pragma unroll
                for (int i = 0; i < 8; i++) {
                    float x = sacc[i >> 2][qt][i & 3] * a.scale_log2;
                    if (needs_mask) {
                        int key = key0 + s * 32 + (i >> 2) * 16 + g * 4 + (i & 3);
                        int rel = key - P;
                        bool vis = rel < 0 || (rel < a.n_tree && ((qmask[qt] >> (rel & 63)) & 1ull));
                        x = vis ? x : -INFINITY;
                    }
                    sv[i] = x;
                    mx = fmaxf(mx, x);
                }
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                float m_new = fmaxf(m_run[qt], mx);
                float m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
                float alpha = __builtin_amdgcn_exp2f(m_run[qt] - m_safe);
                m_run[qt] = m_new;
                float psum = 0.0f;
#pragma unroll
                for (int i = 0; i < 8; i++) {
                    float p = __builtin_amdgcn_exp2f(sv[i] - m_safe);
                    psum += p;
                    pf[qt][i] = (__bf16)p;
                }
                l_run[qt] = l_run[qt] * alpha + psum;
#pragma unroll
                for (int dt = 0; dt < NDT; dt++)
                    oacc[qt][dt] *= alpha;
            }
            // ---- O^T += V^T P^T
#pragma unroll
            for (int dt = 0; dt < NDT; dt++) {
                const uint16_t *vp = tv + (s * 32 + g * 4 + (c >> 2)) * VSTR + dt * 16 + (c & 3) * 4;
                s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(vp));
                s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(vp + 16 * VSTR));
                s16x8 vv = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
                bf16x8 vf = __builtin_bit_cast(bf16x8, vv);
#pragma unroll
                for (int qt = 0; qt < NQT; qt++)
                    oacc[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[qt], oacc[qt][dt], 0, 0, 0);
            }
        }
        buf ^= 1;
    }

    // ---- epilogue
    constexpr float LN2 = 0.6931471805599453f;
#pragma unroll
    for (int qt = 0; qt < NQT; qt++) {
        float l = l_run[qt];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (q_row[qt] < 0)
            continue;
        if (nsplit == 1) {
            float inv = l > 0.0f ? 1.0f / l : 0.0f;
            uint16_t *op = reinterpret_cast<uint16_t *>(a.out) +
                           (((int64_t)b * a.n_q + q_row[qt]) * a.n_q_heads + q_head[qt]) * D + g * 4;
#pragma unroll
            for (int dt = 0; dt < NDT; dt++) {
                bf16x4 o;
#pragma unroll
                for (int r = 0; r < 4; r++)
                    o[r] = (__bf16)(oacc[qt][dt][r] * inv);
                *reinterpret_cast<bf16x4 *>(op + dt * 16) = o;
            }
            if (a.lse && g == 0)
                a.lse[((int64_t)b * a.n_q_heads + q_head[qt]) * a.n_q + q_row[qt]] =
                    l > 0.0f ? (m_run[qt] + log2f(l)) * LN2 : -INFINITY;
        } else {
            int64_t pr = (((int64_t)b * gridDim.y + hc) * nsplit + split) * G::ROWS_PER_WG + (wave * NQT + qt) * 16 + c;
            float *po = a.part_o + pr * D + g * 4;
#pragma unroll
            for (int dt = 0; dt < NDT; dt++)
                *reinterpret_cast<f32x4 *>(po + dt * 16) = oacc[qt][dt];
            if (g == 0) {
                a.part_ml[pr * 2] = m_run[qt];
                a.part_ml[pr * 2 + 1] = l;
            }
        }
    }
}

// Merge the per-split partial results in split order: one thread per 4 output columns.
template <int D>
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnArgs a, int nsplit, int n_chunks, int rows_per_wg, int64_t total)
{
    int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total)
        return;
    int d4 = (int)(idx % (D / 4));
    int64_t r = idx / (D / 4);
    int hq = (int)(r % a.n_q_heads);
    int row = (int)((r / a.n_q_heads) % a.n_q);
    int b = (int)(r / ((int64_t)a.n_q_heads * a.n_q));
    int hc = hq / a.heads_per_wg, hh = hq % a.heads_per_wg;
    int slot = (hh * a.tiles_per_head + row / 16) * 16 + row % 16;
    int64_t base = ((int64_t)b * n_chunks + hc) * nsplit;
    float m = -INFINITY;
    for (int s = 0; s < nsplit; s++)
        m = fmaxf(m, a.part_ml[((base + s) * rows_per_wg + slot) * 2]);
    float m_safe = (m == -INFINITY) ? 0.0f : m;
    float l = 0.0f;
    f32x4 o = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < nsplit; s++) {
        int64_t pr = (base + s) * rows_per_wg + slot;
        float w = __builtin_amdgcn_exp2f(a.part_ml[pr * 2] - m_safe);
        l += w * a.part_ml[pr * 2 + 1];
        f32x4 po = *reinterpret_cast<const f32x4 *>(a.part_o + pr * D + d4 * 4);
        o += po * w;
    }
    float inv = l > 0.0f ? 1.0f / l : 0.0f;
    bf16x4 ob;
#pragma unroll
    for (int i = 0; i < 4; i++)
        ob[i] = (__bf16)(o[i] * inv);
    *reinterpret_cast<bf16x4 *>(reinterpret_cast<uint16_t *>(a.out) + (((int64_t)b * a.n_q + row) * a.n_q_heads + hq) * D + d4 * 4) = ob;
    if (a.lse && d4 == 0)
        a.lse[((int64_t)b * a.n_q_heads + hq) * a.n_q + row] = l > 0.0f ? (m + log2f(l)) * 0.6931471805599453f : -INFINITY;
}

// ------------------------------------------------------------------------------------------------
// float32 path: one workgroup per (query row, head, sequence); 256 keys per pass.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attn_f32_kernel(AttnArgs a, int D)
{
    __shared__ float sq[256];
    __shared__ float sp[256];
    __shared__ float red[8];
    __shared__ uint64_t smask;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
    const int kvh = hq / a.group;
    const int P = a.prefix_len[b];
    const int kv_len = P + a.n_tree;
    const float *q = reinterpret_cast<const float *>(a.q) + (((int64_t)b * a.n_q + row) * a.n_q_heads + hq) * D;
    const float *kb = reinterpret_cast<const float *>(a.k) + ((int64_t)b * a.n_kv_heads + kvh) * a.s_max * D;
    const float *vb = reinterpret_cast<const float *>(a.v) + ((int64_t)b * a.n_kv_heads + kvh) * a.s_max * D;
    if (tid < D)
        sq[tid] = q[tid];
    if (tid == 0) {
        int node = a.q_node ? a.q_node[(int64_t)b * a.n_q + row] : row;
        uint64_t m;
        if (a.tree_mask) {
            m = a.tree_mask[(int64_t)b * a.n_tree + node];
        } else {
            const int32_t *par = a.parent + (int64_t)b * a.n_tree;
            m = a.include_self ? (1ull << node) : 0ull;
            for (int p = par[node]; p >= 0; p = par[p])
                m |= 1ull << p;
        }
        smask = m;
    }
    __syncthreads();
    const uint64_t mask = smask;
    float m_run = -INFINITY, l_run = 0.0f, o = 0.0f;
    for (int k0 = 0; k0 < kv_len; k0 += 256) {
        int key = k0 + tid;
        float s = -INFINITY;
        bool vis = key < P || (key < kv_len && ((mask >> ((key - P) & 63)) & 1ull));
        if (vis) {
            const float4 *kr = reinterpret_cast<const float4 *>(kb + (int64_t)key * D);
            float dot = 0.0f;
            for (int d = 0; d < D / 4; d++) {
                float4 kk = kr[d];
                dot += sq[4 * d] * kk.x + sq[4 * d + 1] * kk.y + sq[4 * d + 2] * kk.z + sq[4 * d + 3] * kk.w;
            }
            s = dot * a.scale;
        }
        float mx = s;
        for (int off = 32; off > 0; off >>= 1)
            mx = fmaxf(mx, __shfl_xor(mx, off));
        if (lane == 0)
            red[wave] = mx;
        __syncthreads();
        mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        float m_new = fmaxf(m_run, mx);
        float m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
        float alpha = expf(m_run - m_safe);
        float p = vis ? expf(s - m_safe) : 0.0f;
        sp[tid] = p;
        float ps = p;
        for (int off = 32; off > 0; off >>= 1)
            ps += __shfl_xor(ps, off);
        if (lane == 0)
            red[4 + wave] = ps;
        __syncthreads();
        l_run = l_run * alpha + ((red[4] + red[5]) + (red[6] + red[7]));
        m_run = m_new;
        if (tid < D) {
            float acc = 0.0f;
            int n = min(256, kv_len - k0);
            for (int j = 0; j < n; j++) {
                float pj = sp[j];
                if (pj != 0.0f)
                    acc += pj * vb[(int64_t)(k0 + j) * D + tid];
            }
            o = o * alpha + acc;
        }
        __syncthreads();
    }
    if (tid < D)
        reinterpret_cast<float *>(a.out)[(((int64_t)b * a.n_q + row) * a.n_q_heads + hq) * D + tid] = l_run > 0.0f ? o / l_run : 0.0f;
    if (a.lse && tid == 0)
        a.lse[((int64_t)b * a.n_q_heads + hq) * a.n_q + row] = l_run > 0.0f ? m_run + logf(l_run) : -INFINITY;
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
struct Plan {
    int tiles_per_head, heads_per_wg, nqt, bn, n_chunks, n_splits, rows_per_wg;
    size_t off_ml, off_o, total;
};

int make_plan(const dream_attn_desc *d, int n_q, int64_t max_kv_len, Plan *p)
{
    const int G = d->n_q_heads / d->n_kv_heads;
    p->tiles_per_head = ceil_div(n_q, 16);
    const int max_tiles = d->head_dim == 256 ? 8 : 16;   // accumulator registers bound the rows per workgroup
    int hpw = G;
    while (hpw > 1 && hpw * p->tiles_per_head > max_tiles)
        hpw--;
    while (G % hpw)
        hpw--;
    if (hpw * p->tiles_per_head > max_tiles)
        return -1;
    p->heads_per_wg = hpw;
    int nt = hpw * p->tiles_per_head;
    p->nqt = nt <= 4 ? 1 : nt <= 8 ? 2 : 4;
    p->bn = d->head_dim == 256 ? 32 : 64;
    p->n_chunks = d->n_q_heads / hpw;
    p->rows_per_wg = 64 * p->nqt;
    const int tiles = ceil_div(max_kv_len, p->bn);
    int s = kv_splits_override();
    if (s <= 0) {
        const int64_t wgs = (int64_t)d->batch * p->n_chunks;
        s = ceil_div(512, wgs);
    }
    if (s > tiles)
        s = tiles;
    if (s < 1)
        s = 1;
    p->n_splits = s;
    p->off_ml = DREAM_WORKSPACE_HEADER_BYTES;
    size_t rows = (size_t)d->batch * p->n_chunks * s * p->rows_per_wg;
    p->off_o = align_up(p->off_ml + rows * 2 * sizeof(float), 256);
    p->total = p->off_o + rows * d->head_dim * sizeof(float);
    if (s == 1 || d->dtype == DREAM_F32)
        p->total = DREAM_WORKSPACE_HEADER_BYTES;
    return 0;
}

int validate_desc(const dream_attn_desc *d, const char *who)
{
    if (!d)
        return fail(DREAM_ERR_INVALID_ARG, "%s: desc is NULL", who);
    if (d->batch < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->s_max < 1)
        return fail(DREAM_ERR_INVALID_ARG, "%s: batch, head counts and s_max must be positive", who);
    if (d->n_q_heads % d->n_kv_heads)
        return fail(DREAM_ERR_INVALID_ARG, "%s: n_q_heads %d is not a multiple of n_kv_heads %d", who, d->n_q_heads, d->n_kv_heads);
    if (d->head_dim != 64 && d->head_dim != 128 && d->head_dim != 256)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: head_dim %d not in {64,128,256}", who, d->head_dim);
    if (d->dtype != DREAM_F32 && d->dtype != DREAM_BF16)
        return fail(DREAM_ERR_INVALID_ARG, "%s: unknown dtype %d", who, d->dtype);
    if (d->batch > 65535 || d->n_q_heads > 65535)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: batch and n_q_heads are limited to 65535", who);
    return DREAM_OK;
}

template <int D, int NQT, int BN>
int launch_bf16(const AttnArgs &a, const Plan &p, int batch, hipStream_t st)
{
    using G = TileGeom<D, NQT, BN>;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_bf16_kernel<D, NQT, BN>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)G::LDS_BYTES) != hipSuccess)
            return fail(DREAM_ERR_HIP, "attention: cannot reserve %zu bytes of LDS", G::LDS_BYTES);
        attr_set = true;
    }
    dim3 grid(p.n_splits, p.n_chunks, batch);
    hipLaunchKernelGGL((attn_bf16_kernel<D, NQT, BN>), grid, dim3(256), G::LDS_BYTES, st, a);
    return check_launch("attn_bf16_kernel");
}

int run_attention(const char *who, const dream_attn_desc *d, const void *q, const void *k, const void *v,
                  const int32_t *prefix_len, int n_tree, const int32_t *parent, const uint64_t *tree_mask,
                  int n_q, const int32_t *q_node, int include_self, int64_t max_kv_len, void *out, float *lse,
                  void *ws, size_t ws_bytes, void *stream)
{
    int rc = validate_desc(d, who);
    if (rc)
        return rc;
    if (!q || !k || !v || !prefix_len || !out)
        return fail(DREAM_ERR_INVALID_ARG, "%s: q, k, v, prefix_len and out must not be NULL", who);
    if (!parent && !tree_mask)
        return fail(DREAM_ERR_INVALID_ARG, "%s: parent is NULL and no tree_mask is given", who);
    if (n_tree < 1 || n_tree > DREAM_MAX_TREE)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: n_tree %d outside [1, %d]", who, n_tree, DREAM_MAX_TREE);
    if (n_q < 1 || n_q > DREAM_MAX_TREE)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: %d query rows outside [1, %d]", who, n_q, DREAM_MAX_TREE);
    if (!q_node && n_q > n_tree)
        return fail(DREAM_ERR_INVALID_ARG, "%s: %d query rows but only %d tree nodes and no q_node", who, n_q, n_tree);
    if (max_kv_len < n_tree || max_kv_len > d->s_max)
        return fail(DREAM_ERR_INVALID_ARG, "%s: max_kv_len %lld outside [n_tree, s_max]", who, (long long)max_kv_len);
    Plan p;
    if (make_plan(d, n_q, max_kv_len, &p))
        return fail(DREAM_ERR_UNSUPPORTED, "%s: %d query rows x head_dim %d does not fit one workgroup", who, n_q, d->head_dim);
    if (!ws || ws_bytes < p.total)
        return fail(DREAM_ERR_WORKSPACE, "%s: workspace of %zu bytes, %zu needed", who, ws_bytes, p.total);

    AttnArgs a;
    a.q = q; a.k = k; a.v = v;
    a.prefix_len = prefix_len; a.parent = parent; a.q_node = q_node; a.tree_mask = tree_mask;
    a.out = out; a.lse = lse;
    a.part_ml = reinterpret_cast<float *>(static_cast<char *>(ws) + p.off_ml);
    a.part_o = reinterpret_cast<float *>(static_cast<char *>(ws) + p.off_o);
    a.n_q_heads = d->n_q_heads; a.n_kv_heads = d->n_kv_heads; a.group = d->n_q_heads / d->n_kv_heads;
    a.n_q = n_q; a.n_tree = n_tree; a.include_self = include_self;
    a.tiles_per_head = p.tiles_per_head; a.heads_per_wg = p.heads_per_wg;
    a.s_max = d->s_max;
    a.scale = d->scale != 0.0f ? d->scale : 1.0f / sqrtf((float)d->head_dim);
    a.scale_log2 = a.scale * 1.4426950408889634f;
    hipStream_t st = as_stream(stream);

    if (d->dtype == DREAM_F32) {
        dim3 grid(n_q, d->n_q_heads, d->batch);
        hipLaunchKernelGGL(attn_f32_kernel, grid, dim3(256), 0, st, a, d->head_dim);
        return check_launch("attn_f32_kernel");
    }

    const int key = d->head_dim * 10 + p.nqt;
    switch (key) {
    case 641:  rc = launch_bf16<64, 1, 64>(a, p, d->batch, st); break;
    case 642:  rc = launch_bf16<64, 2, 64>(a, p, d->batch, st); break;
    case 644:  rc = launch_bf16<64, 4, 64>(a, p, d->batch, st); break;
    case 1281: rc = launch_bf16<128, 1, 64>(a, p, d->batch, st); break;
    case 1282: rc = launch_bf16<128, 2, 64>(a, p, d->batch, st); break;
    case 1284: rc = launch_bf16<128, 4, 64>(a, p, d->batch, st); break;
    case 2561: rc = launch_bf16<256, 1, 32>(a, p, d->batch, st); break;
    case 2562: rc = launch_bf16<256, 2, 32>(a, p, d->batch, st); break;
    default:   return fail(DREAM_ERR_UNSUPPORTED, "%s: no kernel for head_dim %d with %d query tiles per wave", who, d->head_dim, p.nqt);
    }
    if (rc)
        return rc;
    if (p.n_splits > 1) {
        int64_t total = (int64_t)d->batch * n_q * d->n_q_heads * (d->head_dim / 4);
        dim3 grid((unsigned)((total + 255) / 256));
        switch (d->head_dim) {
        case 64:  hipLaunchKernelGGL(attn_combine_kernel<64>, grid, dim3(256), 0, st, a, p.n_splits, p.n_chunks, p.rows_per_wg, total); break;
        case 128: hipLaunchKernelGGL(attn_combine_kernel<128>, grid, dim3(256), 0, st, a, p.n_splits, p.n_chunks, p.rows_per_wg, total); break;
        default:  hipLaunchKernelGGL(attn_combine_kernel<256>, grid, dim3(256), 0, st, a, p.n_splits, p.n_chunks, p.rows_per_wg, total); break;
        }
        return check_launch("attn_combine_kernel");
    }
    return DREAM_OK;
}

size_t workspace_for(const dream_attn_desc *d, int n_q, int64_t max_kv_len)
{
    if (!d || d->n_kv_heads < 1 || d->n_q_heads < 1 || d->n_q_heads % d->n_kv_heads || n_q < 1 || max_kv_len < 1)
        return DREAM_WORKSPACE_HEADER_BYTES;
    Plan p;
    if (make_plan(d, n_q, max_kv_len, &p))
        return DREAM_WORKSPACE_HEADER_BYTES;
    return p.total;
}

}  // namespace

extern "C" {

size_t dream_tree_verify_attn_workspace(const dream_attn_desc *desc, int32_t n_tree, int64_t max_kv_len)
{
    return workspace_for(desc, n_tree, max_kv_len);
}

int dream_tree_verify_attn(const dream_attn_desc *desc, const void *q, const void *k_cache, const void *v_cache,
                           const int32_t *prefix_len, int32_t n_tree, const int32_t *parent,
                           const uint64_t *tree_mask, int64_t max_kv_len, void *out, float *lse,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    return run_attention("dream_tree_verify_attn", desc, q, k_cache, v_cache, prefix_len, n_tree, parent, tree_mask,
                         n_tree, nullptr, 1, max_kv_len, out, lse, workspace, workspace_bytes, stream);
}

size_t dream_draft_xattn_workspace(const dream_attn_desc *desc, int32_t n_q, int64_t max_kv_len)
{
    return workspace_for(desc, n_q, max_kv_len);
}

int dream_draft_xattn(const dream_attn_desc *desc, const void *q, const void *kx_cache, const void *vx_cache,
                      const int32_t *prefix_len, int32_t n_tree, const int32_t *parent, int32_t n_q,
                      const int32_t *q_node, int64_t max_kv_len, void *out, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    if (!parent)
        return fail(DREAM_ERR_INVALID_ARG, "dream_draft_xattn: parent must not be NULL");
    return run_attention("dream_draft_xattn", desc, q, kx_cache, vx_cache, prefix_len, n_tree, parent, nullptr,
                         n_q, q_node, 0, max_kv_len, out, nullptr, workspace, workspace_bytes, stream);
}

}  // extern "C"
