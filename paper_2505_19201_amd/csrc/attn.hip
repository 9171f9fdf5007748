// Tree-masked attention kernels for gfx950: dream_tree_verify_attn and dream_draft_xattn.
//
// Both calls compute softmax(q k^T * scale) v (Section 3.1, Eq. 1) over the keys a tree node may
// see: the whole cached prefix plus its ancestors in the draft tree (Section 3.1, tree-masking
// paragraph); verification includes the node itself, the draft's cross-attention does not.
//
// bf16 path (attn_bf16_kernel).  A workgroup serves one (sequence, KV head, key-range split,
// query group); a query group is QG 16-row query tiles out of the G * ceil(n_q/16) tiles that
// share the KV head (all tree rows of all query heads of the GQA group).  Its 4 waves stream
// disjoint 32-key tiles of the range: a wave loads its tile with 16-byte coalesced loads, parks
// it in a wave-private LDS area (no workgroup barrier in the loop) and reuses every K/V byte
// for all QG*16 query rows.  Scores are formed transposed, S^T = K Q^T, with
// v_mfma_f32_16x16x32_bf16, so a lane owns one query column: the online-softmax state is a
// per-lane scalar and the fp32 score registers, converted to bf16, already are the B operand of
// the second contraction O^T += V^T P^T, whose A operand (V transposed) comes from the LDS
// transpose read ds_read_b64_tr_b16.  At the end the 4 waves merge their (max, sum, O) states
// through LDS in a fixed order.  When B * Hkv * query groups cannot fill 256 CUs the key range is
// split over several workgroups; each writes its state to the workspace, takes a ticket, and
// the last arrival merges all states of its group in split order (deterministic) and writes the
// output - one launch, no separate combine kernel.  Workgroups that read the same K/V stream
// (the query groups of one split) are given ids congruent mod 8 so that they run on one XCD and
// share its L2: HBM sees every K/V byte once.
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
    float *part;        // [groups, splits, state] merged wave states of every split
    int32_t *counters;  // [groups] arrival tickets, zero between calls
    int32_t n_q_heads, n_kv_heads, group;
    int32_t n_q, n_tree, include_self;
    int32_t tiles_per_head;  // 16-row query tiles per head
    int32_t n_qg;            // query groups per KV head
    int32_t n_splits;
    int32_t n_streams;       // B * Hkv * n_splits
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

// LDS traffic inside one wave needs no barrier, only program order.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int D, int QG>
struct Geom {
    static constexpr int KSTR = D + 8;    // K row stride in LDS (elements): 16-byte pad, b128 reads spread over all banks
    static constexpr int VSTR = D + 16;   // V row stride in LDS (elements): 4 consecutive rows land 8 banks apart
    static constexpr int WAVE_ELEMS = 32 * (KSTR + VSTR);
    static constexpr int NDT = D / 16;
    static constexpr int CH = 32 * D / 8 / 64;                       // 16-byte chunks per lane per tensor per tile
    static constexpr int STATE_FLOATS = QG * NDT * 256 + QG * 2 * 64;  // one wave's (O, max, sum) in lane-major order
    static constexpr size_t TILE_BYTES = (size_t)4 * WAVE_ELEMS * 2;
    static constexpr size_t MERGE_BYTES = (size_t)2 * STATE_FLOATS * 4;
    static constexpr size_t LDS_BYTES = (TILE_BYTES > MERGE_BYTES ? TILE_BYTES : MERGE_BYTES) + DREAM_MAX_TREE * sizeof(int32_t);
};

template <int QG, int NDT>
struct WaveState {
    f32x4 o[QG][NDT];
    float m[QG], l[QG];
};

template <int QG, int NDT>
__device__ __forceinline__ void state_store(const WaveState<QG, NDT> &s, float *dst, int lane)
{
#pragma unroll
    for (int qt = 0; qt < QG; qt++) {
#pragma unroll
        for (int dt = 0; dt < NDT; dt++)
            reinterpret_cast<f32x4 *>(dst)[(qt * NDT + dt) * 64 + lane] = s.o[qt][dt];
        dst[QG * NDT * 256 + (qt * 2) * 64 + lane] = s.m[qt];
        dst[QG * NDT * 256 + (qt * 2 + 1) * 64 + lane] = s.l[qt];
    }
}

// s <- s (+) state at src, the associative merge of two online-softmax states
template <int QG, int NDT>
__device__ __forceinline__ void state_merge(WaveState<QG, NDT> &s, const float *src, int lane)
{
#pragma unroll
    for (int qt = 0; qt < QG; qt++) {
        float mo = src[QG * NDT * 256 + (qt * 2) * 64 + lane];
        float lo = src[QG * NDT * 256 + (qt * 2 + 1) * 64 + lane];
        float mn = fmaxf(s.m[qt], mo);
        float ms = (mn == -INFINITY) ? 0.0f : mn;
        float a1 = __builtin_amdgcn_exp2f(s.m[qt] - ms), a2 = __builtin_amdgcn_exp2f(mo - ms);
        s.l[qt] = s.l[qt] * a1 + lo * a2;
        s.m[qt] = mn;
#pragma unroll
        for (int dt = 0; dt < NDT; dt++) {
            f32x4 oo = reinterpret_cast<const f32x4 *>(src)[(qt * NDT + dt) * 64 + lane];
            s.o[qt][dt] = s.o[qt][dt] * a1 + oo * a2;
        }
    }
}

template <int D, int QG>
__global__ __launch_bounds__(256) void attn_bf16_kernel(AttnArgs a)
{
    using G = Geom<D, QG>;
    constexpr int KSTR = G::KSTR, VSTR = G::VSTR, CH = G::CH, NDT = G::NDT;
    constexpr int NKS = D / 32;   // 32-deep contraction steps of q.k
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    uint16_t *lds = reinterpret_cast<uint16_t *>(smem_raw);
    int32_t *lds_parent = reinterpret_cast<int32_t *>(smem_raw + (G::LDS_BYTES - DREAM_MAX_TREE * sizeof(int32_t)));

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;

    // workgroup id -> (K/V stream, query group): ids that share a stream are congruent mod 8 (same XCD)
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int stream = (slot / a.n_qg) * 8 + xcd, qg = slot % a.n_qg;
    if (stream >= a.n_streams)
        return;
    const int nsplit = a.n_splits;
    const int split = stream % nsplit, bk = stream / nsplit;
    const int kvh = bk % a.n_kv_heads, b = bk / a.n_kv_heads;
    const int P = a.prefix_len[b];
    const int kv_len = P + a.n_tree;
    const int tiles_total = (kv_len + 31) / 32;
    const int tps = (tiles_total + nsplit - 1) / nsplit;
    const int t_begin = split * tps;
    const int t_end = min(t_begin + tps, tiles_total);

    const uint16_t *kbase = reinterpret_cast<const uint16_t *>(a.k) + ((int64_t)b * a.n_kv_heads + kvh) * a.s_max * D;
    const uint16_t *vbase = reinterpret_cast<const uint16_t *>(a.v) + ((int64_t)b * a.n_kv_heads + kvh) * a.s_max * D;

    if (!a.tree_mask && tid < a.n_tree)
        lds_parent[tid] = a.parent[(int64_t)b * a.n_tree + tid];

    uint4 kreg[CH], vreg[CH];
    auto load_tile = [&](int t) {
#pragma unroll
        for (int i = 0; i < CH; i++) {
            int chunk = i * 64 + lane;
            int row = chunk / (D / 8), col = chunk % (D / 8);
            int key = t * 32 + row;
            if (key < kv_len) {
                kreg[i] = *reinterpret_cast<const uint4 *>(kbase + (int64_t)key * D + col * 8);
                vreg[i] = *reinterpret_cast<const uint4 *>(vbase + (int64_t)key * D + col * 8);
            } else {
                kreg[i] = make_uint4(0, 0, 0, 0);
                vreg[i] = make_uint4(0, 0, 0, 0);
            }
        }
    };
    uint16_t *wk = lds + wave * G::WAVE_ELEMS;
    uint16_t *wv = wk + 32 * KSTR;
    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < CH; i++) {
            int chunk = i * 64 + lane;
            int row = chunk / (D / 8), col = chunk % (D / 8);
            *reinterpret_cast<uint4 *>(wk + row * KSTR + col * 8) = kreg[i];
            *reinterpret_cast<uint4 *>(wv + row * VSTR + col * 8) = vreg[i];
        }
    };
    int t = t_begin + wave;
    if (t < t_end)
        load_tile(t);

    __syncthreads();   // parents staged

    // per query tile: which (head, row) this lane's column is, its mask, its Q fragments
    bf16x8 qf[QG][NKS];
    uint64_t qmask[QG];
    int q_row[QG], q_head[QG];
    const int n_qtiles = a.group * a.tiles_per_head;
#pragma unroll
    for (int qt = 0; qt < QG; qt++) {
        int tq = qg * QG + qt;
        int hh = tq / a.tiles_per_head, nt = tq % a.tiles_per_head;
        int row = nt * 16 + c;
        bool valid = tq < n_qtiles && row < a.n_q;
        q_row[qt] = valid ? row : -1;
        q_head[qt] = kvh * a.group + hh;
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

    WaveState<QG, NDT> st;
#pragma unroll
    for (int qt = 0; qt < QG; qt++) {
        st.m[qt] = -INFINITY;
        st.l[qt] = 0.0f;
#pragma unroll
        for (int dt = 0; dt < NDT; dt++)
            st.o[qt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    for (; t < t_end; t += 4) {
        store_tile();
        wave_lds_fence();
        if (t + 4 < t_end)
            load_tile(t + 4);
        const int key0 = t * 32;
        const bool needs_mask = key0 + 32 > P;   // tile touches tree rows or the ragged end

        // ---- S^T = K Q^T for 32 keys x (16 * QG) query columns
        f32x4 sacc[2][QG];
#pragma unroll
        for (int qt = 0; qt < QG; qt++) {
            sacc[0][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
            sacc[1][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int ks = 0; ks < NKS; ks++) {
            bf16x8 kf0 = *reinterpret_cast<const bf16x8 *>(wk + c * KSTR + ks * 32 + g * 8);
            bf16x8 kf1 = *reinterpret_cast<const bf16x8 *>(wk + (16 + c) * KSTR + ks * 32 + g * 8);
#pragma unroll
            for (int qt = 0; qt < QG; qt++) {
                sacc[0][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf0, qf[qt][ks], sacc[0][qt], 0, 0, 0);
                sacc[1][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf1, qf[qt][ks], sacc[1][qt], 0, 0, 0);
            }
        }
        // ---- online softmax; lane owns query column c and key rows g*4+r of both 16-key tiles
        bf16x8 pf[QG];
#pragma unroll
        for (int qt = 0; qt < QG; qt++) {
            float sv[8];
            float mx = -INFINITY;
#pragma unroll
            for (int i = 0; i < 8; i++) {
                float x = sacc[i >> 2][qt][i & 3] * a.scale_log2;
                if (needs_mask) {
                    int rel = key0 + (i >> 2) * 16 + g * 4 + (i & 3) - P;
                    bool vis = rel < 0 || (rel < a.n_tree && ((qmask[qt] >> (rel & 63)) & 1ull));
                    x = vis ? x : -INFINITY;
                }
                sv[i] = x;
                mx = fmaxf(mx, x);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            float m_new = fmaxf(st.m[qt], mx);
            float m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
            float alpha = __builtin_amdgcn_exp2f(st.m[qt] - m_safe);
            st.m[qt] = m_new;
            float psum = 0.0f;
#pragma unroll
            for (int i = 0; i < 8; i++) {
                float p = __builtin_amdgcn_exp2f(sv[i] - m_safe);
                psum += p;
                pf[qt][i] = (__bf16)p;
            }
            st.l[qt] = st.l[qt] * alpha + psum;
#pragma unroll
            for (int dt = 0; dt < NDT; dt++)
                st.o[qt][dt] *= alpha;
        }
        // ---- O^T += V^T P^T
#pragma unroll
        for (int dt = 0; dt < NDT; dt++) {
            const uint16_t *vp = wv + (g * 4 + (c >> 2)) * VSTR + dt * 16 + (c & 3) * 4;
            s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(vp));
            s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(vp + 16 * VSTR));
            s16x8 vv = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
            bf16x8 vf = __builtin_bit_cast(bf16x8, vv);
#pragma unroll
            for (int qt = 0; qt < QG; qt++)
                st.o[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[qt], st.o[qt][dt], 0, 0, 0);
        }
        wave_lds_fence();
    }

    // the softmax sum was kept per lane over the lane's own key rows: complete it across the 4 row groups
#pragma unroll
    for (int qt = 0; qt < QG; qt++) {
        float l = st.l[qt];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        st.l[qt] = l;
    }

    // ---- merge the 4 waves through LDS, fixed order: (0<-2, 1<-3), then 0<-1
    float *mbuf = reinterpret_cast<float *>(smem_raw);
    __syncthreads();
    if (wave >= 2)
        state_store<QG, NDT>(st, mbuf + (wave - 2) * G::STATE_FLOATS, lane);
    __syncthreads();
    if (wave < 2)
        state_merge<QG, NDT>(st, mbuf + wave * G::STATE_FLOATS, lane);
    __syncthreads();
    if (wave == 1)
        state_store<QG, NDT>(st, mbuf, lane);
    __syncthreads();
    if (wave != 0)
        return;
    state_merge<QG, NDT>(st, mbuf, lane);

    // ---- several splits: publish this workgroup's state; the last arrival of the group merges all of them
    if (nsplit > 1) {
        const int64_t grp = ((int64_t)b * a.n_kv_heads + kvh) * a.n_qg + qg;
        float *mine = a.part + (grp * nsplit + split) * G::STATE_FLOATS;
        state_store<QG, NDT>(st, mine, lane);
        __threadfence();
        int ticket = 0;
        if (lane == 0)
            ticket = atomicAdd(&a.counters[grp], 1);
        ticket = __shfl(ticket, 0);
        if (ticket != nsplit - 1)
            return;
        __threadfence();
#pragma unroll
        for (int qt = 0; qt < QG; qt++) {
            st.m[qt] = -INFINITY;
            st.l[qt] = 0.0f;
#pragma unroll
            for (int dt = 0; dt < NDT; dt++)
                st.o[qt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        for (int s = 0; s < nsplit; s++)
            state_merge<QG, NDT>(st, a.part + (grp * nsplit + s) * G::STATE_FLOATS, lane);
        if (lane == 0)
            a.counters[grp] = 0;   // ready for the next call on this workspace
    }

    // ---- normalise and write
    constexpr float LN2 = 0.6931471805599453f;
#pragma unroll
    for (int qt = 0; qt < QG; qt++) {
        if (q_row[qt] < 0)
            continue;
        const float l = st.l[qt];
        const float inv = l > 0.0f ? 1.0f / l : 0.0f;
        uint16_t *op = reinterpret_cast<uint16_t *>(a.out) +
                       (((int64_t)b * a.n_q + q_row[qt]) * a.n_q_heads + q_head[qt]) * D + g * 4;
#pragma unroll
        for (int dt = 0; dt < NDT; dt++) {
            bf16x4 o;
#pragma unroll
            for (int r = 0; r < 4; r++)
                o[r] = (__bf16)(st.o[qt][dt][r] * inv);
            *reinterpret_cast<bf16x4 *>(op + dt * 16) = o;
        }
        if (a.lse && g == 0)
            a.lse[((int64_t)b * a.n_q_heads + q_head[qt]) * a.n_q + q_row[qt]] =
                l > 0.0f ? (st.m[qt] + log2f(l)) * LN2 : -INFINITY;
    }
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
    int tiles_per_head, qg, n_qg, n_splits, n_streams, grid;
    size_t state_floats, off_part, total;
};

int make_plan(const dream_attn_desc *d, int n_q, int64_t max_kv_len, Plan *p)
{
    const int G = d->n_q_heads / d->n_kv_heads;
    p->tiles_per_head = ceil_div(n_q, 16);
    const int n_qtiles = G * p->tiles_per_head;
    const int qg_max = d->head_dim == 256 ? 2 : 4;   // accumulator registers bound the query tiles per wave
    const int64_t base = (int64_t)d->batch * d->n_kv_heads;
    int qg = q_tiles_override();
    if (qg <= 0) {
        // largest query group that still yields at least ~half a chip of workgroups before splitting keys
        qg = qg_max;
        while (qg > 1 && base * ceil_div(n_qtiles, qg) < 128)
            qg >>= 1;
    }
    if (qg > qg_max)
        qg = qg_max;
    if (qg != 1 && qg != 2 && qg != 4)
        qg = 1;
    while (qg > 1 && qg / 2 >= n_qtiles)
        qg >>= 1;
    p->qg = qg;
    p->n_qg = ceil_div(n_qtiles, qg);
    const int tiles = ceil_div(max_kv_len, 32);
    int s = kv_splits_override();
    if (s <= 0)
        s = ceil_div(256, base * p->n_qg);
    const int max_split = tiles / 8 > 0 ? tiles / 8 : 1;   // keep at least two 32-key tiles per wave
    if (s > max_split)
        s = max_split;
    if (s < 1)
        s = 1;
    const int64_t groups = base * p->n_qg;
    if (groups > DREAM_WORKSPACE_HEADER_BYTES / 4)
        s = 1;
    p->n_splits = s;
    p->n_streams = (int)(base * s);
    p->grid = ceil_div(p->n_streams, 8) * 8 * p->n_qg;
    p->state_floats = (size_t)qg * (d->head_dim / 16) * 256 + (size_t)qg * 2 * 64;
    p->off_part = DREAM_WORKSPACE_HEADER_BYTES;
    p->total = p->off_part + (s > 1 ? (size_t)groups * s * p->state_floats * sizeof(float) : 0);
    if (d->dtype == DREAM_F32)
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

template <int D, int QG>
int launch_bf16(const AttnArgs &a, const Plan &p, hipStream_t st)
{
    using G = Geom<D, QG>;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_bf16_kernel<D, QG>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)G::LDS_BYTES) != hipSuccess)
            return fail(DREAM_ERR_HIP, "attention: cannot reserve %zu bytes of LDS", G::LDS_BYTES);
        attr_set = true;
    }
    hipLaunchKernelGGL((attn_bf16_kernel<D, QG>), dim3(p.grid), dim3(256), G::LDS_BYTES, st, a);
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
    make_plan(d, n_q, max_kv_len, &p);
    if (!ws || ws_bytes < p.total)
        return fail(DREAM_ERR_WORKSPACE, "%s: workspace of %zu bytes, %zu needed", who, ws_bytes, p.total);

    AttnArgs a;
    a.q = q; a.k = k; a.v = v;
    a.prefix_len = prefix_len; a.parent = parent; a.q_node = q_node; a.tree_mask = tree_mask;
    a.out = out; a.lse = lse;
    a.counters = reinterpret_cast<int32_t *>(ws);
    a.part = reinterpret_cast<float *>(static_cast<char *>(ws) + p.off_part);
    a.n_q_heads = d->n_q_heads; a.n_kv_heads = d->n_kv_heads; a.group = d->n_q_heads / d->n_kv_heads;
    a.n_q = n_q; a.n_tree = n_tree; a.include_self = include_self;
    a.tiles_per_head = p.tiles_per_head; a.n_qg = p.n_qg; a.n_splits = p.n_splits; a.n_streams = p.n_streams;
    a.s_max = d->s_max;
    a.scale = d->scale != 0.0f ? d->scale : 1.0f / sqrtf((float)d->head_dim);
    a.scale_log2 = a.scale * 1.4426950408889634f;
    hipStream_t st = as_stream(stream);

    if (d->dtype == DREAM_F32) {
        dim3 grid(n_q, d->n_q_heads, d->batch);
        hipLaunchKernelGGL(attn_f32_kernel, grid, dim3(256), 0, st, a, d->head_dim);
        return check_launch("attn_f32_kernel");
    }

    switch (d->head_dim * 10 + p.qg) {
    case 641:  return launch_bf16<64, 1>(a, p, st);
    case 642:  return launch_bf16<64, 2>(a, p, st);
    case 644:  return launch_bf16<64, 4>(a, p, st);
    case 1281: return launch_bf16<128, 1>(a, p, st);
    case 1282: return launch_bf16<128, 2>(a, p, st);
    case 1284: return launch_bf16<128, 4>(a, p, st);
    case 2561: return launch_bf16<256, 1>(a, p, st);
    case 2562: return launch_bf16<256, 2>(a, p, st);
    default:   return fail(DREAM_ERR_UNSUPPORTED, "%s: no kernel for head_dim %d with %d query tiles per wave", who, d->head_dim, p.qg);
    }
}

size_t workspace_for(const dream_attn_desc *d, int n_q, int64_t max_kv_len)
{
    if (!d || d->n_kv_heads < 1 || d->n_q_heads < 1 || d->n_q_heads % d->n_kv_heads || n_q < 1 || max_kv_len < 1 ||
        d->batch < 1)
        return DREAM_WORKSPACE_HEADER_BYTES;
    Plan p;
    make_plan(d, n_q, max_kv_len, &p);
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
