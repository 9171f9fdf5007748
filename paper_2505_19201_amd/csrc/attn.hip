// Tree-masked attention kernels for gfx950: dream_tree_verify_attn and dream_draft_xattn.
//
// Both calls compute softmax(q k^T * scale) v (Section 3.1, Eq. 1) over the keys a tree node may
// see: the whole cached prefix plus its ancestors in the draft tree (Section 3.1, tree-masking
// paragraph); verification includes the node itself, the draft's cross-attention does not.
//
// bf16, shared tiles (attn_bf16_kernel).  A workgroup serves one (sequence, KV head, key-range split, query
// group).  The query rows that share a KV head - every tree row of every query head of the GQA
// group - are cut into 16-row tiles; each wave owns QG of them (4 waves, or 8 waves for grouped-query shapes, or
// 8 waves as two key groups for multi-head shapes with one workgroup per CU).  All threads stream the key range in
// 32-key K/V tiles with 16-byte coalesced loads kept one or two steps ahead in registers, park each tile in one of
// two LDS stages (one barrier per step), and every wave reads the tile's MFMA fragments from LDS: a K/V byte leaves
// HBM once and serves all tree rows and all heads of the group.  Scores are formed transposed, S^T = K Q^T, with
// v_mfma_f32_16x16x32_bf16, so a lane owns one query column: the online-softmax state is a
// per-lane scalar and the fp32 score registers, converted to bf16, already are the B operand of
// the second contraction O^T += V^T P^T, whose A operand (V transposed) comes from the LDS
// transpose read ds_read_b64_tr_b16.  The softmax reference of a column is raised only when a
// score exceeds it by 8 octaves, so accumulators are rescaled a handful of times per call.  Where a workgroup is the
// only reader of its K/V rows the loads carry the nontemporal hint; output rows leave as whole lines with it.
//
// One CU can keep only a few tens of KB of loads in flight, so a short stream is bandwidth-starved
// unless all 256 CUs pull a share of it: when B * Hkv * query groups is small either attn_wave_kernel serves a
// query tile per workgroup in one launch (waves stream disjoint key tiles and merge in LDS), or the key range is
// split over several workgroups, each writes its (reference, sum, O) state to the workspace, and
// attn_merge_kernel merges the states of a group in split order (deterministic) and writes the
// rows.  (A merge across workgroups inside one launch costs more than the second launch: the L2s of the XCDs are not
// coherent with each other.)  Workgroups that read the same K/V stream get ids congruent mod 8 so that they run on one
// XCD and share its L2.
//
// fp32 path (attn_f32_kernel): plain vector-ALU kernel, one workgroup per (query row, head,
// sequence), used for float32 tensors (the small correctness configuration).
#include "common.h"
#include "dream_tuning.h"
#include <atomic>
#include <math.h>

using namespace dream;

namespace {

struct AttnArgs {
    const void *q, *k, *v;
    const int32_t *prefix_len, *parent, *q_node;
    const uint64_t *tree_mask;   // [B, n_tree, mask_words] when given
    void *out;
    float *lse;
    float *part;             // [groups, splits, 4 waves, state] per-wave states of every split
    int32_t n_q_heads, n_kv_heads, group;
    int32_t n_q, n_tree, include_self;
    int32_t tiles_per_head;  // 16-row query tiles per head
    int32_t n_qg;            // query groups per KV head
    int32_t mask_words;      // 64-bit words of a node's visibility mask: ceil(n_tree / 64)
    int32_t n_splits;
    int32_t n_streams;       // B * Hkv * n_splits
    int64_t s_max;
    float scale, scale_log2;
};

// Visibility of the tree nodes to one query: bit (a % 64) of word a / 64 is set iff node a is visible.  MW = 1 serves
// trees of up to 64 nodes, MW = 4 up to 256.
template <int MW>
struct NodeMask {
    uint64_t w[MW];
};

template <int MW>
__device__ __forceinline__ void mask_set(NodeMask<MW> &m, int node)
{
    if (MW == 1) {
        m.w[0] |= 1ull << node;
    } else {
#pragma unroll
        for (int i = 0; i < MW; i++)
            m.w[i] |= (node >> 6) == i ? 1ull << (node & 63) : 0ull;
    }
}

// bit `rel` of the mask (the caller has already excluded rel outside [0, n_tree))
template <int MW>
__device__ __forceinline__ uint32_t mask_bit(const NodeMask<MW> &m, int rel)
{
    if (MW == 1)
        return (uint32_t)(m.w[0] >> (rel & 63)) & 1u;
    // (kept as arithmetic on all words: a per-lane choice of the word would become an indexed private array)
    uint32_t bit = 0u;
#pragma unroll
    for (int i = 0; i < MW; i++)
        bit |= (uint32_t)(m.w[i] >> (rel & 63)) & (uint32_t)((rel >> 6) == i);
    return bit & 1u;
}

template <int MW>
__device__ __forceinline__ NodeMask<MW> visible_nodes(const AttnArgs &a, int b, int node, const int32_t *lds_parent)
{
    NodeMask<MW> m;
#pragma unroll
    for (int i = 0; i < MW; i++)
        m.w[i] = 0ull;
    if (a.tree_mask) {
#pragma unroll
        for (int i = 0; i < MW; i++)
            if (i < a.mask_words)
                m.w[i] = a.tree_mask[((int64_t)b * a.n_tree + node) * a.mask_words + i];
        return m;
    }
    if (a.include_self)
        mask_set(m, node);
    for (int p = lds_parent[node]; p >= 0; p = lds_parent[p])
        mask_set(m, p);
    return m;
}

template <int MW>
__device__ __forceinline__ NodeMask<MW> empty_mask()
{
    NodeMask<MW> m;
#pragma unroll
    for (int i = 0; i < MW; i++)
        m.w[i] = 0ull;
    return m;
}

// D: head dimension (K rows, Q); DV: V columns handled (D, or a slice of it when the output columns are split)
template <int D, int QG, int KT, int DV = D>
struct Geom {
    static constexpr int KSTR = D + 8;    // K row stride in LDS (elements): 16-byte pad, b128 reads spread over all banks
    static constexpr int VSTR = DV + 16;  // V row stride in LDS (elements): 4 consecutive rows land 8 banks apart
    static constexpr int TILE_ELEMS = 32 * (KSTR + VSTR);   // one 32-key K tile followed by its V tile
    static constexpr int STAGE_ELEMS = KT * TILE_ELEMS;     // a step handles KT tiles
    static constexpr int NDT = DV / 16;
    static constexpr int NKS = D / 32;
    static constexpr int CH = 32 * D / 8 / 256;             // 16-byte chunks per thread per tensor per tile
    static constexpr size_t LDS_BYTES = (size_t)2 * STAGE_ELEMS * 2 + DREAM_MAX_TREE * sizeof(int32_t);
};

template <int D, int QG>
struct StateGeom {
    static constexpr int NDT = D / 16;
    static constexpr int STATE_FLOATS = QG * NDT * 256 + QG * 2 * 64;   // one wave's (O, reference, sum) in lane-major order
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

// Row ownership of a lane: query tile qt of wave `wave` in query group qg -> (query head, query row) of column c.
struct RowOwner {
    int row, head;
};
__device__ __forceinline__ RowOwner row_owner(const AttnArgs &a, int kvh, int qg, int wave, int QG, int qt, int c, int nw = 4)
{
    int tq = (qg * nw + wave) * QG + qt;
    int hh = tq / a.tiles_per_head, nt = tq % a.tiles_per_head;
    int row = nt * 16 + c;
    bool valid = tq < a.group * a.tiles_per_head && row < a.n_q;
    RowOwner r;
    r.row = valid ? row : -1;
    r.head = kvh * a.group + hh;
    return r;
}

// The softmax reference of a column is only raised when a score exceeds it by more than this many
// octaves, so exp2(score - reference) stays below 2^8 and the accumulators are seldom rescaled.
#define DREAM_SOFTMAX_SLACK 8.0f
// Build-time knobs of the launch shapes (each value is the measured best):
#ifndef DREAM_Q1_WAVES
#define DREAM_Q1_WAVES 2     // waves per SIMD the 4-wave one-tile-per-wave variants are compiled for (3: 1024 workgroups then run as 3 + 1 per CU, 75 against 71 us at 32 LLaVA sequences; 4: spills)
#endif
#ifndef DREAM_KG2_MAX_WG
#define DREAM_KG2_MAX_WG 1   // two key groups while a CU would get at most this many 4-wave workgroups (measured: -5 % at 1, +3 % at 4)
#endif
#ifndef DREAM_W8Q1_WAVES
#define DREAM_W8Q1_WAVES 1   // the same for the 8-wave variants (2 workgroups per CU would need 128 registers: spills, slower)
#endif
#ifndef DREAM_W8_PFD
#define DREAM_W8_PFD 2   // steps in flight of the 8-wave shared-tile form
#endif

// Online softmax of KT 32-key tiles for the QG query tiles of a wave.  sacc holds the raw scores S^T (lane owns
// query column c and key rows g*4+r of every 16-key block); on return pf holds the probabilities as the bf16 B
// operand of O^T += V^T P^T, and the running (reference, sum, accumulators) of `st` are updated.
// Only the first part depends on whether the step needs the visibility test (one wave-uniform branch per step, not
// one per score): a step wholly inside the prefix takes the maximum over the raw scores and leaves the scaling to
// the exponent's fused multiply-add; the general path scales and masks the scores in place.
// softmax_prepare: visibility test, maxima, and the (rare) raise of the references with the rescaling of the
// accumulators; returns what still multiplies the stored scores.  softmax_exponentials: the straight-line rest.
template <int QG, int KT, int NDT, int MW>
__device__ __forceinline__ float softmax_prepare(f32x4 (&sacc)[KT][2][QG], WaveState<QG, NDT> &st, const NodeMask<MW> (&qmask)[QG],
                                                 bool needs_mask, int key0, int P, int key_end, int n_tree, float scale_log2, int g)
{
    float mx_q[QG];
    if (needs_mask) {
#pragma unroll
        for (int qt = 0; qt < QG; qt++) {
            float mx = -INFINITY;
#pragma unroll
            for (int kt = 0; kt < KT; kt++) {
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    float x = sacc[kt][e >> 2][qt][e & 3] * scale_log2;
                    const int key = key0 + kt * 32 + (e >> 2) * 16 + g * 4 + (e & 3);
                    const int rel = key - P;
                    const uint32_t bit = mask_bit(qmask[qt], rel);
                    const uint32_t vis = ((uint32_t)(rel < 0) | ((uint32_t)(rel < n_tree) & bit)) & (uint32_t)(key < key_end);
                    x = vis ? x : -INFINITY;
                    sacc[kt][e >> 2][qt][e & 3] = x;
                    mx = fmaxf(mx, x);
                }
            }
            mx_q[qt] = mx;
        }
    } else {
#pragma unroll
        for (int qt = 0; qt < QG; qt++) {
            float mx = -INFINITY;
#pragma unroll
            for (int kt = 0; kt < KT; kt++)
#pragma unroll
                for (int e = 0; e < 8; e++)
                    mx = fmaxf(mx, sacc[kt][e >> 2][qt][e & 3]);
            mx_q[qt] = mx * scale_log2;   // scale_log2 >= 0 on this path
        }
    }
    const float mult = needs_mask ? 1.0f : scale_log2;   // what still multiplies the stored scores
    bool raise = false;
#pragma unroll
    for (int qt = 0; qt < QG; qt++)
        raise = raise || (mx_q[qt] > st.m[qt] + DREAM_SOFTMAX_SLACK);
    if (__any(raise)) {
        // rare: some column's reference is raised to the true maximum over its 4 row groups
#pragma unroll
        for (int qt = 0; qt < QG; qt++) {
            float mx = mx_q[qt];
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            if (mx > st.m[qt] + DREAM_SOFTMAX_SLACK) {
                float alpha = __builtin_amdgcn_exp2f(st.m[qt] - mx);   // 0 when the old reference was -inf
                st.m[qt] = mx;
                st.l[qt] *= alpha;
#pragma unroll
                for (int dt = 0; dt < NDT; dt++)
                    st.o[qt][dt] *= alpha;
            }
        }
    }
    return mult;
}

template <int QG, int KT, int NDT>
__device__ __forceinline__ void softmax_exponentials(const f32x4 (&sacc)[KT][2][QG], bf16x8 (&pf)[KT][QG], WaveState<QG, NDT> &st, float mult)
{
#pragma unroll
    for (int qt = 0; qt < QG; qt++) {
        const float neg_m = (st.m[qt] == -INFINITY) ? 0.0f : -st.m[qt];
        float psum = 0.0f;
#pragma unroll
        for (int kt = 0; kt < KT; kt++) {
#pragma unroll
            for (int e = 0; e < 8; e++) {
                float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kt][e >> 2][qt][e & 3], mult, neg_m));
                psum += p;
                pf[kt][qt][e] = (__bf16)p;
            }
        }
        st.l[qt] += psum;
    }
}

// S^T = K Q^T for the KT 32-key tiles held in LDS at `stage` (K tile, then V tile, per 32 keys) x the (16 * QG) query
// columns of this wave; independent accumulators keep the MFMA pipe full.
template <int D, int QG, int KT, int DV = D>
__device__ __forceinline__ void tiles_scores(const uint16_t *stage, const bf16x8 (&qf)[QG][D / 32], f32x4 (&sacc)[KT][2][QG], int c, int g)
{
    using G = Geom<D, QG, KT, DV>;
    constexpr int KSTR = G::KSTR, NKS = G::NKS;
#pragma unroll
    for (int kt = 0; kt < KT; kt++) {
        const uint16_t *sk = stage + kt * G::TILE_ELEMS;
        bf16x8 kfr[2][NKS];
#pragma unroll
        for (int ks = 0; ks < NKS; ks++) {
            kfr[0][ks] = *reinterpret_cast<const bf16x8 *>(sk + c * KSTR + ks * 32 + g * 8);
            kfr[1][ks] = *reinterpret_cast<const bf16x8 *>(sk + (16 + c) * KSTR + ks * 32 + g * 8);
        }
#pragma unroll
        for (int qt = 0; qt < QG; qt++) {
            sacc[kt][0][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
            sacc[kt][1][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int ks = 0; ks < NKS; ks++) {
#pragma unroll
            for (int qt = 0; qt < QG; qt++) {
                sacc[kt][0][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kfr[0][ks], qf[qt][ks], sacc[kt][0][qt], 0, 0, 0);
                sacc[kt][1][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kfr[1][ks], qf[qt][ks], sacc[kt][1][qt], 0, 0, 0);
            }
        }
    }
}

// Online softmax of the raw scores `sacc` of the KT tiles at `stage` (first key key0) and O^T += V^T P^T.
template <int D, int QG, int KT, int DV = D, int MW>
__device__ __forceinline__ void tiles_softmax_pv(const uint16_t *stage, int key0, int P, int key_end, int n_tree, float scale_log2,
                                                 f32x4 (&sacc)[KT][2][QG], const NodeMask<MW> (&qmask)[QG], WaveState<QG, DV / 16> &st, int c, int g)
{
    using G = Geom<D, QG, KT, DV>;
    constexpr int KSTR = G::KSTR, VSTR = G::VSTR, NDT = G::NDT;
    // step touches tree rows, the ragged end or the next split (a negative scale also goes the general way)
    const bool needs_mask = key0 + KT * 32 > min(P, key_end) || scale_log2 < 0.0f;
    // ---- V^T fragments of the first tile (first half of the head dimension for D = 256) are requested
    // now, so their LDS latency hides behind the softmax arithmetic
    constexpr int VH = DV == 256 ? 2 : 1, NDH = NDT / VH;
    s16x4 vfr[NDH][2];
    const int v_off = 32 * KSTR + (g * 4 + (c >> 2)) * VSTR + (c & 3) * 4;
    auto read_v = [&](int kt, int h) {
        const uint16_t *vrow = stage + kt * G::TILE_ELEMS + v_off + h * NDH * 16;
#pragma unroll
        for (int dt = 0; dt < NDH; dt++) {
            vfr[dt][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(vrow + dt * 16));
            vfr[dt][1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(vrow + dt * 16 + 16 * VSTR));
        }
    };
    read_v(0, 0);
    // ---- online softmax; lane owns query column c and key rows g*4+r of every 16-key block
    bf16x8 pf[KT][QG];
    const float mult = softmax_prepare<QG, KT, NDT, MW>(sacc, st, qmask, needs_mask, key0, P, key_end, n_tree, scale_log2, g);
    softmax_exponentials<QG, KT, NDT>(sacc, pf, st, mult);
    // ---- O^T += V^T P^T
#pragma unroll
    for (int kt = 0; kt < KT; kt++) {
#pragma unroll
        for (int h = 0; h < VH; h++) {
            if (kt > 0 || h > 0)
                read_v(kt, h);
#pragma unroll
            for (int dt = 0; dt < NDH; dt++) {
                s16x8 vv = __builtin_shufflevector(vfr[dt][0], vfr[dt][1], 0, 1, 2, 3, 4, 5, 6, 7);
                bf16x8 vf = __builtin_bit_cast(bf16x8, vv);
#pragma unroll
                for (int qt = 0; qt < QG; qt++)
                    st.o[qt][h * NDH + dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[kt][qt], st.o[qt][h * NDH + dt], 0, 0, 0);
            }
        }
    }
}

// QK^T, online softmax and PV for KT consecutive 32-key tiles held in LDS at `stage`, for the QG query tiles of this
// wave.  key0 is the global key index of the first row.
template <int D, int QG, int KT, int DV = D, int MW>
__device__ __forceinline__ void tiles_compute(const uint16_t *stage, int key0, int P, int key_end, int n_tree, float scale_log2,
                                              const bf16x8 (&qf)[QG][D / 32], const NodeMask<MW> (&qmask)[QG],
                                              WaveState<QG, DV / 16> &st, int c, int g)
{
    f32x4 sacc[KT][2][QG];
    tiles_scores<D, QG, KT, DV>(stage, qf, sacc, c, g);
    __builtin_amdgcn_sched_barrier(0);
    tiles_softmax_pv<D, QG, KT, DV, MW>(stage, key0, P, key_end, n_tree, scale_log2, sacc, qmask, st, c, g);
}

// LDS traffic inside one wave needs no barrier, only program order.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// KT: 32-key tiles handled per step (per barrier, per softmax update); PFD: steps kept in flight in registers;
// NW: waves per workgroup (4, or 8 when the key range is not split: twice the query tiles share one LDS tile);
// MW: 64-bit words of a node's visibility mask (1: trees of up to 64 nodes; 4: up to 256);
// ONCE: this workgroup is the only reader of its K/V rows (one query group per KV head), so the loads carry the
// nontemporal hint: rows that are used once otherwise displace each other, and the output rows on their way out, in
// L2 (measured at 32 sequences: LLaVA 82.5 -> 71 us, SmolVLM 83.5 -> 74.5 us per launch).  With several query groups per
// KV head the later groups hit the rows in L2, so those launches use the variant without the hint.  (A run-time choice
// between the two kinds of load does not survive the compiler: it merges them into plain loads.)
template <int QG, int NDT>
__device__ __forceinline__ void state_merge(WaveState<QG, NDT> &s, const float *src, int lane);

// KG: key groups (1 or 2).  With 2, the 8 waves are two groups of 4: both serve the same (up to 4·QG) query tiles, a step
// stages 2·KT tiles and each group computes its KT of them; the two partial states of a query tile meet in LDS at the
// end.  For multi-head shapes with few streams per CU: twice the waves and twice the bytes in flight per workgroup.
template <int D, int QG, int KT, int PFD, int NW = 4, int MW = 1, bool ONCE = false, int KG = 1>
__global__ __launch_bounds__(64 * NW, (QG == 1 && D <= 128) ? (NW == 4 ? DREAM_Q1_WAVES : DREAM_W8Q1_WAVES) : 1) void attn_bf16_kernel(AttnArgs a)
{
    using G = Geom<D, QG, KT>;
    using GS = Geom<D, QG, KT * KG>;             // what a step stages
    static_assert(KG == 1 || (KG == 2 && NW == 8), "two key groups: 8 waves");
    constexpr int KSTR = G::KSTR, VSTR = G::VSTR, NDT = G::NDT, NKS = G::NKS;
    constexpr int QW = NW / KG;                  // waves that own different query tiles
    constexpr int NT = 64 * NW, LPR = D / 8, CPT = 32 * LPR;   // threads; 16-byte chunks per row and per tile (one tensor)
    constexpr int NLD = KT * KG * CPT / NT;                    // chunks per thread per tensor per step
    static_assert(NLD >= 1 && NLD * NT == KT * KG * CPT, "the chunks of a step divide evenly among the threads");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    uint16_t *lds = reinterpret_cast<uint16_t *>(smem_raw);
    int32_t *lds_parent = reinterpret_cast<int32_t *>(smem_raw + (size_t)2 * GS::STAGE_ELEMS * 2);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps bookkeeping in scalar registers
    const int wave = wave_all % QW, kgrp = wave_all / QW;             // query-tile slot and key group of this wave
    const int c = lane & 15, g = lane >> 4;

    // workgroup id -> (K/V stream, query group): ids that share a stream are congruent mod 8 (same XCD)
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int stream = (slot / a.n_qg) * 8 + xcd, qg = slot % a.n_qg;
    if (stream >= a.n_streams)
        return;
    const int nsplit = a.n_splits;
    const int split = stream % nsplit, bk = stream / nsplit;
    const int kvh = bk % a.n_kv_heads, b = bk / a.n_kv_heads;

    // tree metadata is requested first: the mask walk then overlaps the K/V loads still in flight
    int32_t my_parent = -1;
    if (!a.tree_mask && tid < a.n_tree)
        my_parent = a.parent[(int64_t)b * a.n_tree + tid];

    const int P = (int)min((int64_t)max(a.prefix_len[b], 0), a.s_max - a.n_tree);   // never past the cache, whatever the array holds
    const int kv_len = P + a.n_tree;
    const int tiles_total = (kv_len + 31) / 32;
    const int tps = (tiles_total + nsplit - 1) / nsplit;
    const int t_begin = split * tps;
    const int t_end = min(t_begin + tps, tiles_total);
    const int n_my = max(t_end - t_begin, 0);
    const int n_steps = (n_my + KT * KG - 1) / (KT * KG);
    const int key_end = min(kv_len, t_end * 32);   // keys at or past it belong to nobody or to the next split

    const uint16_t *kbase = reinterpret_cast<const uint16_t *>(a.k) + ((int64_t)b * a.n_kv_heads + kvh) * a.s_max * D;
    const uint16_t *vbase = reinterpret_cast<const uint16_t *>(a.v) + ((int64_t)b * a.n_kv_heads + kvh) * a.s_max * D;

    // ---- cooperative loads: a thread owns NLD 16-byte chunks of K and of V per step.  Rows past the live
    // range are clamped to the last live row (their scores are masked, so only finite values ever meet a
    // zero probability); tile indices past this workgroup's range are clamped too, so the number of loads
    // issued never depends on control flow and prefetches stay in flight across iterations.
    u32x4 kreg[PFD][NLD], vreg[PFD][NLD];
    // chunk j of this thread within a step: tile ld_tile(j) of the step, row ld_row(j), 16-byte column ld_col(j)
    // (a tile is CPT / NT passes of the workgroup, or, with more threads than a tile has chunks, a pass covers NT / CPT tiles)
    auto ld_tile = [&](int j) {
        if constexpr (CPT >= NT)
            return j / (CPT / NT);
        else
            return tid / CPT + j * (NT / CPT);
    };
    auto ld_row = [&](int j) {
        if constexpr (CPT >= NT)
            return tid / LPR + (j % (CPT / NT)) * (NT / LPR);
        else
            return (tid % CPT) / LPR;
    };
    const int ld_col = tid % LPR;   // (NT is a multiple of LPR)
    auto load_step = [&](int i, u32x4(&kr)[NLD], u32x4(&vr)[NLD]) {
#pragma unroll
        for (int j = 0; j < NLD; j++) {
            const int t = min(t_begin + i * KT * KG + ld_tile(j), t_end - 1);
            const int key = min(t * 32 + ld_row(j), kv_len - 1);
            const u32x4 *kp = reinterpret_cast<const u32x4 *>(kbase + (int64_t)key * D + ld_col * 8);
            const u32x4 *vp = reinterpret_cast<const u32x4 *>(vbase + (int64_t)key * D + ld_col * 8);
            if constexpr (ONCE) {
                kr[j] = __builtin_nontemporal_load(kp);
                vr[j] = __builtin_nontemporal_load(vp);
            } else {
                kr[j] = *kp;
                vr[j] = *vp;
            }
        }
    };
    if (n_my > 0) {
#pragma unroll
        for (int pf = 0; pf < PFD; pf++)
            load_step(pf, kreg[pf], vreg[pf]);
    }

    // ---- this wave's queries: fragments, owning rows, masks
    bf16x8 qf[QG][NKS];
    int q_node_of[QG];
    bool q_valid[QG];
    bool wave_active = false;
#pragma unroll
    for (int qt = 0; qt < QG; qt++) {
        RowOwner ro = row_owner(a, kvh, qg, wave, QG, qt, c, QW);
        q_valid[qt] = ro.row >= 0;
        wave_active = wave_active || q_valid[qt];
        const int row = q_valid[qt] ? ro.row : 0;
        const int head = q_valid[qt] ? ro.head : kvh * a.group;
        q_node_of[qt] = a.q_node ? min(max(a.q_node[(int64_t)b * a.n_q + row], 0), a.n_tree - 1) : row;
        const uint16_t *qp = reinterpret_cast<const uint16_t *>(a.q) + (((int64_t)b * a.n_q + row) * a.n_q_heads + head) * D + g * 8;
#pragma unroll
        for (int ks = 0; ks < NKS; ks++)
            qf[qt][ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 32);
    }
    wave_active = __any(wave_active);
    if (!a.tree_mask && tid < a.n_tree)
        lds_parent[tid] = my_parent < tid ? my_parent : -1;   // a walk up the tree always ends
    __syncthreads();   // parents staged

    NodeMask<MW> qmask[QG];
#pragma unroll
    for (int qt = 0; qt < QG; qt++) {
        qmask[qt] = q_valid[qt] ? visible_nodes<MW>(a, b, q_node_of[qt], lds_parent) : empty_mask<MW>();
        if (!q_valid[qt]) {
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

    // one step of KT tiles: registers -> LDS stage, barrier, refill the register set, compute from LDS
    auto step = [&](int i, u32x4(&kr)[NLD], u32x4(&vr)[NLD]) {
        uint16_t *stage = lds + (i & 1) * GS::STAGE_ELEMS;
#pragma unroll
        for (int j = 0; j < NLD; j++) {
            uint16_t *tile = stage + ld_tile(j) * G::TILE_ELEMS;
            *reinterpret_cast<u32x4 *>(tile + ld_row(j) * KSTR + ld_col * 8) = kr[j];
            *reinterpret_cast<u32x4 *>(tile + 32 * KSTR + ld_row(j) * VSTR + ld_col * 8) = vr[j];
        }
        __syncthreads();
        load_step(i + PFD, kr, vr);
        if (!wave_active)
            return;
        tiles_compute<D, QG, KT, D, MW>(stage + kgrp * KT * G::TILE_ELEMS, (t_begin + (i * KG + kgrp) * KT) * 32, P, key_end, a.n_tree, a.scale_log2, qf,
                                        qmask, st, c, g);
    };

    // every load issued so far (queries, masks, first tiles) has to land before the loop: the in-order
    // load counter then only ever counts tile prefetches inside it
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    {
        int i = 0;
        for (; i + PFD <= n_steps; i += PFD) {
#pragma unroll
            for (int pf = 0; pf < PFD; pf++)
                step(i + pf, kreg[pf], vreg[pf]);
        }
        // leftover steps run outside the loop so that its body always issues the same number of loads
#pragma unroll
        for (int pf = 0; pf < PFD - 1; pf++)
            if (i + pf < n_steps)
                step(i + pf, kreg[pf], vreg[pf]);
    }
    __syncthreads();   // every wave is done with the last tile: the stage areas can be reused for states and output rows
    constexpr int STATE = StateGeom<D, QG>::STATE_FLOATS;
    if (KG == 2) {
        // the second key group parks its states; the first adds them to its own (a barrier in between, so no early exit)
        float *sbuf = reinterpret_cast<float *>(smem_raw) + wave * STATE;
        if (kgrp == 1 && wave_active)
            state_store<QG, NDT>(st, sbuf, lane);
        __syncthreads();
        if (kgrp == 1 || !wave_active)
            return;
        state_merge<QG, NDT>(st, sbuf, lane);
    }
    if (!wave_active)
        return;

    // the softmax sum was kept per lane over the lane's own key rows: complete it across the 4 row groups
#pragma unroll
    for (int qt = 0; qt < QG; qt++) {
        float l = st.l[qt];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        st.l[qt] = l;
    }
    if (NW == 4 && nsplit > 1) {
        // several splits: publish this wave's state for attn_merge_kernel (the launch plan never splits the 8-wave form)
        const int64_t grp = ((int64_t)b * a.n_kv_heads + kvh) * a.n_qg + qg;
        state_store<QG, NDT>(st, a.part + ((grp * nsplit + split) * 4 + wave) * StateGeom<D, QG>::STATE_FLOATS, lane);
        return;
    }
    // Output rows leave through LDS: a lane holds 4 columns of one row per column tile, which stored directly would
    // be 32-byte pieces of 16 rows per instruction; staged in the wave's own LDS area (free by now) the rows go out
    // as whole 16-byte-per-lane rows, full cache lines per instruction, with the nontemporal hint (nobody in this
    // launch reads them; measured together with the staging: 82.5 -> 78 us at 32 LLaVA sequences, either alone nothing).
    constexpr float LN2 = 0.6931471805599453f;
    constexpr int OSTR = D + 8, RPP = 64 / LPR;   // staging row stride; rows per store instruction (LPR lanes per row)
    constexpr size_t OT_BASE = KG == 2 ? (size_t)QW * STATE * sizeof(float) : 0;   // behind the parked states, which may still be read
    static_assert(OT_BASE + (size_t)QW * 16 * OSTR * 2 <= (size_t)2 * GS::STAGE_ELEMS * 2, "states and output staging reuse the tile stages");
    uint16_t *ot = reinterpret_cast<uint16_t *>(smem_raw + OT_BASE) + wave * 16 * OSTR;
#pragma unroll
    for (int qt = 0; qt < QG; qt++) {
        RowOwner ro = row_owner(a, kvh, qg, wave, QG, qt, c, QW);
        const float l = st.l[qt];
        const float inv = l > 0.0f ? 1.0f / l : 0.0f;
#pragma unroll
        for (int dt = 0; dt < NDT; dt++) {
            bf16x4 ob;
#pragma unroll
            for (int r = 0; r < 4; r++)
                ob[r] = (__bf16)(st.o[qt][dt][r] * inv);
            *reinterpret_cast<bf16x4 *>(ot + c * OSTR + dt * 16 + g * 4) = ob;
        }
        if (ro.row >= 0 && a.lse && g == 0)
            a.lse[((int64_t)b * a.n_q_heads + ro.head) * a.n_q + ro.row] = l > 0.0f ? (st.m[qt] + log2f(l)) * LN2 : -INFINITY;
        wave_lds_fence();
#pragma unroll
        for (int pass = 0; pass < 16 / RPP; pass++) {
            const int r2 = pass * RPP + lane / LPR, col = (lane % LPR) * 8;
            RowOwner ro2 = row_owner(a, kvh, qg, wave, QG, qt, r2, QW);
            if (ro2.row >= 0) {
                uint16_t *op = reinterpret_cast<uint16_t *>(a.out) + (((int64_t)b * a.n_q + ro2.row) * a.n_q_heads + ro2.head) * D + col;
                __builtin_nontemporal_store(*reinterpret_cast<const u32x4 *>(ot + r2 * OSTR + col), reinterpret_cast<u32x4 *>(op));
            }
        }
        wave_lds_fence();
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

// Short streams with few query tiles (one sequence; up to 4 query heads per KV head): a workgroup serves ONE 16-row query tile of one
// head over the whole key range, its NW waves stream disjoint 32-key tiles (each through a private LDS
// area, no workgroup barrier in the loop) and merge their states through LDS at the end, in a fixed
// order.  No key split, so no second launch; the workgroups of a head re-read its K/V through the L2 of
// one XCD.  With DS > 1 the output columns are split over DS workgroups: each computes all the scores
// (reads all of K) but only its slice of V and of the output, which multiplies the CUs that pull data when
// there are few query tiles and needs no merge across workgroups.
// Grid: x = (query tile * DS + column slice) * 8 + XCD slot, y = KV head / 8, z = sequence, so that the
// workgroups of one K/V stream share an XCD and the index arithmetic needs no division.  a.n_qg holds
// the number of query tiles per KV head.
//
// Each wave keeps one tile in flight in registers: a CU holds about 64 KB of outstanding loads whatever is
// asked of it, so a second tile in flight per wave only queues behind the first.
// QT: query tiles a workgroup serves (1, or 2 when there are more (KV head, query tile) pairs than CUs: the
// same K/V stream then feeds two tiles and half as many workgroups pull it).
template <int D, int NW, int DS, int QT = 1>
__global__ __launch_bounds__(64 * NW) void attn_wave_kernel(AttnArgs a)
{
    constexpr int DV = D / DS;
    using G = Geom<D, 1, 1, DV>;
    constexpr int KSTR = G::KSTR, VSTR = G::VSTR, NDT = G::NDT, NKS = G::NKS;
    constexpr int CHK = 32 * D / 8 / 64, CHV = 32 * DV / 8 / 64;   // 16-byte chunks per lane per tile of K, V
    constexpr int STATE = StateGeom<DV, QT>::STATE_FLOATS;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    uint16_t *lds = reinterpret_cast<uint16_t *>(smem_raw);
    int32_t *lds_parent = reinterpret_cast<int32_t *>(smem_raw + (size_t)NW * G::TILE_ELEMS * 2);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, g = lane >> 4;
    const int unit = blockIdx.x >> 3;
    const int kvh = blockIdx.y * 8 + (blockIdx.x & 7), tq0 = (unit / DS) * QT, ds = unit % DS, b = blockIdx.z;
    if (kvh >= a.n_kv_heads)
        return;
    const uint16_t *kbase = reinterpret_cast<const uint16_t *>(a.k) + ((int64_t)b * a.n_kv_heads + kvh) * a.s_max * D;
    const uint16_t *vbase = reinterpret_cast<const uint16_t *>(a.v) + ((int64_t)b * a.n_kv_heads + kvh) * a.s_max * D + ds * DV;

    int32_t my_parent = -1;
    if (!a.tree_mask && tid < a.n_tree)
        my_parent = a.parent[(int64_t)b * a.n_tree + tid];
    const int P = (int)min((int64_t)max(a.prefix_len[b], 0), a.s_max - a.n_tree);   // never past the cache, whatever the array holds
    const int kv_len = P + a.n_tree;
    const int t_end = (kv_len + 31) / 32;
    const int n = t_end > wave ? (t_end - wave + NW - 1) / NW : 0;   // tiles of this wave: wave, wave + NW, ...

    u32x4 kr[CHK], vr[CHV];
    const int k_row = lane / (D / 8), k_col = lane % (D / 8), v_row = lane / (DV / 8), v_col = lane % (DV / 8);
    // Unconditional (the tile index is clamped), so the number of loads in flight does not depend on
    // control flow; the prefetch past the last tile re-reads it and is dropped.
    auto issue = [&](int t) {
        t = min(t, t_end - 1);
#pragma unroll
        for (int j = 0; j < CHK; j++) {
            const int key = min(t * 32 + k_row + j * (512 / D), kv_len - 1);
            kr[j] = *reinterpret_cast<const u32x4 *>(kbase + key * D + k_col * 8);
        }
#pragma unroll
        for (int j = 0; j < CHV; j++) {
            const int key = min(t * 32 + v_row + j * (512 / DV), kv_len - 1);
            vr[j] = *reinterpret_cast<const u32x4 *>(vbase + key * D + v_col * 8);
        }
    };
    issue(wave);

    // the query tiles: head hh of the group, rows nt*16 .. nt*16+15 (at most 4 heads per group, so three compares instead of a division)
    const int tph = a.tiles_per_head;
    int row[QT], head[QT], node[QT];
    bool valid[QT];
    bf16x8 qf[QT][NKS];
#pragma unroll
    for (int qt = 0; qt < QT; qt++) {
        const int tq = tq0 + qt;
        const int hh = (tq >= tph) + (tq >= 2 * tph) + (tq >= 3 * tph), nt = tq - hh * tph;
        row[qt] = nt * 16 + c;
        valid[qt] = hh < a.group && row[qt] < a.n_q;     // (the second tile of the last pair may not exist)
        head[qt] = kvh * a.group + (hh < a.group ? hh : 0);
        const int rr = valid[qt] ? row[qt] : 0;
        node[qt] = a.q_node ? min(max(a.q_node[(int64_t)b * a.n_q + rr], 0), a.n_tree - 1) : rr;
        const uint16_t *qp = reinterpret_cast<const uint16_t *>(a.q) + (((int64_t)b * a.n_q + rr) * a.n_q_heads + head[qt]) * D + g * 8;
#pragma unroll
        for (int ks = 0; ks < NKS; ks++)
            qf[qt][ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 32);
    }
    if (!a.tree_mask && tid < a.n_tree)
        lds_parent[tid] = my_parent < tid ? my_parent : -1;   // a walk up the tree always ends
    __syncthreads();
    NodeMask<1> qmask[QT];
    WaveState<QT, NDT> st;
#pragma unroll
    for (int qt = 0; qt < QT; qt++) {
        qmask[qt] = valid[qt] ? visible_nodes<1>(a, b, node[qt], lds_parent) : empty_mask<1>();
        if (!valid[qt]) {
#pragma unroll
            for (int ks = 0; ks < NKS; ks++)
#pragma unroll
                for (int i = 0; i < 8; i++)
                    qf[qt][ks][i] = (__bf16)0.0f;
        }
        st.m[qt] = -INFINITY;
        st.l[qt] = 0.0f;
#pragma unroll
        for (int dt = 0; dt < NDT; dt++)
            st.o[qt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): from here on only tile prefetches are in flight

    uint16_t *wt = lds + wave * G::TILE_ELEMS;
    for (int i = 0; i < n; i++) {
        const int t = wave + i * NW;
        uint16_t *dk = wt + k_row * KSTR + k_col * 8, *dv = wt + 32 * KSTR + v_row * VSTR + v_col * 8;
#pragma unroll
        for (int j = 0; j < CHK; j++)
            *reinterpret_cast<u32x4 *>(dk + j * (512 / D) * KSTR) = kr[j];
#pragma unroll
        for (int j = 0; j < CHV; j++)
            *reinterpret_cast<u32x4 *>(dv + j * (512 / DV) * VSTR) = vr[j];
        wave_lds_fence();
        issue(t + NW);
        tiles_compute<D, QT, 1, DV, 1>(wt, t * 32, P, kv_len, a.n_tree, a.scale_log2, qf, qmask, st, c, g);
        wave_lds_fence();
    }
#pragma unroll
    for (int qt = 0; qt < QT; qt++) {
        float l = st.l[qt];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        st.l[qt] = l;
    }
    // merge the waves through LDS (the tile areas are free by then) in one round: every wave parks its
    // state, then wave w sums the 16-wide output column tiles w, w+NW, ... over the states in wave order
    float *mbuf = reinterpret_cast<float *>(smem_raw);
    __syncthreads();
    state_store<QT, NDT>(st, mbuf + wave * STATE, lane);
    __syncthreads();
#pragma unroll
    for (int qt = 0; qt < QT; qt++) {
        if (!valid[qt])
            continue;
        float mj[NW], m = -INFINITY;
#pragma unroll
        for (int j = 0; j < NW; j++) {
            mj[j] = mbuf[j * STATE + QT * NDT * 256 + (qt * 2) * 64 + lane];
            m = fmaxf(m, mj[j]);
        }
        const float ms = (m == -INFINITY) ? 0.0f : m;
        float l = 0.0f;
#pragma unroll
        for (int j = 0; j < NW; j++) {
            mj[j] = __builtin_amdgcn_exp2f(mj[j] - ms);
            l += mj[j] * mbuf[j * STATE + QT * NDT * 256 + (qt * 2 + 1) * 64 + lane];
        }
        const float inv = l > 0.0f ? 1.0f / l : 0.0f;
        uint16_t *op = reinterpret_cast<uint16_t *>(a.out) + (((int64_t)b * a.n_q + row[qt]) * a.n_q_heads + head[qt]) * D + ds * DV + g * 4;
        for (int dt = wave; dt < NDT; dt += NW) {
            f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < NW; j++)
                o += reinterpret_cast<const f32x4 *>(mbuf + j * STATE)[(qt * NDT + dt) * 64 + lane] * mj[j];
            bf16x4 ob;
#pragma unroll
            for (int r = 0; r < 4; r++)
                ob[r] = (__bf16)(o[r] * inv);
            *reinterpret_cast<bf16x4 *>(op + dt * 16) = ob;
        }
        if (wave == 0 && ds == 0 && a.lse && g == 0)
            a.lse[((int64_t)b * a.n_q_heads + head[qt]) * a.n_q + row[qt]] = l > 0.0f ? (m + log2f(l)) * 0.6931471805599453f : -INFINITY;
    }
}

// Merge the split states of one (group, wave, query tile) in split order and write the rows.  One
// workgroup of 4 waves per state; wave w owns the 16-wide output column tiles w, w+4, ...; loads of
// up to 8 splits are in flight at once.
template <int D, int QG>
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a)
{
    constexpr int NDT = D / 16, NDW = NDT / 4;
    constexpr int STATE = StateGeom<D, QG>::STATE_FLOATS;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int qt = blockIdx.x % QG;
    const int wave = (blockIdx.x / QG) % 4;
    const int64_t grp = blockIdx.x / (QG * 4);
    const int qg = (int)(grp % a.n_qg);
    const int kvh = (int)((grp / a.n_qg) % a.n_kv_heads), b = (int)(grp / ((int64_t)a.n_qg * a.n_kv_heads));
    RowOwner ro = row_owner(a, kvh, qg, wave, QG, qt, lane & 15);
    if (__all(ro.row < 0))
        return;
    const int nsplit = a.n_splits;
    const float *base = a.part + (grp * nsplit * 4 + wave) * STATE;
    const int64_t stride = (int64_t)4 * STATE;
    const int ml = QG * NDT * 256 + (qt * 2) * 64 + lane;
    float m = -INFINITY;
    for (int s0 = 0; s0 < nsplit; s0 += 8) {
        float mm[8];
#pragma unroll
        for (int j = 0; j < 8; j++)
            mm[j] = s0 + j < nsplit ? base[(s0 + j) * stride + ml] : -INFINITY;
#pragma unroll
        for (int j = 0; j < 8; j++)
            m = fmaxf(m, mm[j]);
    }
    const float ms = (m == -INFINITY) ? 0.0f : m;
    float l = 0.0f;
    f32x4 o[NDW];
#pragma unroll
    for (int d = 0; d < NDW; d++)
        o[d] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < nsplit; s0 += 8) {
        float mm[8], ll[8];
        f32x4 oo[8][NDW];
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const bool live = s0 + j < nsplit;
            const float *src = base + (live ? s0 + j : s0) * stride;
            mm[j] = live ? src[ml] : -INFINITY;
            ll[j] = src[ml + 64];
#pragma unroll
            for (int d = 0; d < NDW; d++)
                oo[j][d] = reinterpret_cast<const f32x4 *>(src)[(qt * NDT + w + 4 * d) * 64 + lane];
        }
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const float wgt = __builtin_amdgcn_exp2f(mm[j] - ms);   // 0 for splits past the end
            l += wgt * ll[j];
#pragma unroll
            for (int d = 0; d < NDW; d++)
                o[d] += oo[j][d] * wgt;
        }
    }
    if (ro.row < 0)
        return;
    const int g = lane >> 4;
    const float inv = l > 0.0f ? 1.0f / l : 0.0f;
    uint16_t *op = reinterpret_cast<uint16_t *>(a.out) + (((int64_t)b * a.n_q + ro.row) * a.n_q_heads + ro.head) * D + g * 4;
#pragma unroll
    for (int d = 0; d < NDW; d++) {
        bf16x4 ob;
#pragma unroll
        for (int r = 0; r < 4; r++)
            ob[r] = (__bf16)(o[d][r] * inv);
        *reinterpret_cast<bf16x4 *>(op + (w + 4 * d) * 16) = ob;
    }
    if (a.lse && g == 0 && w == 0)
        a.lse[((int64_t)b * a.n_q_heads + ro.head) * a.n_q + ro.row] = l > 0.0f ? (m + log2f(l)) * 0.6931471805599453f : -INFINITY;
}

// ------------------------------------------------------------------------------------------------
// float32 path: one workgroup per (query row, head, sequence); 256 keys per pass.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attn_f32_kernel(AttnArgs a, int D)
{
    __shared__ float sq[256];
    __shared__ float sp[256];
    __shared__ float red[8];
    __shared__ uint64_t smask[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
    const int kvh = hq / a.group;
    const int P = (int)min((int64_t)max(a.prefix_len[b], 0), a.s_max - a.n_tree);   // never past the cache, whatever the array holds
    const int kv_len = P + a.n_tree;
    const float *q = reinterpret_cast<const float *>(a.q) + (((int64_t)b * a.n_q + row) * a.n_q_heads + hq) * D;
    const float *kb = reinterpret_cast<const float *>(a.k) + ((int64_t)b * a.n_kv_heads + kvh) * a.s_max * D;
    const float *vb = reinterpret_cast<const float *>(a.v) + ((int64_t)b * a.n_kv_heads + kvh) * a.s_max * D;
    if (tid < D)
        sq[tid] = q[tid];
    if (tid == 0) {
        const int node = a.q_node ? min(max(a.q_node[(int64_t)b * a.n_q + row], 0), a.n_tree - 1) : row;
        NodeMask<4> m = empty_mask<4>();
        if (a.tree_mask) {
#pragma unroll
            for (int i = 0; i < 4; i++)
                if (i < a.mask_words)
                    m.w[i] = a.tree_mask[((int64_t)b * a.n_tree + node) * a.mask_words + i];
        } else {
            const int32_t *par = a.parent + (int64_t)b * a.n_tree;
            if (a.include_self)
                mask_set(m, node);
            for (int prev = node, p = par[node]; p >= 0 && p < prev; prev = p, p = par[p])   // parents decrease: the walk ends
                mask_set(m, p);
        }
#pragma unroll
        for (int i = 0; i < 4; i++)
            smask[i] = m.w[i];
    }
    __syncthreads();
    float m_run = -INFINITY, l_run = 0.0f, o = 0.0f;
    for (int k0 = 0; k0 < kv_len; k0 += 256) {
        int key = k0 + tid;
        float s = -INFINITY;
        bool vis = key < P || (key < kv_len && ((smask[((key - P) >> 6) & 3] >> ((key - P) & 63)) & 1ull));
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
    int tiles_per_head, qg, n_qg, n_splits, n_streams, grid, n_groups, kt, pfd;
    int nw;           // waves per workgroup of the shared-tile kernel (4 or 8)
    int mw;           // 64-bit words of a node's visibility mask (1, or 4 for trees above 64 nodes)
    int once;         // 1: the variant whose K/V loads carry the nontemporal hint (one query group per KV head)
    int kg;           // key groups per workgroup of the shared-tile kernel (1; 2 = 8 waves as two groups of 4)
    bool wave_mode;   // one query tile per workgroup, waves split the keys, no key split (attn_wave_kernel)
    int wave_nw;      // waves per workgroup in that mode
    int wave_ds;      // workgroups that share the output columns of a query tile in that mode (1, 2 or 4)
    int wave_qt;      // query tiles per workgroup in that mode (1 or 2)
    size_t state_floats, off_part, total;
};

int make_plan(const dream_attn_desc *d, int n_q, int64_t max_kv_len, Plan *p)
{
    const int G = d->n_q_heads / d->n_kv_heads;
    p->wave_qt = 1;
    p->tiles_per_head = ceil_div(n_q, 16);
    const int n_qtiles = G * p->tiles_per_head;
    const int qg_max = d->head_dim == 256 ? 2 : 4;   // accumulator registers bound the query tiles per wave
    const int64_t base = (int64_t)d->batch * d->n_kv_heads;
    const int tiles = ceil_div(max_kv_len, 32);
    // throughput regime: as many query tiles per wave as registers allow, so that a K/V byte read from
    // LDS serves the most rows.  Latency regime (too few streams to fill the chip): one tile per wave keeps
    // the per-workgroup state small; the query groups of a KV head then re-read its K/V through L2.
    int qg = q_tiles_override();
    if (qg <= 0) {
        qg = n_qtiles <= 4 ? 1 : n_qtiles <= 8 ? 2 : 4;
        if (qg > qg_max)
            qg = qg_max;
        if (base * ceil_div(n_qtiles, 4 * qg) < 256)
            qg = 1;
        // measured at 32 sequences of a 4-way grouped-query model: below about four workgroups per CU the
        // chip hides latency better with more, smaller workgroups than it gains from sharing LDS reads
        // (head_dim 256 is the exception: its tiles are twice the bytes to re-read)
        while (d->head_dim <= 128 && qg > 1 && base * ceil_div(n_qtiles, 4 * qg) < 1024)
            qg /= 2;
    }
    if (qg > qg_max)
        qg = qg_max;
    if (qg != 1 && qg != 2 && qg != 4)
        qg = 1;
    p->qg = qg;
    p->nw = 4;
    p->mw = 1;
    p->once = 0;
    p->kg = 1;
    p->n_qg = ceil_div(n_qtiles, 4 * qg);
    // few, short streams with at most 16 query tiles each: a workgroup per query tile fills at least half the chip
    // without splitting keys, which saves the merge launch (short: up to 64 key tiles at head_dim 128, twice that
    // at 64: the measured crossover against the key-split path, which comes a little later for grouped-query
    // shapes because their split states are larger)
    p->wave_mode = q_tiles_override() == 0 && kv_splits_override() == 0 && tile_waves_override() == 0 &&
                   d->dtype == DREAM_BF16 && n_qtiles <= 16 && G <= 4 && base * n_qtiles <= 512 && base * n_qtiles >= 32 &&
                   (base * n_qtiles <= 256 || d->head_dim <= 128) && (int64_t)tiles * d->head_dim <= (G > 1 ? 12288 : 8192) &&
                   d->s_max * d->head_dim < (1ll << 31);
    if (p->wave_mode) {
        p->qg = 1;
        p->n_qg = n_qtiles;
        // output columns split over 2 or 4 workgroups while that still leaves at most one workgroup per CU
        p->wave_ds = 1;
        while (p->wave_ds < 4 && base * n_qtiles * p->wave_ds * 2 <= 256 && d->head_dim / (p->wave_ds * 2) >= 32)
            p->wave_ds *= 2;
        // more pairs than CUs (up to twice as many; beyond that the shared-tile kernel measures faster): a
        // workgroup serves two query tiles from the one K/V stream
        p->wave_qt = base * n_qtiles > 256 ? 2 : 1;
        // 8 waves (two per SIMD) where the registers allow it and each wave still gets a few tiles
        p->wave_nw = (d->head_dim <= 128 && (tiles > 32 || p->wave_ds > 1)) ? 8 : 4;
        p->n_splits = 1;
        p->n_groups = (int)base;
        p->n_streams = (int)base;
        p->grid = ceil_div(p->n_streams, 8) * 8 * n_qtiles;
        p->kt = 1;
        p->pfd = 1;
        p->state_floats = 0;
        p->off_part = DREAM_WORKSPACE_MIN_BYTES;
        p->total = DREAM_WORKSPACE_MIN_BYTES;
        return 0;
    }
    // grouped-query shapes with enough streams to give every CU a workgroup without splitting keys: 8 waves share
    // one LDS tile, so the 8-16 query tiles of a KV head are served by ONE workgroup (K/V leave L2 once per head
    // instead of once per 4 query tiles) while the CU still holds 8 waves.  head_dim 64 tiles are too small to
    // spread over 512 threads; with more than 16 (8 at head_dim 256) query tiles a KV head takes several workgroups.
    {
        const int tw = tile_waves_override();
        const int qg8_max = d->head_dim == 256 ? 1 : 2;
        int qg8 = q_tiles_override() > 0 ? (q_tiles_override() > qg8_max ? qg8_max : q_tiles_override()) : (n_qtiles > 8 ? qg8_max : 1);
        const bool can8 = d->dtype == DREAM_BF16 && d->head_dim >= 128 && kv_splits_override() <= 1 && tw != 4;
        const bool want8 = n_qtiles > 4 && (tw == 8 || (q_tiles_override() == 0 && base >= 256));   // (up to 4 tiles: see the two key groups below)
        // (the 8-wave variants read K/V with the nontemporal hint, so a KV head must not need two of them)
        if (can8 && want8 && ceil_div(n_qtiles, 8 * qg8) == 1) {
            p->nw = 8;
            p->qg = qg = qg8;
            p->n_qg = 1;
            p->once = 1;
        }
    }
    int s = kv_splits_override();
    if (p->nw == 8)
        s = 1;
    if (s <= 0) {
        s = ceil_div(256, base * p->n_qg);   // one workgroup per CU before anything is split further
        if (s > 8)
            s = 8;                           // more splits cost more in the merge than they save
    }
    if (s > tiles)
        s = tiles;
    if (s < 1)
        s = 1;
    const int64_t groups = base * p->n_qg;
    if (groups * qg * p->nw > 0x7fffffff)
        s = 1;
    p->n_splits = s;
    p->n_groups = (int)groups;
    p->n_streams = (int)(base * s);
    p->grid = ceil_div(p->n_streams, 8) * 8 * p->n_qg;
    // short streams (latency regime): the whole share of a workgroup is one step, everything in flight at once;
    // long streams: one tile per step (two at head_dim 64, whose tiles are half the bytes), two steps in flight
    const int tps = ceil_div(tiles, s);
    if (qg == 1 && d->head_dim <= 128 && tps <= 4) {
        p->kt = tps < 2 ? 2 : tps;
        p->pfd = 1;
    } else {
        p->kt = (qg == 1 && d->head_dim == 64) ? 2 : 1;
        p->pfd = 2;
        // the widest variants keep one step in flight: with two their accumulators and staging registers no
        // longer fit the 512 registers of a wave (same speed, no spills)
        if ((qg == 4 && d->head_dim == 128) || (qg == 2 && d->head_dim == 256))
            p->pfd = 1;
    }
    if (p->nw == 8) {
        p->kt = 1;
        p->pfd = DREAM_W8_PFD;
    } else if (qg == 1 && p->pfd == 2 && p->n_qg == 1) {
        p->once = 1;
        // multi-head shapes that leave a CU with at most DREAM_KG2_MAX_WG 4-wave workgroups: 8 waves as two key groups
        const int tw = tile_waves_override();
        if (s == 1 && d->head_dim <= 128 && tw != 4 && (tw == 8 || groups <= 256 * DREAM_KG2_MAX_WG)) {
            p->nw = 8;
            p->kg = 2;
        }
    }
    p->state_floats = (size_t)qg * (d->head_dim / 16) * 256 + (size_t)qg * 2 * 64;
    p->off_part = DREAM_WORKSPACE_MIN_BYTES;
    p->total = p->off_part + (s > 1 ? (size_t)groups * s * 4 * p->state_floats * sizeof(float) : 0);
    if (d->dtype == DREAM_F32)
        p->total = DREAM_WORKSPACE_MIN_BYTES;
    return 0;
}

// Trees above 64 nodes: the shared-tile kernel with four mask words, one query tile per wave, the key range unsplit
// (no split states, so the workspace need never exceeds what the query for any other shape returns), streamed.
void make_wide_plan(const dream_attn_desc *d, int n_q, Plan *p)
{
    const int G = d->n_q_heads / d->n_kv_heads;
    const int64_t base = (int64_t)d->batch * d->n_kv_heads;
    p->tiles_per_head = ceil_div(n_q, 16);
    p->wave_mode = false;
    p->wave_nw = p->wave_ds = p->wave_qt = 0;
    p->qg = 1;
    p->nw = 4;
    p->mw = 4;
    p->once = 0;
    p->kg = 1;
    p->n_qg = ceil_div(G * p->tiles_per_head, 4);
    p->n_splits = 1;
    p->n_groups = (int)(base * p->n_qg);
    p->n_streams = (int)base;
    p->grid = ceil_div(p->n_streams, 8) * 8 * p->n_qg;
    p->kt = d->head_dim == 64 ? 2 : 1;
    p->pfd = 2;
    p->state_floats = 0;
    p->off_part = DREAM_WORKSPACE_MIN_BYTES;
    p->total = DREAM_WORKSPACE_MIN_BYTES;
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

// The dynamic-LDS limit of a kernel is raised once (dream_init does it for every variant up front; a variant
// that is reached first by a call does it then).  Two threads may both set it once: harmless.
template <int D, int QG, int KT, int PFD, int NW = 4, int MW = 1, bool ONCE = false, int KG = 1>
int ensure_bf16_lds()
{
    using G = Geom<D, QG, KT * KG>;
    static std::atomic<bool> attr_set{false};
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_bf16_kernel<D, QG, KT, PFD, NW, MW, ONCE, KG>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)G::LDS_BYTES) != hipSuccess)
            return fail(DREAM_ERR_HIP, "attention: cannot reserve %zu bytes of LDS", G::LDS_BYTES);
        attr_set = true;
    }
    return DREAM_OK;
}

template <int D, int QG, int KT, int PFD, int NW = 4, int MW = 1, bool ONCE = false, int KG = 1>
int launch_bf16(const AttnArgs &a, const Plan &p, hipStream_t st)
{
    using G = Geom<D, QG, KT * KG>;
    if (int rc = ensure_bf16_lds<D, QG, KT, PFD, NW, MW, ONCE, KG>())
        return rc;
    if (ONCE && a.n_qg != 1)
        return fail(DREAM_ERR_INVALID_ARG, "attention: the read-once kernel variant needs one query group per KV head, not %d", a.n_qg);
    if (NW != 4 && p.n_splits != 1)
        return fail(DREAM_ERR_INVALID_ARG, "attention: the 8-wave shared-tile kernel does not split the key range");
    if (a.mask_words > MW)
        return fail(DREAM_ERR_INVALID_ARG, "attention: a tree of %d nodes needs %d mask words, this kernel has %d", a.n_tree, a.mask_words, MW);
    hipLaunchKernelGGL((attn_bf16_kernel<D, QG, KT, PFD, NW, MW, ONCE, KG>), dim3(p.grid), dim3(64 * NW), G::LDS_BYTES, st, a);
    int rc = check_launch("attn_bf16_kernel");
    if (rc || p.n_splits == 1)
        return rc;
    hipLaunchKernelGGL((attn_merge_kernel<D, QG>), dim3(p.n_groups * 4 * QG), dim3(256), 0, st, a);
    return check_launch("attn_merge_kernel");
}

template <int D, int NW, int DS, int QT>
struct WaveLds {
    using G = Geom<D, 1, 1, D / DS>;
    static constexpr size_t tile_bytes = (size_t)NW * G::TILE_ELEMS * 2, merge_bytes = (size_t)NW * StateGeom<D / DS, QT>::STATE_FLOATS * 4;
    static constexpr size_t bytes = (tile_bytes > merge_bytes ? tile_bytes : merge_bytes) + DREAM_MAX_TREE * sizeof(int32_t);
    static_assert(merge_bytes <= tile_bytes, "the wave merge buffers reuse the tile area");
};

template <int D, int NW, int DS, int QT = 1>
int ensure_wave_lds()
{
    static std::atomic<bool> attr_set{false};
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_wave_kernel<D, NW, DS, QT>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)WaveLds<D, NW, DS, QT>::bytes) != hipSuccess)
            return fail(DREAM_ERR_HIP, "attention: cannot reserve %zu bytes of LDS", WaveLds<D, NW, DS, QT>::bytes);
        attr_set = true;
    }
    return DREAM_OK;
}

template <int D, int NW, int DS, int QT = 1>
int launch_wave(const AttnArgs &a, const Plan &p, hipStream_t st)
{
    constexpr size_t lds_bytes = WaveLds<D, NW, DS, QT>::bytes;
    if (int rc = ensure_wave_lds<D, NW, DS, QT>())
        return rc;
    if (a.n_qg > 16 || a.group > 4)
        return fail(DREAM_ERR_INVALID_ARG, "attention: the wave kernel serves at most 16 query tiles and 4 query heads per KV head");
    const dim3 grid(8 * ceil_div(a.n_qg, QT) * DS, ceil_div(a.n_kv_heads, 8), p.n_streams / a.n_kv_heads);
    hipLaunchKernelGGL((attn_wave_kernel<D, NW, DS, QT>), grid, dim3(64 * NW), lds_bytes, st, a);
    return check_launch("attn_wave_kernel");
}

// Every bf16 kernel variant the launch plan can choose, in one table: the plan names a variant by
// (kernel family, head_dim, three template arguments); the table gives its launcher and the routine that raises
// its dynamic-LDS limit.  The launch, dream_init, dream_attn_plan_describe and dream_attn_variants all read it.
enum { FAMILY_TILE = 0, FAMILY_WAVE = 1 };
struct Variant {
    int family, d, p1, p2, p3, p4, p5, p6, p7;   // tile: (QG, KT, PFD, waves, mask words, read-once, key groups); wave: (NW, DS, QT, 0, 1, 0, 1)
    int (*launch)(const AttnArgs &, const Plan &, hipStream_t);
    int (*ensure)();
};
#define TILE_VARIANT(D, QG, KT, PFD) {FAMILY_TILE, D, QG, KT, PFD, 4, 1, 0, 1, &launch_bf16<D, QG, KT, PFD>, &ensure_bf16_lds<D, QG, KT, PFD>}
#define ONCE_VARIANT(D, QG, KT, PFD) {FAMILY_TILE, D, QG, KT, PFD, 4, 1, 1, 1, &launch_bf16<D, QG, KT, PFD, 4, 1, true>, &ensure_bf16_lds<D, QG, KT, PFD, 4, 1, true>}
#define KG2_VARIANT(D, QG, KT, PFD) {FAMILY_TILE, D, QG, KT, PFD, 8, 1, 1, 2, &launch_bf16<D, QG, KT, PFD, 8, 1, true, 2>, &ensure_bf16_lds<D, QG, KT, PFD, 8, 1, true, 2>}
#define WIDE_VARIANT(D, QG, KT, PFD) {FAMILY_TILE, D, QG, KT, PFD, 4, 4, 0, 1, &launch_bf16<D, QG, KT, PFD, 4, 4>, &ensure_bf16_lds<D, QG, KT, PFD, 4, 4>}
#define TILE8_VARIANT(D, QG, KT, PFD) {FAMILY_TILE, D, QG, KT, PFD, 8, 1, 1, 1, &launch_bf16<D, QG, KT, PFD, 8, 1, true>, &ensure_bf16_lds<D, QG, KT, PFD, 8, 1, true>}
#define WAVE_VARIANT(D, NW, DS, QT) {FAMILY_WAVE, D, NW, DS, QT, 0, 1, 0, 1, &launch_wave<D, NW, DS, QT>, &ensure_wave_lds<D, NW, DS, QT>}
const Variant VARIANTS[] = {
    // shared-tile kernel, one query tile per wave: a short key range in one step (2-4 tiles), or streamed
    TILE_VARIANT(64, 1, 2, 1), TILE_VARIANT(64, 1, 3, 1), TILE_VARIANT(64, 1, 4, 1), TILE_VARIANT(64, 1, 2, 2),
    TILE_VARIANT(128, 1, 2, 1), TILE_VARIANT(128, 1, 3, 1), TILE_VARIANT(128, 1, 4, 1), TILE_VARIANT(128, 1, 1, 2),
    TILE_VARIANT(256, 1, 1, 2),
    // several query tiles per wave
    TILE_VARIANT(64, 2, 1, 2), TILE_VARIANT(64, 4, 1, 2), TILE_VARIANT(128, 2, 1, 2), TILE_VARIANT(128, 4, 1, 1), TILE_VARIANT(256, 2, 1, 1),
    // streamed, the workgroup the only reader of its K/V rows (one query group per KV head): name arguments ...,4,1,1
    ONCE_VARIANT(64, 1, 2, 2), ONCE_VARIANT(128, 1, 1, 2), ONCE_VARIANT(256, 1, 1, 2),
    // the same with 8 waves as two key groups (few streams per CU): name arguments ...,8,1,1,2
    KG2_VARIANT(64, 1, 2, 2), KG2_VARIANT(128, 1, 1, 2),
    // 8 waves per workgroup (unsplit key range, grouped queries, always the only reader): a fifth name argument 8
    TILE8_VARIANT(128, 1, 1, DREAM_W8_PFD), TILE8_VARIANT(128, 2, 1, DREAM_W8_PFD), TILE8_VARIANT(256, 1, 1, DREAM_W8_PFD),
    // trees of 65-256 nodes (four mask words): a sixth name argument 4
    WIDE_VARIANT(64, 1, 2, 2), WIDE_VARIANT(128, 1, 1, 2), WIDE_VARIANT(256, 1, 1, 2),
    // single-launch wave kernel: (waves, column slices, query tiles per workgroup); split output columns always come
    // with 8 waves at head_dim <= 128
    WAVE_VARIANT(64, 8, 1, 1), WAVE_VARIANT(64, 8, 2, 1), WAVE_VARIANT(64, 4, 1, 1),
    WAVE_VARIANT(64, 8, 1, 2), WAVE_VARIANT(64, 4, 1, 2),
    WAVE_VARIANT(128, 8, 1, 1), WAVE_VARIANT(128, 8, 2, 1), WAVE_VARIANT(128, 8, 4, 1), WAVE_VARIANT(128, 4, 1, 1),
    WAVE_VARIANT(128, 8, 1, 2), WAVE_VARIANT(128, 4, 1, 2),
    WAVE_VARIANT(256, 4, 1, 1), WAVE_VARIANT(256, 4, 2, 1), WAVE_VARIANT(256, 4, 4, 1),
};
#undef TILE_VARIANT
#undef TILE8_VARIANT
#undef ONCE_VARIANT
#undef KG2_VARIANT
#undef WIDE_VARIANT
#undef WAVE_VARIANT
constexpr int N_VARIANTS = sizeof(VARIANTS) / sizeof(VARIANTS[0]);

// the variant a plan asks for, or nullptr
const Variant *find_variant(const dream_attn_desc *d, const Plan &p)
{
    const int family = p.wave_mode ? FAMILY_WAVE : FAMILY_TILE;
    const int p1 = p.wave_mode ? p.wave_nw : p.qg, p2 = p.wave_mode ? p.wave_ds : p.kt, p3 = p.wave_mode ? p.wave_qt : p.pfd;
    const int p4 = p.wave_mode ? 0 : p.nw, p5 = p.wave_mode ? 1 : p.mw, p6 = p.wave_mode ? 0 : p.once, p7 = p.wave_mode ? 1 : p.kg;
    for (int i = 0; i < N_VARIANTS; i++) {
        const Variant &v = VARIANTS[i];
        if (v.family == family && v.d == d->head_dim && v.p1 == p1 && v.p2 == p2 && v.p3 == p3 && v.p4 == p4 && v.p5 == p5 && v.p6 == p6 && v.p7 == p7)
            return &v;
    }
    return nullptr;
}

void variant_name(const Variant &v, char *buf, size_t n)
{
    if (v.family == FAMILY_WAVE)
        snprintf(buf, n, "attn_wave_kernel<%d,%d,%d,%d>", v.d, v.p1, v.p2, v.p3);
    else if (v.p7 != 1)
        snprintf(buf, n, "attn_bf16_kernel<%d,%d,%d,%d,%d,%d,%d,%d>", v.d, v.p1, v.p2, v.p3, v.p4, v.p5, v.p6, v.p7);
    else if (v.p6 && v.p4 == 4)
        snprintf(buf, n, "attn_bf16_kernel<%d,%d,%d,%d,%d,%d,%d>", v.d, v.p1, v.p2, v.p3, v.p4, v.p5, v.p6);
    else if (v.p5 != 1)
        snprintf(buf, n, "attn_bf16_kernel<%d,%d,%d,%d,%d,%d>", v.d, v.p1, v.p2, v.p3, v.p4, v.p5);
    else if (v.p4 != 4)
        snprintf(buf, n, "attn_bf16_kernel<%d,%d,%d,%d,%d>", v.d, v.p1, v.p2, v.p3, v.p4);
    else
        snprintf(buf, n, "attn_bf16_kernel<%d,%d,%d,%d>", v.d, v.p1, v.p2, v.p3);
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
    if (n_tree > 64 && d->dtype == DREAM_BF16)
        make_wide_plan(d, n_q, &p);
    if (!ws || ws_bytes < p.total)
        return fail(DREAM_ERR_WORKSPACE, "%s: workspace of %zu bytes, %zu needed", who, ws_bytes, p.total);

    AttnArgs a;
    a.q = q; a.k = k; a.v = v;
    a.prefix_len = prefix_len; a.parent = parent; a.q_node = q_node; a.tree_mask = tree_mask;
    a.out = out; a.lse = lse;
    a.part = reinterpret_cast<float *>(static_cast<char *>(ws) + p.off_part);
    a.n_q_heads = d->n_q_heads; a.n_kv_heads = d->n_kv_heads; a.group = d->n_q_heads / d->n_kv_heads;
    a.n_q = n_q; a.n_tree = n_tree; a.include_self = include_self;
    a.mask_words = ceil_div(n_tree, 64);
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

    const Variant *variant = find_variant(d, p);
    if (!variant)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: no kernel variant for head_dim %d with launch parameters (%d, %d, %d)", who, d->head_dim,
                    p.wave_mode ? p.wave_nw : p.qg, p.wave_mode ? p.wave_ds : p.kt, p.wave_mode ? p.wave_qt : p.pfd);
    return variant->launch(a, p, st);
}

size_t workspace_for(const dream_attn_desc *d, int n_q, int64_t max_kv_len)
{
    if (!d || d->n_kv_heads < 1 || d->n_q_heads < 1 || d->n_q_heads % d->n_kv_heads || n_q < 1 || max_kv_len < 1 ||
        d->batch < 1)
        return DREAM_WORKSPACE_MIN_BYTES;
    Plan p;
    make_plan(d, n_q, max_kv_len, &p);
    return p.total;
}

}  // namespace

namespace dream {
// every attention kernel variant the launch plan can choose (part of dream_init)
int attn_init()
{
    for (int i = 0; i < N_VARIANTS; i++)
        if (int rc = VARIANTS[i].ensure())
            return rc;
    return DREAM_OK;
}
}  // namespace dream

extern "C" {

int dream_attn_plan_describe(const dream_attn_desc *desc, int32_t n_q, int64_t max_kv_len, char *buf, size_t buf_bytes)
{
    const char *who = "dream_attn_plan_describe";
    if (!buf || buf_bytes == 0)
        return fail(DREAM_ERR_INVALID_ARG, "%s: no buffer", who);
    int rc = validate_desc(desc, who);
    if (rc)
        return rc;
    if (n_q < 1 || max_kv_len < 1 || max_kv_len > desc->s_max)
        return fail(DREAM_ERR_INVALID_ARG, "%s: need n_q >= 1 and 1 <= max_kv_len <= s_max", who);
    Plan p;
    make_plan(desc, n_q, max_kv_len, &p);
    if (n_q > 64 && desc->dtype == DREAM_BF16)   // more than 64 query rows: taken as a verification call over a tree of n_q nodes
        make_wide_plan(desc, n_q, &p);
    if (desc->dtype == DREAM_F32) {
        snprintf(buf, buf_bytes, "attn_f32_kernel workgroups=%lld", (long long)desc->batch * desc->n_q_heads * n_q);
        return DREAM_OK;
    }
    const Variant *v = find_variant(desc, p);
    if (!v)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: the plan names a kernel variant that is not built", who);
    char name[64];
    variant_name(*v, name, sizeof name);
    if (p.wave_mode)
        snprintf(buf, buf_bytes, "%s workgroups=%d splits=1 merge_launch=0", name,
                 ceil_div(p.n_qg, p.wave_qt) * p.wave_ds * desc->n_kv_heads * desc->batch);
    else
        snprintf(buf, buf_bytes, "%s workgroups=%d splits=%d merge_launch=%d", name, p.n_groups * p.n_splits, p.n_splits,
                 p.n_splits > 1 ? 1 : 0);
    return DREAM_OK;
}

int dream_attn_variants(char *buf, size_t buf_bytes)
{
    if (!buf || buf_bytes == 0)
        return fail(DREAM_ERR_INVALID_ARG, "dream_attn_variants: no buffer");
    size_t used = 0;
    buf[0] = 0;
    for (int i = 0; i < N_VARIANTS; i++) {
        char name[64];
        variant_name(VARIANTS[i], name, sizeof name);
        const int n = snprintf(buf + used, buf_bytes - used, "%s%s", i ? ";" : "", name);
        if (n < 0 || (size_t)n >= buf_bytes - used)
            return fail(DREAM_ERR_INVALID_ARG, "dream_attn_variants: buffer of %zu bytes is too small", buf_bytes);
        used += (size_t)n;
    }
    return DREAM_OK;
}

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
