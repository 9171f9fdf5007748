// Draft-tree construction (Section 3.1, last paragraph: width-k tree expansion with the top-k reordering of
// EAGLE-2; Section 4: k children per node, a depth, a maximum number of drafted tokens).
//
// dream_tree_expand_level  one level of the expansion: for every frontier node the log-softmax of its draft
//   logits, its k most probable tokens as candidate children with score = score(node) + log p(token | node),
//   and the k best candidates of the level as the next frontier.
//     expand_partial_kernel  one workgroup per 8192-logit chunk of a row: the chunk is read once (16-byte
//       loads) into registers; block reductions give the chunk's maximum and sum of exponentials, then k rounds
//       of a block-wide arg-max pick the chunk's k largest logits.  The order is (logit descending, token
//       ascending) and compares the logits themselves, so the chosen tokens are exact whatever the chunking.
//     expand_merge_kernel    one workgroup per sequence, one wave per frontier row: merges the chunk partials
//       (log-sum-exp; k rounds of a wave arg-max over the chunk candidates), writes tokens and scores, then
//       ranks the F*k candidates by counting (score descending, index ascending) for the next frontier.
// dream_tree_finalize  the root and the `budget` best candidates of all levels, in creation order, parents
//   re-indexed: rank by counting in LDS, block scan for the new indices.
// Roofline: the expansion is an HBM scan of B*F*V logits (launch-latency bound at one sequence); the rest is
// latency bound by construction (a few hundred candidates).
#include "common.h"

using namespace dream;

namespace {

constexpr int CHUNK = 8192;          // logits per workgroup of the partial kernel
constexpr int PER_THREAD = CHUNK / 256;
constexpr int MAX_K = 16;            // DREAM_MAX_TREE_WIDTH
constexpr int MAX_F = 16;            // frontier rows per sequence (one wave each in the merge kernel)

// (value, index) pairs are ranked as one 64-bit key: the float mapped to an unsigned integer with the same
// order in the high word, the complemented index in the low word, so a larger key is a larger value or, among
// equal values, a lower index.  One integer compare per candidate instead of a float/integer cascade.
__device__ __forceinline__ uint32_t order_bits(float x)
{
    x += 0.0f;   // -0 and +0 are equal values: give them one key
    const uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float value_of(uint32_t k) { return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k); }
__device__ __forceinline__ uint64_t make_key(float v, int i) { return ((uint64_t)order_bits(v) << 32) | (uint32_t)(0xffffffffu - (uint32_t)i); }
__device__ __forceinline__ int index_of(uint64_t k) { return (int)(0xffffffffu - (uint32_t)k); }

// Maximum of a 64-bit key over the wave, returned in every lane.  Inside each row of 16 lanes the key is
// combined with its rotations by 8, 4, 2 and 1 lanes (DPP row_ror: a VALU move, no LDS round trip), which
// leaves the row maximum in all 16 lanes; the four row maxima are then read as scalars.
template <int ROT>
__device__ __forceinline__ uint64_t row_rotate(uint64_t k)
{
    constexpr int ctrl = 0x120 + ROT;   // DPP row_ror:ROT
    const uint32_t lo = __builtin_amdgcn_update_dpp(0u, (uint32_t)k, ctrl, 0xf, 0xf, false);
    const uint32_t hi = __builtin_amdgcn_update_dpp(0u, (uint32_t)(k >> 32), ctrl, 0xf, 0xf, false);
    return ((uint64_t)hi << 32) | lo;
}
template <int ROT>
__device__ __forceinline__ float row_rotate_f(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 + ROT, 0xf, 0xf, false));
}
__device__ __forceinline__ uint64_t lane_value(uint64_t k, int lane)
{
    return ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(k >> 32), lane) << 32) | (uint32_t)__builtin_amdgcn_readlane((int)k, lane);
}
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t k)
{
    uint64_t o = row_rotate<8>(k);
    k = o > k ? o : k;
    o = row_rotate<4>(k);
    k = o > k ? o : k;
    o = row_rotate<2>(k);
    k = o > k ? o : k;
    o = row_rotate<1>(k);
    k = o > k ? o : k;
    const uint64_t a = lane_value(k, 0), b = lane_value(k, 16), c = lane_value(k, 32), d = lane_value(k, 48);
    const uint64_t ab = a > b ? a : b, cd = c > d ? c : d;
    return ab > cd ? ab : cd;
}

template <bool BF16>
__global__ __launch_bounds__(256) void expand_partial_kernel(const void *logits, int vocab, int n_chunks, int k, float *part_m,
                                                             float *part_s, uint64_t *part_key)
{
    __shared__ float s_f[4];
    __shared__ uint64_t s_k[4];
    const int chunk = blockIdx.x;
    const int64_t row = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int begin = chunk * CHUNK;
    // element e of this thread is token begin + (e / 8) * 2048 + tid * 8 + e % 8: 16-byte loads when the row allows
    float x[PER_THREAD];
    if (BF16) {
        const uint16_t *p = reinterpret_cast<const uint16_t *>(logits) + row * vocab;
        const bool aligned = ((reinterpret_cast<uintptr_t>(p)) & 15) == 0;
#pragma unroll
        for (int j = 0; j < PER_THREAD / 8; j++) {
            const int t0 = begin + j * 2048 + tid * 8;
            if (aligned && t0 + 8 <= vocab) {
                const u32x4 u = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p + t0));   // logits: read once
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    x[j * 8 + 2 * q] = __uint_as_float(u[q] << 16);
                    x[j * 8 + 2 * q + 1] = __uint_as_float(u[q] & 0xffff0000u);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; e++)
                    x[j * 8 + e] = t0 + e < vocab ? bf16_bits_to_float(p[t0 + e]) : -INFINITY;
            }
        }
    } else {
        const float *p = reinterpret_cast<const float *>(logits) + row * vocab;
        const bool aligned = ((reinterpret_cast<uintptr_t>(p)) & 15) == 0;
#pragma unroll
        for (int j = 0; j < PER_THREAD / 8; j++) {
            const int t0 = begin + j * 2048 + tid * 8;
            if (aligned && t0 + 8 <= vocab) {
                const f32x4 u0 = *reinterpret_cast<const f32x4 *>(p + t0), u1 = *reinterpret_cast<const f32x4 *>(p + t0 + 4);
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    x[j * 8 + q] = u0[q];
                    x[j * 8 + 4 + q] = u1[q];
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; e++)
                    x[j * 8 + e] = t0 + e < vocab ? p[t0 + e] : -INFINITY;
            }
        }
    }

    // chunk maximum and sum of exponentials relative to it
    float m = -INFINITY;
#pragma unroll
    for (int e = 0; e < PER_THREAD; e++)
        m = fmaxf(m, x[e]);
    const float tmax = m;   // this thread's maximum (padding is -inf)
    for (int off = 32; off > 0; off >>= 1)
        m = fmaxf(m, __shfl_xor(m, off));
    if (lane == 0)
        s_f[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(s_f[0], s_f[1]), fmaxf(s_f[2], s_f[3]));
    __syncthreads();
    float s = 0.0f;
#pragma unroll
    for (int e = 0; e < PER_THREAD; e++)
        s += x[e] == -INFINITY ? 0.0f : __expf(x[e] - m);
    for (int off = 32; off > 0; off >>= 1)
        s += __shfl_xor(s, off);
    if (lane == 0)
        s_f[wave] = s;
    __syncthreads();
    if (tid == 0) {
        part_m[row * n_chunks + chunk] = m;
        part_s[row * n_chunks + chunk] = (s_f[0] + s_f[1]) + (s_f[2] + s_f[3]);
    }

    // ---- the chunk's k largest.  A lower bound of the k-th largest value first: the 256 thread maxima fall into
    // 16 rows of 16 lanes, and the k-th largest of the 16 row maxima has at least k elements at or above it.
    // Elements at or above that bound (a few dozen for ordinary logits) are collected in LDS and ranked by
    // counting; more than 256 of them (heavy ties) fall back to k rounds of a block-wide arg-max.
    __shared__ float s_row[16];
    __shared__ float s_tau;
    __shared__ int s_count;
    __shared__ uint64_t s_cand[256];
    float rm = tmax;
    rm = fmaxf(rm, row_rotate_f<8>(rm));
    rm = fmaxf(rm, row_rotate_f<4>(rm));
    rm = fmaxf(rm, row_rotate_f<2>(rm));
    rm = fmaxf(rm, row_rotate_f<1>(rm));
    if ((lane & 15) == 0)
        s_row[tid >> 4] = rm;
    if (tid == 0)
        s_count = 0;
    __syncthreads();
    if (tid < 16) {
        const float mine = s_row[tid];
        int rank = 0;
#pragma unroll
        for (int j = 0; j < 16; j++) {
            const float o = s_row[j];
            rank += (o > mine || (o == mine && j < tid)) ? 1 : 0;
        }
        if (rank == min(k, 16) - 1)
            s_tau = mine;
    }
    __syncthreads();
    const float tau = s_tau;
    int overflow = 0;
#pragma unroll
    for (int e = 0; e < PER_THREAD; e++) {
        const int t = begin + (e >> 3) * 2048 + tid * 8 + (e & 7);
        if (t < vocab && x[e] >= tau) {
            const int slot = atomicAdd(&s_count, 1);
            if (slot < 256)
                s_cand[slot] = make_key(x[e], t);
            else
                overflow = 1;
        }
    }
    __syncthreads();
    const int n_cand = s_count;
    uint64_t *out_key = part_key + (row * n_chunks + chunk) * k;
    if (n_cand <= 256) {
        if (tid < n_cand) {
            const uint64_t mine = s_cand[tid];
            int rank = 0;
#pragma unroll 8
            for (int j = 0; j < n_cand; j++)
                rank += s_cand[j] > mine ? 1 : 0;
            if (rank < k)
                out_key[rank] = mine;
        }
        if (tid >= n_cand && tid < k)
            out_key[tid] = 0ull;   // fewer than k tokens in the chunk
        return;
    }
    (void)overflow;
    // keys of this thread's elements (0 for tokens past the vocabulary: below every real key)
    uint64_t key[PER_THREAD];
#pragma unroll
    for (int e = 0; e < PER_THREAD; e++) {
        const int t = begin + (e >> 3) * 2048 + tid * 8 + (e & 7);
        key[e] = t < vocab ? make_key(x[e], t) : 0ull;
    }
    // k rounds: the largest key below the previous pick
    uint64_t prev = ~0ull;
    for (int r = 0; r < k; r++) {
        uint64_t best = 0ull;
#pragma unroll
        for (int e = 0; e < PER_THREAD; e++) {
            const uint64_t c = key[e] < prev ? key[e] : 0ull;
            best = c > best ? c : best;
        }
        best = wave_max_u64(best);
        if (lane == 0)
            s_k[wave] = best;
        __syncthreads();
        best = s_k[0];
#pragma unroll
        for (int w = 1; w < 4; w++)
            best = s_k[w] > best ? s_k[w] : best;
        __syncthreads();
        if (tid == 0)
            out_key[r] = best;   // 0 once the chunk is exhausted
        prev = best;
    }
}

// One workgroup of 16 waves per sequence; wave f merges the chunk partials of frontier row f.
__global__ __launch_bounds__(64 * MAX_F) void expand_merge_kernel(const float *part_m, const float *part_s, const uint64_t *part_key,
                                                                  int n_frontier, int n_chunks, int k, const float *cum_in,
                                                                  int32_t *cand_token, float *cand_score, int32_t *next_frontier)
{
    __shared__ uint64_t s_key[MAX_F * MAX_K];   // (score, flat index) keys of the level's candidates
    constexpr int MAX_PART = 8;                 // chunk candidates per lane: 64 * 8 = 32 chunks * 16
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
    const int f = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_cand = n_frontier * k;
    if (f < n_frontier) {
        const int64_t row = (int64_t)b * n_frontier + f;
        const int n_part = n_chunks * k;
        uint64_t pk[MAX_PART];
#pragma unroll
        for (int j = 0; j < MAX_PART; j++)
            pk[j] = lane + j * 64 < n_part ? part_key[row * n_part + lane + j * 64] : 0ull;
        // log-sum-exp of the row from the chunk partials
        float M = -INFINITY;
        for (int ch = lane; ch < n_chunks; ch += 64)
            M = fmaxf(M, part_m[row * n_chunks + ch]);
        for (int off = 32; off > 0; off >>= 1)
            M = fmaxf(M, __shfl_xor(M, off));
        float S = 0.0f;
        for (int ch = lane; ch < n_chunks; ch += 64) {
            const float mc = part_m[row * n_chunks + ch];
            S += mc == -INFINITY ? 0.0f : part_s[row * n_chunks + ch] * __expf(mc - M);
        }
        for (int off = 32; off > 0; off >>= 1)
            S += __shfl_xor(S, off);
        const float lse = M + __logf(S);
        const float cum = cum_in[row];
        uint64_t prev = ~0ull;
        for (int r = 0; r < k; r++) {
            uint64_t best = 0ull;
#pragma unroll
            for (int j = 0; j < MAX_PART; j++) {
                const uint64_t c = pk[j] < prev ? pk[j] : 0ull;
                best = c > best ? c : best;
            }
            best = wave_max_u64(best);
            if (lane == 0) {
                const float sc = cum + (value_of((uint32_t)(best >> 32)) - lse);
                cand_token[row * k + r] = index_of(best);
                cand_score[row * k + r] = sc;
                s_key[f * k + r] = make_key(sc, f * k + r);
            }
            prev = best;
        }
    }
    __syncthreads();
    // next frontier: rank of every candidate = number of larger keys; 4 threads share a candidate
    const int kf = min(k, n_cand);
    const int cand = tid >> 2, part = tid & 3;
    int rank = 0;
    if (cand < n_cand) {
        const uint64_t mine = s_key[cand];
#pragma unroll 8
        for (int j = part; j < n_cand; j += 4)
            rank += s_key[j] > mine ? 1 : 0;
    }
    rank += __shfl_xor(rank, 1);
    rank += __shfl_xor(rank, 2);
    if (cand < n_cand && part == 0 && rank < kf)
        next_frontier[(int64_t)b * kf + rank] = cand;
}

// One workgroup of 1024 threads per sequence.  `share` threads (a power of two, adjacent lanes) count the
// rank of one pool entry together.
__global__ __launch_bounds__(1024) void tree_finalize_kernel(const float *pool_score, const int32_t *pool_parent, const int32_t *pool_token,
                                                             int n_pool, int keep_n, int share_log2, int32_t *tree_parent,
                                                             int32_t *tree_token, int32_t *tree_pool_index)
{
    __shared__ uint64_t s_key[DREAM_MAX_POOL];
    __shared__ int32_t s_new[DREAM_MAX_POOL];   // new index of a kept entry, -2 for a dropped one
    __shared__ uint8_t s_keep[DREAM_MAX_POOL];
    __shared__ int s_wave[16];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *sc = pool_score + (int64_t)b * n_pool;
    if (tid < n_pool)
        s_key[tid] = tid == 0 ? ~0ull : make_key(sc[tid], tid);   // the root outranks everything
    __syncthreads();
    {
        const int share = 1 << share_log2;
        const int e = tid >> share_log2, part = tid & (share - 1);
        int rank = 0;
        if (e < n_pool) {
            const uint64_t mine = s_key[e];
#pragma unroll 8
            for (int j = part; j < n_pool; j += share)
                rank += s_key[j] > mine ? 1 : 0;
        }
        for (int off = 1; off < share; off <<= 1)
            rank += __shfl_xor(rank, off);
        if (e < n_pool && part == 0)
            s_keep[e] = rank <= keep_n ? 1 : 0;   // rank counts the root too: root has rank 0
    }
    __syncthreads();
    const bool keep = tid < n_pool && s_keep[tid];
    // exclusive scan of the keep flags: ballot inside a wave, wave totals through LDS
    const uint64_t bal = __ballot(keep);
    const int within = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0)
        s_wave[wave] = __popcll(bal);
    __syncthreads();
    int base = 0;
    for (int w = 0; w < wave; w++)
        base += s_wave[w];
    const int my_new = base + within;
    if (tid < n_pool)
        s_new[tid] = keep ? my_new : -2;
    __syncthreads();
    if (keep) {
        const int T = 1 + keep_n;
        const int64_t o = (int64_t)b * T + my_new;
        const int pp = pool_parent[(int64_t)b * n_pool + tid];
        tree_parent[o] = tid == 0 ? -1 : ((pp >= 0 && pp < n_pool) ? s_new[pp] : -2);
        tree_token[o] = pool_token[(int64_t)b * n_pool + tid];
        tree_pool_index[o] = tid;
    }
}

struct ExpandPlan {
    int n_chunks;
    size_t off_m, off_s, off_key, total;
};

ExpandPlan expand_plan(int batch, int n_frontier, int vocab, int k)
{
    ExpandPlan p;
    p.n_chunks = ceil_div(vocab, CHUNK);
    const size_t rows = (size_t)batch * n_frontier;
    p.off_m = DREAM_WORKSPACE_MIN_BYTES;
    p.off_s = align_up(p.off_m + rows * p.n_chunks * sizeof(float), 256);
    p.off_key = align_up(p.off_s + rows * p.n_chunks * sizeof(float), 256);
    p.total = align_up(p.off_key + rows * p.n_chunks * k * sizeof(uint64_t), 256);
    return p;
}

}  // namespace

extern "C" {

size_t dream_tree_expand_workspace(int32_t batch, int32_t n_frontier, int32_t vocab, int32_t k)
{
    if (batch < 1 || n_frontier < 1 || vocab < 1 || k < 1)
        return DREAM_WORKSPACE_MIN_BYTES;
    return expand_plan(batch, n_frontier, vocab, k).total;
}

int dream_tree_expand_level(const void *logits, int32_t logits_dtype, int32_t batch, int32_t n_frontier, int32_t vocab,
                            const float *cum_in, int32_t k, int32_t *cand_token, float *cand_score, int32_t *next_frontier,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    const char *who = "dream_tree_expand_level";
    if (!logits || !cum_in || !cand_token || !cand_score || !next_frontier)
        return fail(DREAM_ERR_INVALID_ARG, "%s: NULL argument", who);
    if (logits_dtype != DREAM_F32 && logits_dtype != DREAM_BF16)
        return fail(DREAM_ERR_INVALID_ARG, "%s: unknown dtype %d", who, logits_dtype);
    if (batch < 1 || batch > 65535)
        return fail(DREAM_ERR_INVALID_ARG, "%s: batch %d outside [1, 65535]", who, batch);
    if (n_frontier < 1 || n_frontier > MAX_F)
        return fail(DREAM_ERR_INVALID_ARG, "%s: n_frontier %d outside [1, %d]", who, n_frontier, MAX_F);
    if (k < 1 || k > DREAM_MAX_TREE_WIDTH || k > vocab)
        return fail(DREAM_ERR_INVALID_ARG, "%s: k %d outside [1, min(%d, vocab)]", who, k, DREAM_MAX_TREE_WIDTH);
    if (ceil_div(vocab, CHUNK) * k > 64 * 8)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: vocab %d with k %d exceeds the 512 chunk candidates a wave merges", who, vocab, k);
    if (vocab < 1 || (int64_t)batch * n_frontier > 65535)
        return fail(DREAM_ERR_INVALID_ARG, "%s: vocab must be positive and batch * n_frontier at most 65535", who);
    ExpandPlan p = expand_plan(batch, n_frontier, vocab, k);
    if (!workspace || workspace_bytes < p.total)
        return fail(DREAM_ERR_WORKSPACE, "%s: workspace of %zu bytes, %zu needed", who, workspace_bytes, p.total);
    char *ws = static_cast<char *>(workspace);
    float *pm = reinterpret_cast<float *>(ws + p.off_m), *ps = reinterpret_cast<float *>(ws + p.off_s);
    uint64_t *pkey = reinterpret_cast<uint64_t *>(ws + p.off_key);
    hipStream_t st = as_stream(stream);
    const dim3 grid(p.n_chunks, batch * n_frontier);
    if (logits_dtype == DREAM_BF16)
        hipLaunchKernelGGL(expand_partial_kernel<true>, grid, dim3(256), 0, st, logits, vocab, p.n_chunks, k, pm, ps, pkey);
    else
        hipLaunchKernelGGL(expand_partial_kernel<false>, grid, dim3(256), 0, st, logits, vocab, p.n_chunks, k, pm, ps, pkey);
    int rc = check_launch("expand_partial_kernel");
    if (rc)
        return rc;
    hipLaunchKernelGGL(expand_merge_kernel, dim3(batch), dim3(64 * MAX_F), 0, st, pm, ps, pkey, n_frontier, p.n_chunks, k, cum_in,
                       cand_token, cand_score, next_frontier);
    return check_launch("expand_merge_kernel");
}

int dream_tree_finalize(const float *pool_score, const int32_t *pool_parent, const int32_t *pool_token, int32_t batch, int32_t n_pool,
                        int32_t budget, int32_t *tree_parent, int32_t *tree_token, int32_t *tree_pool_index, int32_t *n_tree_host,
                        void *stream)
{
    const char *who = "dream_tree_finalize";
    if (!pool_score || !pool_parent || !pool_token || !tree_parent || !tree_token || !tree_pool_index)
        return fail(DREAM_ERR_INVALID_ARG, "%s: NULL argument", who);
    if (batch < 1 || batch > 65535)
        return fail(DREAM_ERR_INVALID_ARG, "%s: batch %d outside [1, 65535]", who, batch);
    if (n_pool < 1 || n_pool > DREAM_MAX_POOL)
        return fail(DREAM_ERR_INVALID_ARG, "%s: n_pool %d outside [1, %d]", who, n_pool, DREAM_MAX_POOL);
    if (budget < 0)
        return fail(DREAM_ERR_INVALID_ARG, "%s: negative budget", who);
    const int keep_n = budget < n_pool - 1 ? budget : n_pool - 1;
    if (n_tree_host)
        *n_tree_host = 1 + keep_n;
    int share_log2 = 0;   // threads that count one entry's rank together: 1024 / next power of two >= n_pool
    while ((n_pool << (share_log2 + 1)) <= 1024 && share_log2 < 6)
        share_log2++;
    hipLaunchKernelGGL(tree_finalize_kernel, dim3(batch), dim3(1024), 0, as_stream(stream), pool_score, pool_parent, pool_token, n_pool,
                       keep_n, share_log2, tree_parent, tree_token, tree_pool_index);
    return check_launch("tree_finalize_kernel");
}

}  // extern "C"
