// dream_spec_accept: acceptance over the verified tree at a sampling temperature (Section 2.1: a drafted token
// d is accepted with probability min(1, P_target(d) / P_draft(d)); after a rejection the rest is discarded and
// the target's distribution decides the next token; Section 4 evaluates at temperature 1).  For a tree the
// children of the current node are tried in node order; after a rejected child the target distribution becomes
// the positive part of (target - draft), the rejected token leaves the draft distribution, and the next child is
// tried against those; the first accepted child becomes the current node.  With no accepted child the next
// token is drawn from the current target distribution by inverting its cumulative sum in token order.  The
// uniform random numbers are inputs.
//
// One workgroup of 1024 threads walks one sequence (the walk is a dependent chain of at most depth+1 nodes).
// The target and draft distributions of the current node live unnormalised in the workspace (P, Q and a spare
// R, V floats each, L2-resident) with their normalisers as scalars, so
//   a node visit     = two passes over the two logit rows (maxima; exponentials and their sums),
//   a rejection      = one pass (R = max(P/Zp - Q/Zq, 0) and its sum; then P and R swap; Q[x] = 0, Zq -= Q[x]),
//   the final draw   = one pass of per-thread contiguous partial sums, a block scan, one thread's rescan.
// Every reduction has a fixed order, so the result is reproducible.  Roofline: HBM/L2 scans of V logits per
// visited node; latency bound at one sequence.
#include "common.h"

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

template <bool BF16>
__global__ __launch_bounds__(NT) void spec_accept_kernel(const void *tlogits, const void *dlogits, int n_tree, int vocab,
                                                         const int32_t *token, const int32_t *parent, const float *u_accept,
                                                         const float *u_bonus, int max_depth, float inv_temp, float *work,
                                                         int32_t *accept_len, int32_t *accept_path, int32_t *bonus_token)
{
    __shared__ int32_t s_par[DREAM_MAX_TREE_ACCEPT];
    __shared__ int32_t s_tok[DREAM_MAX_TREE_ACCEPT];
    __shared__ float s_redf[16];
    __shared__ int s_redi[16];
    __shared__ float s_scan[16];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < n_tree; i += NT) {
        s_par[i] = parent[(int64_t)b * n_tree + i];
        s_tok[i] = token[(int64_t)b * n_tree + i];
    }
    float *P = work + (int64_t)b * 3 * vocab, *Q = P + vocab, *R = Q + vocab;
    int32_t *path = accept_path + (int64_t)b * (max_depth + 1);
    if (tid <= max_depth)
        path[tid] = tid == 0 ? 0 : -1;
    __syncthreads();

    int cur = 0, depth = 0;
    for (;;) {
        // first child of the current node (children have larger indices than their parent), if depth allows
        int first = 0x7fffffff;
        if (depth < max_depth)
            for (int i = tid; i < n_tree; i += NT)
                if (i > cur && s_par[i] == cur)
                    first = min(first, i);
        first = block_min_int(first, s_redi, tid);
        const bool has_kids = first != 0x7fffffff;
        const int64_t row = ((int64_t)b * n_tree + cur) * vocab;

        // ---- node visit: unnormalised target (and draft) distributions of the current node
        float mt = -INFINITY, md = -INFINITY;
        for (int t = tid; t < vocab; t += NT) {
            mt = fmaxf(mt, load_logit<BF16>(tlogits, row + t) * inv_temp);
            if (has_kids)
                md = fmaxf(md, load_logit<BF16>(dlogits, row + t) * inv_temp);
        }
        mt = block_max(mt, s_redf, tid);
        if (has_kids)
            md = block_max(md, s_redf, tid);
        float zp = 0.0f, zq = 0.0f;
        for (int t = tid; t < vocab; t += NT) {
            const float e = __expf(load_logit<BF16>(tlogits, row + t) * inv_temp - mt);
            P[t] = e;
            zp += e;
            if (has_kids) {
                const float f = __expf(load_logit<BF16>(dlogits, row + t) * inv_temp - md);
                Q[t] = f;
                zq += f;
            }
        }
        float Zp = block_sum(zp, s_redf, tid);
        float Zq = has_kids ? block_sum(zq, s_redf, tid) : 0.0f;
        __syncthreads();   // P and Q are complete and visible to the whole workgroup

        // ---- try the children in node order
        int accepted = -1;
        int child = first;
        while (has_kids && child != 0x7fffffff) {
            const int x = min(max(s_tok[child], 0), vocab - 1);   // device metadata is trusted but kept inside the row
            const float px = P[x], qx = Q[x];
            const float ratio = qx > 0.0f ? (px / Zp) / (qx / Zq) : (px > 0.0f ? INFINITY : 0.0f);
            if (u_accept[(int64_t)b * n_tree + child] < fminf(1.0f, ratio)) {
                accepted = child;
                break;
            }
            // rejected: residual target into the spare array, then swap; the token leaves the draft distribution
            const float ip = 1.0f / Zp, iq = Zq > 0.0f ? 1.0f / Zq : 0.0f;
            float s = 0.0f;
            for (int t = tid; t < vocab; t += NT) {
                const float r = fmaxf(P[t] * ip - Q[t] * iq, 0.0f);
                R[t] = r;
                s += r;
            }
            s = block_sum(s, s_redf, tid);
            if (s > 0.0f) {   // (a zero residual means target == draft, which the test above never rejects)
                float *tmp = P;
                P = R;
                R = tmp;
                Zp = s;
            }
            __syncthreads();   // everybody has read Q[x] before it is cleared
            if (tid == 0)
                Q[x] = 0.0f;
            Zq = fmaxf(Zq - qx, 0.0f);
            // next child of the current node
            int next = 0x7fffffff;
            for (int i = tid; i < n_tree; i += NT)
                if (i > child && s_par[i] == cur)
                    next = min(next, i);
            child = block_min_int(next, s_redi, tid);   // (its barriers also publish Q[x] = 0 and the new P)
        }
        if (accepted >= 0) {
            cur = accepted;
            depth++;
            if (tid == 0)
                path[depth] = cur;
            continue;
        }

        // ---- no child accepted: draw the next token from P by inverting the cumulative sum in token order
        const int cpt = (vocab + NT - 1) / NT;          // contiguous tokens per thread
        const int t0 = min(tid * cpt, vocab), t1 = min(t0 + cpt, vocab);
        float local = 0.0f;
        for (int t = t0; t < t1; t++)
            local += P[t];
        // inclusive scan of the per-thread sums: inside a wave by shuffles, wave totals through LDS
        float inc = local;
        for (int off = 1; off < 64; off <<= 1) {
            const float o = __shfl_up(inc, off);
            if (lane >= off)
                inc += o;
        }
        __syncthreads();
        if (lane == 63)
            s_scan[wave] = inc;
        __syncthreads();
        float base = 0.0f, total = 0.0f;
#pragma unroll
        for (int w = 0; w < 16; w++) {
            if (w < wave)
                base += s_scan[w];
            total += s_scan[w];
        }
        const float before = base + inc - local;        // sum of all tokens below t0
        const float target = u_bonus[b] * total;
        // the first thread whose inclusive sum exceeds the target holds the token
        int owner = (before + local > target && t1 > t0) ? tid : 0x7fffffff;
        owner = block_min_int(owner, s_redi, tid);
        if (owner == 0x7fffffff) {
            // rounding left the target at or above the total: the last token with mass
            int last = -1;
            for (int t = t0; t < t1; t++)
                if (P[t] > 0.0f)
                    last = t;
            last = -block_min_int(-last, s_redi, tid);
            if (tid == 0)
                bonus_token[b] = max(last, 0);
        } else if (tid == owner) {
            float run = before;
            int pick = t1 - 1;
            for (int t = t0; t < t1; t++) {
                run += P[t];
                if (run > target) {
                    pick = t;
                    break;
                }
            }
            bonus_token[b] = pick;
        }
        if (tid == 0)
            accept_len[b] = depth;
        return;
    }
}

}  // namespace

extern "C" {

size_t dream_spec_accept_workspace(int32_t batch, int32_t vocab)
{
    if (batch < 1 || vocab < 1)
        return DREAM_WORKSPACE_HEADER_BYTES;
    return DREAM_WORKSPACE_HEADER_BYTES + align_up((size_t)batch * 3 * vocab * sizeof(float), 256);
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
    if (!(temperature > 0.0f))
        return fail(DREAM_ERR_INVALID_ARG, "%s: temperature must be positive (use dream_accept_path for the greedy rule)", who);
    const size_t need = dream_spec_accept_workspace(batch, vocab);
    if (!workspace || workspace_bytes < need)
        return fail(DREAM_ERR_WORKSPACE, "%s: workspace of %zu bytes, %zu needed", who, workspace_bytes, need);
    float *work = reinterpret_cast<float *>(static_cast<char *>(workspace) + DREAM_WORKSPACE_HEADER_BYTES);
    if (logits_dtype == DREAM_BF16)
        hipLaunchKernelGGL(spec_accept_kernel<true>, dim3(batch), dim3(NT), 0, as_stream(stream), target_logits, draft_logits, n_tree, vocab,
                           token, parent, u_accept, u_bonus, max_depth, 1.0f / temperature, work, accept_len, accept_path, bonus_token);
    else
        hipLaunchKernelGGL(spec_accept_kernel<false>, dim3(batch), dim3(NT), 0, as_stream(stream), target_logits, draft_logits, n_tree, vocab,
                           token, parent, u_accept, u_bonus, max_depth, 1.0f / temperature, work, accept_len, accept_path, bonus_token);
    return check_launch("spec_accept_kernel");
}

}  // extern "C"
