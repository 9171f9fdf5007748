// dream_kv_commit: after verification the K/V rows of the accepted root-to-node path become the next rows of
// the cached prefix and every other tree row is dropped (Section 2.1: everything after the first rejected
// token is discarded and decoding continues from the accepted prefix; Section 4: KV caching).
//
// One launch serves many caches of one shape (K and V of every layer, the draft's feature caches): the cache
// pointers travel in the launch arguments.  One workgroup per (group of KV heads, sequence, cache) moves the
// accepted rows of its heads in place: every 16-byte chunk is loaded into a register first, the workgroup meets
// at a barrier, then the chunks are stored, so a row that is both a source and a destination (path 0,2,3: row 2
// is written by the second entry and read by the first) is always read before it is overwritten.  A head's
// accepted rows are only a few hundred bytes to a few KB, so a workgroup takes as many heads as its 64 KB of
// registers hold while the grid still has about a thousand workgroups: with one head each, a launch over many
// sequences is tens of thousands of workgroups that each keep a fifth of their threads busy for one round trip.
// Roofline: HBM (read and write of rows x heads x caches); at one sequence the call is one launch latency.
#include "common.h"

using namespace dream;

namespace {

constexpr int MAX_CACHES_PER_LAUNCH = 128;
constexpr int CHUNKS_PER_THREAD = 16;   // 256 threads x 16 chunks x 16 bytes = 64 KB of rows per workgroup

struct CommitArgs {
    void *cache[MAX_CACHES_PER_LAUNCH];
    const int32_t *prefix_len, *path, *accept_len;
    int32_t *prefix_len_out;
    int32_t n_kv_heads, n_tree, path_stride, chunks_per_row, first_cache, heads_per_wg;
    int64_t s_max;
};

__global__ __launch_bounds__(256) void kv_commit_kernel(CommitArgs a)
{
    const int h0 = blockIdx.x * a.heads_per_wg, b = blockIdx.y, ci = blockIdx.z;
    const int n_heads = min(a.heads_per_wg, a.n_kv_heads - h0);
    const int tid = threadIdx.x;
    const int P = (int)min((int64_t)max(a.prefix_len[b], 0), a.s_max - a.n_tree);
    // device metadata is trusted, but stay inside the tree rows whatever it holds
    const int n = min(max(a.accept_len[b], 0), min(a.path_stride, a.n_tree) - 1);
    if (blockIdx.x == 0 && ci == 0 && a.first_cache == 0 && tid == 0 && a.prefix_len_out)
        a.prefix_len_out[b] = P + n + 1;
    const int cpr = a.chunks_per_row;
    const int per_head = (n + 1) * cpr;          // chunks of one head: destination rows 0..n of its tree area are contiguous
    const int total = n_heads * per_head;
    const int64_t head_stride = a.s_max * cpr;   // chunks between the same row of consecutive heads
    u32x4 *tree = reinterpret_cast<u32x4 *>(a.cache[ci]) + (((int64_t)b * a.n_kv_heads + h0) * a.s_max + P) * cpr;
    const int32_t *path = a.path + (int64_t)b * a.path_stride;
    u32x4 r[CHUNKS_PER_THREAD];
#pragma unroll
    for (int i = 0; i < CHUNKS_PER_THREAD; i++) {
        const int idx = tid + i * 256;
        if (idx < total) {
            const int hl = idx / per_head, rest = idx - hl * per_head;
            const int j = rest / cpr, c = rest - j * cpr;
            const int node = min(max(path[j], 0), a.n_tree - 1);
            r[i] = tree[hl * head_stride + (int64_t)node * cpr + c];
        }
    }
    __syncthreads();   // every source chunk of these heads is in a register
#pragma unroll
    for (int i = 0; i < CHUNKS_PER_THREAD; i++) {
        const int idx = tid + i * 256;
        if (idx < total) {
            const int hl = idx / per_head, rest = idx - hl * per_head;
            tree[hl * head_stride + rest] = r[i];
        }
    }
}

}  // namespace

extern "C" {

int dream_kv_commit(const dream_attn_desc *desc, void *const *caches_host, int32_t n_caches, const int32_t *prefix_len,
                    int32_t n_tree, const int32_t *accept_path, int32_t path_stride, const int32_t *accept_len,
                    int32_t *prefix_len_out, void *stream)
{
    const char *who = "dream_kv_commit";
    if (!desc || !caches_host || !prefix_len || !accept_path || !accept_len)
        return fail(DREAM_ERR_INVALID_ARG, "%s: NULL argument", who);
    if (desc->batch < 1 || desc->batch > 65535 || desc->n_kv_heads < 1 || desc->s_max < 1 || desc->head_dim < 1)
        return fail(DREAM_ERR_INVALID_ARG, "%s: batch in [1, 65535], n_kv_heads, head_dim and s_max must be positive", who);
    if (desc->dtype != DREAM_F32 && desc->dtype != DREAM_BF16)
        return fail(DREAM_ERR_INVALID_ARG, "%s: unknown dtype %d", who, desc->dtype);
    if (n_caches < 1)
        return fail(DREAM_ERR_INVALID_ARG, "%s: n_caches %d < 1", who, n_caches);
    if (n_tree < 1 || n_tree > DREAM_MAX_TREE_ACCEPT || n_tree > desc->s_max)
        return fail(DREAM_ERR_INVALID_ARG, "%s: n_tree %d outside [1, min(%d, s_max)]", who, n_tree, DREAM_MAX_TREE_ACCEPT);
    if (path_stride < 1)
        return fail(DREAM_ERR_INVALID_ARG, "%s: path_stride %d < 1", who, path_stride);
    if (prefix_len_out == prefix_len)
        return fail(DREAM_ERR_INVALID_ARG, "%s: prefix_len_out must not alias prefix_len", who);
    const int64_t row_bytes = (int64_t)desc->head_dim * (desc->dtype == DREAM_F32 ? 4 : 2);
    if (row_bytes % 16)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: rows of %lld bytes are not a multiple of 16", who, (long long)row_bytes);
    const int64_t max_rows = path_stride < n_tree ? path_stride : n_tree;
    if (max_rows * (row_bytes / 16) > 256 * CHUNKS_PER_THREAD)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: up to %lld rows of %lld bytes exceed the 64 KB a workgroup moves", who,
                    (long long)max_rows, (long long)row_bytes);
    for (int32_t i = 0; i < n_caches; i++) {
        if (!caches_host[i])
            return fail(DREAM_ERR_INVALID_ARG, "%s: cache %d is NULL", who, i);
        if (reinterpret_cast<uintptr_t>(caches_host[i]) & 15)
            return fail(DREAM_ERR_INVALID_ARG, "%s: cache %d is not 16-byte aligned", who, i);
    }
    CommitArgs a;
    a.prefix_len = prefix_len; a.path = accept_path; a.accept_len = accept_len; a.prefix_len_out = prefix_len_out;
    a.n_kv_heads = desc->n_kv_heads; a.n_tree = n_tree; a.path_stride = path_stride;
    a.chunks_per_row = (int)(row_bytes / 16); a.s_max = desc->s_max;
    // heads per workgroup: as many as the registers of a workgroup hold, while about a thousand workgroups remain
    const int64_t fit = (256 * CHUNKS_PER_THREAD) / (max_rows * a.chunks_per_row);
    const int64_t spare = ((int64_t)desc->n_kv_heads * desc->batch * (n_caches < MAX_CACHES_PER_LAUNCH ? n_caches : MAX_CACHES_PER_LAUNCH)) / 1024;
    int64_t hpw = fit < spare ? fit : spare;
    if (hpw > desc->n_kv_heads)
        hpw = desc->n_kv_heads;
    if (hpw < 1)
        hpw = 1;
    a.heads_per_wg = (int)hpw;
    for (int32_t first = 0; first < n_caches; first += MAX_CACHES_PER_LAUNCH) {
        const int m = n_caches - first < MAX_CACHES_PER_LAUNCH ? n_caches - first : MAX_CACHES_PER_LAUNCH;
        for (int i = 0; i < MAX_CACHES_PER_LAUNCH; i++)
            a.cache[i] = i < m ? caches_host[first + i] : nullptr;
        a.first_cache = first;
        hipLaunchKernelGGL(kv_commit_kernel, dim3(ceil_div(desc->n_kv_heads, a.heads_per_wg), desc->batch, m), dim3(256), 0, as_stream(stream), a);
        int rc = check_launch("kv_commit_kernel");
        if (rc)
            return rc;
    }
    return DREAM_OK;
}

}  // extern "C"
