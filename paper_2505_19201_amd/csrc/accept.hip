// dream_accept_path: per-node arg-max over the vocabulary and the greedy accepted path.
//
// At temperature 0 the acceptance rule of Section 2.1 accepts a drafted token exactly when it is
// the target's arg-max at its parent; everything after the first mismatch on a path is dropped and
// the target's own choice at the last accepted node is emitted as the bonus token (Section 4).
//
// argmax_partial_kernel streams the logits once (16-byte loads, one workgroup per row chunk) and
// reduces (value, index) pairs with wavefront shuffles; ties always keep the lower index, so the
// result does not depend on how rows are chunked.  accept_walk_kernel merges the chunk results and
// walks the tree in node order in a single wavefront per sequence.
#include "common.h"
#include <mutex>

using namespace dream;

// Scratch of dream_accept_path_static: the per-chunk (value, index) partial results live here instead of in a
// caller's workspace.  One copy per GPU, held until the process ends; host code only ever uses the address
// hipGetSymbolAddress reports for the current device, never the symbol itself.
static __device__ __align__(256) unsigned char scratch[DREAM_ACCEPT_STATIC_SCRATCH_BYTES];

namespace {

constexpr int CHUNK_ELEMS = 8192;   // logits handled by one workgroup
constexpr int MAX_DEVICES = 64;

__device__ __forceinline__ void better(float &v, int &i, float ov, int oi)
{
    if (ov > v || (ov == v && oi < i)) {
        v = ov;
        i = oi;
    }
}

template <bool BF16>
__global__ __launch_bounds__(256) void argmax_partial_kernel(const void *logits, int vocab, int n_chunks,
                                                             float *part_val, int32_t *part_idx)
{
    const int chunk = blockIdx.x;
    const int64_t row = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int begin = chunk * CHUNK_ELEMS;
    const int end = min(begin + CHUNK_ELEMS, vocab);
    float best = -INFINITY;
    int best_i = 0x7fffffff;
    if (BF16) {
        const uint16_t *p = reinterpret_cast<const uint16_t *>(logits) + row * vocab;
        // 16-byte vector loads when the row start allows it, scalar loads otherwise and for the tail
        const bool aligned = (((uintptr_t)(p + begin)) & 15) == 0;
        int vec_end = aligned ? begin + ((end - begin) & ~7) : begin;
        for (int i = begin + tid * 8; i < vec_end; i += 256 * 8) {
            const u32x4 u = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p + i));   // logits: read once
            uint32_t w[4] = {u[0], u[1], u[2], u[3]};
#pragma unroll
            for (int j = 0; j < 4; j++) {
                float lo = __uint_as_float(w[j] << 16), hi = __uint_as_float(w[j] & 0xffff0000u);
                if (lo > best) { best = lo; best_i = i + 2 * j; }
                if (hi > best) { best = hi; best_i = i + 2 * j + 1; }
            }
        }
        for (int i = vec_end + tid; i < end; i += 256) {
            float x = bf16_bits_to_float(p[i]);
            if (x > best || (x == best && i < best_i)) { best = x; best_i = i; }
        }
    } else {
        const float *p = reinterpret_cast<const float *>(logits) + row * vocab;
        const bool aligned = (((uintptr_t)(p + begin)) & 15) == 0;
        int vec_end = aligned ? begin + ((end - begin) & ~3) : begin;
        for (int i = begin + tid * 4; i < vec_end; i += 256 * 4) {
            float4 u = *reinterpret_cast<const float4 *>(p + i);
            if (u.x > best) { best = u.x; best_i = i; }
            if (u.y > best) { best = u.y; best_i = i + 1; }
            if (u.z > best) { best = u.z; best_i = i + 2; }
            if (u.w > best) { best = u.w; best_i = i + 3; }
        }
        for (int i = vec_end + tid; i < end; i += 256) {
            float x = p[i];
            if (x > best || (x == best && i < best_i)) { best = x; best_i = i; }
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        float ov = __shfl_xor(best, off);
        int oi = __shfl_xor(best_i, off);
        better(best, best_i, ov, oi);
    }
    __shared__ float sv[4];
    __shared__ int si[4];
    if (lane == 0) {
        sv[wave] = best;
        si[wave] = best_i;
    }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; w++)
            better(best, best_i, sv[w], si[w]);
        part_val[row * n_chunks + chunk] = best;
        part_idx[row * n_chunks + chunk] = best_i;
    }
}

// One wave per sequence.  Every node checks its own root path in parallel (a node is accepted iff every
// edge above it matches the target's arg-max and it is not deeper than max_depth); the deepest accepted
// node, lowest index among equals, wins a wave reduction; lane 0 writes its path.
__global__ __launch_bounds__(64) void accept_walk_kernel(const float *part_val, const int32_t *part_idx, int n_chunks,
                                                         int n_tree, const int32_t *token, const int32_t *parent,
                                                         int max_depth, int32_t *node_argmax, int32_t *accept_len,
                                                         int32_t *accept_path, int32_t *bonus_token)
{
    __shared__ int32_t s_am[DREAM_MAX_TREE_ACCEPT];
    __shared__ int32_t s_par[DREAM_MAX_TREE_ACCEPT];
    __shared__ int32_t s_tok[DREAM_MAX_TREE_ACCEPT];
    const int b = blockIdx.x, lane = threadIdx.x;
    for (int i = lane; i < n_tree; i += 64) {
        int64_t row = (int64_t)b * n_tree + i;
        float v = part_val[row * n_chunks];
        int idx = part_idx[row * n_chunks];
        for (int ch = 1; ch < n_chunks; ch++)
            better(v, idx, part_val[row * n_chunks + ch], part_idx[row * n_chunks + ch]);
        s_am[i] = idx;
        const int par = parent[row];
        s_par[i] = par < i ? par : -1;   // a walk up the tree always ends
        s_tok[i] = token[row];
        node_argmax[row] = idx;
    }
    __syncthreads();
    int best_d = -1, best_i = 0x7fffffff;
    for (int i = lane; i < n_tree; i += 64) {
        int d = 0;
        bool ok = true;
        for (int a = i; a > 0 && ok; d++) {
            const int p = s_par[a];
            ok = p >= 0 && s_tok[a] == s_am[p];
            a = p;
        }
        if (ok && d <= max_depth && d > best_d) {   // nodes are visited in increasing index: strict '>' keeps the lowest
            best_d = d;
            best_i = i;
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        const int od = __shfl_xor(best_d, off), oi = __shfl_xor(best_i, off);
        if (od > best_d || (od == best_d && oi < best_i)) {
            best_d = od;
            best_i = oi;
        }
    }
    if (lane == 0) {
        accept_len[b] = best_d;
        int32_t *path = accept_path + (int64_t)b * (max_depth + 1);
        for (int t = best_d + 1; t <= max_depth; t++)
            path[t] = -1;
        int d = best_d;
        for (int n = best_i; n >= 0 && d >= 0; n = s_par[n])
            path[d--] = n;
        bonus_token[b] = s_am[best_i];
    }
}

size_t partial_bytes(int batch, int n_tree, int vocab)
{
    const size_t n = (size_t)batch * n_tree * ceil_div(vocab, CHUNK_ELEMS);
    return align_up(n * 4, 256) + align_up(n * 4, 256);
}

int validate_accept(const char *who, const void *logits, int logits_dtype, int batch, int n_tree, int vocab, const int32_t *token,
                    const int32_t *parent, int max_depth, const int32_t *node_argmax, const int32_t *accept_len,
                    const int32_t *accept_path, const int32_t *bonus_token)
{
    if (!logits || !token || !parent || !node_argmax || !accept_len || !accept_path || !bonus_token)
        return fail(DREAM_ERR_INVALID_ARG, "%s: NULL argument", who);
    if (logits_dtype != DREAM_F32 && logits_dtype != DREAM_BF16)
        return fail(DREAM_ERR_INVALID_ARG, "%s: unknown logits dtype %d", who, logits_dtype);
    if (batch < 1 || vocab < 1 || max_depth < 0)
        return fail(DREAM_ERR_INVALID_ARG, "%s: batch, vocab must be positive and max_depth non-negative", who);
    if (n_tree < 1 || n_tree > DREAM_MAX_TREE_ACCEPT)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: n_tree %d outside [1, %d]", who, n_tree, DREAM_MAX_TREE_ACCEPT);
    if ((int64_t)batch * n_tree > 65535)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: batch * n_tree = %lld exceeds 65535 rows", who, (long long)batch * n_tree);
    return DREAM_OK;
}

// The two launches; `partials` is device memory of partial_bytes() bytes (a workspace or the static scratch).
int launch_accept(const void *logits, int logits_dtype, int batch, int n_tree, int vocab, const int32_t *token, const int32_t *parent,
                  int max_depth, int32_t *node_argmax, int32_t *accept_len, int32_t *accept_path, int32_t *bonus_token, void *partials,
                  void *stream)
{
    const int n_chunks = ceil_div(vocab, CHUNK_ELEMS);
    const size_t n = (size_t)batch * n_tree * n_chunks;
    float *part_val = reinterpret_cast<float *>(partials);
    int32_t *part_idx = reinterpret_cast<int32_t *>(static_cast<char *>(partials) + align_up(n * 4, 256));
    hipStream_t st = as_stream(stream);
    dim3 grid(n_chunks, batch * n_tree);
    if (logits_dtype == DREAM_BF16)
        hipLaunchKernelGGL(argmax_partial_kernel<true>, grid, dim3(256), 0, st, logits, vocab, n_chunks, part_val, part_idx);
    else
        hipLaunchKernelGGL(argmax_partial_kernel<false>, grid, dim3(256), 0, st, logits, vocab, n_chunks, part_val, part_idx);
    int rc = check_launch("argmax_partial_kernel");
    if (rc)
        return rc;
    hipLaunchKernelGGL(accept_walk_kernel, dim3(batch), dim3(64), 0, st, part_val, part_idx, n_chunks, n_tree, token, parent,
                       max_depth, node_argmax, accept_len, accept_path, bonus_token);
    return check_launch("accept_walk_kernel");
}

// Device address of `scratch` on the current GPU, looked up once per device (each GPU holds its own copy).
int static_scratch_address(const char *who, void **out)
{
    static std::mutex mu;
    static void *address[MAX_DEVICES] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES)
        return fail(DREAM_ERR_HIP, "%s: no current HIP device (or its index is not below %d)", who, MAX_DEVICES);
    std::lock_guard<std::mutex> lock(mu);
    if (!address[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(DREAM_ERR_HIP, "%s: hipGetSymbolAddress(scratch) on device %d: %s", who, dev, hipGetErrorString(e));
        address[dev] = p;
    }
    *out = address[dev];
    return DREAM_OK;
}

}  // namespace

extern "C" {

size_t dream_accept_path_workspace(int32_t batch, int32_t n_tree, int32_t vocab)
{
    if (batch < 1 || n_tree < 1 || vocab < 1)
        return DREAM_WORKSPACE_MIN_BYTES;
    return DREAM_WORKSPACE_MIN_BYTES + partial_bytes(batch, n_tree, vocab);
}

int dream_accept_path(const void *logits, int32_t logits_dtype, int32_t batch, int32_t n_tree, int32_t vocab,
                      const int32_t *token, const int32_t *parent, int32_t max_depth, int32_t *node_argmax,
                      int32_t *accept_len, int32_t *accept_path, int32_t *bonus_token, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    const char *who = "dream_accept_path";
    int rc = validate_accept(who, logits, logits_dtype, batch, n_tree, vocab, token, parent, max_depth, node_argmax, accept_len,
                             accept_path, bonus_token);
    if (rc)
        return rc;
    const size_t need = dream_accept_path_workspace(batch, n_tree, vocab);
    if (!workspace || workspace_bytes < need)
        return fail(DREAM_ERR_WORKSPACE, "%s: workspace of %zu bytes, %zu needed", who, workspace_bytes, need);
    return launch_accept(logits, logits_dtype, batch, n_tree, vocab, token, parent, max_depth, node_argmax, accept_len, accept_path,
                         bonus_token, static_cast<char *>(workspace) + DREAM_WORKSPACE_MIN_BYTES, stream);
}

int dream_accept_path_static(const void *logits, int32_t logits_dtype, int32_t batch, int32_t n_tree, int32_t vocab,
                             const int32_t *token, const int32_t *parent, int32_t max_depth, int32_t *node_argmax,
                             int32_t *accept_len, int32_t *accept_path, int32_t *bonus_token, void *stream)
{
    const char *who = "dream_accept_path_static";
    int rc = validate_accept(who, logits, logits_dtype, batch, n_tree, vocab, token, parent, max_depth, node_argmax, accept_len,
                             accept_path, bonus_token);
    if (rc)
        return rc;
    const size_t need = partial_bytes(batch, n_tree, vocab);
    if (need > DREAM_ACCEPT_STATIC_SCRATCH_BYTES)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: batch * n_tree * ceil(vocab / %d) = %zu partial results need %zu bytes, the static scratch "
                    "holds %d; use dream_accept_path with a workspace", who, CHUNK_ELEMS,
                    (size_t)batch * n_tree * ceil_div(vocab, CHUNK_ELEMS), need, DREAM_ACCEPT_STATIC_SCRATCH_BYTES);
    void *base = nullptr;
    rc = static_scratch_address(who, &base);
    if (rc)
        return rc;
    // every partial result the walk reads is written by this call's first kernel: nothing has to start at zero
    return launch_accept(logits, logits_dtype, batch, n_tree, vocab, token, parent, max_depth, node_argmax, accept_len, accept_path,
                         bonus_token, base, stream);
}

int dream_accept_static_init(void)
{
    void *base = nullptr;
    return static_scratch_address("dream_accept_static_init", &base);
}

}  // extern "C"
