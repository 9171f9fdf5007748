// dream_visual_compress: visual-token importance scores, top-k keep and row gather (Section 3.3).
//
// The importance of key token j is the attention weight it receives, summed over the rows and
// heads of the last-layer causal attention matrix.  The probabilities need each row's softmax
// normaliser first, so stage A runs two passes over q k^T (both on v_mfma_f32_16x16x32_bf16, no
// attention matrix is ever stored):
//   scores_lse_*     one wave per 16 query rows: log-sum-exp of every causal row;
//   scores_colsum_*  one wave per 16 visual keys: sum over rows of exp(score - lse), per head.
// Each (sequence, head, key) partial sum is produced by exactly one wave in a fixed order, and the
// sum over heads is taken in head order by the selection kernel, so scores are reproducible
// bit for bit.  Stage B ranks every visual token by counting the tokens that beat it under
// (higher score, then lower index), keeps ranks below k and compacts the survivors in position
// order; the optional gather copies the surviving rows of a [rows, row_elems] matrix.
#include "common.h"

using namespace dream;

namespace {

struct ScoreArgs {
    const void *q, *k;
    const int32_t *q_pos;
    float *lse2;   // [B, Hq, n_q_pad]  log2-domain log-sum-exp of each row
    float *part;   // [B, Hq, vis_len]  per-head column sums
    int32_t n_q, n_q_pad, n_keys, n_q_heads, n_kv_heads, vis_start, vis_len;
    int64_t s_max;
    float scale, scale_log2;
};

template <int D>
__global__ __launch_bounds__(256) void scores_lse_bf16_kernel(ScoreArgs a)
{
    constexpr int NKS = D / 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int row0 = (blockIdx.x * 4 + wave) * 16, h = blockIdx.y, b = blockIdx.z;
    if (row0 >= a.n_q)
        return;
    const int kvh = h / (a.n_q_heads / a.n_kv_heads);
    const int row = row0 + c;
    const bool valid = row < a.n_q;
    const int pos = valid ? (a.q_pos ? a.q_pos[(int64_t)b * a.n_q + row] : row) : -1;
    bf16x8 qf[NKS];
    const uint16_t *qp = reinterpret_cast<const uint16_t *>(a.q) + (((int64_t)b * a.n_q + (valid ? row : 0)) * a.n_q_heads + h) * D + g * 8;
#pragma unroll
    for (int ks = 0; ks < NKS; ks++) {
        qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 32);
        if (!valid)
#pragma unroll
            for (int i = 0; i < 8; i++)
                qf[ks][i] = (__bf16)0.0f;
    }
    int lim = pos + 1;
    for (int off = 32; off > 0; off >>= 1)
        lim = max(lim, __shfl_xor(lim, off));
    lim = min(lim, a.n_keys);
    const uint16_t *kb = reinterpret_cast<const uint16_t *>(a.k) + ((int64_t)b * a.n_kv_heads + kvh) * a.s_max * D + g * 8;
    float m = -INFINITY, l = 0.0f;
    for (int key0 = 0; key0 < lim; key0 += 16) {
        const int key = key0 + c;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        if (key < a.n_keys) {
            const uint16_t *kp = kb + (int64_t)key * D;
            bf16x8 kf[NKS];
#pragma unroll
            for (int ks = 0; ks < NKS; ks++)
                kf[ks] = *reinterpret_cast<const bf16x8 *>(kp + ks * 32);
#pragma unroll
            for (int ks = 0; ks < NKS; ks++)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[ks], qf[ks], acc, 0, 0, 0);
        } else {
            bf16x8 z;
#pragma unroll
            for (int i = 0; i < 8; i++)
                z[i] = (__bf16)0.0f;
#pragma unroll
            for (int ks = 0; ks < NKS; ks++)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(z, qf[ks], acc, 0, 0, 0);
        }
        float x[4], mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 4; r++) {
            int kk = key0 + g * 4 + r;
            x[r] = (kk <= pos && kk < a.n_keys) ? acc[r] * a.scale_log2 : -INFINITY;
            mx = fmaxf(mx, x[r]);
        }
        float m_new = fmaxf(m, mx);
        float m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
        float s = 0.0f;
#pragma unroll
        for (int r = 0; r < 4; r++)
            s += __builtin_amdgcn_exp2f(x[r] - m_safe);
        l = l * __builtin_amdgcn_exp2f(m - m_safe) + s;
        m = m_new;
    }
    float mt = fmaxf(m, __shfl_xor(m, 16));
    mt = fmaxf(mt, __shfl_xor(mt, 32));
    float ms = (mt == -INFINITY) ? 0.0f : mt;
    float lw = l * __builtin_amdgcn_exp2f(m - ms);
    lw += __shfl_xor(lw, 16);
    lw += __shfl_xor(lw, 32);
    if (g == 0 && valid)
        a.lse2[((int64_t)b * a.n_q_heads + h) * a.n_q_pad + row] = lw > 0.0f ? mt + log2f(lw) : INFINITY;
}

template <int D>
__global__ __launch_bounds__(256) void scores_colsum_bf16_kernel(ScoreArgs a)
{
    constexpr int NKS = D / 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int vis_end = a.vis_start + a.vis_len;
    const int j0 = a.vis_start + (blockIdx.x * 4 + wave) * 16, h = blockIdx.y, b = blockIdx.z;
    if (j0 >= vis_end)
        return;
    const int kvh = h / (a.n_q_heads / a.n_kv_heads);
    const int key = j0 + c;
    const bool kvalid = key < vis_end && key < a.n_keys;
    bf16x8 kf[NKS];
    const uint16_t *kp = reinterpret_cast<const uint16_t *>(a.k) + (((int64_t)b * a.n_kv_heads + kvh) * a.s_max + (kvalid ? key : 0)) * D + g * 8;
#pragma unroll
    for (int ks = 0; ks < NKS; ks++) {
        kf[ks] = *reinterpret_cast<const bf16x8 *>(kp + ks * 32);
        if (!kvalid)
#pragma unroll
            for (int i = 0; i < 8; i++)
                kf[ks][i] = (__bf16)0.0f;
    }
    const int n_rt = (a.n_q + 15) / 16;
    const int rt_begin = a.q_pos ? 0 : j0 / 16;   // without explicit positions row r sits at position r: rows below j0 see none of these keys
    const uint16_t *qb = reinterpret_cast<const uint16_t *>(a.q) + ((int64_t)b * a.n_q * a.n_q_heads + h) * D + g * 8;
    const float *lrow = a.lse2 + ((int64_t)b * a.n_q_heads + h) * a.n_q_pad;
    float cs = 0.0f;
    for (int rt = rt_begin; rt < n_rt; rt++) {
        const int row_a = rt * 16 + c;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        bf16x8 qf[NKS];
        const uint16_t *qp = qb + (int64_t)(row_a < a.n_q ? row_a : 0) * a.n_q_heads * D;
#pragma unroll
        for (int ks = 0; ks < NKS; ks++) {
            qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 32);
            if (row_a >= a.n_q)
#pragma unroll
                for (int i = 0; i < 8; i++)
                    qf[ks][i] = (__bf16)0.0f;
        }
#pragma unroll
        for (int ks = 0; ks < NKS; ks++)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[ks], kf[ks], acc, 0, 0, 0);
        const int rbase = rt * 16 + g * 4;
        f32x4 L = *reinterpret_cast<const f32x4 *>(lrow + rbase);
#pragma unroll
        for (int r = 0; r < 4; r++) {
            int row = rbase + r;
            if (row < a.n_q) {
                int pos = a.q_pos ? a.q_pos[(int64_t)b * a.n_q + row] : row;
                if (key <= pos)
                    cs += __builtin_amdgcn_exp2f(acc[r] * a.scale_log2 - L[r]);
            }
        }
    }
    cs += __shfl_xor(cs, 16);
    cs += __shfl_xor(cs, 32);
    if (g == 0 && key < vis_end)
        a.part[((int64_t)b * a.n_q_heads + h) * a.vis_len + (key - a.vis_start)] = kvalid ? cs : 0.0f;
}

// ---- float32 tensors: plain vector-ALU versions of the two passes -------------------------------
__global__ __launch_bounds__(256) void scores_lse_f32_kernel(ScoreArgs a, int D)
{
    __shared__ float sq[256];
    __shared__ float red_m[4], red_l[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int kvh = h / (a.n_q_heads / a.n_kv_heads);
    const int pos = a.q_pos ? a.q_pos[(int64_t)b * a.n_q + row] : row;
    const float *q = reinterpret_cast<const float *>(a.q) + (((int64_t)b * a.n_q + row) * a.n_q_heads + h) * D;
    const float *kb = reinterpret_cast<const float *>(a.k) + ((int64_t)b * a.n_kv_heads + kvh) * a.s_max * D;
    if (tid < D)
        sq[tid] = q[tid];
    __syncthreads();
    float m = -INFINITY, l = 0.0f;
    const int lim = min(pos + 1, a.n_keys);
    for (int key = tid; key < lim; key += 256) {
        const float *kr = kb + (int64_t)key * D;
        float dot = 0.0f;
        for (int d = 0; d < D; d++)
            dot += sq[d] * kr[d];
        float x = dot * a.scale;
        float mn = fmaxf(m, x);
        l = l * expf(m - mn) + expf(x - mn);
        m = mn;
    }
    for (int off = 32; off > 0; off >>= 1) {
        float om = __shfl_xor(m, off), ol = __shfl_xor(l, off);
        float mn = fmaxf(m, om);
        float ms = (mn == -INFINITY) ? 0.0f : mn;
        l = l * expf(m - ms) + ol * expf(om - ms);
        m = mn;
    }
    if (lane == 0) {
        red_m[wave] = m;
        red_l[wave] = l;
    }
    __syncthreads();
    if (tid == 0) {
        float mm = fmaxf(fmaxf(red_m[0], red_m[1]), fmaxf(red_m[2], red_m[3]));
        float ms = (mm == -INFINITY) ? 0.0f : mm;
        float ll = 0.0f;
        for (int w = 0; w < 4; w++)
            ll += red_l[w] * expf(red_m[w] - ms);
        a.lse2[((int64_t)b * a.n_q_heads + h) * a.n_q_pad + row] = ll > 0.0f ? mm + logf(ll) : INFINITY;   // natural log here
    }
}

__global__ __launch_bounds__(64) void scores_colsum_f32_kernel(ScoreArgs a, int D)
{
    const int j = blockIdx.x * 64 + threadIdx.x, h = blockIdx.y, b = blockIdx.z;
    if (j >= a.vis_len)
        return;
    const int key = a.vis_start + j;
    const int kvh = h / (a.n_q_heads / a.n_kv_heads);
    float cs = 0.0f;
    if (key < a.n_keys) {
        const float *kr = reinterpret_cast<const float *>(a.k) + (((int64_t)b * a.n_kv_heads + kvh) * a.s_max + key) * D;
        const float *lrow = a.lse2 + ((int64_t)b * a.n_q_heads + h) * a.n_q_pad;
        for (int row = 0; row < a.n_q; row++) {
            int pos = a.q_pos ? a.q_pos[(int64_t)b * a.n_q + row] : row;
            if (key > pos)
                continue;
            const float *q = reinterpret_cast<const float *>(a.q) + (((int64_t)b * a.n_q + row) * a.n_q_heads + h) * D;
            float dot = 0.0f;
            for (int d = 0; d < D; d++)
                dot += q[d] * kr[d];
            cs += expf(dot * a.scale - lrow[row]);
        }
    }
    a.part[((int64_t)b * a.n_q_heads + h) * a.vis_len + j] = cs;
}

// ---- stage B ----------------------------------------------------------------------------------
// One workgroup of 1024 threads per sequence.  Dynamic LDS: vis_len floats + vis_len bytes + 1024 ints.
__global__ __launch_bounds__(1024) void topk_keep_kernel(const float *part, int n_heads, const float *scores_in,
                                                         float *scores_out, int vis_start, int vis_len, int k,
                                                         int32_t *kept_idx)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    float *s = reinterpret_cast<float *>(smem_raw);
    int32_t *cnt = reinterpret_cast<int32_t *>(s + vis_len);
    uint8_t *keep = reinterpret_cast<uint8_t *>(cnt + 1024);
    const int b = blockIdx.x, tid = threadIdx.x;
    for (int j = tid; j < vis_len; j += 1024) {
        float x;
        if (scores_in) {
            x = scores_in[(int64_t)b * vis_len + j];
        } else {
            x = 0.0f;
            for (int h = 0; h < n_heads; h++)
                x += part[((int64_t)b * n_heads + h) * vis_len + j];
        }
        s[j] = x;
        if (scores_out)
            scores_out[(int64_t)b * vis_len + j] = x;
    }
    __syncthreads();
    for (int j = tid; j < vis_len; j += 1024) {
        const float x = s[j];
        int rank = 0;
        for (int i = 0; i < vis_len; i++) {
            float y = s[i];
            rank += (y > x) || (y == x && i < j);
        }
        keep[j] = rank < k;
    }
    __syncthreads();
    // ordered compaction: thread t owns the contiguous slice [t*per, (t+1)*per)
    const int per = (vis_len + 1023) / 1024;
    const int lo = min(tid * per, vis_len), hi = min(lo + per, vis_len);
    int mine = 0;
    for (int j = lo; j < hi; j++)
        mine += keep[j];
    cnt[tid] = mine;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {   // inclusive scan
        int v = tid >= off ? cnt[tid - off] : 0;
        __syncthreads();
        cnt[tid] += v;
        __syncthreads();
    }
    int out = cnt[tid] - mine;
    for (int j = lo; j < hi; j++)
        if (keep[j])
            kept_idx[(int64_t)b * k + out++] = vis_start + j;
}

__global__ __launch_bounds__(256) void gather_rows_kernel(const unsigned char *src, int64_t n_rows_src, int64_t row_bytes,
                                                          const int32_t *kept_idx, int k, unsigned char *dst)
{
    const int t = blockIdx.x, b = blockIdx.y;
    const int64_t srow = kept_idx[(int64_t)b * k + t];
    const unsigned char *s = src + ((int64_t)b * n_rows_src + srow) * row_bytes;
    unsigned char *d = dst + ((int64_t)b * k + t) * row_bytes;
    if (((row_bytes | (uintptr_t)s | (uintptr_t)d) & 15) == 0) {
        for (int64_t i = threadIdx.x; i < row_bytes / 16; i += 256)
            reinterpret_cast<uint4 *>(d)[i] = reinterpret_cast<const uint4 *>(s)[i];
    } else {
        for (int64_t i = threadIdx.x; i < row_bytes; i += 256)
            d[i] = s[i];
    }
}

struct CompressPlan {
    int n_q_pad;
    size_t off_lse, off_part, total;
};

CompressPlan compress_plan(int batch, int n_heads, int n_q, int vis_len)
{
    CompressPlan p;
    p.n_q_pad = (n_q + 15) / 16 * 16;
    p.off_lse = DREAM_WORKSPACE_HEADER_BYTES;
    p.off_part = align_up(p.off_lse + (size_t)batch * n_heads * p.n_q_pad * sizeof(float), 256);
    p.total = align_up(p.off_part + (size_t)batch * n_heads * (vis_len > 0 ? vis_len : 1) * sizeof(float), 256);
    return p;
}

}  // namespace

extern "C" {

size_t dream_visual_compress_workspace(const dream_attn_desc *desc, int32_t n_q, int32_t vis_len)
{
    if (!desc || desc->batch < 1 || desc->n_q_heads < 1 || n_q < 1)
        return DREAM_WORKSPACE_HEADER_BYTES;
    return compress_plan(desc->batch, desc->n_q_heads, n_q, vis_len).total;
}

int dream_visual_compress(const dream_attn_desc *desc, const void *q, const int32_t *q_pos, int32_t n_q,
                          const void *k_cache, int32_t n_keys, int32_t vis_start, int32_t vis_len,
                          int32_t keep_num, int32_t keep_den, const float *scores_in, float *scores_out,
                          int32_t *kept_idx, int32_t *n_kept_host, const void *gather_src, int64_t n_rows_src,
                          void *gather_dst, int64_t row_elems, void *workspace, size_t workspace_bytes, void *stream)
{
    const char *who = "dream_visual_compress";
    if (!desc)
        return fail(DREAM_ERR_INVALID_ARG, "%s: desc is NULL", who);
    if (desc->batch < 1 || desc->batch > 65535)
        return fail(DREAM_ERR_INVALID_ARG, "%s: batch %d outside [1, 65535]", who, desc->batch);
    if (keep_den <= 0 || keep_num < 0 || keep_num > keep_den)
        return fail(DREAM_ERR_INVALID_ARG, "%s: keep ratio %d/%d is not in [0, 1]", who, keep_num, keep_den);
    if (vis_start < 0 || vis_len < 0)
        return fail(DREAM_ERR_INVALID_ARG, "%s: negative visual span", who);
    if (vis_len > DREAM_MAX_VISUAL)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: vis_len %d exceeds %d", who, vis_len, DREAM_MAX_VISUAL);
    if (desc->dtype != DREAM_F32 && desc->dtype != DREAM_BF16)
        return fail(DREAM_ERR_INVALID_ARG, "%s: unknown dtype %d", who, desc->dtype);
    const int k = (int)(((int64_t)vis_len * keep_num + keep_den / 2) / keep_den);
    if (k > 0 && !kept_idx)
        return fail(DREAM_ERR_INVALID_ARG, "%s: kept_idx is NULL", who);
    if ((gather_src == nullptr) != (gather_dst == nullptr))
        return fail(DREAM_ERR_INVALID_ARG, "%s: gather_src and gather_dst must be given together", who);
    if (gather_src && (row_elems < 1 || n_rows_src < (int64_t)vis_start + vis_len))
        return fail(DREAM_ERR_INVALID_ARG, "%s: gather needs row_elems >= 1 and n_rows_src >= vis_start + vis_len", who);
    hipStream_t st = as_stream(stream);
    const float *part = nullptr;
    int n_heads = 0;
    if (!scores_in && vis_len > 0) {
        if (desc->n_q_heads < 1 || desc->n_kv_heads < 1 || desc->n_q_heads % desc->n_kv_heads || desc->n_q_heads > 65535)
            return fail(DREAM_ERR_INVALID_ARG, "%s: bad head counts %d / %d", who, desc->n_q_heads, desc->n_kv_heads);
        if (desc->head_dim != 64 && desc->head_dim != 128 && desc->head_dim != 256)
            return fail(DREAM_ERR_UNSUPPORTED, "%s: head_dim %d not in {64,128,256}", who, desc->head_dim);
        if (!q || !k_cache)
            return fail(DREAM_ERR_INVALID_ARG, "%s: q and k_cache are required when scores_in is NULL", who);
        if (n_q < 1 || n_keys < 1 || n_keys > desc->s_max)
            return fail(DREAM_ERR_INVALID_ARG, "%s: need n_q >= 1 and 1 <= n_keys <= s_max", who);
        if (!q_pos && n_q > n_keys)
            return fail(DREAM_ERR_INVALID_ARG, "%s: %d rows at positions 0..n_q-1 but only %d keys", who, n_q, n_keys);
        if ((int64_t)vis_start + vis_len > n_keys)
            return fail(DREAM_ERR_INVALID_ARG, "%s: visual span [%d, %d) exceeds the %d live keys", who, vis_start, vis_start + vis_len, n_keys);
        CompressPlan p = compress_plan(desc->batch, desc->n_q_heads, n_q, vis_len);
        if (!workspace || workspace_bytes < p.total)
            return fail(DREAM_ERR_WORKSPACE, "%s: workspace of %zu bytes, %zu needed", who, workspace_bytes, p.total);
        ScoreArgs a;
        a.q = q; a.k = k_cache; a.q_pos = q_pos;
        a.lse2 = reinterpret_cast<float *>(static_cast<char *>(workspace) + p.off_lse);
        a.part = reinterpret_cast<float *>(static_cast<char *>(workspace) + p.off_part);
        a.n_q = n_q; a.n_q_pad = p.n_q_pad; a.n_keys = n_keys;
        a.n_q_heads = desc->n_q_heads; a.n_kv_heads = desc->n_kv_heads;
        a.vis_start = vis_start; a.vis_len = vis_len; a.s_max = desc->s_max;
        a.scale = desc->scale != 0.0f ? desc->scale : 1.0f / sqrtf((float)desc->head_dim);
        a.scale_log2 = a.scale * 1.4426950408889634f;
        if (desc->dtype == DREAM_BF16) {
            dim3 g1(ceil_div(n_q, 64), desc->n_q_heads, desc->batch), g2(ceil_div(vis_len, 64), desc->n_q_heads, desc->batch);
            switch (desc->head_dim) {
            case 64:
                hipLaunchKernelGGL(scores_lse_bf16_kernel<64>, g1, dim3(256), 0, st, a);
                hipLaunchKernelGGL(scores_colsum_bf16_kernel<64>, g2, dim3(256), 0, st, a);
                break;
            case 128:
                hipLaunchKernelGGL(scores_lse_bf16_kernel<128>, g1, dim3(256), 0, st, a);
                hipLaunchKernelGGL(scores_colsum_bf16_kernel<128>, g2, dim3(256), 0, st, a);
                break;
            default:
                hipLaunchKernelGGL(scores_lse_bf16_kernel<256>, g1, dim3(256), 0, st, a);
                hipLaunchKernelGGL(scores_colsum_bf16_kernel<256>, g2, dim3(256), 0, st, a);
                break;
            }
        } else {
            if (n_q > 65535 * 1)
                return fail(DREAM_ERR_UNSUPPORTED, "%s: too many rows for the float32 path", who);
            hipLaunchKernelGGL(scores_lse_f32_kernel, dim3(n_q, desc->n_q_heads, desc->batch), dim3(256), 0, st, a, desc->head_dim);
            hipLaunchKernelGGL(scores_colsum_f32_kernel, dim3(ceil_div(vis_len, 64), desc->n_q_heads, desc->batch), dim3(64), 0, st, a, desc->head_dim);
        }
        int rc = check_launch("visual score kernels");
        if (rc)
            return rc;
        part = a.part;
        n_heads = desc->n_q_heads;
    }
    if (n_kept_host)
        *n_kept_host = k;
    if (vis_len > 0 && (k > 0 || scores_out)) {
        size_t lds = (size_t)vis_len * 4 + 1024 * 4 + (size_t)vis_len;
        static bool attr_set = false;
        if (!attr_set) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(&topk_keep_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    DREAM_MAX_VISUAL * 5 + 4096) != hipSuccess)
                return fail(DREAM_ERR_HIP, "%s: cannot reserve LDS for the selection kernel", who);
            attr_set = true;
        }
        hipLaunchKernelGGL(topk_keep_kernel, dim3(desc->batch), dim3(1024), lds, st, part, n_heads, scores_in, scores_out,
                           vis_start, vis_len, k, kept_idx);
        int rc = check_launch("topk_keep_kernel");
        if (rc)
            return rc;
    }
    if (gather_src && k > 0) {
        const int64_t row_bytes = row_elems * (desc->dtype == DREAM_F32 ? 4 : 2);
        hipLaunchKernelGGL(gather_rows_kernel, dim3(k, desc->batch), dim3(256), 0, st,
                           static_cast<const unsigned char *>(gather_src), n_rows_src, row_bytes, kept_idx, k,
                           static_cast<unsigned char *>(gather_dst));
        return check_launch("gather_rows_kernel");
    }
    return DREAM_OK;
}

}  // extern "C"
