// dream_visual_compress: visual-token importance scores, top-k keep and row gather (Section 3.3).
//
// The importance of key token j is the attention weight it receives, summed over the rows and
// heads of the last-layer causal attention matrix.  The probabilities need each row's softmax
// normaliser first, so stage A runs two passes over q k^T (both on v_mfma_f32_16x16x32_bf16, no
// attention matrix is ever stored):
//   scores_lse_*     one workgroup per 64 query rows, K streamed through LDS: log-sum-exp of every causal row;
//   scores_colsum_*  one workgroup per 64 visual keys, query rows streamed through LDS: sum over rows of
//                    exp(score - lse), per head.
// Each (sequence, head, key) partial sum is produced by exactly one wave in a fixed order, and the
// sum over heads is taken in head order by the selection kernel, so scores are reproducible
// bit for bit.  Stage B finds the k-th largest score with a radix select, keeps everything above it
// plus the first ties in position order, and compacts the survivors in position order; the optional
// gather copies the surviving rows of a [rows, row_elems] matrix.
#include "common.h"
#include <atomic>

using namespace dream;

namespace {

struct ScoreArgs {
    const void *q, *k;
    const int32_t *q_pos;
    float *lse2;   // [ns1, B, Hq, n_q_pad]  log2-domain log-sum-exp of each row over the keys of split s (-inf: none)
    const float *lse_in;   // nullable [B, Hq, n_q]: the caller's natural-log log-sum-exp of every row (pass 1 is skipped)
    float *part;   // [B, Hq, ns2, vis_len]  column sums per head and row split
    int32_t n_q, n_q_pad, n_keys, n_q_heads, n_kv_heads, vis_start, vis_len;
    float *ent_part;    // [ns1, B, Hq, n_q_pad]  expected score of the row under its attention weights, per split (entropy only)
    int32_t ns1, ns2;   // splits of the streamed axis: keys in pass 1, query rows in pass 2
    int64_t lse_split_stride;   // B * Hq * n_q_pad
    int64_t s_max;
    float scale, scale_log2;
};

// Pass 1: log-sum-exp of every causal row.  One workgroup per (64 query rows, head, sequence, key split); wave w
// owns rows w*16..w*16+15; with ns1 > 1 the block's key tiles are divided evenly over ns1 workgroups, each of
// which writes a partial log-sum-exp that pass 2 combines.  All 256 threads stream K in 32-key tiles (two tiles ahead in registers, two LDS stages,
// one barrier per tile); scores are formed transposed (lane = query column), so a lane keeps a private running
// (max, sum) over its own key rows and the four row groups are combined once at the end.
// With ENT the kernel also keeps t = sum_j 2^(x_j - m) x_j, so that the expected score sum_j A_j x_j = t / l of
// the row is known and the row's entropy -sum A log A = LSE - sum A_j s_j (Eq. 2, Section 3.2) needs no
// second pass.
template <int D, bool ENT>
__global__ __launch_bounds__(256) void scores_lse_bf16_kernel(ScoreArgs a)
{
    constexpr int NKS = D / 32, STR = D + 8, CH = 32 * D / 8 / 256;
    __shared__ __attribute__((aligned(16))) uint16_t lds[2][32 * STR];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, g = lane >> 4;
    // x walks the heads with the KV head fastest: workgroup ids that share a KV head are congruent mod 8
    // (when there are 8 or more KV heads), so its K is fetched into one XCD's L2 only
    const int kvh = blockIdx.x % a.n_kv_heads, h = kvh * (a.n_q_heads / a.n_kv_heads) + blockIdx.x / a.n_kv_heads;
    // later row blocks see more keys: they are dispatched first so that the launch does not end on the longest workgroups
    const int blk = gridDim.y - 1 - blockIdx.y, b = blockIdx.z / a.ns1, split = blockIdx.z % a.ns1;
    const int row = blk * 64 + wave * 16 + c;
    const bool valid = row < a.n_q;
    const int pos = valid ? (a.q_pos ? a.q_pos[(int64_t)b * a.n_q + row] : row) : -1;
    // keys this workgroup has to see: without explicit positions, up to its last row
    const int key_lim = a.q_pos ? a.n_keys : min(min(blk * 64 + 64, a.n_q), a.n_keys);
    const int n_tiles_all = (key_lim + 31) / 32;
    const int tps = (n_tiles_all + a.ns1 - 1) / a.ns1;
    const int t0 = split * tps, n_tiles = max(min(tps, n_tiles_all - t0), 0);   // tiles t0 .. t0 + n_tiles - 1
    int wave_max_pos = pos;
    for (int off = 32; off > 0; off >>= 1)
        wave_max_pos = max(wave_max_pos, __shfl_xor(wave_max_pos, off));
    wave_max_pos = __builtin_amdgcn_readfirstlane(wave_max_pos);
    int wave_min_pos = valid ? pos : 0x7fffffff;   // rows that do not exist keep nothing, so they do not count
    for (int off = 32; off > 0; off >>= 1)
        wave_min_pos = min(wave_min_pos, __shfl_xor(wave_min_pos, off));
    wave_min_pos = __builtin_amdgcn_readfirstlane(wave_min_pos);

    const uint16_t *kb = reinterpret_cast<const uint16_t *>(a.k) + ((int64_t)b * a.n_kv_heads + kvh) * a.s_max * D;
    u32x4 kreg[2][CH];
    const int ld_row = tid / (D / 8), ld_col = tid % (D / 8);
    auto load_tile = [&](int i, u32x4(&kr)[CH]) {
        const int t = t0 + max(min(i, n_tiles - 1), 0);
#pragma unroll
        for (int j = 0; j < CH; j++) {
            const int key = min(t * 32 + ld_row + j * (2048 / D), a.n_keys - 1);
            kr[j] = *reinterpret_cast<const u32x4 *>(kb + (int64_t)key * D + ld_col * 8);
        }
    };
    load_tile(0, kreg[0]);
    load_tile(1, kreg[1]);
    bf16x8 qf[NKS];
    {
        const uint16_t *qp = reinterpret_cast<const uint16_t *>(a.q) + (((int64_t)b * a.n_q + (valid ? row : 0)) * a.n_q_heads + h) * D + g * 8;
#pragma unroll
        for (int ks = 0; ks < NKS; ks++)
            qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 32);
    }
    float m = -INFINITY, l = 0.0f, tx = 0.0f;
    auto step = [&](int i, u32x4(&kr)[CH]) {
        uint16_t *st = lds[i & 1];
#pragma unroll
        for (int j = 0; j < CH; j++)
            *reinterpret_cast<u32x4 *>(st + (ld_row + j * (2048 / D)) * STR + ld_col * 8) = kr[j];
        __syncthreads();
        load_tile(i + 2, kr);
        const int key0 = (t0 + i) * 32;
        if (key0 > wave_max_pos)
            return;   // causal: nothing in this tile is visible to this wave's rows
        bf16x8 kfr[2][NKS];
#pragma unroll
        for (int ks = 0; ks < NKS; ks++) {
            kfr[0][ks] = *reinterpret_cast<const bf16x8 *>(st + c * STR + ks * 32 + g * 8);
            kfr[1][ks] = *reinterpret_cast<const bf16x8 *>(st + (16 + c) * STR + ks * 32 + g * 8);
        }
        f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < NKS; ks++) {
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kfr[0][ks], qf[ks], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kfr[1][ks], qf[ks], acc1, 0, 0, 0);
        }
        float sum = 0.0f, xsum = 0.0f, m_new, m_safe;
        if (key0 + 31 <= wave_min_pos && key0 + 31 < a.n_keys && a.scale_log2 > 0.0f) {
            // every key of the tile is visible to every row of the wave (all but the tiles on the diagonal):
            // no masking, the maximum is taken before scaling and the scale rides in the exponent's fma
            float mx = fmaxf(fmaxf(fmaxf(acc0[0], acc0[1]), fmaxf(acc0[2], acc0[3])), fmaxf(fmaxf(acc1[0], acc1[1]), fmaxf(acc1[2], acc1[3])));
            m_new = fmaxf(m, mx * a.scale_log2);
            m_safe = m_new;   // finite: the tile has visible keys
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const float raw = e < 4 ? acc0[e & 3] : acc1[e & 3];
                const float p = __builtin_amdgcn_exp2f(fmaf(raw, a.scale_log2, -m_safe));
                sum += p;
                if (ENT)
                    xsum += p * (raw * a.scale_log2);
            }
        } else {
            float x[8], mx = -INFINITY;
            const int lim = min(pos, a.n_keys - 1);
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const int kk = key0 + (e >> 2) * 16 + g * 4 + (e & 3);
                const float v = (e < 4 ? acc0[e & 3] : acc1[e & 3]) * a.scale_log2;
                x[e] = kk <= lim ? v : -INFINITY;
                mx = fmaxf(mx, x[e]);
            }
            m_new = fmaxf(m, mx);
            m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const float p = __builtin_amdgcn_exp2f(x[e] - m_safe);
                sum += p;
                if (ENT)
                    xsum += p * (x[e] == -INFINITY ? 0.0f : x[e]);
            }
        }
        const float alpha = __builtin_amdgcn_exp2f(m - m_safe);
        l = l * alpha + sum;
        if (ENT)
            tx = tx * alpha + xsum;
        m = m_new;
    };
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): only tile prefetches are counted inside the loop
    {
        int t = 0;
        for (; t + 2 <= n_tiles; t += 2) {
            step(t, kreg[0]);
            step(t + 1, kreg[1]);
        }
        if (t < n_tiles)
            step(t, kreg[0]);
    }
    float mt = fmaxf(m, __shfl_xor(m, 16));
    mt = fmaxf(mt, __shfl_xor(mt, 32));
    const float ms = (mt == -INFINITY) ? 0.0f : mt;
    const float wgt = __builtin_amdgcn_exp2f(m - ms);
    float lw = l * wgt;
    lw += __shfl_xor(lw, 16);
    lw += __shfl_xor(lw, 32);
    const int64_t o = split * a.lse_split_stride + ((int64_t)b * a.n_q_heads + h) * a.n_q_pad + row;
    if (g == 0 && valid)
        a.lse2[o] = lw > 0.0f ? mt + log2f(lw) : -INFINITY;
    if (ENT) {
        float tw = tx * wgt;
        tw += __shfl_xor(tw, 16);
        tw += __shfl_xor(tw, 32);
        if (g == 0 && valid)
            a.ent_part[o] = lw > 0.0f ? tw / lw : 0.0f;
    }
}

// Entropy of every row from pass 1's per-split (log-sum-exp, expected score) pairs (Eq. 2).  One thread per
// (head, row); each workgroup also leaves the sum of its 256 entropies for entropy_mean_kernel, which adds the
// workgroup sums of a sequence in index order, so the mean is reproducible.
// log2_domain: bf16 path (scores in log2 units); otherwise natural units and a single split.
__global__ __launch_bounds__(256) void entropy_rows_kernel(ScoreArgs a, int log2_domain, float *row_entropy, float *block_sum)
{
    __shared__ float s_part[4];
    const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_rows = a.n_q_heads * a.n_q;
    const int i = blockIdx.x * 256 + tid;
    float H = 0.0f;
    if (i < n_rows) {
        const int h = i / a.n_q, r = i - h * a.n_q;
        const int64_t o = ((int64_t)b * a.n_q_heads + h) * a.n_q_pad + r;
        if (log2_domain) {
            float M = -INFINITY;
            for (int s = 0; s < a.ns1; s++)
                M = fmaxf(M, a.lse2[s * a.lse_split_stride + o]);
            if (M != -INFINITY) {
                float W = 0.0f, U = 0.0f;
                for (int s = 0; s < a.ns1; s++) {
                    const float w = __builtin_amdgcn_exp2f(a.lse2[s * a.lse_split_stride + o] - M);
                    W += w;
                    U += w * a.ent_part[s * a.lse_split_stride + o];
                }
                H = 0.6931471805599453f * ((M + log2f(W)) - U / W);
            }
        } else {
            const float L = a.lse2[o];
            H = L == INFINITY ? 0.0f : L - a.ent_part[o];
        }
        H = fmaxf(H, 0.0f);   // rounding can leave a tiny negative value for a one-hot row
        if (row_entropy)
            row_entropy[((int64_t)b * a.n_q_heads + h) * a.n_q + r] = H;
    }
    float acc = H;
    for (int off = 32; off > 0; off >>= 1)
        acc += __shfl_xor(acc, off);
    if (lane == 0)
        s_part[wave] = acc;
    __syncthreads();
    if (tid == 0)
        block_sum[(int64_t)b * gridDim.x + blockIdx.x] = (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
}

__global__ __launch_bounds__(64) void entropy_mean_kernel(const float *block_sum, int n_blocks, int n_rows, float *ae)
{
    const int b = blockIdx.x;
    if (threadIdx.x == 0) {
        float t = 0.0f;
        for (int i = 0; i < n_blocks; i++)
            t += block_sum[(int64_t)b * n_blocks + i];
        ae[b] = t / (float)n_rows;
    }
}

// Pass 2: column sums of the probabilities.  One workgroup per (64 visual keys, head, sequence, row split); wave w keeps
// the K fragments of its 16 keys in registers and all 256 threads stream the query rows (with their
// log-sum-exp and positions) in 32-row tiles through LDS.  A lane sums its key column over the rows it
// holds; the four row groups are combined at the end, so every (head, row split, key) sum has one fixed order.
// The row's log-sum-exp is combined from pass 1's ns1 partial values when its tile is loaded.
template <int D, int NS1>
__global__ __launch_bounds__(256) void scores_colsum_bf16_kernel(ScoreArgs a)
{
    constexpr int NKS = D / 32, STR = D + 8, CH = 32 * D / 8 / 256;
    __shared__ __attribute__((aligned(16))) uint16_t lds[2][32 * STR];
    __shared__ __attribute__((aligned(16))) float lds_lse[2][32];
    __shared__ __attribute__((aligned(16))) int32_t lds_pos[2][32];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, g = lane >> 4;
    const int vis_end = a.vis_start + a.vis_len;
    // x walks the heads with the KV head fastest (see pass 1): the query rows of a head stay in one XCD's L2
    const int kvh = blockIdx.x % a.n_kv_heads, h = kvh * (a.n_q_heads / a.n_kv_heads) + blockIdx.x / a.n_kv_heads;
    const int blk0 = a.vis_start + blockIdx.y * 64, b = blockIdx.z / a.ns2, split = blockIdx.z % a.ns2;
    const int j0 = blk0 + wave * 16;
    const int key = j0 + c;
    const bool kvalid = key < vis_end && key < a.n_keys;
    bf16x8 kf[NKS];
    {
        const uint16_t *kp = reinterpret_cast<const uint16_t *>(a.k) + (((int64_t)b * a.n_kv_heads + kvh) * a.s_max + (kvalid ? key : 0)) * D + g * 8;
#pragma unroll
        for (int ks = 0; ks < NKS; ks++)
            kf[ks] = *reinterpret_cast<const bf16x8 *>(kp + ks * 32);
    }
    // row tiles: without explicit positions row r sits at position r, so rows below the block's first key see nothing
    const int n_tiles_all = (a.n_q + 31) / 32;
    const int t_begin = a.q_pos ? 0 : min(blk0 / 32, n_tiles_all);
    const int tps = (n_tiles_all - t_begin + a.ns2 - 1) / a.ns2;
    const int t_first = t_begin + split * tps, n_tiles = max(min(tps, n_tiles_all - t_first), 0);
    const uint16_t *qb = reinterpret_cast<const uint16_t *>(a.q) + ((int64_t)b * a.n_q * a.n_q_heads + h) * D;
    const float *lrow = a.lse2 + ((int64_t)b * a.n_q_heads + h) * a.n_q_pad;
    u32x4 qreg[2][CH];
    float lreg[2][NS1];
    int32_t preg[2];
    const int ld_row = tid / (D / 8), ld_col = tid % (D / 8);
    auto load_tile = [&](int i, u32x4(&qr)[CH], float(&lr)[NS1], int32_t &pr) {
        const int t = t_first + max(min(i, n_tiles - 1), 0);
#pragma unroll
        for (int j = 0; j < CH; j++) {
            const int r = min(t * 32 + ld_row + j * (2048 / D), a.n_q - 1);
            qr[j] = *reinterpret_cast<const u32x4 *>(qb + (int64_t)r * a.n_q_heads * D + ld_col * 8);
        }
        if (tid < 32) {
            const int r = t * 32 + tid;
            const bool live = r < a.n_q;
            if (a.lse_in) {      // (only with NS1 = 1) natural logarithm -> the log2 units of the scores here
                lr[0] = live ? a.lse_in[((int64_t)b * a.n_q_heads + h) * a.n_q + r] * 1.4426950408889634f : -INFINITY;
            } else {
#pragma unroll
                for (int s = 0; s < NS1; s++)
                    lr[s] = live ? lrow[s * a.lse_split_stride + r] : -INFINITY;
            }
            pr = live ? (a.q_pos ? a.q_pos[(int64_t)b * a.n_q + r] : r) : -1;
        }
    };
    if (n_tiles > 0) {
        load_tile(0, qreg[0], lreg[0], preg[0]);
        load_tile(1, qreg[1], lreg[1], preg[1]);
    }
    float cs = 0.0f;
    auto step = [&](int i, u32x4(&qr)[CH], float(&lr)[NS1], int32_t &pr) {
        const int sidx = i & 1;
        uint16_t *st = lds[sidx];
#pragma unroll
        for (int j = 0; j < CH; j++)
            *reinterpret_cast<u32x4 *>(st + (ld_row + j * (2048 / D)) * STR + ld_col * 8) = qr[j];
        if (tid < 32) {
            // log-sum-exp over all keys from pass 1's per-split values; a single split is taken as it is
            float mx = lr[0];
#pragma unroll
            for (int s = 1; s < NS1; s++)
                mx = fmaxf(mx, lr[s]);
            float L = mx;
            if (NS1 > 1) {
                float sum = 0.0f;
#pragma unroll
                for (int s = 0; s < NS1; s++)
                    sum += __builtin_amdgcn_exp2f(lr[s] - (mx == -INFINITY ? 0.0f : mx));
                L = mx + log2f(sum);
            }
            // +inf makes the probability zero: padding rows and rows that see no key
            lds_lse[sidx][tid] = mx == -INFINITY ? INFINITY : L;
            lds_pos[sidx][tid] = pr;
        }
        __syncthreads();
        load_tile(i + 2, qr, lr, pr);
        const int r0 = (t_first + i) * 32;
        if (!a.q_pos && r0 + 31 < j0)
            return;   // causal: these rows sit before this wave's keys
        bf16x8 qfr[2][NKS];
#pragma unroll
        for (int ks = 0; ks < NKS; ks++) {
            qfr[0][ks] = *reinterpret_cast<const bf16x8 *>(st + c * STR + ks * 32 + g * 8);
            qfr[1][ks] = *reinterpret_cast<const bf16x8 *>(st + (16 + c) * STR + ks * 32 + g * 8);
        }
        const f32x4 L0 = *reinterpret_cast<const f32x4 *>(&lds_lse[sidx][g * 4]);
        const f32x4 L1 = *reinterpret_cast<const f32x4 *>(&lds_lse[sidx][16 + g * 4]);
        const int32_t *pp = &lds_pos[sidx][g * 4];
        f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < NKS; ks++) {
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qfr[0][ks], kf[ks], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qfr[1][ks], kf[ks], acc1, 0, 0, 0);
        }
        if (!a.q_pos && r0 >= j0 + 15) {
            // every row of the tile sits at or after every key of this wave: nothing to mask
#pragma unroll
            for (int r = 0; r < 4; r++) {
                cs += __builtin_amdgcn_exp2f(fmaf(acc0[r], a.scale_log2, -L0[r]));
                cs += __builtin_amdgcn_exp2f(fmaf(acc1[r], a.scale_log2, -L1[r]));
            }
        } else {
#pragma unroll
            for (int r = 0; r < 4; r++) {
                const float p0 = __builtin_amdgcn_exp2f(acc0[r] * a.scale_log2 - L0[r]);
                const float p1 = __builtin_amdgcn_exp2f(acc1[r] * a.scale_log2 - L1[r]);
                cs += key <= pp[r] ? p0 : 0.0f;
                cs += key <= pp[16 + r] ? p1 : 0.0f;
            }
        }
    };
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    {
        int i = 0;
        for (; i + 2 <= n_tiles; i += 2) {
            step(i, qreg[0], lreg[0], preg[0]);
            step(i + 1, qreg[1], lreg[1], preg[1]);
        }
        if (i < n_tiles)
            step(i, qreg[0], lreg[0], preg[0]);
    }
    cs += __shfl_xor(cs, 16);
    cs += __shfl_xor(cs, 32);
    if (g == 0 && key < vis_end)
        a.part[(((int64_t)b * a.n_q_heads + h) * a.ns2 + split) * a.vis_len + (key - a.vis_start)] = kvalid ? cs : 0.0f;
}

// ---- float32 tensors: plain vector-ALU versions of the two passes -------------------------------
__global__ __launch_bounds__(256) void scores_lse_f32_kernel(ScoreArgs a, int D)
{
    __shared__ float sq[256];
    __shared__ float red_m[4], red_l[4], red_t[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int kvh = h / (a.n_q_heads / a.n_kv_heads);
    const int pos = a.q_pos ? a.q_pos[(int64_t)b * a.n_q + row] : row;
    const float *q = reinterpret_cast<const float *>(a.q) + (((int64_t)b * a.n_q + row) * a.n_q_heads + h) * D;
    const float *kb = reinterpret_cast<const float *>(a.k) + ((int64_t)b * a.n_kv_heads + kvh) * a.s_max * D;
    if (tid < D)
        sq[tid] = q[tid];
    __syncthreads();
    float m = -INFINITY, l = 0.0f, tx = 0.0f;   // tx = sum_j exp(x_j - m) x_j (used for the entropy only)
    const int lim = min(pos + 1, a.n_keys);
    for (int key = tid; key < lim; key += 256) {
        const float *kr = kb + (int64_t)key * D;
        float dot = 0.0f;
        for (int d = 0; d < D; d++)
            dot += sq[d] * kr[d];
        float x = dot * a.scale;
        float mn = fmaxf(m, x);
        const float al = expf(m - mn), p = expf(x - mn);
        l = l * al + p;
        tx = tx * al + p * x;
        m = mn;
    }
    for (int off = 32; off > 0; off >>= 1) {
        float om = __shfl_xor(m, off), ol = __shfl_xor(l, off), ot = __shfl_xor(tx, off);
        float mn = fmaxf(m, om);
        float ms = (mn == -INFINITY) ? 0.0f : mn;
        l = l * expf(m - ms) + ol * expf(om - ms);
        tx = tx * expf(m - ms) + ot * expf(om - ms);
        m = mn;
    }
    if (lane == 0) {
        red_m[wave] = m;
        red_l[wave] = l;
        red_t[wave] = tx;
    }
    __syncthreads();
    if (tid == 0) {
        float mm = fmaxf(fmaxf(red_m[0], red_m[1]), fmaxf(red_m[2], red_m[3]));
        float ms = (mm == -INFINITY) ? 0.0f : mm;
        float ll = 0.0f, tt = 0.0f;
        for (int w = 0; w < 4; w++) {
            ll += red_l[w] * expf(red_m[w] - ms);
            tt += red_t[w] * expf(red_m[w] - ms);
        }
        const int64_t o = ((int64_t)b * a.n_q_heads + h) * a.n_q_pad + row;
        a.lse2[o] = ll > 0.0f ? mm + logf(ll) : INFINITY;   // natural log here
        if (a.ent_part)
            a.ent_part[o] = ll > 0.0f ? tt / ll : 0.0f;
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
        const float *lrow = a.lse_in ? a.lse_in + ((int64_t)b * a.n_q_heads + h) * a.n_q : a.lse2 + ((int64_t)b * a.n_q_heads + h) * a.n_q_pad;
        for (int row = 0; row < a.n_q; row++) {
            int pos = a.q_pos ? a.q_pos[(int64_t)b * a.n_q + row] : row;
            if (key > pos || lrow[row] == -INFINITY)   // (a caller's log-sum-exp of a row that sees no key)
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
// One workgroup of 1024 threads per sequence; everything lives in LDS.  Scores are mapped to unsigned keys
// whose order is the order of the floats; the k-th largest key is found by a most-significant-digit radix
// select (4 passes of 256-bin histograms built with integer LDS atomics, so nothing depends on scheduling).
// A token is kept iff its key is above the threshold, or equal to it and among the first `need` such tokens
// in position order (equal scores resolve toward the lower index); survivors are compacted in position order.
// Dynamic LDS: vis_len keys, then 256 histogram bins, 32 wave totals and 4 control words.
__device__ __forceinline__ uint32_t order_key(float x)
{
    x += 0.0f;   // -0 and +0 are equal scores: give them one key
    const uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(1024) void topk_keep_kernel(const float *part, int n_heads, const float *scores_in,
                                                         float *scores_out, int vis_start, int vis_len, int k,
                                                         int32_t *kept_idx)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    uint32_t *key = reinterpret_cast<uint32_t *>(smem_raw);
    int32_t *hist = reinterpret_cast<int32_t *>(key + vis_len);
    int32_t *wave_tot = hist + 256;   // [2][16]
    int32_t *ctl = wave_tot + 32;     // [0] chosen bin, [1] remaining need
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int j = tid; j < vis_len; j += 1024) {
        float x;
        if (scores_in) {
            x = scores_in[(int64_t)b * vis_len + j];
        } else {
            x = 0.0f;
            for (int h0 = 0; h0 < n_heads; h0 += 32) {   // up to 32 loads in flight, added in head order
                float t32[32];
#pragma unroll
                for (int i = 0; i < 32; i++)
                    t32[i] = h0 + i < n_heads ? part[((int64_t)b * n_heads + h0 + i) * vis_len + j] : 0.0f;
#pragma unroll
                for (int i = 0; i < 32; i++)
                    x += t32[i];
            }
        }
        if (scores_out)
            scores_out[(int64_t)b * vis_len + j] = x;
        key[j] = order_key(x);
    }
    if (k <= 0)
        return;
    // ---- radix select of the k-th largest key
    uint32_t prefix = 0, mask = 0;
    int need = k;
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256)
            hist[tid] = 0;
        __syncthreads();
        for (int j = tid; j < vis_len; j += 1024) {
            const uint32_t u = key[j];
            if ((u & mask) == prefix)
                atomicAdd(&hist[(u >> shift) & 255u], 1);
        }
        __syncthreads();
        if (wave == 0) {
            // lane l owns bins 4l..4l+3; walk down from the top bin until `need` keys are covered
            int c4[4], tot = 0;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                c4[i] = hist[4 * lane + i];
                tot += c4[i];
            }
            // suffix scan over lanes: keys in bins owned by higher lanes
            int incl = tot;
            for (int off = 1; off < 64; off <<= 1) {
                int v = __shfl_down(incl, off);
                if (lane + off < 64)
                    incl += v;
            }
            const int above = incl - tot;
            if (above < need && need <= above + tot) {
                int rem = need - above, bin = 4 * lane + 3;
#pragma unroll
                for (int i = 3; i >= 0; i--) {
                    if (rem > 0) {
                        bin = 4 * lane + i;
                        if (rem <= c4[i]) {
                            ctl[0] = bin;
                            ctl[1] = rem;
                            rem = 0;
                        } else {
                            rem -= c4[i];
                        }
                    }
                }
            }
        }
        __syncthreads();
        prefix |= (uint32_t)ctl[0] << shift;
        mask |= 255u << shift;
        need = ctl[1];
        __syncthreads();
    }
    const uint32_t tau = prefix;   // key of the k-th largest; `need` of the keys equal to it are kept
    // ---- ordered compaction: thread t owns the contiguous slice [t*per, (t+1)*per)
    const int per = (vis_len + 1023) / 1024;
    const int lo = min(tid * per, vis_len), hi = min(lo + per, vis_len);
    int gt = 0, eq = 0;
    for (int j = lo; j < hi; j++) {
        const uint32_t u = key[j];
        gt += u > tau;
        eq += u == tau;
    }
    int gi = gt, ei = eq;   // inclusive scans inside the wave
    for (int off = 1; off < 64; off <<= 1) {
        int a = __shfl_up(gi, off), c = __shfl_up(ei, off);
        if (lane >= off) {
            gi += a;
            ei += c;
        }
    }
    if (lane == 63) {
        wave_tot[wave] = gi;
        wave_tot[16 + wave] = ei;
    }
    __syncthreads();
    int g_before = gi - gt, e_before = ei - eq;
    for (int w = 0; w < wave; w++) {
        g_before += wave_tot[w];
        e_before += wave_tot[16 + w];
    }
    int out = g_before + min(e_before, need);
    for (int j = lo; j < hi; j++) {
        const uint32_t u = key[j];
        bool keep = u > tau;
        if (u == tau) {
            keep = e_before < need;
            e_before++;
        }
        if (keep)
            kept_idx[(int64_t)b * k + out++] = vis_start + j;
    }
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

template <int D>
void launch_colsum(int ns1, dim3 grid, hipStream_t st, const ScoreArgs &a)
{
    switch (ns1) {
    case 1:  hipLaunchKernelGGL((scores_colsum_bf16_kernel<D, 1>), grid, dim3(256), 0, st, a); break;
    case 2:  hipLaunchKernelGGL((scores_colsum_bf16_kernel<D, 2>), grid, dim3(256), 0, st, a); break;
    case 4:  hipLaunchKernelGGL((scores_colsum_bf16_kernel<D, 4>), grid, dim3(256), 0, st, a); break;
    default: hipLaunchKernelGGL((scores_colsum_bf16_kernel<D, 8>), grid, dim3(256), 0, st, a); break;
    }
}

struct CompressPlan {
    int n_q_pad, ns1, ns2;
    size_t off_lse, off_part, total;
};

// Splits of the streamed axis of a score pass: enough that a workgroup walks about 8 tiles, at most 8 splits,
// and only while the grid stays near 2048 workgroups (beyond that the chip is busy anyway and more, shorter
// workgroups only add start-up cost).
int score_splits(int64_t grid, int tiles)
{
    int ns = ceil_div(tiles, 8);
    if (ns > 8)
        ns = 8;
    const int64_t room = 2048 / (grid > 0 ? grid : 1);
    if (ns > room)
        ns = (int)room;
    int pow2 = 1;   // 1, 2, 4 or 8: pass 2 is compiled for these counts of pass-1 splits
    while (pow2 * 2 <= ns)
        pow2 *= 2;
    return pow2;
}

CompressPlan compress_plan(int batch, int n_heads, int n_q, int vis_len, int dtype)
{
    CompressPlan p;
    p.n_q_pad = (n_q + 15) / 16 * 16;
    p.ns1 = p.ns2 = 1;
    if (dtype == DREAM_BF16) {
        p.ns1 = score_splits((int64_t)ceil_div(n_q, 64) * n_heads * batch, ceil_div(n_q, 32));
        p.ns2 = score_splits((int64_t)ceil_div(vis_len > 0 ? vis_len : 1, 64) * n_heads * batch, ceil_div(n_q, 32));
    }
    p.off_lse = DREAM_WORKSPACE_MIN_BYTES;
    p.off_part = align_up(p.off_lse + (size_t)p.ns1 * batch * n_heads * p.n_q_pad * sizeof(float), 256);
    p.total = align_up(p.off_part + (size_t)p.ns2 * batch * n_heads * (vis_len > 0 ? vis_len : 1) * sizeof(float), 256);
    return p;
}

// the selection kernel's dynamic LDS holds up to DREAM_MAX_VISUAL scores: raise its limit once
int ensure_topk_lds(const char *who)
{
    static std::atomic<bool> attr_set{false};   // (two threads may both set the attribute once: harmless)
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&topk_keep_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                DREAM_MAX_VISUAL * 4 + (256 + 32 + 4) * 4) != hipSuccess)
            return fail(DREAM_ERR_HIP, "%s: cannot reserve LDS for the selection kernel", who);
        attr_set = true;
    }
    return DREAM_OK;
}

}  // namespace

namespace dream {
int compress_init() { return ensure_topk_lds("dream_init"); }
}  // namespace dream

extern "C" {

size_t dream_visual_compress_workspace(const dream_attn_desc *desc, int32_t n_q, int32_t vis_len)
{
    if (!desc || desc->batch < 1 || desc->n_q_heads < 1 || n_q < 1)
        return DREAM_WORKSPACE_MIN_BYTES;
    return compress_plan(desc->batch, desc->n_q_heads, n_q, vis_len, desc->dtype).total;
}

int dream_visual_compress(const dream_attn_desc *desc, const void *q, const int32_t *q_pos, int32_t n_q,
                          const void *k_cache, int32_t n_keys, int32_t vis_start, int32_t vis_len,
                          int32_t keep_num, int32_t keep_den, const float *scores_in, const float *row_lse_in,
                          float *scores_out, int32_t *kept_idx, int32_t *n_kept_host, const void *gather_src, int64_t n_rows_src,
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
        CompressPlan p = compress_plan(desc->batch, desc->n_q_heads, n_q, vis_len, desc->dtype);
        if (!workspace || workspace_bytes < p.total)
            return fail(DREAM_ERR_WORKSPACE, "%s: workspace of %zu bytes, %zu needed", who, workspace_bytes, p.total);
        ScoreArgs a;
        a.q = q; a.k = k_cache; a.q_pos = q_pos;
        a.lse2 = reinterpret_cast<float *>(static_cast<char *>(workspace) + p.off_lse);
        a.part = reinterpret_cast<float *>(static_cast<char *>(workspace) + p.off_part);
        a.n_q = n_q; a.n_q_pad = p.n_q_pad; a.n_keys = n_keys;
        a.ns1 = row_lse_in ? 1 : p.ns1; a.ns2 = p.ns2; a.ent_part = nullptr; a.lse_in = row_lse_in;
        a.lse_split_stride = (int64_t)desc->batch * desc->n_q_heads * p.n_q_pad;
        a.n_q_heads = desc->n_q_heads; a.n_kv_heads = desc->n_kv_heads;
        a.vis_start = vis_start; a.vis_len = vis_len; a.s_max = desc->s_max;
        a.scale = desc->scale != 0.0f ? desc->scale : 1.0f / sqrtf((float)desc->head_dim);
        a.scale_log2 = a.scale * 1.4426950408889634f;
        if (desc->dtype == DREAM_BF16) {
            if ((int64_t)desc->batch * (p.ns1 > p.ns2 ? p.ns1 : p.ns2) > 65535 || ceil_div(n_q, 64) > 65535)
                return fail(DREAM_ERR_UNSUPPORTED, "%s: batch %d or n_q %d too large for the score grids", who, desc->batch, n_q);
            dim3 g1(desc->n_q_heads, ceil_div(n_q, 64), desc->batch * p.ns1), g2(desc->n_q_heads, ceil_div(vis_len, 64), desc->batch * p.ns2);
            // pass 1 (the rows' log-sum-exps) only when the caller does not bring them
            switch (desc->head_dim) {
            case 64:
                if (!row_lse_in) {
                    hipLaunchKernelGGL((scores_lse_bf16_kernel<64, false>), g1, dim3(256), 0, st, a);
                }
                launch_colsum<64>(a.ns1, g2, st, a);
                break;
            case 128:
                if (!row_lse_in) {
                    hipLaunchKernelGGL((scores_lse_bf16_kernel<128, false>), g1, dim3(256), 0, st, a);
                }
                launch_colsum<128>(a.ns1, g2, st, a);
                break;
            default:
                if (!row_lse_in) {
                    hipLaunchKernelGGL((scores_lse_bf16_kernel<256, false>), g1, dim3(256), 0, st, a);
                }
                launch_colsum<256>(a.ns1, g2, st, a);
                break;
            }
        } else {
            if (n_q > 65535 * 1)
                return fail(DREAM_ERR_UNSUPPORTED, "%s: too many rows for the float32 path", who);
            if (!row_lse_in) {
                hipLaunchKernelGGL(scores_lse_f32_kernel, dim3(n_q, desc->n_q_heads, desc->batch), dim3(256), 0, st, a, desc->head_dim);
            }
            hipLaunchKernelGGL(scores_colsum_f32_kernel, dim3(ceil_div(vis_len, 64), desc->n_q_heads, desc->batch), dim3(64), 0, st, a, desc->head_dim);
        }
        int rc = check_launch("visual score kernels");
        if (rc)
            return rc;
        part = a.part;
        n_heads = desc->n_q_heads * p.ns2;
    }
    if (n_kept_host)
        *n_kept_host = k;
    if (vis_len > 0 && (k > 0 || scores_out)) {
        size_t lds = (size_t)vis_len * 4 + (256 + 32 + 4) * 4;
        if (int rc = ensure_topk_lds(who))
            return rc;
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

size_t dream_attention_entropy_workspace(const dream_attn_desc *desc, int32_t n_q)
{
    if (!desc || desc->batch < 1 || desc->n_q_heads < 1 || n_q < 1)
        return DREAM_WORKSPACE_MIN_BYTES;
    const CompressPlan p = compress_plan(desc->batch, desc->n_q_heads, n_q, 0, desc->dtype);
    const size_t part = align_up((size_t)p.ns1 * desc->batch * desc->n_q_heads * p.n_q_pad * sizeof(float), 256);
    const size_t sums = align_up((size_t)desc->batch * ceil_div((int64_t)desc->n_q_heads * n_q, 256) * sizeof(float), 256);
    return DREAM_WORKSPACE_MIN_BYTES + 2 * part + sums;
}

int dream_attention_entropy(const dream_attn_desc *desc, const void *q, const int32_t *q_pos, int32_t n_q, const void *k_cache,
                            int32_t n_keys, float *row_entropy, float *ae, void *workspace, size_t workspace_bytes, void *stream)
{
    const char *who = "dream_attention_entropy";
    if (!desc || !q || !k_cache || !ae)
        return fail(DREAM_ERR_INVALID_ARG, "%s: NULL argument", who);
    if (desc->batch < 1 || desc->batch > 65535)
        return fail(DREAM_ERR_INVALID_ARG, "%s: batch %d outside [1, 65535]", who, desc->batch);
    if (desc->dtype != DREAM_F32 && desc->dtype != DREAM_BF16)
        return fail(DREAM_ERR_INVALID_ARG, "%s: unknown dtype %d", who, desc->dtype);
    if (desc->n_q_heads < 1 || desc->n_kv_heads < 1 || desc->n_q_heads % desc->n_kv_heads || desc->n_q_heads > 65535)
        return fail(DREAM_ERR_INVALID_ARG, "%s: bad head counts %d / %d", who, desc->n_q_heads, desc->n_kv_heads);
    if (desc->head_dim != 64 && desc->head_dim != 128 && desc->head_dim != 256)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: head_dim %d not in {64,128,256}", who, desc->head_dim);
    if (n_q < 1 || n_keys < 1 || n_keys > desc->s_max)
        return fail(DREAM_ERR_INVALID_ARG, "%s: need n_q >= 1 and 1 <= n_keys <= s_max", who);
    if (!q_pos && n_q > n_keys)
        return fail(DREAM_ERR_INVALID_ARG, "%s: %d rows at positions 0..n_q-1 but only %d keys", who, n_q, n_keys);
    const CompressPlan p = compress_plan(desc->batch, desc->n_q_heads, n_q, 0, desc->dtype);
    const size_t part = align_up((size_t)p.ns1 * desc->batch * desc->n_q_heads * p.n_q_pad * sizeof(float), 256);
    const int n_blocks = ceil_div((int64_t)desc->n_q_heads * n_q, 256);
    const size_t need = DREAM_WORKSPACE_MIN_BYTES + 2 * part + align_up((size_t)desc->batch * n_blocks * sizeof(float), 256);
    if (!workspace || workspace_bytes < need)
        return fail(DREAM_ERR_WORKSPACE, "%s: workspace of %zu bytes, %zu needed", who, workspace_bytes, need);
    hipStream_t st = as_stream(stream);
    ScoreArgs a;
    a.q = q; a.k = k_cache; a.q_pos = q_pos;
    a.lse2 = reinterpret_cast<float *>(static_cast<char *>(workspace) + DREAM_WORKSPACE_MIN_BYTES);
    a.lse_in = nullptr;
    a.ent_part = reinterpret_cast<float *>(static_cast<char *>(workspace) + DREAM_WORKSPACE_MIN_BYTES + part);
    a.part = nullptr;
    a.n_q = n_q; a.n_q_pad = p.n_q_pad; a.n_keys = n_keys;
    a.n_q_heads = desc->n_q_heads; a.n_kv_heads = desc->n_kv_heads;
    a.vis_start = 0; a.vis_len = 0; a.s_max = desc->s_max;
    a.ns1 = p.ns1; a.ns2 = 1;
    a.lse_split_stride = (int64_t)desc->batch * desc->n_q_heads * p.n_q_pad;
    a.scale = desc->scale != 0.0f ? desc->scale : 1.0f / sqrtf((float)desc->head_dim);
    a.scale_log2 = a.scale * 1.4426950408889634f;
    if (desc->dtype == DREAM_BF16) {
        if ((int64_t)desc->batch * p.ns1 > 65535 || ceil_div(n_q, 64) > 65535)
            return fail(DREAM_ERR_UNSUPPORTED, "%s: batch %d or n_q %d too large for the score grid", who, desc->batch, n_q);
        dim3 g1(desc->n_q_heads, ceil_div(n_q, 64), desc->batch * p.ns1);
        switch (desc->head_dim) {
        case 64:  hipLaunchKernelGGL((scores_lse_bf16_kernel<64, true>), g1, dim3(256), 0, st, a); break;
        case 128: hipLaunchKernelGGL((scores_lse_bf16_kernel<128, true>), g1, dim3(256), 0, st, a); break;
        default:  hipLaunchKernelGGL((scores_lse_bf16_kernel<256, true>), g1, dim3(256), 0, st, a); break;
        }
    } else {
        if (n_q > 65535)
            return fail(DREAM_ERR_UNSUPPORTED, "%s: too many rows for the float32 path", who);
        hipLaunchKernelGGL(scores_lse_f32_kernel, dim3(n_q, desc->n_q_heads, desc->batch), dim3(256), 0, st, a, desc->head_dim);
    }
    int rc = check_launch("entropy score kernel");
    if (rc)
        return rc;
    float *block_sum = reinterpret_cast<float *>(static_cast<char *>(workspace) + DREAM_WORKSPACE_MIN_BYTES + 2 * part);
    hipLaunchKernelGGL(entropy_rows_kernel, dim3(n_blocks, desc->batch), dim3(256), 0, st, a, desc->dtype == DREAM_BF16 ? 1 : 0, row_entropy,
                       block_sum);
    hipLaunchKernelGGL(entropy_mean_kernel, dim3(desc->batch), dim3(64), 0, st, block_sum, n_blocks, desc->n_q_heads * n_q, ae);
    return check_launch("entropy reduction kernels");
}

}  // extern "C"
