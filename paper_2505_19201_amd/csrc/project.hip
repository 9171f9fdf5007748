// dream_project_rows: the linear maps of Eq. 1 (Section 3.1), Q = E W_Q, K = S W_K, V = S W_V, for the few
// feature rows a decode step adds (the frontier's draft features, the accepted tokens' target features), with
// the result written straight to where attention reads it: head-split rows of a K/V cache
// [B, H, s_max, D] at row_base[b] + row_index[b, r] (cache append), or a dense [B, R, H, D] tensor (queries).
//
// M = B*R is small (<= a few hundred) and the weight matrix [N, hidden] is large, so the call is bound by
// streaming the weights once from HBM.  One workgroup owns 16 output features (16 weight rows, contiguous in
// memory); its 4 waves split the hidden dimension, each computing C^T[n][m] += W[n][k] X[m][k] with
// v_mfma_f32_16x16x32_bf16 (A = weight rows, B = feature rows).  With at most 16 feature rows (the paper's
// shapes) a wave fetches 256 contiguous bytes of each row at a time and passes them through a private LDS area
// to reach the operand layout: nobody else reads those bytes, but an operand-layout load touches 16 rows x 64
// bytes per instruction, half cache lines, and measures 10-13 % slower.  With more rows (up to 4 tiles of 16 at
// a time) the operands are loaded directly.  The 4 partial tiles are summed through LDS in wave order and the
// rows are rounded to bf16 and scattered.  Roofline: HBM, N*hidden*2 weight bytes per call.
#include "common.h"

using namespace dream;

namespace {

constexpr int NWAVE = 4;   // (8 waves measured 5-8 % slower on the narrower maps, 2 no faster)
static_assert(NWAVE >= 4, "the final reduction gives each of up to 4 feature-row tiles to one wave");

__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

struct ProjJob {
    const uint16_t *x, *w;
    uint16_t *out;
    const int32_t *row_base, *row_index;
    int32_t n_heads;
    int32_t tile_end;    // one past this job's last workgroup (jobs occupy consecutive workgroup ranges)
};

struct ProjArgs {
    ProjJob job[DREAM_MAX_PROJ_JOBS];
    int32_t n_jobs;
    int32_t n_rows;      // R: rows per sequence
    int32_t m_total;     // B * R
    int32_t hidden, head_dim;
    int64_t s_max;       // cache mode only
};

// MT: tiles of 16 feature rows handled per pass (1, 2 or 4)
template <int MT>
__global__ __launch_bounds__(64 * NWAVE) void project_kernel(ProjArgs args)
{
    // the job this workgroup belongs to (uniform: scalar selects)
    int ji = 0;
    for (int j = 0; j + 1 < args.n_jobs; j++)
        ji += (int)blockIdx.x >= args.job[j].tile_end;
    struct {
        const uint16_t *x, *w;
        uint16_t *out;
        const int32_t *row_base, *row_index;
        int32_t n_heads, n_rows, m_total, hidden, head_dim;
        int64_t s_max;
    } a;
    int tile0 = 0;
    a.x = args.job[0].x; a.w = args.job[0].w; a.out = args.job[0].out; a.row_base = args.job[0].row_base;
    a.row_index = args.job[0].row_index; a.n_heads = args.job[0].n_heads;
#pragma unroll
    for (int j = 1; j < DREAM_MAX_PROJ_JOBS; j++)
        if (ji == j) {
            a.x = args.job[j].x; a.w = args.job[j].w; a.out = args.job[j].out; a.row_base = args.job[j].row_base;
            a.row_index = args.job[j].row_index; a.n_heads = args.job[j].n_heads;
            tile0 = args.job[j - 1].tile_end;
        }
    a.n_rows = args.n_rows; a.m_total = args.m_total; a.hidden = args.hidden; a.head_dim = args.head_dim; a.s_max = args.s_max;

    __shared__ __attribute__((aligned(16))) float s_part[NWAVE][MT][64][4];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, g = lane >> 4;
    const int n0 = ((int)blockIdx.x - tile0) * 16;
    const int K = a.hidden, kw = K / NWAVE;          // this wave's slice of the hidden dimension
    const uint16_t *wrow = a.w + (int64_t)(n0 + c) * K + wave * kw + g * 8;
    const int h = n0 / a.head_dim, d0 = n0 % a.head_dim;

    for (int m0 = 0; m0 < a.m_total; m0 += 16 * MT) {
        f32x4 acc[MT];
        const uint16_t *xrow[MT];
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
            const int m = min(m0 + mt * 16 + c, a.m_total - 1);   // padding rows repeat the last row; never stored
            xrow[mt] = a.x + (int64_t)m * K + wave * kw + g * 8;
        }
        if (MT == 1) {
            // Rows are fetched 256 contiguous bytes at a time (4 rows per load instruction: full cache lines) into
            // a wave-private LDS area and read back in operand layout; loading the operands directly would make
            // every instruction touch 16 rows x 64 bytes.
            constexpr int SS = 128, RSTR = SS + 8;             // elements of a row per super-step; padded LDS row stride
            constexpr int LPR = SS / 8, RPI = 64 / LPR, NI = 16 / RPI;   // lanes per row, rows per instruction, instructions per 16 rows
            __shared__ __attribute__((aligned(16))) uint16_t s_stage[NWAVE][2][16 * RSTR];
            uint16_t *lw = s_stage[wave][0], *lx = s_stage[wave][1];
            const int lrow = lane / LPR, lcol = (lane % LPR) * 8;
            const int n_ss = (kw + SS - 1) / SS;
            const uint16_t *wsrc = a.w + (int64_t)n0 * K + wave * kw;
            const uint16_t *xsrc = a.x + wave * kw;
            const int xj = min((a.m_total - m0 + RPI - 1) / RPI, NI);
            auto issue = [&](int s, u32x4 (&wr)[NI], u32x4 (&xr)[NI]) {
                s = min(s, n_ss - 1);                              // the prefetch past the end re-reads and is dropped
                const int nvalid = min(SS, kw - s * SS);
                const int col = s * SS + (lcol < nvalid ? lcol : 0);
#pragma unroll
                for (int j = 0; j < NI; j++) {
                    wr[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wsrc + (int64_t)(j * RPI + lrow) * K + col));   // weights: read once
                    if (j < xj) {   // feature rows are fetched RPI at a time, only as many as exist
                        const int m = min(m0 + j * RPI + lrow, a.m_total - 1);
                        xr[j] = *reinterpret_cast<const u32x4 *>(xsrc + (int64_t)m * K + col);
                    }
                }
            };
            // one super-step: registers -> LDS, request the super-step that reuses these registers, multiply
            auto step = [&](int s, u32x4 (&wr)[NI], u32x4 (&xr)[NI]) {
#pragma unroll
                for (int j = 0; j < NI; j++) {
                    *reinterpret_cast<u32x4 *>(lw + (j * RPI + lrow) * RSTR + lcol) = wr[j];
                    if (j < xj)     // (the other LDS rows feed output columns that are never stored)
                        *reinterpret_cast<u32x4 *>(lx + (j * RPI + lrow) * RSTR + lcol) = xr[j];
                }
                issue(s + 1, wr, xr);
                wave_lds_fence();
                const int nvalid = min(SS, kw - s * SS);
#pragma unroll
                for (int ks = 0; ks < SS / 32; ks++) {
                    if (ks * 32 < nvalid) {
                        const bf16x8 af = *reinterpret_cast<const bf16x8 *>(lw + c * RSTR + ks * 32 + g * 8);
                        const bf16x8 bfr = *reinterpret_cast<const bf16x8 *>(lx + c * RSTR + ks * 32 + g * 8);
                        acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, bfr, acc[0], 0, 0, 0);
                    }
                }
                wave_lds_fence();
            };
            u32x4 wr[NI], xr[NI];
            issue(0, wr, xr);
            for (int s = 0; s < n_ss; s++)
                step(s, wr, xr);
        } else
        {
        constexpr int U = 8 / MT;        // k-steps whose loads are in flight together
            for (int k = 0; k < kw; k += 32 * U) {
                bf16x8 wf[U], xf[U][MT];
#pragma unroll
                for (int u = 0; u < U; u++) {
                    const int kk = min(k + 32 * u, kw - 32);            // (kw is a multiple of 32; a short tail re-reads and is skipped below)
                    wf[u] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8 *>(wrow + kk));   // weights: read once
#pragma unroll
                    for (int mt = 0; mt < MT; mt++)
                        xf[u][mt] = *reinterpret_cast<const bf16x8 *>(xrow[mt] + kk);
                }
#pragma unroll
                for (int u = 0; u < U; u++) {
                    if (k + 32 * u < kw) {
#pragma unroll
                        for (int mt = 0; mt < MT; mt++)
                            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[u], xf[u][mt], acc[mt], 0, 0, 0);
                    }
                }
            }
        }
        // sum the waves' partial tiles in wave order; thread (wave, lane) finishes tile mt = wave % MT ... spread evenly
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
            *reinterpret_cast<f32x4 *>(s_part[wave][mt][lane]) = acc[mt];
        __syncthreads();
        if (wave < MT) {
            const int mt = wave;
            f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < NWAVE; w++)
                sum += *reinterpret_cast<const f32x4 *>(s_part[w][mt][lane]);
            const int m = m0 + mt * 16 + c;                          // lane holds outputs n0 + g*4 .. +3 of feature row m
            if (m < a.m_total) {
                const int b = m / a.n_rows, r = m - b * a.n_rows;
                bf16x4 o;
#pragma unroll
                for (int i = 0; i < 4; i++)
                    o[i] = (__bf16)sum[i];
                int64_t dst;
                if (a.row_base) {
                    const int row = a.row_base[b] + (a.row_index ? a.row_index[(int64_t)b * a.n_rows + r] : r);
                    dst = row >= 0 && row < a.s_max ? (((int64_t)b * a.n_heads + h) * a.s_max + row) * a.head_dim + d0 + g * 4 : -1;
                } else {
                    dst = (((int64_t)b * a.n_rows + r) * a.n_heads + h) * a.head_dim + d0 + g * 4;
                }
                if (dst >= 0)                                        // a row outside the cache is dropped, never written
                    *reinterpret_cast<bf16x4 *>(a.out + dst) = o;
            }
        }
    }
}

}  // namespace

extern "C" {

int dream_project_rows_multi(const dream_attn_desc *desc, const dream_proj_job *jobs, int32_t n_jobs, int32_t n_rows, int32_t hidden,
                             void *stream)
{
    const char *who = "dream_project_rows";
    if (!desc || !jobs)
        return fail(DREAM_ERR_INVALID_ARG, "%s: NULL argument", who);
    if (n_jobs < 1 || n_jobs > DREAM_MAX_PROJ_JOBS)
        return fail(DREAM_ERR_INVALID_ARG, "%s: %d jobs outside [1, %d]", who, n_jobs, DREAM_MAX_PROJ_JOBS);
    if (desc->dtype != DREAM_BF16)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: bf16 tensors only", who);
    if (desc->batch < 1 || n_rows < 1 || (int64_t)desc->batch * n_rows > (1 << 20))
        return fail(DREAM_ERR_INVALID_ARG, "%s: batch and n_rows must be positive, batch * n_rows at most 2^20", who);
    if (desc->head_dim < 16 || desc->head_dim % 16)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: head_dim %d is not a positive multiple of 16", who, desc->head_dim);
    if (hidden < 256 || hidden % 256)
        return fail(DREAM_ERR_UNSUPPORTED, "%s: hidden %d is not a positive multiple of 256", who, hidden);
    ProjArgs a = {};
    int64_t tiles = 0;
    for (int j = 0; j < n_jobs; j++) {
        const dream_proj_job &jb = jobs[j];
        if (!jb.x || !jb.w || !jb.out)
            return fail(DREAM_ERR_INVALID_ARG, "%s: NULL tensor in job %d", who, j);
        if (jb.n_heads < 1)
            return fail(DREAM_ERR_INVALID_ARG, "%s: n_heads of job %d must be positive", who, j);
        if (jb.row_base && desc->s_max < 1)
            return fail(DREAM_ERR_INVALID_ARG, "%s: cache output needs s_max", who);
        if (!jb.row_base && jb.row_index)
            return fail(DREAM_ERR_INVALID_ARG, "%s: row_index without row_base in job %d", who, j);
        if ((reinterpret_cast<uintptr_t>(jb.x) | reinterpret_cast<uintptr_t>(jb.w) | reinterpret_cast<uintptr_t>(jb.out)) & 15)
            return fail(DREAM_ERR_INVALID_ARG, "%s: x, w and out must be 16-byte aligned", who);
        tiles += (int64_t)jb.n_heads * desc->head_dim / 16;
        if (tiles > (1 << 24))
            return fail(DREAM_ERR_UNSUPPORTED, "%s: more than 2^24 tiles of 16 output features", who);
        a.job[j].x = static_cast<const uint16_t *>(jb.x); a.job[j].w = static_cast<const uint16_t *>(jb.w);
        a.job[j].out = static_cast<uint16_t *>(jb.out); a.job[j].row_base = jb.row_base; a.job[j].row_index = jb.row_index;
        a.job[j].n_heads = jb.n_heads; a.job[j].tile_end = (int32_t)tiles;
    }
    a.n_jobs = n_jobs; a.n_rows = n_rows; a.m_total = desc->batch * n_rows; a.hidden = hidden; a.head_dim = desc->head_dim;
    a.s_max = desc->s_max;
    const dim3 grid((unsigned)tiles);
    hipStream_t st = as_stream(stream);
    if (a.m_total <= 16)
        hipLaunchKernelGGL(project_kernel<1>, grid, dim3(64 * NWAVE), 0, st, a);
    else if (a.m_total <= 32)
        hipLaunchKernelGGL(project_kernel<2>, grid, dim3(64 * NWAVE), 0, st, a);
    else
        hipLaunchKernelGGL(project_kernel<4>, grid, dim3(64 * NWAVE), 0, st, a);
    return check_launch("project_kernel");
}

int dream_project_rows(const dream_attn_desc *desc, const void *x, int32_t n_rows, int32_t hidden, const void *w, int32_t n_heads,
                       const int32_t *row_base, const int32_t *row_index, void *out, void *stream)
{
    dream_proj_job job = {x, w, n_heads, row_base, row_index, out};
    return dream_project_rows_multi(desc, &job, 1, n_rows, hidden, stream);
}

}  // extern "C"
