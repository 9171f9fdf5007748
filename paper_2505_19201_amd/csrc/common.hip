// Error reporting, launch-shape overrides, the read-only measurement kernel and tree validation shared by all entry points.
#include "common.h"
#include "dream_tuning.h"
#include <atomic>
#include <string.h>

namespace dream {

static thread_local char g_error[512] = "";
static std::atomic<int> g_kv_splits{0};
static std::atomic<int> g_q_tiles{0};
static std::atomic<int> g_tile_waves{0};

char *error_buffer() { return g_error; }

int fail(int status, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof g_error, fmt, ap);
    va_end(ap);
    return status;
}

int check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail(DREAM_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return DREAM_OK;
}

int kv_splits_override() { return g_kv_splits.load(std::memory_order_relaxed); }
int q_tiles_override() { return g_q_tiles.load(std::memory_order_relaxed); }
int tile_waves_override() { return g_tile_waves.load(std::memory_order_relaxed); }

// Reads n16 16-byte words once, grid-stride, and folds them into one word per thread; the fold is stored only
// if it equals a value the caller does not expect, which keeps the loads alive without a write stream.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4 *src, size_t n16, uint32_t *sink, uint32_t never)
{
    u32x4 acc = {0u, 0u, 0u, 0u};
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        acc ^= __builtin_nontemporal_load(src + i);   // read once: the hint keeps the stream from thrashing L2
    const uint32_t fold = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (fold == never)
        *sink = fold;
}

}  // namespace dream

using namespace dream;

extern "C" {

const char *dream_last_error(void) { return error_buffer(); }

void dream_set_kv_splits(int32_t n_splits) { dream::g_kv_splits.store(n_splits < 0 ? 0 : n_splits, std::memory_order_relaxed); }

void dream_set_q_tiles(int32_t q_tiles) { dream::g_q_tiles.store(q_tiles < 0 ? 0 : q_tiles, std::memory_order_relaxed); }

void dream_set_tile_waves(int32_t waves) { dream::g_tile_waves.store(waves == 4 || waves == 8 ? waves : 0, std::memory_order_relaxed); }

int dream_init(void)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess)
        return fail(DREAM_ERR_HIP, "dream_init: no usable HIP device");
    int rc = attn_init();
    if (!rc)
        rc = compress_init();
    if (!rc)
        rc = dream_accept_static_init();
    return rc;
}

int dream_stream_read(const void *src, size_t bytes, void *sink, void *stream)
{
    if (!src || !sink || bytes < 16 || (reinterpret_cast<uintptr_t>(src) & 15))
        return fail(DREAM_ERR_INVALID_ARG, "dream_stream_read: need a 16-byte aligned source of at least 16 bytes and a sink");
    const size_t n16 = bytes / 16;
    size_t wgs = (n16 + 255) / 256;
    if (wgs > 2048)
        wgs = 2048;   // 8 workgroups per CU, grid-stride beyond that
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)wgs), dim3(256), 0, as_stream(stream),
                       reinterpret_cast<const u32x4 *>(src), n16, reinterpret_cast<uint32_t *>(sink), 0x9e3779b9u);
    return check_launch("dream_stream_read");
}

int dream_tree_validate_host(const int32_t *parent_host, int32_t n_tree, int32_t *max_depth_out)
{
    if (!parent_host || n_tree < 1)
        return fail(DREAM_ERR_INVALID_ARG, "dream_tree_validate_host: NULL parent array or n_tree < 1");
    if (parent_host[0] != -1)
        return fail(DREAM_ERR_INVALID_ARG, "dream_tree_validate_host: parent[0] is %d, expected -1", parent_host[0]);
    int max_depth = 0;
    // depth of node i fits in the slot of an int array only for small trees; recompute by walking, trees are tiny
    for (int i = 1; i < n_tree; i++) {
        if (parent_host[i] < 0 || parent_host[i] >= i)
            return fail(DREAM_ERR_INVALID_ARG, "dream_tree_validate_host: parent[%d] = %d is not in [0, %d)", i, parent_host[i], i);
        int d = 0;
        for (int a = i; a > 0; a = parent_host[a])
            d++;
        if (d > max_depth)
            max_depth = d;
    }
    if (max_depth_out)
        *max_depth_out = max_depth;
    return DREAM_OK;
}

}  // extern "C"
