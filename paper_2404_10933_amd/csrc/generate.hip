// Seeded synthetic inputs generated on the device (the draws themselves are in
// grid_draws.h), and the small host-only entry points of the library.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/llmem.h"
#include "grid_draws.h"

namespace llmem {

typedef unsigned long long u64;

static thread_local char g_error_text[256] = "";
void set_hip_error(hipError_t e)
{
    snprintf(g_error_text, sizeof(g_error_text), "HIP error: %s", hipGetErrorString(e));
}
const char *last_hip_error();   // the estimator keeps its own buffer

// grid_id 6: the queries of the method decision; tp_out is only written for that grid
__global__ __launch_bounds__(256) void grid_kernel(int grid_id, u64 seed, long long first, long long n,
                                                   llmem_configs c, uint8_t *tp_out)
{
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n) return;
    const DrawnConfig g = draw_config(grid_id, seed, (u64)(first + t));
    if (grid_id == 6) tp_out[t] = (uint8_t)g.tp_n;
    c.arch_id[t] = (uint8_t)g.arch_id; c.h[t] = g.h; c.L[t] = (uint16_t)g.L; c.n_heads[t] = (uint16_t)g.n_heads;
    c.n_kv[t] = (uint16_t)g.n_kv; c.ffn[t] = g.ffn; c.V[t] = g.V; c.P[t] = g.P; c.bs[t] = (uint16_t)g.bs;
    c.sl[t] = (uint16_t)g.sl; c.method[t] = (uint8_t)g.method; c.d[t] = (uint8_t)g.d; c.chunk_k[t] = (int8_t)g.chunk_k;
    c.flags[t] = (uint8_t)g.flags;
}

// ---- explicit event lists ---------------------------------------------------------
// One list = one iteration: a forward pass of n_fwd operators (n_fwd in [2800, 3450]),
// each output transient (released after the next allocation) or, with probability
// 0.3, saved; a backward pass over the saved outputs in reverse (gradient of equal
// size, release the saved output, release the previous gradient); an optimizer pass
// with one short-lived temporary per saved output.  Sizes are log-uniform in
// [2^5, 2^28).  Per-operator draws use index = list * 8192 + operator.
enum { F_NFWD = 100, F_EXP = 101, F_MANT = 102, F_SAVED = 103 };

__device__ inline long long n_forward(u64 seed, long long c) { return 2800 + (long long)(mix64(seed, (u64)c, F_NFWD) % 651); }
__device__ inline long long op_size(u64 seed, long long c, long long j)
{
    const u64 idx = (u64)c * 8192 + (u64)j;
    const unsigned e = 5 + (unsigned)(mix64(seed, idx, F_EXP) % 23);
    return (long long)((1ull << e) + (mix64(seed, idx, F_MANT) & ((1ull << e) - 1)));
}
__device__ inline bool op_saved(u64 seed, long long c, long long j)
{
    return (mix64(seed, (u64)c * 8192 + (u64)j, F_SAVED) % 10) < 3;
}

__global__ __launch_bounds__(256) void events_count_kernel(u64 seed, long long first, long long n,
                                                           long long *counts)
{
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n) return;
    const long long c = first + t, nf = n_forward(seed, c);
    long long ns = 0;
    for (long long j = 0; j < nf; ++j) ns += op_saved(seed, c, j) ? 1 : 0;
    counts[t] = 2 * nf + 4 * ns;
}

__global__ __launch_bounds__(256) void events_fill_kernel(u64 seed, long long first, long long n,
                                                          const long long *offsets, long long *events)
{
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n) return;
    const long long c = first + t, nf = n_forward(seed, c);
    long long *out = events + offsets[t];
    long long *const end = events + offsets[t + 1];     // never write past the caller's slot
    bool prev_saved = true;
    long long prev_size = 0;
    for (long long j = 0; j < nf; ++j) {
        const long long s = op_size(seed, c, j);
        if (out < end) *out++ = s;
        if (!prev_saved && out < end) *out++ = -prev_size;
        prev_saved = op_saved(seed, c, j);
        prev_size = s;
    }
    if (!prev_saved && out < end) *out++ = -prev_size;
    long long prev_grad = 0;
    for (long long j = nf - 1; j >= 0; --j) {
        if (!op_saved(seed, c, j)) continue;
        const long long s = op_size(seed, c, j);
        if (out < end) *out++ = s;
        if (out < end) *out++ = -s;
        if (prev_grad && out < end) *out++ = -prev_grad;
        prev_grad = s;
    }
    if (prev_grad && out < end) *out++ = -prev_grad;
    for (long long j = 0; j < nf; ++j) {
        if (!op_saved(seed, c, j)) continue;
        const long long s = op_size(seed, c, j);
        if (out < end) *out++ = s;
        if (out < end) *out++ = -s;
    }
}

static int check_launch()
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e); return LLMEM_EHIP; }
    return LLMEM_OK;
}

}  // namespace llmem

extern "C" int llmem_grid_generate(int grid_id, uint64_t seed, int64_t first, int64_t n,
                                   const llmem_configs *c, void *hip_stream)
{
    using namespace llmem;
    if (!c) return LLMEM_EINVAL_NULL;
    if (n < 0 || first < 0) return LLMEM_EINVAL_N;
    if (grid_id < 1 || grid_id > 4) return LLMEM_EINVAL_ARG;
    if (grid_id == 1 && first + n > 432) return LLMEM_EINVAL_ARG;
    if (n == 0) return LLMEM_OK;
    if (!c->arch_id || !c->h || !c->L || !c->n_heads || !c->n_kv || !c->ffn || !c->V || !c->P || !c->bs
        || !c->sl || !c->method || !c->d || !c->chunk_k || !c->flags) return LLMEM_EINVAL_NULL;
    const unsigned blocks = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(grid_kernel, dim3(blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream),
                       grid_id, (u64)seed, (long long)first, (long long)n, *c, (uint8_t *)nullptr);
    return check_launch();
}

extern "C" int llmem_queries_generate(uint64_t seed, int64_t first, int64_t n, const llmem_configs *c,
                                      uint8_t *tp_n_out, void *hip_stream)
{
    using namespace llmem;
    if (!c) return LLMEM_EINVAL_NULL;
    if (n < 0 || first < 0) return LLMEM_EINVAL_N;
    if (n == 0) return LLMEM_OK;
    if (!tp_n_out || !c->arch_id || !c->h || !c->L || !c->n_heads || !c->n_kv || !c->ffn || !c->V || !c->P
        || !c->bs || !c->sl || !c->method || !c->d || !c->chunk_k || !c->flags) return LLMEM_EINVAL_NULL;
    const unsigned blocks = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(grid_kernel, dim3(blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream),
                       6, (u64)seed, (long long)first, (long long)n, *c, tp_n_out);
    return check_launch();
}

extern "C" int llmem_events_count(uint64_t seed, int64_t first, int64_t n, int64_t *counts, void *hip_stream)
{
    using namespace llmem;
    if (n < 0 || first < 0) return LLMEM_EINVAL_N;
    if (n == 0) return LLMEM_OK;
    if (!counts) return LLMEM_EINVAL_NULL;
    hipLaunchKernelGGL(events_count_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                       reinterpret_cast<hipStream_t>(hip_stream), (u64)seed, (long long)first, (long long)n,
                       reinterpret_cast<long long *>(counts));
    return check_launch();
}

extern "C" int llmem_events_generate(uint64_t seed, int64_t first, int64_t n, const int64_t *offsets,
                                     int64_t *events, void *hip_stream)
{
    using namespace llmem;
    if (n < 0 || first < 0) return LLMEM_EINVAL_N;
    if (n == 0) return LLMEM_OK;
    if (!offsets || !events) return LLMEM_EINVAL_NULL;
    hipLaunchKernelGGL(events_fill_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                       reinterpret_cast<hipStream_t>(hip_stream), (u64)seed, (long long)first, (long long)n,
                       reinterpret_cast<const long long *>(offsets), reinterpret_cast<long long *>(events));
    return check_launch();
}

extern "C" size_t llmem_config_bytes(int64_t n)
{
    // arch_id, method, d, chunk_k, flags: 1 byte; L, n_heads, n_kv, bs, sl: 2; h, ffn, V, P: 4
    return n < 0 ? 0 : (size_t)n * (5 * 1 + 5 * 2 + 4 * 4);
}

extern "C" size_t llmem_events_bytes(int64_t n)
{
    // at most 2 * 3450 + 4 * 3450 events of 8 bytes per list
    return n < 0 ? 0 : (size_t)n * (6 * 3450) * sizeof(int64_t);
}

extern "C" const char *llmem_strerror(int code)
{
    switch (code) {
    case LLMEM_OK: return "ok";
    case LLMEM_EINVAL_NULL: return "a required pointer is NULL";
    case LLMEM_EINVAL_N: return "negative count";
    case LLMEM_EINVAL_TABLE: return "malformed architecture tables or constants";
    case LLMEM_EHIP: {
        const char *a = llmem::last_hip_error();
        return (a && a[0]) ? a : (llmem::g_error_text[0] ? llmem::g_error_text : "HIP error");
    }
    case LLMEM_EINVAL_ARG: return "invalid argument";
    default: return "unknown error code";
    }
}

extern "C" int llmem_abi_version(void) { return LLMEM_ABI_VERSION; }
