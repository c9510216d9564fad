// Seeded synthetic inputs generated on the device, and the small host-only
// entry points of the library.
//
// Every draw is  lo + mix64(seed, index, field) mod span  with splitmix64's
// finaliser over  seed + 0x9E3779B97F4A7C15*(index+1) + 0xD1B54A32D192ED03*(field+1).
// The grids draw decoder shapes of the model families the paper fine-tunes
// (Sec. 7.1: OPT / GPT-style and LLaMA-style decoders); they stand in for its
// real models, whose weights and dataset the estimator never reads.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/llmem.h"

namespace llmem {

typedef unsigned long long u64;

static thread_local char g_error_text[256] = "";
void set_hip_error(hipError_t e)
{
    snprintf(g_error_text, sizeof(g_error_text), "HIP error: %s", hipGetErrorString(e));
}
const char *last_hip_error();   // the estimator keeps its own buffer

__host__ __device__ inline u64 mix64(u64 seed, u64 index, u64 field)
{
    u64 x = seed + 0x9E3779B97F4A7C15ull * (index + 1) + 0xD1B54A32D192ED03ull * (field + 1);
    x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27; x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

// hash field ids of the configuration grids
enum { F_H, F_L, F_V, F_BS, F_SL, F_METHOD, F_D, F_K, F_NKV, F_TP };

__device__ inline u64 uniform(u64 seed, u64 i, int field, u64 lo, u64 hi)
{
    return lo + mix64(seed, i, (u64)field) % (hi - lo + 1);
}

// grid_id 6: the queries of the method decision (grid 4's shapes; gpu_n, the batch-size cap and
// tp_n instead of d, bs and method); tp_out is only written for that grid
__global__ __launch_bounds__(256) void grid_kernel(int grid_id, u64 seed, long long first, long long n,
                                                   llmem_configs c, uint8_t *tp_out)
{
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n) return;
    const u64 i = (u64)(first + t);
    unsigned arch = 0, h, L, n_heads, n_kv, ffn, V, P, bs, sl, method, d, flags;
    int k;
    if (grid_id == 1) {
        // full Cartesian product, last factor fastest: bs x sl x method x d x chunk
        u64 r = i;
        const unsigned ik = r % 3; r /= 3;
        const unsigned id = r % 4; r /= 4;
        method = r % 3; r /= 3;
        const unsigned isl = r % 3; r /= 3;
        const unsigned ibs = r % 4;
        h = 256; L = 4; n_heads = 4; n_kv = 4; ffn = 1024; V = 8192; P = 512;
        bs = 1u << ibs; sl = 128u << isl; d = id + 1; k = 4 + (int)ik;
        flags = LLMEM_CFG_GRAD_ALIAS;
    } else if (grid_id == 2) {
        const unsigned hs[5] = {768, 1024, 2048, 2560, 4096};
        const unsigned vs[2] = {32000, 50272};
        const unsigned sls[4] = {256, 512, 1024, 2048};
        h = hs[mix64(seed, i, F_H) % 5];
        L = (unsigned)uniform(seed, i, F_L, 12, 32);
        n_heads = h / 64; n_kv = n_heads; ffn = 4 * h;
        V = vs[mix64(seed, i, F_V) % 2]; P = 2048;
        bs = (unsigned)uniform(seed, i, F_BS, 1, 32);
        sl = sls[mix64(seed, i, F_SL) % 4];
        method = (unsigned)uniform(seed, i, F_METHOD, 0, 2);
        d = (unsigned)uniform(seed, i, F_D, 1, 16);
        k = (int)uniform(seed, i, F_K, 4, 8);
        flags = LLMEM_CFG_TIED_LM_HEAD | LLMEM_CFG_GRAD_ALIAS;
    } else {
        const unsigned hs[4] = {2048, 4096, 5120, 8192};
        const unsigned kvs[3] = {1, 4, 8};
        const unsigned vs[2] = {32000, 128256};
        const unsigned sls[5] = {512, 1024, 2048, 4096, 8192};
        h = hs[mix64(seed, i, F_H) % 4];
        L = (unsigned)uniform(seed, i, F_L, 16, 80);
        n_heads = h / 128;
        n_kv = kvs[mix64(seed, i, F_NKV) % 3];
        ffn = ((8 * h + 2) / 3 + 255) / 256 * 256;       // SwiGLU width: 8h/3 rounded up to 256
        V = vs[mix64(seed, i, F_V) % 2]; P = 0;
        bs = (unsigned)uniform(seed, i, F_BS, 1, 64);
        sl = sls[mix64(seed, i, F_SL) % 5];
        method = (unsigned)uniform(seed, i, F_METHOD, 0, 2);
        d = (unsigned)uniform(seed, i, F_D, 1, 16);
        k = grid_id >= 4 ? LLMEM_CHUNK_SEARCH : (int)uniform(seed, i, F_K, 4, 8);
        flags = LLMEM_CFG_LOGITS_FP32 | LLMEM_CFG_GRAD_ALIAS;
        if (grid_id == 6) {
            const unsigned log_g = (unsigned)(mix64(seed, i, F_D) % 5);
            const unsigned log_t = (unsigned)(mix64(seed, i, F_TP) % (log_g + 1));
            d = 1u << log_g; bs = LLMEM_QUERY_BS_CAP; method = 0;
            tp_out[t] = (uint8_t)(1u << log_t);
        }
    }
    c.arch_id[t] = (uint8_t)arch; c.h[t] = h; c.L[t] = (uint16_t)L; c.n_heads[t] = (uint16_t)n_heads;
    c.n_kv[t] = (uint16_t)n_kv; c.ffn[t] = ffn; c.V[t] = V; c.P[t] = P; c.bs[t] = (uint16_t)bs;
    c.sl[t] = (uint16_t)sl; c.method[t] = (uint8_t)method; c.d[t] = (uint8_t)d; c.chunk_k[t] = (int8_t)k;
    c.flags[t] = (uint8_t)flags;
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
