// Seeded draws of the synthetic configuration grids, one configuration at a time
// (device code: the generator kernels store them, the sweep estimates them in
// registers).
//
// Every draw is  lo + mix64(seed, index, field) mod span  with splitmix64's
// finaliser over  seed + 0x9E3779B97F4A7C15*(index+1) + 0xD1B54A32D192ED03*(field+1).
// The grids draw decoder shapes of the model families the paper fine-tunes
// (Sec. 7.1: OPT / GPT-style and LLaMA-style decoders); they stand in for its
// real models, whose weights and dataset the estimator never reads.
#pragma once

#ifndef __HIPCC_RTC__
#include <hip/hip_runtime.h>
#include <stdint.h>
#endif

#ifdef __HIPCC_RTC__
#include "llmem.h"                 // the run-time compiler gets every file by its bare name
#else
#include "../../include/llmem.h"
#endif

namespace llmem {

__host__ __device__ inline unsigned long long mix64(unsigned long long seed, unsigned long long index,
                                                    unsigned long long field)
{
    unsigned long long x = seed + 0x9E3779B97F4A7C15ull * (index + 1) + 0xD1B54A32D192ED03ull * (field + 1);
    x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27; x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

// hash field ids of the configuration grids
enum { F_H, F_L, F_V, F_BS, F_SL, F_METHOD, F_D, F_K, F_NKV, F_TP };

__device__ inline unsigned long long uniform(unsigned long long seed, unsigned long long i, int field,
                                             unsigned long long lo, unsigned long long hi)
{
    return lo + mix64(seed, i, (unsigned long long)field) % (hi - lo + 1);
}

struct DrawnConfig {
    unsigned arch_id, h, L, n_heads, n_kv, ffn, V, P, bs, sl, method, d, flags, tp_n;
    int chunk_k;
};

// Configuration `i` of grid `grid_id`: 1 the tiny Cartesian grid, 2 the OPT/GPT-style grid, 3 the
// Llama-style grid, 4 the same with chunk search, 6 the queries of the method decision (grid 4's
// shapes; gpu_n, the batch-size cap and tp_n instead of d, bs and method).
__device__ inline DrawnConfig draw_config(int grid_id, unsigned long long seed, unsigned long long i)
{
    DrawnConfig c;
    c.arch_id = 0; c.tp_n = 0;
    if (grid_id == 1) {
        // full Cartesian product, last factor fastest: bs x sl x method x d x chunk
        unsigned long long r = i;
        const unsigned ik = r % 3; r /= 3;
        const unsigned id = r % 4; r /= 4;
        c.method = r % 3; r /= 3;
        const unsigned isl = r % 3; r /= 3;
        const unsigned ibs = r % 4;
        c.h = 256; c.L = 4; c.n_heads = 4; c.n_kv = 4; c.ffn = 1024; c.V = 8192; c.P = 512;
        c.bs = 1u << ibs; c.sl = 128u << isl; c.d = id + 1; c.chunk_k = 4 + (int)ik;
        c.flags = LLMEM_CFG_GRAD_ALIAS;
    } else if (grid_id == 2) {
        const unsigned ih = (unsigned)(mix64(seed, i, F_H) % 5);
        c.h = ih == 0 ? 768u : ih == 1 ? 1024u : ih == 2 ? 2048u : ih == 3 ? 2560u : 4096u;
        c.L = (unsigned)uniform(seed, i, F_L, 12, 32);
        c.n_heads = c.h / 64; c.n_kv = c.n_heads; c.ffn = 4 * c.h;
        c.V = (mix64(seed, i, F_V) % 2) ? 50272u : 32000u; c.P = 2048;
        c.bs = (unsigned)uniform(seed, i, F_BS, 1, 32);
        c.sl = 256u << (unsigned)(mix64(seed, i, F_SL) % 4);
        c.method = (unsigned)uniform(seed, i, F_METHOD, 0, 2);
        c.d = (unsigned)uniform(seed, i, F_D, 1, 16);
        c.chunk_k = (int)uniform(seed, i, F_K, 4, 8);
        c.flags = LLMEM_CFG_TIED_LM_HEAD | LLMEM_CFG_GRAD_ALIAS;
    } else {
        const unsigned ih = (unsigned)(mix64(seed, i, F_H) % 4);
        c.h = ih == 0 ? 2048u : ih == 1 ? 4096u : ih == 2 ? 5120u : 8192u;
        c.L = (unsigned)uniform(seed, i, F_L, 16, 80);
        c.n_heads = c.h / 128;
        const unsigned ikv = (unsigned)(mix64(seed, i, F_NKV) % 3);
        c.n_kv = ikv == 0 ? 1u : ikv == 1 ? 4u : 8u;
        c.ffn = ((8 * c.h + 2) / 3 + 255) / 256 * 256;       // SwiGLU width: 8h/3 rounded up to 256
        c.V = (mix64(seed, i, F_V) % 2) ? 128256u : 32000u; c.P = 0;
        c.bs = (unsigned)uniform(seed, i, F_BS, 1, 64);
        c.sl = 512u << (unsigned)(mix64(seed, i, F_SL) % 5);
        c.method = (unsigned)uniform(seed, i, F_METHOD, 0, 2);
        c.d = (unsigned)uniform(seed, i, F_D, 1, 16);
        c.chunk_k = grid_id >= 4 ? LLMEM_CHUNK_SEARCH : (int)uniform(seed, i, F_K, 4, 8);
        c.flags = LLMEM_CFG_LOGITS_FP32 | LLMEM_CFG_GRAD_ALIAS;
        if (grid_id == 6) {
            const unsigned log_g = (unsigned)(mix64(seed, i, F_D) % 5);
            const unsigned log_t = (unsigned)(mix64(seed, i, F_TP) % (log_g + 1));
            c.d = 1u << log_g; c.bs = LLMEM_QUERY_BS_CAP; c.method = 0;
            c.tp_n = 1u << log_t;
        }
    }
    return c;
}

}  // namespace llmem
