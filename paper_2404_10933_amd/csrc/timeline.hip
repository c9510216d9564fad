// Peaks of explicit allocator timelines: one wavefront per event list.
//
// Sequential traversal with live tensors and 512-byte blocks (Sec. 2.1 / Sec. 3.1
// of arXiv 2404.10933) as a scan: every lane walks a run of consecutive events
// keeping running sums and running maxima of the two pools relative to the run's
// start; a wave prefix sum over the runs' totals places each run on the list's
// timeline; per-lane absolute maxima are carried from tile to tile and reduced
// once per list.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/llmem.h"
#include "wave.h"

namespace llmem {

constexpr int TL_WAVES = 4;
constexpr int TL_BLOCK = 64 * TL_WAVES;
constexpr int TL_RUN = 16;                 // consecutive events per lane and tile
constexpr int TL_TILE = 64 * TL_RUN;

extern const char *last_hip_error();
void set_hip_error(hipError_t e);

__global__ __launch_bounds__(TL_BLOCK) void timeline_kernel(const long long *__restrict__ events,
                                                            const long long *__restrict__ offsets,
                                                            long long n, long long *__restrict__ out_alloc,
                                                            long long *__restrict__ out_resv)
{
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    for (long long li = (long long)blockIdx.x * TL_WAVES + wave; li < n;
         li += (long long)gridDim.x * TL_WAVES) {
        const long long first = offsets[li], last = offsets[li + 1];
        i64 carry_s = 0, carry_l = 0;                 // live bytes of the pools before the tile
        i64 best_s = 0, best_l = 0, best_t = 0;       // per-lane maxima; the empty prefix counts
        for (long long base = first; base < last; base += TL_TILE) {
            const long long e0 = base + (long long)lane * TL_RUN;
            i64 run_s = 0, run_l = 0;
            i64 top_s = 0, top_l = 0, top_t = 0;      // maxima relative to the run's start (>= 0: the start itself)
#pragma unroll
            for (int j = 0; j < TL_RUN; ++j) {
                const long long e = e0 + j;
                const i64 raw = e < last ? events[e] : 0;
                const u64 mag = raw < 0 ? (u64)0 - (u64)raw : (u64)raw;
                const u64 r = (mag + (LLMEM_BLOCK - 1)) & ~(u64)(LLMEM_BLOCK - 1);
                const i64 delta = raw < 0 ? -(i64)r : (i64)r;
                const bool small = r < (u64)LLMEM_POOL_SPLIT;
                run_s += small ? delta : 0;
                run_l += small ? 0 : delta;
                top_s = max64(top_s, run_s);
                top_l = max64(top_l, run_l);
                top_t = max64(top_t, run_s + run_l);
            }
            const i64 incl_s = wave_scan_add(run_s), incl_l = wave_scan_add(run_l);
            const i64 start_s = carry_s + incl_s - run_s, start_l = carry_l + incl_l - run_l;
            best_s = max64(best_s, start_s + top_s);
            best_l = max64(best_l, start_l + top_l);
            best_t = max64(best_t, start_s + start_l + top_t);
            carry_s += read_lane(incl_s, 63);
            carry_l += read_lane(incl_l, 63);
        }
        const i64 peak_s = wave_max(best_s), peak_l = wave_max(best_l), peak_t = wave_max(best_t);
        if (lane == 0) {
            const u64 seg = (u64)LLMEM_SEGMENT - 1;
            out_alloc[li] = peak_t;
            out_resv[li] = (i64)((((u64)peak_s + seg) & ~seg) + (((u64)peak_l + seg) & ~seg));
        }
    }
}

}  // namespace llmem

extern "C" int llmem_timeline_peaks(const int64_t *events, const int64_t *offsets, int64_t n,
                                    int64_t *out_allocated, int64_t *out_reserved, void *hip_stream)
{
    using namespace llmem;
    if (n < 0) return LLMEM_EINVAL_N;
    if (n == 0) return LLMEM_OK;
    if (!offsets || !out_allocated || !out_reserved) return LLMEM_EINVAL_NULL;
    int64_t blocks = (n + TL_WAVES - 1) / TL_WAVES;
    const int64_t max_blocks = 256 * 64;
    if (blocks > max_blocks) blocks = max_blocks;
    hipLaunchKernelGGL(timeline_kernel, dim3((unsigned)blocks), dim3(TL_BLOCK), 0,
                       reinterpret_cast<hipStream_t>(hip_stream),
                       reinterpret_cast<const long long *>(events),
                       reinterpret_cast<const long long *>(offsets), (long long)n,
                       reinterpret_cast<long long *>(out_allocated),
                       reinterpret_cast<long long *>(out_reserved));
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e); return LLMEM_EHIP; }
    return LLMEM_OK;
}
