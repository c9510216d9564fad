// Peaks of explicit allocator timelines: one wavefront per event list.
//
// Sequential traversal with live tensors and 512-byte blocks (Sec. 2.1 / Sec. 3.1
// of arXiv 2404.10933) as a scan.  A wave streams its list in tiles of 1024
// events: coalesced 16-byte streaming loads into registers (the next tile is
// requested before the current one is walked), a transpose through wave-private LDS so that
// every lane owns 16 consecutive events, a sequential walk of those 16 keeping
// running sums and running maxima of the two pools relative to the run's start,
// then a wave prefix sum over the runs' totals that places each run on the list's
// timeline.  Per-lane absolute maxima are carried from tile to tile and reduced
// once per list.
//
// While every event of a tile is below 2^35 bytes the walk is done in 32-bit
// block counts (a run of 16 such events cannot overflow); otherwise the tile
// takes the 64-bit path.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/llmem.h"
#include "wave.h"

namespace llmem {

constexpr int TL_WAVES = 4;
constexpr int TL_BLOCK = 64 * TL_WAVES;
constexpr int TL_RUN = 16;                       // consecutive events per lane and tile
constexpr int TL_TILE = 64 * TL_RUN;             // events per tile
constexpr int TL_ROW = TL_RUN * 8 + 16;          // bytes of LDS per lane: 16 events + padding against bank conflicts
constexpr int BLOCK_SHIFT = 9;                   // log2(LLMEM_BLOCK)
constexpr int SPLIT_BLOCKS = LLMEM_POOL_SPLIT / LLMEM_BLOCK;
static_assert((1 << BLOCK_SHIFT) == LLMEM_BLOCK, "block size");

typedef long long pair64 __attribute__((ext_vector_type(2)));

void set_hip_error(hipError_t e);

__global__ __launch_bounds__(TL_BLOCK) void timeline_kernel(const long long *__restrict__ events,
                                                            const long long *__restrict__ offsets,
                                                            long long n, long long *__restrict__ out_alloc,
                                                            long long *__restrict__ out_resv)
{
    __shared__ __attribute__((aligned(16))) char stage[TL_WAVES][64 * TL_ROW];
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    char *mine = stage[wave];
    // where this lane's pair of events of load j lands: tile index t = j*128 + 2*lane,
    // owner lane t / 16, position t % 16
    const int put0 = ((2 * lane) / TL_RUN) * TL_ROW + ((2 * lane) % TL_RUN) * 8;
    const char *get = mine + lane * TL_ROW;

    for (long long li = (long long)blockIdx.x * TL_WAVES + wave; li < n;
         li += (long long)gridDim.x * TL_WAVES) {
        const long long first = offsets[li], last = offsets[li + 1];
        i64 carry_s = 0, carry_l = 0;                 // live bytes of the pools before the tile
        i64 best_s = 0, best_l = 0, best_t = 0;       // per-lane maxima; the empty prefix counts
        // tiles start at a 128-byte boundary of the event array, so that no cache line is shared by
        // two load instructions (a streaming load does not find it in the L2 the second time); what
        // lies before `first` or at and after `last` is read as 0 (an event of 0 bytes changes nothing)
        const long long lead = (long long)((reinterpret_cast<uintptr_t>(events + first) >> 3) & 15);
        // coalesced loads of one tile into registers: load j covers events base + j*128 .. +127, two per lane
        auto request = [&](long long base, i64 (&v)[2 * (TL_TILE / 128)]) {
            if (base >= first && base + TL_TILE <= last) {                // a tile inside the list: nothing to mask
#pragma unroll
                for (int j = 0; j < TL_TILE / 128; ++j) {
                    const pair64 p = __builtin_nontemporal_load(reinterpret_cast<const pair64 *>(events + base + j * 128 + 2 * lane));
                    v[2 * j] = p.x; v[2 * j + 1] = p.y;
                }
                return;
            }
#pragma unroll
            for (int j = 0; j < TL_TILE / 128; ++j) {
                const long long e = base + j * 128 + 2 * lane;
                i64 a0 = 0, a1 = 0;
                if (e >= first && e + 1 < last) {
                    // every event is read once: a streaming load, which does not keep the line in the L2
                    const pair64 p = __builtin_nontemporal_load(reinterpret_cast<const pair64 *>(events + e));
                    a0 = p.x; a1 = p.y;
                } else {
                    if (e >= first && e < last) a0 = events[e];
                    if (e + 1 >= first && e + 1 < last) a1 = events[e + 1];
                }
                v[2 * j] = a0; v[2 * j + 1] = a1;
            }
        };
        // the next tile is requested before the current one is walked, so that its loads are in
        // flight meanwhile (past `last` nothing is loaded)
        i64 tile[2 * (TL_TILE / 128)];
        request(first - lead, tile);
        for (long long base = first - lead; base < last; base += TL_TILE) {
            u32 high_bits = 0;
#pragma unroll
            for (int j = 0; j < TL_TILE / 128; ++j) {
                const i64 a0 = tile[2 * j], a1 = tile[2 * j + 1];
                const u32 h0 = (u32)((u64)a0 >> 32), h1 = (u32)((u64)a1 >> 32);
                high_bits |= (h0 ^ (u32)((int)h0 >> 31)) | (h1 ^ (u32)((int)h1 >> 31));
                *reinterpret_cast<longlong2 *>(mine + put0 + j * (128 / TL_RUN) * TL_ROW) = make_longlong2(a0, a1);
            }
            request(base + TL_TILE, tile);
            wave_lds_fence();                         // the tile as all lanes stored it, before any lane reads its run
            const bool narrow = __builtin_amdgcn_ballot_w64(high_bits >= 8u) == 0;   // all |raw| < 2^35

            i64 run_s, run_l, top_s, top_l, top_t;    // relative to the run's start; tops >= 0 (the start itself)
            if (narrow) {
                int rs = 0, rl = 0, ts = 0, tl = 0, tt = 0;          // in blocks
#pragma unroll
                for (int q = 0; q < TL_RUN / 2; ++q) {
                    const longlong2 p = *reinterpret_cast<const longlong2 *>(get + q * 16);
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const i64 raw = u ? p.y : p.x;
                        // signed block count: ceil(raw / 512) for raw >= 0, -ceil(-raw / 512) = floor(raw / 512) below
                        const int sb = (int)((raw + (raw >= 0 ? (i64)(LLMEM_BLOCK - 1) : 0)) >> BLOCK_SHIFT);
                        const int mag = sb < 0 ? -sb : sb;
                        const int ds = mag < SPLIT_BLOCKS ? sb : 0;
                        rs += ds;
                        rl += sb - ds;
                        ts = rs > ts ? rs : ts;
                        tl = rl > tl ? rl : tl;
                        const int t = rs + rl;
                        tt = t > tt ? t : tt;
                    }
                }
                run_s = (i64)rs << BLOCK_SHIFT; run_l = (i64)rl << BLOCK_SHIFT;
                top_s = (i64)ts << BLOCK_SHIFT; top_l = (i64)tl << BLOCK_SHIFT; top_t = (i64)tt << BLOCK_SHIFT;
            } else {
                run_s = 0; run_l = 0; top_s = 0; top_l = 0; top_t = 0;
#pragma unroll
                for (int q = 0; q < TL_RUN; ++q) {
                    const i64 raw = *reinterpret_cast<const i64 *>(get + q * 8);
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
            }
            const i64 incl_s = wave_scan_add(run_s), incl_l = wave_scan_add(run_l);
            const i64 start_s = carry_s + incl_s - run_s, start_l = carry_l + incl_l - run_l;
            best_s = max64(best_s, start_s + top_s);
            best_l = max64(best_l, start_l + top_l);
            best_t = max64(best_t, start_s + start_l + top_t);
            carry_s += read_lane(incl_s, 63);
            carry_l += read_lane(incl_l, 63);
            wave_lds_fence();                         // every run has been read before the next tile is stored
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
