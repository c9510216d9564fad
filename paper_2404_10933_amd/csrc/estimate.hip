// Batched peak-GPU-memory estimator: one wavefront per configuration.
//
// A wave takes 64 consecutive configurations with one coalesced load per column
// (lane i holds configuration i), then visits them one by one: the fields of the
// current configuration are broadcast to wave-uniform values, the lanes spread
// over the parameter-table entries and over the timeline events of its
// architecture (both staged in LDS once per workgroup), and wave reductions
// produce the sums, maxima and the prefix-sum/max of the timeline.  Results are
// parked in lane i of per-wave accumulators and stored coalesced.
//
// Closed form: Sec. 4.2 (m_p, m_os, m_out, m_lm, m_peak^s) and Sec. 5 (m_peak^dp,
// m_peak^tp, m_back^tp) of arXiv 2404.10933; chunk size per Sec. 4.1; timeline
// traversal per Sec. 2.1 / Sec. 3.1.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "../../include/llmem.h"
#include "estimate_args.h"
#include "wave.h"

namespace llmem {

constexpr int WAVES_PER_BLOCK = 4;
constexpr int BLOCK = 64 * WAVES_PER_BLOCK;

// x / d and ceil(x / d) for wave-uniform or per-lane x, 1 <= d <= 255, x < 2^63
__device__ __forceinline__ u64 div_small(u64 x, u32 d, u64 mul, u32 shift)
{
    return d == 1 ? x : (__umul64hi(x, mul) >> shift);
}
__device__ __forceinline__ u64 cdiv_small(u64 x, u32 d, u64 mul, u32 shift)
{
    return div_small(x + (d - 1), d, mul, shift);
}
__device__ __forceinline__ u64 round_up_shift(u64 x, int shift)
{
    return ((x + ((1ull << shift) - 1)) >> shift) << shift;
}

// coef * D[dim0] * D[dim1] * D[dim2] * D[dim3]; lane i < 16 of `dvec` holds D[i]
__device__ __forceinline__ u64 monomial(u32 coef, u32 dims, u32 dvec)
{
    u64 x = coef;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        u32 sel = (dims >> (8 * j)) & 15u;
        u32 dv = (u32)__builtin_amdgcn_ds_bpermute((int)(sel << 2), (int)dvec);
        x *= (u64)dv;
    }
    return x;
}

template <bool DETAIL>
__global__ __launch_bounds__(BLOCK) void estimate_kernel(const EstimateArgs a)
{
    extern __shared__ uint4 lds[];
    uint4 *lds_param = lds;
    uint4 *lds_event = lds + a.n_param_total;

    // ---- stage the tables: parameters verbatim, events dealt to lanes ----------
    for (int t = threadIdx.x; t < a.n_param_total; t += BLOCK) lds_param[t] = a.params_dev[t];
    for (int ar = 0; ar < a.n_arch; ++ar) {
        const ArchLayout &al = a.arch[ar];
        const int slots = al.per_lane * 64;
        for (int t = threadIdx.x; t < slots; t += BLOCK) {
            const int l = t & 63, j = t >> 6;
            uint4 e = make_uint4(0, 0, 0, 0);          // padding: method_mask 0, never active
            int s = 0;
            while (s < LLMEM_NSEG && l >= al.lane0[s + 1]) ++s;
            if (s < LLMEM_NSEG) {
                const int idx = al.seg_first[s] + (l - al.lane0[s]) * al.per_lane + j;
                if (idx < al.seg_first[s + 1]) e = a.events_dev[al.event_first + idx];
            }
            lds_event[al.slot_first + t] = e;
        }
    }
    __syncthreads();

    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const long long n = a.n;
    const long long n_batch = (n + 63) >> 6;
    const int cu_shift = a.cu_shift, align_shift = a.align_shift;

    for (long long b = (long long)blockIdx.x * WAVES_PER_BLOCK + wave; b < n_batch;
         b += (long long)gridDim.x * WAVES_PER_BLOCK) {
        const long long i = (b << 6) + lane;
        const bool in_range = i < n;
        // coalesced column loads, packed into 8 dwords per lane
        u32 w_h = 0, w_ffn = 0, w_V = 0, w_P = 0, w_a = 0, w_b = 0, w_c = 0, w_d = 0;
        if (in_range) {
            w_h = a.cfg.h[i]; w_ffn = a.cfg.ffn[i]; w_V = a.cfg.V[i]; w_P = a.cfg.P[i];
            w_a = (u32)a.cfg.arch_id[i] | ((u32)a.cfg.method[i] << 8) | ((u32)a.cfg.d[i] << 16)
                  | ((u32)a.cfg.flags[i] << 24);
            w_b = (u32)a.cfg.L[i] | ((u32)a.cfg.n_heads[i] << 16);
            w_c = (u32)a.cfg.n_kv[i] | ((u32)(uint8_t)a.cfg.chunk_k[i] << 16);
            w_d = (u32)a.cfg.bs[i] | ((u32)a.cfg.sl[i] << 16);
        }
        const int count = (int)((n - (b << 6)) < 64 ? (n - (b << 6)) : 64);

        i64 acc[LLMEM_NDETAIL];
#pragma unroll
        for (int q = 0; q < LLMEM_NDETAIL; ++q) acc[q] = 0;

        for (int c = 0; c < count; ++c) {
            // ---- broadcast configuration c ------------------------------------
            const u32 h = read_lane(w_h, c), ffn = read_lane(w_ffn, c), V = read_lane(w_V, c),
                      P = read_lane(w_P, c);
            const u32 pa = read_lane(w_a, c), pb = read_lane(w_b, c), pc = read_lane(w_c, c),
                      pd = read_lane(w_d, c);
            const u32 arch_id = pa & 255u, method = (pa >> 8) & 255u, d = (pa >> 16) & 255u,
                      cflags = pa >> 24;
            const u32 L = pb & 0xffffu, n_heads = pb >> 16, n_kv = pc & 0xffffu;
            const int chunk_k = (int)(int8_t)((pc >> 16) & 255u);
            const u32 bs = pd & 0xffffu, sl = pd >> 16;

            u32 err = 0;
            if (arch_id >= (u32)a.n_arch) err |= LLMEM_F_ERR_ARCH;
            if (method > 2) err |= LLMEM_F_ERR_METHOD;
            if (d == 0) err |= LLMEM_F_ERR_D;
            if (n_heads == 0) err |= LLMEM_F_ERR_HEADS;
            if (!(chunk_k == -1 || (chunk_k >= 0 && chunk_k <= K_FIXED_MAX))) err |= LLMEM_F_ERR_CHUNK;

            i64 r[LLMEM_NDETAIL];
#pragma unroll
            for (int q = 0; q < LLMEM_NDETAIL; ++q) r[q] = 0;

            if (err) {
                r[LLMEM_D_PEAK] = -1;
                r[LLMEM_D_FLAGS] = err;
            } else {
                const ArchLayout &al = a.arch[arch_id];
                const u64 div_mul = c_div.t[d].mul;
                const u32 div_shift = c_div.t[d].shift;
                const u32 head_dim = h / n_heads;
                const u32 kv_dim = n_kv * head_dim;
                const u32 sl_m1 = sl > 0 ? sl - 1 : 0;
                const u32 Blog = (cflags & LLMEM_CFG_LOGITS_FP32) ? B32 : B16;

                // dimension vector: lane j < LLMEM_NDIM holds D[j]
                u32 dvec = 0;
                dvec = write_lane(dvec, 1u, LLMEM_DIM_ONE, lane);
                dvec = write_lane(dvec, bs, LLMEM_DIM_BS, lane);
                dvec = write_lane(dvec, sl, LLMEM_DIM_SL, lane);
                dvec = write_lane(dvec, sl_m1, LLMEM_DIM_SL_M1, lane);
                dvec = write_lane(dvec, h, LLMEM_DIM_H, lane);
                dvec = write_lane(dvec, ffn, LLMEM_DIM_FFN, lane);
                dvec = write_lane(dvec, n_heads, LLMEM_DIM_N_HEADS, lane);
                dvec = write_lane(dvec, n_kv, LLMEM_DIM_N_KV, lane);
                dvec = write_lane(dvec, head_dim, LLMEM_DIM_HEAD_DIM, lane);
                dvec = write_lane(dvec, kv_dim, LLMEM_DIM_KV_DIM, lane);
                dvec = write_lane(dvec, V, LLMEM_DIM_V, lane);
                dvec = write_lane(dvec, P, LLMEM_DIM_P, lane);
                dvec = write_lane(dvec, L, LLMEM_DIM_L, lane);
                dvec = write_lane(dvec, Blog, LLMEM_DIM_B_LOGITS, lane);
                dvec = write_lane(dvec, d, LLMEM_DIM_D, lane);

                // ---- parameter table: one entry per lane ---------------------------
                // Notation table (embed_p, lm_p, other_p) and Sec. 4.2, equation for m_os
                uint4 pe = make_uint4(0, 0, 0, 0);
                const bool has_p = lane < al.n_param;
                if (has_p) pe = lds_param[al.param_first + lane];
                const u32 p_cls = pe.z & 255u, p_role = (pe.z >> 8) & 255u, p_layer = (pe.z >> 16) & 255u;
                const u64 t_p = monomial(pe.x, pe.y, dvec);
                const u64 copies = p_layer ? (u64)L : 1ull;
                const u64 tot = has_p ? t_p * copies : 0ull;
                const bool in_os = has_p && p_cls <= LLMEM_CLS_LINEAR && p_role != LLMEM_ROLE_LM_HEAD;
                const u64 os_one = round_up_shift(t_p * (u64)(B32 + B32), cu_shift);
                const u64 embed_p = (u64)wave_sum((i64)(p_role == LLMEM_ROLE_EMBED_TOK ? tot : 0ull));
                const u64 lm_p = (u64)wave_sum((i64)(p_role == LLMEM_ROLE_LM_HEAD ? tot : 0ull));
                const u64 other_p = (u64)wave_sum((i64)(p_role == LLMEM_ROLE_OTHER ? tot : 0ull));
                const u64 m_os = (u64)wave_sum((i64)(in_os ? os_one * copies : 0ull));
                const u64 t_max = (u64)wave_max((i64)((has_p && p_role == LLMEM_ROLE_OTHER) ? t_p : 0ull));
                const u64 e_n = (u64)__builtin_popcountll(__builtin_amdgcn_ballot_w64(
                    has_p && p_cls == LLMEM_CLS_EMBEDDING && p_role != LLMEM_ROLE_LM_HEAD));
                const u64 n_params = embed_p + other_p + ((cflags & LLMEM_CFG_TIED_LM_HEAD) ? 0ull : lm_p);

                // ---- Sec. 4.2: m_out, m_lm; Sec. 5: m_back^tp --------------------------
                const u64 A = (u64)bs * sl * h;
                const u64 m_out = round_up_shift((e_n + L) * A * B16, cu_shift);
                const u64 row = (u64)bs * V * Blog;
                const u64 m_lm = round_up_shift(row * sl, cu_shift) + 2 * round_up_shift(row * sl_m1, cu_shift)
                                 + lm_p * B16;
                u64 m_back = 0;
                if (method == LLMEM_METHOD_TP) {
                    // ceil(x / (d * cu_p)) = ceil(ceil(x / cu_p) / d)
                    const u64 pages = ((u64)L * A * (d - 1) * B16 + ((1ull << cu_shift) - 1)) >> cu_shift;
                    m_back = cdiv_small(pages, d, div_mul, div_shift) << cu_shift;
                }

                // ---- Sec. 4.1: gradients alias param fp16 unless switched off ----------
                const u64 grad_bytes = (embed_p + other_p) * B16;
                const u64 grad_logical = method == LLMEM_METHOD_CDP ? grad_bytes
                                                                     : cdiv_small(grad_bytes, d, div_mul, div_shift);
                u64 grad_extra = 0;
                if (!(cflags & LLMEM_CFG_GRAD_ALIAS)) {
                    const u64 g = round_up_shift(grad_bytes, cu_shift);
                    grad_extra = method == LLMEM_METHOD_CDP
                                     ? g : round_up_shift(cdiv_small(g, d, div_mul, div_shift), align_shift);
                }

                // ---- chunk size, m_p and the method's peak ------------------------------
                // Sec. 4.1: least padding waste among the candidates that hold the largest
                // tensor, ties to the smaller chunk.  Lanes 0..8 each estimate one candidate
                // k = 2..10; a fixed chunk size is estimated by every lane alike.
                const bool search = chunk_k == -1;
                const int k_lane = search ? (K_SEARCH_MIN + (lane < 9 ? lane : 8)) : chunk_k;
                const int cs_shift = k_lane + 20 - 1;                       // 2^k MiB of fp16 values
                const u64 cs_mask = (1ull << cs_shift) - 1;
                const u64 other_chunked = (other_p + cs_mask) & ~cs_mask;   // ceil(other_p / cs) * cs
                const u64 chunked = embed_p + other_chunked;
                const u64 m_p = round_up_shift(chunked * (B16 + B32), cu_shift);
                const u64 m_p16 = round_up_shift(chunked * B16, cu_shift);
                const u64 m_p32 = round_up_shift(chunked * B32, cu_shift);
                u64 peak_lane;
                if (method == LLMEM_METHOD_CDP)
                    peak_lane = (u64)a.m_base + m_p + m_os + m_out + m_lm;
                else if (method == LLMEM_METHOD_ZERO3)
                    peak_lane = (u64)a.m_base + m_p16
                                + round_up_shift(cdiv_small(m_p32 + m_os, d, div_mul, div_shift), align_shift)
                                + m_out + m_lm;
                else
                    peak_lane = (u64)a.m_base
                                + round_up_shift(cdiv_small(m_p + m_os, d, div_mul, div_shift), align_shift)
                                + m_out + m_lm + m_back;
                peak_lane += grad_extra;

                int pick = 0;                                               // lane whose candidate is used
                if (search) {
                    const u64 waste = other_chunked - other_p;
                    const bool feasible = lane < 9 && t_max <= (1ull << cs_shift);
                    // smallest waste, then smallest k: waste < 2^40, so (waste << 8 | lane) orders both
                    const u64 key = feasible ? ((waste << 8) | (u64)lane) : ~0ull >> 1;
                    const u64 best = (u64)(-wave_max(-(i64)key));
                    pick = best == (~0ull >> 1) ? 8 : (int)(best & 255u);
                }
                const int k_used = search ? K_SEARCH_MIN + pick : chunk_k;
                const u64 m_peak = (u64)read_lane((i64)peak_lane, pick);
                const u64 mp = (u64)read_lane((i64)m_p, pick), mp16 = (u64)read_lane((i64)m_p16, pick),
                          mp32 = (u64)read_lane((i64)m_p32, pick);
                const u32 flags = t_max > (1ull << (k_used + 19)) ? LLMEM_F_CHUNK_INFEASIBLE : 0;

                u64 param_gpu, os_gpu;
                if (method == LLMEM_METHOD_CDP) {
                    param_gpu = mp; os_gpu = m_os;
                } else if (method == LLMEM_METHOD_ZERO3) {
                    param_gpu = mp16 + round_up_shift(cdiv_small(mp32, d, div_mul, div_shift), align_shift);
                    os_gpu = round_up_shift(cdiv_small(m_os, d, div_mul, div_shift), align_shift);
                } else {
                    param_gpu = round_up_shift(cdiv_small(mp, d, div_mul, div_shift), align_shift);
                    os_gpu = round_up_shift(cdiv_small(m_os, d, div_mul, div_shift), align_shift);
                }

                r[LLMEM_D_PEAK] = (i64)m_peak;
                if (DETAIL) {
                    // ---- timeline: Sec. 2.1 / Sec. 3.1 traversal with live tensors ------
                    // Each lane sums its own events in order (running sum and running maximum
                    // relative to the lane's start); a wave prefix sum places the lanes on the
                    // one-block timeline A F H B Z.  The L equal blocks shift the prefix
                    // linearly: repetition r of F adds r * dF, so its maximum over r is at
                    // r = 0 or r = L-1; likewise for B.  Everything after a repeated segment
                    // is shifted by (L-1) * its net change.
                    i64 run = 0, run_max = (i64)0x8000000000000000ull;
                    const uint4 *ev = lds_event + al.slot_first + lane;
                    for (int j = 0; j < al.per_lane; ++j) {
                        const uint4 e = ev[j * 64];
                        const u32 eb = e.z & 255u, efl = (e.z >> 16) & 255u, emask = e.z >> 24;
                        u64 x = monomial(e.x, e.y, dvec) * (u64)eb;
                        if (__builtin_amdgcn_ballot_w64((efl & LLMEM_EV_TP_GATHER) != 0)) {
                            const u64 g = cdiv_small(x * (u64)(d - 1), d, div_mul, div_shift);
                            x = (efl & LLMEM_EV_TP_GATHER) ? g : x;
                        }
                        u64 rnd = round_up_shift(x, align_shift);
                        if (efl & LLMEM_EV_TIMES_L) rnd *= (u64)L;
                        i64 v = (efl & LLMEM_EV_FREE) ? -(i64)rnd : (i64)rnd;
                        if (!((emask >> method) & 1u)) v = 0;
                        run += v;
                        run_max = max64(run_max, run);
                    }
                    const i64 incl = wave_scan_add(run);
                    const i64 start = incl - run;                     // prefix before the lane's events
                    // net change of one F block and one B block
                    const i64 end_A = al.lane0[1] > 0 ? read_lane(incl, al.lane0[1] - 1) : 0;
                    const i64 end_F = al.lane0[2] > 0 ? read_lane(incl, al.lane0[2] - 1) : 0;
                    const i64 end_H = al.lane0[3] > 0 ? read_lane(incl, al.lane0[3] - 1) : 0;
                    const i64 end_B = al.lane0[4] > 0 ? read_lane(incl, al.lane0[4] - 1) : 0;
                    const i64 dF = end_F - end_A, dB = end_B - end_H;
                    const i64 Lm1 = (i64)L - 1;
                    const i64 shift_F = Lm1 * dF, shift_B = Lm1 * dB;
                    const i64 lowest = (i64)0x8000000000000000ull;
                    i64 adj;
                    if (lane < al.lane0[1]) adj = 0;
                    else if (lane < al.lane0[2]) adj = L ? (shift_F > 0 ? shift_F : 0) : lowest;
                    else if (lane < al.lane0[3]) adj = shift_F;
                    else if (lane < al.lane0[4]) adj = L ? shift_F + (shift_B > 0 ? shift_B : 0) : lowest;
                    else if (lane < al.lane0[5]) adj = shift_F + shift_B;
                    else adj = lowest;
                    i64 cand = (adj == lowest || run_max == lowest) ? lowest : start + run_max + adj;
                    const i64 top = wave_max(cand);
                    const i64 prelude = (i64)((u64)a.m_base + param_gpu + os_gpu + lm_p * B16 + grad_extra);
                    const i64 peak_live = prelude + (top > 0 ? top : 0);

                    r[LLMEM_D_PARAM_GPU] = (i64)param_gpu;
                    r[LLMEM_D_GRAD_GPU] = (i64)grad_logical;
                    r[LLMEM_D_OS_GPU] = (i64)os_gpu;
                    r[LLMEM_D_OUT] = (i64)m_out;
                    r[LLMEM_D_LM] = (i64)m_lm;
                    r[LLMEM_D_BACK] = (i64)m_back;
                    r[LLMEM_D_K] = (i64)k_used;
                    r[LLMEM_D_PEAK_LIVE] = peak_live;
                    r[LLMEM_D_NPARAMS] = (i64)n_params;
                    r[LLMEM_D_TMAX] = (i64)t_max;
                    r[LLMEM_D_FLAGS] = (i64)flags;
                }
            }
            // park the results of configuration c in lane c
            acc[LLMEM_D_PEAK] = write_lane(acc[LLMEM_D_PEAK], r[LLMEM_D_PEAK], c, lane);
            if (DETAIL) {
#pragma unroll
                for (int q = 1; q < LLMEM_NDETAIL; ++q) acc[q] = write_lane(acc[q], r[q], c, lane);
            }
        }

        if (in_range) {
            if (a.out_peaks) a.out_peaks[i] = acc[LLMEM_D_PEAK];
            if (DETAIL) {
#pragma unroll
                for (int q = 0; q < LLMEM_NDETAIL; ++q) a.out_detail[(long long)q * n + i] = acc[q];
            }
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
static thread_local char g_hip_error[256] = "";

static int log2_exact(int64_t v)
{
    if (v < 1 || (v & (v - 1))) return -1;
    int s = 0;
    while ((int64_t(1) << s) < v) ++s;
    return s;
}

// Size expression as the compiled tables carry it: the selectors that are not LLMEM_DIM_ONE and
// their number.  `sorted_dims` holds four selectors in ascending order, one per byte.  One batch
// size and one sequence length together become the selector DIM_BS_SL of their product, which
// the kernel keeps ready (both are below 2^16, so it fits 32 bits): one multiplication less.
static uint32_t descriptor_of(uint32_t sorted_dims)
{
    uint32_t sel[4], n = 0;
    bool has_bs = false, has_sl = false;
    for (int q = 0; q < 4; ++q) {
        const uint32_t v = (sorted_dims >> (8 * q)) & 15u;
        has_bs = has_bs || v == LLMEM_DIM_BS;
        has_sl = has_sl || v == LLMEM_DIM_SL;
    }
    bool pair = has_bs && has_sl, bs_done = false, sl_done = false;
    for (int q = 0; q < 4; ++q) {
        const uint32_t v = (sorted_dims >> (8 * q)) & 15u;
        if (v == LLMEM_DIM_ONE) continue;
        if (pair && v == LLMEM_DIM_BS && !bs_done) { bs_done = true; sel[n++] = DIM_BS_SL; continue; }
        if (pair && v == LLMEM_DIM_SL && !sl_done) { sl_done = true; continue; }
        sel[n++] = v;
    }
    uint32_t desc = n;
    for (uint32_t q = 0; q < n; ++q) desc |= sel[q] << (4 + 4 * q);
    return desc;
}

// Parameter entries of one architecture grouped by size expression, in the compiled tables'
// format (estimate_args.h): four words per group into `words`, which holds up to `max_groups`
// groups.  Returns the number of groups, or -1 if there are more; *e_n: the embedding tables
// whose outputs are kept (Sec. 4.2, m_out).
int compile_param_groups(const llmem_param_entry *pe, int n_param, uint32_t *words, int max_groups, uint32_t *e_n)
{
    struct Group { uint32_t coef, dims; uint32_t cnt[8]; };      // E, LM, OTHER, OS x once, per block
    std::vector<Group> groups;
    *e_n = 0;
    for (int j = 0; j < n_param; ++j) {
        const uint32_t *w = reinterpret_cast<const uint32_t *>(&pe[j]);
        const ClassKey k = make_class_key(w[0], w[1], 0u);         // sorts the selectors
        size_t g = 0;
        for (; g < groups.size(); ++g) if (groups[g].coef == k.coef && groups[g].dims == k.dims) break;
        if (g == groups.size()) groups.push_back(Group{k.coef, k.dims, {0, 0, 0, 0, 0, 0, 0, 0}});
        const int layer = pe[j].per_layer ? 1 : 0;
        const int role = pe[j].role == LLMEM_ROLE_EMBED_TOK ? 0 : pe[j].role == LLMEM_ROLE_LM_HEAD ? 1 : 2;
        ++groups[g].cnt[2 * role + layer];
        if (pe[j].cls <= LLMEM_CLS_LINEAR && pe[j].role != LLMEM_ROLE_LM_HEAD) ++groups[g].cnt[6 + layer];
        if (pe[j].cls == LLMEM_CLS_EMBEDDING && pe[j].role != LLMEM_ROLE_LM_HEAD) ++*e_n;
    }
    if ((int)groups.size() > max_groups) return -1;
    for (const Group &g : groups) {
        *words++ = g.coef;
        *words++ = descriptor_of(g.dims);
        *words++ = g.cnt[0] | (g.cnt[1] << 8) | (g.cnt[2] << 16) | (g.cnt[3] << 24);
        *words++ = g.cnt[4] | (g.cnt[5] << 8) | (g.cnt[6] << 16) | (g.cnt[7] << 24);
    }
    return (int)groups.size();
}

// Compiles the tables of one architecture for the lane-per-configuration kernel: parameter
// entries grouped by size expression; size classes of the events; then per segment the
// class-count vectors at the peak points (an allocation followed by a release or by the end of the
// segment), minus those another point dominates component-wise (class values are never negative,
// so a dominated point cannot hold the maximum), then the segment's net change.  Appends 32-bit
// words to `prog`; returns false if the architecture does not fit.
static bool compile_tables(const llmem_param_entry *pe, int n_param, const llmem_event_entry *ev, int n_event,
                           const int *seg_first, ArchLayout *al, std::vector<uint32_t> *prog, int *p_slots,
                           int *stats)
{
    // ---- parameter groups ----
    uint32_t group_words[4 * 255], e_n = 0;
    const int n_groups = compile_param_groups(pe, n_param, group_words, 255, &e_n);
    // ---- size classes ----
    std::vector<ClassKey> classes;
    std::vector<int> cls_of(n_event);
    for (int j = 0; j < n_event; ++j) {
        const uint32_t *w = reinterpret_cast<const uint32_t *>(&ev[j]);
        const ClassKey k = make_class_key(w[0], w[1], w[2]);
        int c = 0;
        for (; c < (int)classes.size(); ++c)
            if (classes[c].coef == k.coef && classes[c].dims == k.dims && classes[c].meta == k.meta) break;
        if (c == (int)classes.size()) classes.push_back(k);
        cls_of[j] = c;
    }
    const int nc = (int)classes.size();
    if (nc > CLS_MAX || n_groups < 0 || e_n > 255) return false;
    // Classes with the same dimensions become neighbours, the smaller coefficient * element width
    // first: where the next one's is 2^k times as large, its raw size is the previous one shifted.
    {
        std::vector<int> order(nc), place(nc);
        for (int c = 0; c < nc; ++c) order[c] = c;
        auto c64_of = [&](int c) { return (uint64_t)classes[c].coef * (classes[c].meta & 255u); };
        std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
            if (classes[a].dims != classes[b].dims) return classes[a].dims < classes[b].dims;
            return c64_of(a) < c64_of(b);
        });
        std::vector<ClassKey> sorted(nc);
        for (int q = 0; q < nc; ++q) { sorted[q] = classes[order[q]]; place[order[q]] = q; }
        classes = sorted;
        for (int j = 0; j < n_event; ++j) cls_of[j] = place[cls_of[j]];
    }
    al->prog_first = (int)prog->size();
    prog->push_back((uint32_t)n_groups | (e_n << 8) | ((uint32_t)nc << 16));
    for (int q = 1; q < PROG_HEADER; ++q) prog->push_back(0u);     // segment boundaries, filled in below
    for (int q = 0; q < 4 * n_groups; ++q) prog->push_back(group_words[q]);
    // ---- peak points and net change of every segment ----
    std::vector<std::vector<int>> seg_sums[LLMEM_NSEG];           // kept points, then the net change last
    const int n_slots = nc + 1;                                   // slot 0 holds 0, slot c + 1 minus the value of class c
    for (int s = 0; s < LLMEM_NSEG; ++s) {
        std::vector<std::vector<int>> points;
        std::vector<int> count(nc, 0);
        for (int j = seg_first[s]; j < seg_first[s + 1]; ++j) {
            const bool is_free = ev[j].flags & LLMEM_EV_FREE;
            count[cls_of[j]] += is_free ? -1 : 1;
            if (!is_free && (j + 1 == seg_first[s + 1] || (ev[j + 1].flags & LLMEM_EV_FREE))) points.push_back(count);
        }
        for (size_t j = 0; j < points.size(); ++j) {
            bool dominated = false;
            for (size_t k = 0; k < points.size() && !dominated; ++k) {
                if (k == j) continue;
                bool le = true, lt = false;
                for (int c = 0; c < nc; ++c) { le = le && points[j][c] <= points[k][c]; lt = lt || points[j][c] < points[k][c]; }
                dominated = le && (lt || k < j);
            }
            if (!dominated) seg_sums[s].push_back(points[j]);
        }
        seg_sums[s].push_back(count);
    }
    if (n_slots > PROG_SLOT_MAX) return false;
    stats[0] += n_groups;
    stats[1] += nc;
    if (n_slots > *p_slots) *p_slots = n_slots;
    // ---- emit: classes, then the terms of every segment ----
    for (int c = 0; c < nc; ++c) {
        const ClassKey &k = classes[c];
        const uint64_t c64 = (uint64_t)k.coef * (k.meta & 255u);   // coefficient * element bytes
        if (c64 >> 32) return false;
        const uint32_t flags = (k.meta >> 8) & 255u, mask = (k.meta >> 16) & 7u;
        uint32_t first_word = (uint32_t)c64, size_desc = descriptor_of(k.dims);
        if (c > 0 && classes[c - 1].dims == k.dims) {
            const uint64_t before = (uint64_t)classes[c - 1].coef * (classes[c - 1].meta & 255u);
            for (uint32_t shift = 0; shift < 32 && before != 0; ++shift)
                if (before << shift == c64) { first_word = shift; size_desc = DESC_FROM_PREVIOUS; break; }
        }
        prog->push_back(first_word);
        prog->push_back(size_desc | ((flags & LLMEM_EV_TP_GATHER) ? DESC_TP_GATHER : 0u)
                        | ((flags & LLMEM_EV_TIMES_L) ? DESC_TIMES_L : 0u) | (mask << DESC_MASK_SHIFT));
    }
    for (int c = nc; c % PROG_CLASS_FETCH; ++c) { prog->push_back(0u); prog->push_back(0u); }   // empty classes
    for (int s = 0; s < LLMEM_NSEG; ++s) {
        al->prog_seg[s] = (int)prog->size();
        for (size_t j = 0; j < seg_sums[s].size(); ++j) {
            const std::vector<int> &v = seg_sums[s][j];
            const bool is_point = j + 1 < seg_sums[s].size();     // the last sum is the net change: stays open
            const size_t group_first = prog->size();
            for (int c = 0; c < nc; ++c) {
                if (v[c] == 0) continue;
                if (v[c] > 32767 || v[c] < -32767) return false;
                // the slot holds minus the value: the factor is minus the count, as a signed 16-bit field
                prog->push_back((uint32_t)(c + 1) * SLOT_ROW | ((uint32_t)(uint16_t)(int16_t)(-v[c]) << 16));
                ++stats[2];                                                         // (class, count) terms
            }
            stats[3] += is_point ? 1 : 0;                                           // peak points
            if (prog->size() == group_first) prog->push_back(0u);                   // an empty sum still has a group
            while ((prog->size() - group_first) % PROG_GROUP) prog->push_back(0u);
            // the flag sits in the first word of the sum's last group
            (*prog)[prog->size() - PROG_GROUP] |= is_point ? PROG_END_POINT : PROG_END_SEGMENT;
        }
    }
    // the kernel fetches PROG_FETCH words at a time: groups of padding terms fill the tail
    while ((prog->size() - (size_t)al->prog_seg[0]) % PROG_FETCH) prog->push_back(0u);
    al->prog_seg[LLMEM_NSEG] = (int)prog->size();
    for (int q = 0; q <= LLMEM_NSEG; ++q) (*prog)[al->prog_first + 1 + q] = (uint32_t)al->prog_seg[q];
    return prog->size() <= (size_t)PROG_WORDS;
}

// Checks the host copy of the tables and derives the lane layout of every
// architecture's events.  Returns LLMEM_OK or LLMEM_EINVAL_*.
static int plan_tables(const llmem_tables *t, EstimateArgs *out, bool *wave_ok, bool *batch_ok, bool *prog_ok,
                       int *prog_words = nullptr, int *prog_stats = nullptr)
{
    int stats_local[4] = {0, 0, 0, 0};
    int *stats = prog_stats ? prog_stats : stats_local;
    *wave_ok = true;
    *batch_ok = true;
    *prog_ok = true;
    std::vector<uint32_t> prog;
    if (!t->params_host && t->n_param_total > 0) return LLMEM_EINVAL_NULL;
    if (!t->events_host && t->n_event_total > 0) return LLMEM_EINVAL_NULL;
    if (!t->params_dev && t->n_param_total > 0) return LLMEM_EINVAL_NULL;
    if (!t->events_dev && t->n_event_total > 0) return LLMEM_EINVAL_NULL;
    if (t->n_arch < 1 || t->n_arch > LLMEM_MAX_ARCH) return LLMEM_EINVAL_TABLE;
    if (t->n_param_total < 0 || t->n_event_total < 0) return LLMEM_EINVAL_TABLE;
    if (t->n_param_total > LLMEM_MAX_ARCH * LLMEM_MAX_PARAM_ENTRIES) return LLMEM_EINVAL_TABLE;
    const int cu_shift = log2_exact(t->cu_p), align_shift = log2_exact(t->align);
    if (cu_shift < 0 || align_shift < 0 || cu_shift > 40 || t->align > t->cu_p || t->m_base < 0)
        return LLMEM_EINVAL_TABLE;
    out->cu_shift = cu_shift;
    out->align_shift = align_shift;
    out->m_base = t->m_base;
    out->n_arch = t->n_arch;
    out->n_param_total = t->n_param_total;
    int slot = 0, code = 0;
    for (int ar = 0; ar < t->n_arch; ++ar) {
        const llmem_arch_desc &d = t->arch[ar];
        ArchLayout &al = out->arch[ar];
        if (d.param_first < 0 || d.n_param < 0 || d.n_param > LLMEM_MAX_PARAM_ENTRIES
            || (int64_t)d.param_first + d.n_param > t->n_param_total) return LLMEM_EINVAL_TABLE;
        if (d.event_first < 0 || d.n_event < 0 || d.n_event > LLMEM_MAX_EVENT_ENTRIES
            || (int64_t)d.event_first + d.n_event > t->n_event_total) return LLMEM_EINVAL_TABLE;
        for (int j = 0; j < d.n_param; ++j) {
            const llmem_param_entry &p = t->params_host[d.param_first + j];
            for (int q = 0; q < 4; ++q) if (p.dim[q] >= LLMEM_NDIM) return LLMEM_EINVAL_TABLE;
            if (p.cls > LLMEM_CLS_NORM || p.role > LLMEM_ROLE_OTHER || p.per_layer > 1) return LLMEM_EINVAL_TABLE;
        }
        int seg_count[LLMEM_NSEG] = {0, 0, 0, 0, 0};
        int prev_seg = 0;
        for (int j = 0; j < d.n_event; ++j) {
            const llmem_event_entry &e = t->events_host[d.event_first + j];
            for (int q = 0; q < 4; ++q) if (e.dim[q] >= LLMEM_NDIM) return LLMEM_EINVAL_TABLE;
            if (e.seg >= LLMEM_NSEG || e.seg < prev_seg) return LLMEM_EINVAL_TABLE;
            if (e.flags & ~(LLMEM_EV_FREE | LLMEM_EV_TIMES_L | LLMEM_EV_TP_GATHER)) return LLMEM_EINVAL_TABLE;
            if (e.method_mask & ~7u) return LLMEM_EINVAL_TABLE;
            prev_seg = e.seg;
            ++seg_count[e.seg];
        }
        al.param_first = d.param_first;
        al.n_param = d.n_param;
        al.event_first = d.event_first;
        al.seg_first[0] = 0;
        for (int s = 0; s < LLMEM_NSEG; ++s) al.seg_first[s + 1] = al.seg_first[s] + seg_count[s];
        // smallest events-per-lane such that whole lanes per segment fit in one wave
        int per_lane = 1;
        for (;; ++per_lane) {
            int lanes = 0;
            for (int s = 0; s < LLMEM_NSEG; ++s) lanes += (seg_count[s] + per_lane - 1) / per_lane;
            if (lanes <= 64) break;
        }
        if (d.n_event == 0) per_lane = 0;
        al.per_lane = per_lane;
        al.lane0[0] = 0;
        for (int s = 0; s < LLMEM_NSEG; ++s)
            al.lane0[s + 1] = al.lane0[s] + (per_lane ? (seg_count[s] + per_lane - 1) / per_lane : 0);
        al.slot_first = slot;
        slot += per_lane * 64;
        // lane-per-configuration kernel: padded event codes, size classes and value slots
        al.code_first = code;
        al.seg_code[0] = 0;
        for (int s = 0; s < LLMEM_NSEG; ++s)
            al.seg_code[s + 1] = al.seg_code[s] + (seg_count[s] + CODE_GROUP - 1) / CODE_GROUP * CODE_GROUP;
        code += al.seg_code[LLMEM_NSEG];
        if (d.n_event > out->max_events) out->max_events = d.n_event;
        int n_class = 0;
        for (int j = 0; j < d.n_event && n_class <= CLS_MAX; ++j) {
            const uint32_t *w = reinterpret_cast<const uint32_t *>(&t->events_host[d.event_first + j]);
            const ClassKey kj = make_class_key(w[0], w[1], w[2]);
            bool first_of_class = true;
            for (int q = 0; q < j && first_of_class; ++q) {
                const uint32_t *v = reinterpret_cast<const uint32_t *>(&t->events_host[d.event_first + q]);
                const ClassKey kq = make_class_key(v[0], v[1], v[2]);
                first_of_class = !(kq.coef == kj.coef && kq.dims == kj.dims && kq.meta == kj.meta);
            }
            if (first_of_class) ++n_class;
        }
        if (n_class > CLS_MAX) *batch_ok = false;
        if (n_class + 1 > out->s_slots) out->s_slots = n_class + 1;
        if (*prog_ok && !compile_tables(t->params_host + d.param_first, d.n_param, t->events_host + d.event_first, d.n_event,
                                        al.seg_first, &al, &prog, &out->p_slots, stats))
            *prog_ok = false;
    }
    if (*prog_ok) for (size_t q = 0; q < prog.size(); ++q) out->prog[q] = prog[q];
    if (prog_words) *prog_words = (int)prog.size();
    out->n_slot_total = slot;
    out->code_count = code;
    if (out->s_slots < 1) out->s_slots = 1;
    if (out->p_slots < 1) out->p_slots = 1;
    // each lane form needs its value slots to fit the LDS of a workgroup of at least one wavefront
    out->use_program = 1;
    if (*prog_ok && batch_kernel_waves(*out) == 0) *prog_ok = false;
    out->use_program = 0;
    if (*batch_ok && batch_kernel_waves(*out) == 0) *batch_ok = false;
    out->waves = BATCH_WAVES;                 // the launch sets it for the form it takes
    *wave_ok = slot <= LLMEM_MAX_EVENT_SLOTS;
    return LLMEM_OK;
}

// plan_tables costs tens to hundreds of microseconds (the classes and the dominance test of the
// peak points are quadratic in the events), more than a launch over a small grid.  Its result
// depends on the contents of the host tables alone, so each host thread keeps the plans of the last
// few table sets it was called with and takes one over when every byte it was made from is the
// same: constants, ranges and the entries inside the ranges (a comparison of a few KB).  The
// tables are still checked in full whenever anything in them differs; a plan that was refused is
// not kept.  `out` arrives zeroed, as plan_tables expects.
namespace {

struct PlanKey {
    int64_t m_base, cu_p, align;
    int32_t n_arch, n_param_total, n_event_total;
    llmem_arch_desc arch[LLMEM_MAX_ARCH];
};

struct KeptPlan {
    bool used = false;
    PlanKey key;
    std::vector<llmem_param_entry> params;      // the entries inside the ranges, architecture by architecture
    std::vector<llmem_event_entry> events;
    EstimateArgs args;
    bool wave_ok, batch_ok, prog_ok;
    int words, stats[4];
};

constexpr int KEPT_PLANS = 4;

bool ranges_readable(const llmem_tables *t)
{
    if ((!t->params_host || !t->params_dev) && t->n_param_total > 0) return false;
    if ((!t->events_host || !t->events_dev) && t->n_event_total > 0) return false;
    if (t->n_arch < 1 || t->n_arch > LLMEM_MAX_ARCH || t->n_param_total < 0 || t->n_event_total < 0) return false;
    for (int ar = 0; ar < t->n_arch; ++ar) {
        const llmem_arch_desc &d = t->arch[ar];
        if (d.param_first < 0 || d.n_param < 0 || d.n_param > LLMEM_MAX_PARAM_ENTRIES
            || (int64_t)d.param_first + d.n_param > t->n_param_total) return false;
        if (d.event_first < 0 || d.n_event < 0 || d.n_event > LLMEM_MAX_EVENT_ENTRIES
            || (int64_t)d.event_first + d.n_event > t->n_event_total) return false;
    }
    return true;
}

bool same_tables(const KeptPlan &k, const PlanKey &key, const llmem_tables *t)
{
    if (!k.used || memcmp(&k.key, &key, sizeof(key)) != 0) return false;
    size_t p = 0, e = 0;
    for (int ar = 0; ar < t->n_arch; ++ar) {
        const llmem_arch_desc &d = t->arch[ar];
        if (d.n_param && memcmp(&k.params[p], t->params_host + d.param_first, sizeof(llmem_param_entry) * d.n_param)) return false;
        if (d.n_event && memcmp(&k.events[e], t->events_host + d.event_first, sizeof(llmem_event_entry) * d.n_event)) return false;
        p += d.n_param;
        e += d.n_event;
    }
    return true;
}

}  // namespace

static int plan_tables_kept(const llmem_tables *t, EstimateArgs *out, bool *wave_ok, bool *batch_ok, bool *prog_ok,
                            int *prog_words = nullptr, int *prog_stats = nullptr)
{
    if (!ranges_readable(t)) return plan_tables(t, out, wave_ok, batch_ok, prog_ok, prog_words, prog_stats);   // reports what is wrong
    static thread_local KeptPlan kept[KEPT_PLANS];
    static thread_local int next = 0;
    PlanKey key;
    memset(&key, 0, sizeof(key));                           // padding and unused architectures compare equal
    key.m_base = t->m_base; key.cu_p = t->cu_p; key.align = t->align;
    key.n_arch = t->n_arch; key.n_param_total = t->n_param_total; key.n_event_total = t->n_event_total;
    for (int ar = 0; ar < t->n_arch; ++ar) key.arch[ar] = t->arch[ar];
    for (int q = 0; q < KEPT_PLANS; ++q) {
        const KeptPlan &k = kept[q];
        if (!same_tables(k, key, t)) continue;
        *out = k.args;
        *wave_ok = k.wave_ok; *batch_ok = k.batch_ok; *prog_ok = k.prog_ok;
        if (prog_words) *prog_words = k.words;
        if (prog_stats) for (int i = 0; i < 4; ++i) prog_stats[i] += k.stats[i];
        return LLMEM_OK;
    }
    int words = 0, stats[4] = {0, 0, 0, 0};
    const int rc = plan_tables(t, out, wave_ok, batch_ok, prog_ok, &words, stats);
    if (prog_words) *prog_words = words;
    if (prog_stats) for (int i = 0; i < 4; ++i) prog_stats[i] += stats[i];
    if (rc != LLMEM_OK) return rc;
    KeptPlan &k = kept[next];
    next = (next + 1) % KEPT_PLANS;
    k.used = false;
    k.key = key;
    k.params.clear();
    k.events.clear();
    for (int ar = 0; ar < t->n_arch; ++ar) {
        const llmem_arch_desc &d = t->arch[ar];
        if (d.n_param) k.params.insert(k.params.end(), t->params_host + d.param_first, t->params_host + d.param_first + d.n_param);
        if (d.n_event) k.events.insert(k.events.end(), t->events_host + d.event_first, t->events_host + d.event_first + d.n_event);
    }
    k.args = *out;
    k.wave_ok = *wave_ok; k.batch_ok = *batch_ok; k.prog_ok = *prog_ok;
    k.words = words;
    for (int i = 0; i < 4; ++i) k.stats[i] = stats[i];
    k.used = true;
    return rc;
}

int check_tables(const llmem_tables *tables, EstimateArgs *out)
{
    memset(out, 0, sizeof(*out));
    bool wave_ok, batch_ok, prog_ok;
    return plan_tables_kept(tables, out, &wave_ok, &batch_ok, &prog_ok);
}

static int launch_estimate(const llmem_configs *cfg, int64_t n, const llmem_tables *tables,
                           int64_t *out_peaks, int64_t *out_detail, hipStream_t stream)
{
    if (!cfg || !tables) return LLMEM_EINVAL_NULL;
    if (!out_peaks && !out_detail) return LLMEM_EINVAL_NULL;
    if (n < 0) return LLMEM_EINVAL_N;
    EstimateArgs args;
    memset(&args, 0, sizeof(args));
    bool wave_ok, batch_ok, prog_ok;
    int rc = plan_tables_kept(tables, &args, &wave_ok, &batch_ok, &prog_ok);
    if (rc != LLMEM_OK) return rc;
    // which kernel (see LLMEM_KERNEL_* in the header)
    const int hint = tables->kernel;
    const int flavour = out_detail ? 1 : 0;
    args.use_program = prog_ok ? 1 : 0;
    const int lane_form = !prog_ok ? (batch_ok ? LLMEM_KERNEL_LANE_EVENTS : LLMEM_KERNEL_LANE_DIRECT)
                          : has_prebuilt(args, flavour) ? LLMEM_KERNEL_LANE_SPECIALIZED : LLMEM_KERNEL_LANE_COMPILED;
    int choice;
    switch (hint) {
    case LLMEM_KERNEL_AUTO:
    case LLMEM_KERNEL_LANE: choice = lane_form; break;
    case LLMEM_KERNEL_WAVE: choice = wave_ok ? hint : -1; break;
    case LLMEM_KERNEL_LANE_EVENTS: choice = batch_ok ? hint : -1; break;
    case LLMEM_KERNEL_LANE_COMPILED:
    case LLMEM_KERNEL_LANE_SPECIALIZED:
    case LLMEM_KERNEL_LANE_RUNTIME: choice = prog_ok ? hint : -1; break;
    case LLMEM_KERNEL_LANE_DIRECT: choice = hint; break;
    default: choice = -1;
    }
    if (choice < 0) return LLMEM_EINVAL_TABLE;
    const bool use_batch = choice != LLMEM_KERNEL_WAVE;
    args.use_program = (choice >= LLMEM_KERNEL_LANE_COMPILED && choice != LLMEM_KERNEL_LANE_DIRECT) ? 1 : 0;
    args.direct = choice == LLMEM_KERNEL_LANE_DIRECT ? 1 : 0;
    if (use_batch) args.waves = batch_kernel_waves(args);
    if (n == 0) return LLMEM_OK;
    if (!cfg->arch_id || !cfg->h || !cfg->L || !cfg->n_heads || !cfg->n_kv || !cfg->ffn || !cfg->V
        || !cfg->P || !cfg->bs || !cfg->sl || !cfg->method || !cfg->d || !cfg->chunk_k || !cfg->flags)
        return LLMEM_EINVAL_NULL;
    args.cfg = *cfg;
    args.n = n;
    args.params_dev = reinterpret_cast<const uint4 *>(tables->params_dev);
    args.events_dev = reinterpret_cast<const uint4 *>(tables->events_dev);
    args.out_peaks = reinterpret_cast<long long *>(out_peaks);
    args.out_detail = reinterpret_cast<long long *>(out_detail);

    const int64_t n_batch = (n + 63) / 64;
    if (choice == LLMEM_KERNEL_LANE_SPECIALIZED || choice == LLMEM_KERNEL_LANE_RUNTIME)
        return launch_specialized(args, flavour, n_batch, stream, choice == LLMEM_KERNEL_LANE_RUNTIME);
    if (use_batch) {
        launch_batch_kernel(args, out_detail != nullptr, n_batch, stream);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) {
            snprintf(g_hip_error, sizeof(g_hip_error), "HIP error: %s", hipGetErrorString(e));
            return LLMEM_EHIP;
        }
        return LLMEM_OK;
    }
    const size_t lds_bytes = sizeof(uint4) * (size_t)(args.n_param_total + args.n_slot_total);
    int64_t blocks = (n_batch + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
    const int64_t max_blocks = 256 * 16;          // 256 CUs, a few resident workgroups each
    if (blocks > max_blocks) blocks = max_blocks;
    if (out_detail)
        hipLaunchKernelGGL(estimate_kernel<true>, dim3((unsigned)blocks), dim3(BLOCK), lds_bytes, stream, args);
    else
        hipLaunchKernelGGL(estimate_kernel<false>, dim3((unsigned)blocks), dim3(BLOCK), lds_bytes, stream, args);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        snprintf(g_hip_error, sizeof(g_hip_error), "HIP error: %s", hipGetErrorString(e));
        return LLMEM_EHIP;
    }
    return LLMEM_OK;
}

static int launch_status()
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        snprintf(g_hip_error, sizeof(g_hip_error), "HIP error: %s", hipGetErrorString(e));
        return LLMEM_EHIP;
    }
    return LLMEM_OK;
}

static int launch_sweep(int grid_id, uint64_t seed, int64_t first, int64_t n, const llmem_tables *tables,
                        int64_t m_total, int64_t *stats, hipStream_t stream)
{
    if (!tables || !stats) return LLMEM_EINVAL_NULL;
    if (n < 0 || first < 0) return LLMEM_EINVAL_N;
    if (grid_id < 1 || grid_id > 4) return LLMEM_EINVAL_ARG;
    if (grid_id == 1 && first + n > 432) return LLMEM_EINVAL_ARG;
    if (first > (1ll << SWEEP_INDEX_BITS) || n > (1ll << SWEEP_INDEX_BITS) - first) return LLMEM_EINVAL_ARG;
    EstimateArgs args;
    memset(&args, 0, sizeof(args));
    bool wave_ok, batch_ok, prog_ok;
    int rc = plan_tables_kept(tables, &args, &wave_ok, &batch_ok, &prog_ok);
    if (rc != LLMEM_OK) return rc;
    // the lane forms only; a hint that names one of them is honoured
    const int hint = tables->kernel;
    args.use_program = prog_ok ? 1 : 0;
    const int lane_form = !prog_ok ? (batch_ok ? LLMEM_KERNEL_LANE_EVENTS : LLMEM_KERNEL_LANE_DIRECT)
                          : has_prebuilt(args, 2) ? LLMEM_KERNEL_LANE_SPECIALIZED : LLMEM_KERNEL_LANE_COMPILED;
    int choice;
    switch (hint) {
    case LLMEM_KERNEL_AUTO:
    case LLMEM_KERNEL_LANE: choice = lane_form; break;
    case LLMEM_KERNEL_LANE_EVENTS: choice = batch_ok ? hint : -1; break;
    case LLMEM_KERNEL_LANE_COMPILED:
    case LLMEM_KERNEL_LANE_SPECIALIZED:
    case LLMEM_KERNEL_LANE_RUNTIME: choice = prog_ok ? hint : -1; break;
    case LLMEM_KERNEL_LANE_DIRECT: choice = hint; break;
    default: choice = -1;
    }
    if (choice < 0) return LLMEM_EINVAL_TABLE;
    if (n == 0) return LLMEM_OK;
    args.use_program = (choice >= LLMEM_KERNEL_LANE_COMPILED && choice != LLMEM_KERNEL_LANE_DIRECT) ? 1 : 0;
    args.direct = choice == LLMEM_KERNEL_LANE_DIRECT ? 1 : 0;
    args.waves = batch_kernel_waves(args);
    args.n = n;
    args.params_dev = reinterpret_cast<const uint4 *>(tables->params_dev);
    args.events_dev = reinterpret_cast<const uint4 *>(tables->events_dev);
    args.sweep_grid = grid_id;
    args.sweep_seed = seed;
    args.sweep_first = first;
    args.m_total = m_total;
    args.sweep_stats = reinterpret_cast<unsigned long long *>(stats);
    if (choice == LLMEM_KERNEL_LANE_SPECIALIZED || choice == LLMEM_KERNEL_LANE_RUNTIME)
        return launch_specialized(args, 2, (n + 63) / 64, stream, choice == LLMEM_KERNEL_LANE_RUNTIME);
    launch_sweep_kernel(args, (n + 63) / 64, stream);
    return launch_status();
}

const char *last_hip_error() { return g_hip_error; }
void set_error_text(const char *text) { snprintf(g_hip_error, sizeof(g_hip_error), "%s", text); }

}  // namespace llmem

extern "C" int llmem_kernel_forms(const llmem_tables *tables, int32_t info[8])
{
    using namespace llmem;
    if (!tables || !info) return LLMEM_EINVAL_NULL;
    static_assert(LLMEM_PROGRAM_WORDS == PROG_WORDS, "header and kernel arguments disagree");
    EstimateArgs args;
    memset(&args, 0, sizeof(args));
    bool wave_ok, batch_ok, prog_ok;
    int words = 0;
    int stats[4] = {0, 0, 0, 0};
    const int rc = plan_tables_kept(tables, &args, &wave_ok, &batch_ok, &prog_ok, &words, stats);
    if (rc != LLMEM_OK) return rc;
    for (int q = 0; q < 8; ++q) info[q] = 0;
    info[0] = (wave_ok ? 1 << LLMEM_KERNEL_WAVE : 0) | (batch_ok ? 1 << LLMEM_KERNEL_LANE_EVENTS : 0)
              | (prog_ok ? 1 << LLMEM_KERNEL_LANE_COMPILED : 0) | (1 << LLMEM_KERNEL_LANE) | (1 << LLMEM_KERNEL_LANE_DIRECT)
              | (prog_ok ? (1 << LLMEM_KERNEL_LANE_SPECIALIZED) | (1 << LLMEM_KERNEL_LANE_RUNTIME) : 0);
    if (prog_ok) {
        args.use_program = 1;
        for (int flavour = 0; flavour < 3; ++flavour)
            if (has_prebuilt(args, flavour)) info[0] |= LLMEM_FORMS_PREBUILT_PEAKS << flavour;
    }
    info[1] = words;
    info[2] = args.p_slots;
    info[3] = args.s_slots;
    info[4] = args.n_slot_total;
    if (prog_ok) { info[5] = stats[0] | (stats[1] << 16); info[6] = stats[2]; info[7] = stats[3]; }
    return LLMEM_OK;
}

extern "C" int llmem_compiled_tables(const llmem_tables *tables, uint32_t *words, int32_t max_words,
                                     int32_t first[LLMEM_MAX_ARCH])
{
    using namespace llmem;
    if (!tables || !words || !first) return LLMEM_EINVAL_NULL;
    EstimateArgs args;
    memset(&args, 0, sizeof(args));
    bool wave_ok, batch_ok, prog_ok;
    int n_words = 0;
    const int rc = plan_tables_kept(tables, &args, &wave_ok, &batch_ok, &prog_ok, &n_words);
    if (rc != LLMEM_OK) return rc;
    if (!prog_ok) return LLMEM_EINVAL_TABLE;
    if (n_words > max_words) return LLMEM_EINVAL_ARG;
    for (int q = 0; q < n_words; ++q) words[q] = args.prog[q];
    for (int q = 0; q < LLMEM_MAX_ARCH; ++q) first[q] = q < args.n_arch ? args.arch[q].prog_first : 0;
    return n_words;
}

extern "C" int llmem_kernels_release(void) { return llmem::release_built(); }

extern "C" uint64_t llmem_selftest_divide(uint64_t x, uint32_t d)
{
    static constexpr llmem::DivMagicTable table = llmem::DivMagicTable();
    if (d < 1 || d > 255) return 0;
    if (d == 1) return x;
    const unsigned __int128 prod = (unsigned __int128)x * table.t[d].mul;
    return (uint64_t)(prod >> 64) >> table.t[d].shift;
}

extern "C" int llmem_sweep(int grid_id, uint64_t seed, int64_t first, int64_t n, const llmem_tables *method_tables,
                           int64_t m_total, int64_t *stats, void *hip_stream)
{
    return llmem::launch_sweep(grid_id, seed, first, n, method_tables, m_total, stats,
                               reinterpret_cast<hipStream_t>(hip_stream));
}

extern "C" int llmem_sweep_reset(int64_t *stats, void *hip_stream)
{
    if (!stats) return LLMEM_EINVAL_NULL;
    llmem::launch_sweep_reset(reinterpret_cast<long long *>(stats), reinterpret_cast<hipStream_t>(hip_stream));
    return llmem::launch_status();
}

extern "C" int llmem_estimate(const llmem_configs *cfg, int64_t n, const llmem_tables *method_tables,
                              int64_t *out_peaks)
{
    if (!out_peaks) return LLMEM_EINVAL_NULL;
    return llmem::launch_estimate(cfg, n, method_tables, out_peaks, nullptr, nullptr);
}

extern "C" int llmem_estimate_ex(const llmem_configs *cfg, int64_t n, const llmem_tables *method_tables,
                                 int64_t *out_peaks, int64_t *out_detail, void *hip_stream)
{
    return llmem::launch_estimate(cfg, n, method_tables, out_peaks, out_detail,
                                  reinterpret_cast<hipStream_t>(hip_stream));
}
