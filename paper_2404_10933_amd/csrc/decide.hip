// Estimates of all four fine-tuning methods and the method decision, one lane
// per query.
//
// A query is a model shape with gpu_n and sl.  What does not depend on the batch
// size is computed once per query: the parameter census (embed_p, lm_p, other_p,
// the largest tensor, m_os tensor by tensor), the chunk size, m_p / m_p16 / m_p32,
// the sharded model states of ZeRO-3 and TP, the share of param fp16 that DP+TP
// removes.  What grows with bs is a handful of products with per-query factors:
//   m_out(bs) = up(bs * (e_n + L) * sl * h * 2),  logits up(bs * V * B * sl) and
//   2 * up(bs * V * B * (sl - 1)),  m_back^tp(bs; t) = ceil(L * bs * sl * h * (t-1) * 2
//   / (t * cu_p)) * cu_p.
// llmem_estimate_methods evaluates the four estimates at the query's own bs.
// llmem_decide finds, per method, the largest bs whose estimate does not exceed
// m_total (the estimates never decrease with bs, so this is the batch size
// Algorithm 1 reaches by adding one at a time): a bracket from the linear growth
// of the estimate, then bisection inside it; then it scores and chooses.
// The parameter census reads the entries grouped by size expression (the groups
// travel in the kernel arguments) and the probes of the search count pages in 32
// bits where a query's sizes allow it; tables with too many groups and waves with
// a query beyond that take the entry-by-entry and the 64-bit forms of the same
// arithmetic.
//
// Closed forms: Sec. 4.2 and Sec. 5 of arXiv 2404.10933 (incl. the DP+TP equation);
// chunk size: Sec. 4.1; decision: Sec. 6, Algorithm 1.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/llmem.h"
#include "estimate_args.h"
#include "wave.h"

namespace llmem {

void set_hip_error(hipError_t e);

namespace {

constexpr int DC_WAVES = 4;
constexpr int DC_BLOCK = 64 * DC_WAVES;
constexpr int DC_GROUPS_MAX = 160;             // parameter groups of all architectures that fit the kernel arguments

struct DecideArgs {
    llmem_configs cfg;
    const uint8_t *tp_n;             // may be null: no DP+TP set-up anywhere
    long long n;
    long long m_base, m_total;
    int cu_shift, align_shift, n_arch;
    int param_first[LLMEM_MAX_ARCH], n_param[LLMEM_MAX_ARCH];
    const uint4 *params_dev;
    long long *out_peaks, *out_flags;          // estimate_methods
    int *out_method, *out_bs;                  // decide
    long long *out_detail;
    // parameter entries grouped by size expression (four words per group, the compiled tables'
    // format): architecture ar owns groups[group_first[ar] ..] (a word index), n_groups[ar] of them
    int use_groups;
    int group_first[LLMEM_MAX_ARCH], n_groups[LLMEM_MAX_ARCH], e_n[LLMEM_MAX_ARCH];
    uint32_t groups[4 * DC_GROUPS_MAX];
};
static_assert(sizeof(DecideArgs) <= 4096, "kernel arguments are limited to 4 KB");

__device__ __forceinline__ u64 d_div(u64 x, u32 d, DivMagic m) { return d == 1 ? x : (__umul64hi(x, m.mul) >> m.shift); }
__device__ __forceinline__ u64 d_cdiv(u64 x, u32 d, DivMagic m) { return d_div(x + (d - 1), d, m); }
__device__ __forceinline__ u64 d_up(u64 x, int shift) { return ((x + ((1ull << shift) - 1)) >> shift) << shift; }
__device__ __forceinline__ u32 d_uni(u32 v) { return (u32)__builtin_amdgcn_readfirstlane((int)v); }
// Results are written once and not read again: streaming stores, which do not keep the lines in
// the L2 (with ordinary stores the decision columns cost a quarter of the kernel's time).
__device__ __forceinline__ void put(long long *p, i64 v) { __builtin_nontemporal_store((long long)v, p); }
__device__ __forceinline__ void put(int *p, int v) { __builtin_nontemporal_store(v, p); }
// acc + x * m (mod 2^64): the low half's 64-bit product added in one instruction, the low 32 bits of
// the high half's product added to the upper word (three instructions where the plain expression
// compiles to five)
__device__ __forceinline__ u64 d_mad(u64 acc, u64 x, u32 m)
{
    const u64 low = (u64)(u32)x * (u64)m + acc;
    const u32 high = (u32)(x >> 32) * m;
    return low + ((u64)high << 32);
}
__device__ __forceinline__ u64 d_mul(u64 x, u32 m) { return d_mad(0ull, x, m); }
// ceil(x / d) for x + d - 1 < 2^32: the multiply-high of the 64-bit constant with a 32-bit dividend
__device__ __forceinline__ u32 d_cdiv32(u32 x, u32 d, DivMagic m)
{
    const u32 dividend = x + (d - 1);
    const u64 low = (u64)dividend * (u32)m.mul;
    const u64 high = (u64)dividend * (u32)(m.mul >> 32) + (low >> 32);
    return d == 1 ? x : (u32)(high >> 32) >> m.shift;
}

// what a query needs to evaluate any method at any batch size
struct QueryTerms {
    u64 fixed[4];        // batch-independent part of m_peak^s, m_peak^dp, m_peak^tp, m_peak^{dp+tp}
    u64 c_out;           // (e_n + L) * sl * h * B16
    u64 c_logits, c_shifted;   // V * B * sl,  V * B * max(sl - 1, 0)
    u64 c_back_tp, c_back_hy;  // L * sl * h * (t - 1) * B16 for t = gpu_n and t = tp_n
    u32 gpu_n, tp_n;
    DivMagic div_g, div_t;
    int cu_shift;
};

__device__ __forceinline__ u64 pages_over(u64 bytes, u32 t, DivMagic m, int cu_shift)
{
    const u64 pages = (bytes + ((1ull << cu_shift) - 1)) >> cu_shift;
    return d_cdiv(pages, t, m) << cu_shift;             // ceil(bytes / (t * cu_p)) * cu_p
}

// m_peak of method m (0..3) at batch size bs
__device__ __forceinline__ i64 peak_at(const QueryTerms &q, int m, u32 bs)
{
    const u64 b = bs;
    u64 x = q.fixed[m] + d_up(b * q.c_out, q.cu_shift) + d_up(b * q.c_logits, q.cu_shift)
            + 2 * d_up(b * q.c_shifted, q.cu_shift);
    if (m == LLMEM_METHOD_TP) x += pages_over(b * q.c_back_tp, q.gpu_n, q.div_g, q.cu_shift);
    if (m == LLMEM_METHOD_HYBRID) x += pages_over(b * q.c_back_hy, q.tp_n, q.div_t, q.cu_shift);
    return (i64)x;
}

template <bool DECIDE>
__global__ __launch_bounds__(DC_BLOCK) void decide_kernel(const DecideArgs a)
{
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const long long n = a.n;
    const long long n_batch = (n + 63) >> 6;
    const int cu_shift = a.cu_shift, align_shift = a.align_shift;

    for (long long b = (long long)blockIdx.x * DC_WAVES + wave; b < n_batch; b += (long long)gridDim.x * DC_WAVES) {
        // The 64 queries of a batch start at a wave-uniform position: every column is read at that
        // position plus the lane (a 32-bit offset); lanes past the end read the last query again and
        // are masked afterwards.  The column pointers are read from the argument segment again for
        // every batch (scalar loads) instead of occupying 30 scalar registers through all of it.
        const long long first = b << 6, left = n - first;
        const bool in_range = (long long)lane < left;
        const u32 last = left < 64 ? (u32)left - 1u : 63u;
        const u32 lane_at = (u32)lane < last ? (u32)lane : last;
        const char __attribute__((address_space(4))) *segment =
            (const char __attribute__((address_space(4))) *)__builtin_amdgcn_kernarg_segment_ptr();
        asm volatile("" : "+s"(segment));
#define LLMEM_COLUMN(field) (*(decltype(a.cfg.field) const __attribute__((address_space(4))) *)( \
        segment + __builtin_offsetof(DecideArgs, cfg) + __builtin_offsetof(llmem_configs, field)))
        const u32 h = (LLMEM_COLUMN(h) + first)[lane_at], ffn = (LLMEM_COLUMN(ffn) + first)[lane_at], V = (LLMEM_COLUMN(V) + first)[lane_at],
                  P = (LLMEM_COLUMN(P) + first)[lane_at], arch_id = (LLMEM_COLUMN(arch_id) + first)[lane_at],
                  g = (LLMEM_COLUMN(d) + first)[lane_at], cflags = (LLMEM_COLUMN(flags) + first)[lane_at],
                  L = (LLMEM_COLUMN(L) + first)[lane_at], n_heads = (LLMEM_COLUMN(n_heads) + first)[lane_at],
                  n_kv = (LLMEM_COLUMN(n_kv) + first)[lane_at], bs = (LLMEM_COLUMN(bs) + first)[lane_at],
                  sl = (LLMEM_COLUMN(sl) + first)[lane_at];
        const int chunk_k = (LLMEM_COLUMN(chunk_k) + first)[lane_at];
#undef LLMEM_COLUMN
        const u32 tp = a.tp_n ? (a.tp_n + first)[lane_at] : 0u;
        u32 err = 0;
        if (arch_id >= (u32)a.n_arch) err |= LLMEM_F_ERR_ARCH;
        if (g == 0) err |= LLMEM_F_ERR_D;
        if (n_heads == 0) err |= LLMEM_F_ERR_HEADS;
        if (!(chunk_k == -1 || (chunk_k >= 0 && chunk_k <= K_FIXED_MAX))) err |= LLMEM_F_ERR_CHUNK;
        const DivMagic div_g = c_div.t[g & 255u], div_t = c_div.t[tp & 255u];
        if (tp > 0 && g > 0 && g - (u32)d_div(g, tp, div_t) * tp != 0) err |= LLMEM_F_ERR_TP;
        const bool valid = in_range && err == 0;

        const u32 head_dim = h / (n_heads ? n_heads : 1u);
        u32 D[16];
        D[LLMEM_DIM_ONE] = 1; D[LLMEM_DIM_BS] = bs; D[LLMEM_DIM_SL] = sl; D[LLMEM_DIM_SL_M1] = sl ? sl - 1 : 0;
        D[LLMEM_DIM_H] = h; D[LLMEM_DIM_FFN] = ffn; D[LLMEM_DIM_N_HEADS] = n_heads; D[LLMEM_DIM_N_KV] = n_kv;
        D[LLMEM_DIM_HEAD_DIM] = head_dim; D[LLMEM_DIM_KV_DIM] = n_kv * head_dim; D[LLMEM_DIM_V] = V;
        D[LLMEM_DIM_P] = P; D[LLMEM_DIM_L] = L;
        const u32 Blog = (cflags & LLMEM_CFG_LOGITS_FP32) ? B32 : B16;
        D[LLMEM_DIM_B_LOGITS] = Blog; D[LLMEM_DIM_D] = g; D[DIM_BS_SL] = bs * sl;      // both below 2^16

        // ---- parameter table (Notation table; Sec. 4.2, equation for m_os), architecture by architecture
        u64 embed_p = 0, lm_p = 0, other_p = 0, t_max = 0, m_os = 0;
        u32 e_n = 0;
        unsigned long long todo = __builtin_amdgcn_ballot_w64(valid);
        while (todo) {
            const int first = __builtin_ctzll(todo);
            const u32 ar = read_lane(arch_id, first);
            const bool mine = valid && arch_id == ar;
            todo &= ~__builtin_amdgcn_ballot_w64(mine);
            if (!mine) continue;
            if (a.use_groups) {
                // entries with the same size expression arrive as one group with the number of
                // entries that count towards each sum, once and once per block
                const int n_groups = (int)d_uni((u32)a.n_groups[ar]);
                int at = (int)d_uni((u32)a.group_first[ar]);
                e_n = d_uni((u32)a.e_n[ar]);
                for (int j = 0; j < n_groups; ++j, at += 4) {
                    const u32 coef = a.groups[at], desc = a.groups[at + 1], w2 = a.groups[at + 2], w3 = a.groups[at + 3];
                    const u32 nd = desc & 7u;
                    u64 t_p = coef;
                    if (nd > 0) t_p = (u64)coef * D[(desc >> 4) & 15u];
                    if (nd > 1) t_p = d_mul(t_p, D[(desc >> 8) & 15u]);
                    if (nd > 2) t_p = d_mul(t_p, D[(desc >> 12) & 15u]);
                    if (nd > 3) t_p = d_mul(t_p, D[(desc >> 16) & 15u]);
                    // (how many tensors: so many once, so many in each of the L blocks)
                    if (w2 & 0xffffu) embed_p = d_mad(embed_p, t_p, (w2 & 255u) + ((w2 >> 8) & 255u) * L);
                    if (w2 >> 16) lm_p = d_mad(lm_p, t_p, ((w2 >> 16) & 255u) + (w2 >> 24) * L);
                    if (w3 & 0xffffu) {
                        other_p = d_mad(other_p, t_p, (w3 & 255u) + ((w3 >> 8) & 255u) * L);
                        t_max = t_p > t_max ? t_p : t_max;
                    }
                    if (w3 >> 16)
                        m_os = d_mad(m_os, d_up(t_p * (u64)(B32 + B32), cu_shift), ((w3 >> 16) & 255u) + (w3 >> 24) * L);
                }
                continue;
            }
            const int n_param = (int)d_uni((u32)a.n_param[ar]), param_first = (int)d_uni((u32)a.param_first[ar]);
            for (int j = 0; j < n_param; ++j) {
                const uint4 pe = a.params_dev[param_first + j];               // wave-uniform
                const u32 cls = pe.z & 255u, role = (pe.z >> 8) & 255u, per_layer = (pe.z >> 16) & 255u;
                u64 t_p = (u64)pe.x * D[pe.y & 15u];
                t_p *= D[(pe.y >> 8) & 15u];
                t_p *= D[(pe.y >> 16) & 15u];
                t_p *= D[(pe.y >> 24) & 15u];
                const u64 copies = per_layer ? (u64)L : 1ull;
                const u64 tot = t_p * copies;
                if (role == LLMEM_ROLE_EMBED_TOK) embed_p += tot;
                else if (role == LLMEM_ROLE_LM_HEAD) lm_p += tot;
                else { other_p += tot; t_max = t_p > t_max ? t_p : t_max; }
                if (cls <= LLMEM_CLS_LINEAR && role != LLMEM_ROLE_LM_HEAD)
                    m_os += d_up(t_p * (u64)(B32 + B32), cu_shift) * copies;
                if (cls == LLMEM_CLS_EMBEDDING && role != LLMEM_ROLE_LM_HEAD) ++e_n;
            }
        }

        // ---- chunk size (Sec. 4.1): given, or the feasible candidate with the least padding waste,
        // ties to the smaller chunk.  The waste of candidate k, (-other_p) mod 2^(k+19), never
        // decreases with k and the candidates from some k on are the feasible ones: the search
        // ends at the smallest feasible candidate (the last one when none is feasible).
        int k_used = chunk_k;
        if (chunk_k == -1) {
            const int need = t_max > 1 ? 64 - __builtin_clzll(t_max - 1) : 0;       // least s with t_max <= 2^s
            const int k = need - 19;
            k_used = k < K_SEARCH_MIN ? K_SEARCH_MIN : k > K_SEARCH_MAX ? K_SEARCH_MAX : k;
        }
        k_used = (k_used < 0 || k_used > K_FIXED_MAX) ? 0 : k_used;          // invalid lanes: any defined shift
        const int cs_shift = k_used + 19;                                    // 2^k MiB of fp16 values
        u32 flags = t_max > (1ull << cs_shift) ? LLMEM_F_CHUNK_INFEASIBLE : 0;

        // ---- Sec. 4.1: gradients alias param fp16 unless switched off
        u64 grad_cdp = 0, grad_sharded = 0;
        if (!(cflags & LLMEM_CFG_GRAD_ALIAS)) {
            grad_cdp = d_up((embed_p + other_p) * B16, cu_shift);
            grad_sharded = d_up(d_cdiv(grad_cdp, g, div_g), align_shift);
        }

        // ---- batch-independent parts (Sec. 4.2, Sec. 5)
        QueryTerms q;
        const u64 head = lm_p * B16;
        const u32 tp1 = tp ? tp : 1u;
        // Model states in 32-bit counts of pages and allocator blocks.  A chunk of 2^(k+19) elements is
        // a whole number of pages at 2, 4 and 6 bytes per element once k + 20 >= log2 cu_p: the chunked
        // part of m_p, m_p16, m_p32 needs no rounding, the embedding's part is rounded on its own, and a
        // page is a whole number of blocks, so each shard is one 32-bit division of a block count (the
        // DP+TP share: of m_p16's blocks times tp_n).  Used by waves whose queries all keep every count
        // below 2^31 (checked through an upper bound in bytes); the same values as the byte form below.
        const u64 states_bound = ((other_p + embed_p + (1ull << cs_shift)) * (B16 + B32) + m_os + (4ull << cu_shift)) * tp1;
        const bool states_ok = cu_shift >= 1 && cs_shift + 1 >= cu_shift && ((other_p | embed_p) >> 48) == 0
                               && (m_os >> 54) == 0 && (states_bound >> (align_shift + 31)) == 0;
        if (__builtin_amdgcn_ballot_w64(valid && !states_ok) == 0) {
            const int half_shift = cu_shift - 1, page_shift = cu_shift - align_shift;
            const int rel_shift = states_ok ? cs_shift - half_shift : 0;     // lanes that take no part: any defined shift
            const u64 half_round = (1ull << half_shift) - 1;
            const u32 chunks = (u32)((other_p + ((1ull << cs_shift) - 1)) >> cs_shift);      // ceil(other_p / cs)
            const u32 chunk_pages = chunks << rel_shift;                                     // at 2 bytes per element
            const u32 p16_pages = chunk_pages + (u32)((embed_p + half_round) >> half_shift);
            const u32 p32_pages = 2u * chunk_pages + (u32)((embed_p * 2 + half_round) >> half_shift);
            const u32 p_pages = 3u * chunk_pages + (u32)((embed_p * 3 + half_round) >> half_shift);
            const u32 os_pages = (u32)(m_os >> cu_shift);
            const u32 p16_blocks = p16_pages << page_shift;
            const u64 common = (u64)a.m_base + head;
            const u32 z_shard = d_cdiv32((p32_pages + os_pages) << page_shift, g, div_g);
            const u32 t_shard = d_cdiv32((p_pages + os_pages) << page_shift, g, div_g);
            const u32 removed = d_cdiv32(p16_blocks * tp1, g, div_g);
            const u32 removed_other = d_cdiv32(p16_blocks * (tp1 - 1), tp1, div_t);
            q.fixed[LLMEM_METHOD_CDP] = common + ((u64)(p_pages + os_pages) << cu_shift) + grad_cdp;
            q.fixed[LLMEM_METHOD_ZERO3] = common + ((u64)(p16_blocks + z_shard) << align_shift) + grad_sharded;
            q.fixed[LLMEM_METHOD_TP] = common + ((u64)t_shard << align_shift) + grad_sharded;
            q.fixed[LLMEM_METHOD_HYBRID] = common + ((u64)(p16_blocks + z_shard - removed) << align_shift) + grad_sharded;
            if (tp > 0 && removed != removed_other) flags |= LLMEM_F_HYBRID_READINGS_DIFFER;
        } else {
            const u64 cs_mask = (1ull << cs_shift) - 1;
            const u64 chunked = embed_p + ((other_p + cs_mask) & ~cs_mask);
            const u64 m_p = d_up(chunked * (B16 + B32), cu_shift);
            const u64 m_p16 = d_up(chunked * B16, cu_shift);
            const u64 m_p32 = d_up(chunked * B32, cu_shift);
            q.fixed[LLMEM_METHOD_CDP] = (u64)a.m_base + m_p + m_os + head + grad_cdp;
            q.fixed[LLMEM_METHOD_ZERO3] = (u64)a.m_base + m_p16 + d_up(d_cdiv(m_p32 + m_os, g, div_g), align_shift) + head + grad_sharded;
            q.fixed[LLMEM_METHOD_TP] = (u64)a.m_base + d_up(d_cdiv(m_p + m_os, g, div_g), align_shift) + head + grad_sharded;
            // DP+TP: m_peak^dp minus the share of param fp16 that tensor parallelism removes
            const u64 removed = d_up(d_cdiv(m_p16 * tp1, g, div_g), align_shift);
            const u64 removed_other = d_up(d_cdiv(m_p16 * (tp1 - 1), tp1, div_t), align_shift);
            q.fixed[LLMEM_METHOD_HYBRID] = q.fixed[LLMEM_METHOD_ZERO3] - removed;
            if (tp > 0 && removed != removed_other) flags |= LLMEM_F_HYBRID_READINGS_DIFFER;
        }
        const u64 slh = (u64)sl * h;
        q.c_out = ((u64)e_n + L) * slh * B16;
        q.c_logits = (u64)V * Blog * sl;
        q.c_shifted = (u64)V * Blog * D[LLMEM_DIM_SL_M1];
        q.c_back_tp = (u64)L * slh * (g - 1) * B16;
        q.c_back_hy = (u64)L * slh * (tp1 - 1) * B16;
        q.gpu_n = g; q.tp_n = tp1; q.div_g = div_g; q.div_t = div_t; q.cu_shift = cu_shift;

        if (!DECIDE) {
            if (in_range) {
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    i64 v = peak_at(q, m, bs);
                    if (err || (m == LLMEM_METHOD_HYBRID && tp == 0)) v = -1;
                    put(&(a.out_peaks + (long long)m * n + first)[(u32)lane], v);
                }
                if (a.out_flags) put(&(a.out_flags + first)[(u32)lane], err ? (i64)err : (i64)flags);
            }
            continue;
        }

        // ---- Algorithm 1: largest batch size per method ---------------------------------------
        // The estimates never decrease with bs, so the largest batch size that fits is found by
        // bisection; and they are a fixed part plus terms that grow linearly with bs up to page
        // rounding, which brackets it first:
        //   fixed + bs * growth  <=  m_peak(bs)  <=  fixed + bs * growth + 6 pages
        // (growth: bytes per sample of m_out, the logits, the two shifted copies and 1/t of the TP
        // buffer; four round-ups to a page plus two in the buffer).  Both ends are moved out by more
        // than the rounding of the single-precision quotient can amount to; where that cannot be
        // shown for the lower end it is checked by an estimate of its own and dropped to 0 if that
        // does not fit.
        const u32 cap = valid ? bs : 0u;
        u32 best[4], top[4];                                                // the bracket: lower and upper end

        // Page form of the probes.  The batch-dependent part of an estimate is a whole number of
        // pages: with c = w * cu_p + r per term, ceil(b * c / cu_p) = b * w + ceil(b * r / cu_p), so
        // the whole parts of m_out, the logits and the two shifted copies share one product and
        // everything after the b * r products is 32-bit; an estimate fits iff its pages do not
        // exceed floor((m_total - fixed) / cu_p).  Used by waves whose queries all keep every
        // count below 2^31 at their largest batch size; the others probe in bytes.
        const u64 page_mask = (1ull << cu_shift) - 1;
        const u64 whole_sum = (q.c_out >> cu_shift) + (q.c_logits >> cu_shift) + 2 * (q.c_shifted >> cu_shift)
                              + (q.c_back_tp >> cu_shift) + (q.c_back_hy >> cu_shift);
        const bool pages_ok = cu_shift <= 31 && ((q.c_out | q.c_logits | q.c_shifted | q.c_back_tp | q.c_back_hy) >> 58) == 0
                              && (whole_sum >> 31) == 0 && (((whole_sum + 8) * cap) >> 31) == 0;
        const bool page_form = __builtin_amdgcn_ballot_w64(valid && !pages_ok) == 0;
        const u32 plain_whole = (u32)(q.c_out >> cu_shift) + (u32)(q.c_logits >> cu_shift) + 2u * (u32)(q.c_shifted >> cu_shift);
        const u32 r_out = (u32)(q.c_out & page_mask), r_logits = (u32)(q.c_logits & page_mask),
                  r_shifted = (u32)(q.c_shifted & page_mask);
        const u32 back_whole_tp = (u32)(q.c_back_tp >> cu_shift), r_back_tp = (u32)(q.c_back_tp & page_mask);
        const u32 back_whole_hy = (u32)(q.c_back_hy >> cu_shift), r_back_hy = (u32)(q.c_back_hy & page_mask);
        auto ceil_pages = [&](u32 b, u32 r) -> u32 { return (u32)(((u64)b * r + page_mask) >> cu_shift); };
        auto plain_pages = [&](u32 b) -> u32 {
            return b * plain_whole + ceil_pages(b, r_out) + ceil_pages(b, r_logits) + 2u * ceil_pages(b, r_shifted);
        };
        auto back_pages = [&](u32 b, u32 whole, u32 r, u32 t, DivMagic div) -> u32 {
            return d_cdiv32(b * whole + ceil_pages(b, r), t, div);
        };

        // lower end checked where the bracket's derivation does not vouch for it (`confirm`, the same
        // for the whole wave), then the bracket bisected
        auto search = [&](auto fits, const bool confirm) {
            u32 span = 0;
            if (confirm) {
#pragma unroll
                for (int m = 0; m < 4; ++m)
                    if (best[m] > 0 && !fits(m, best[m])) best[m] = 0;
            }
#pragma unroll
            for (int m = 0; m < 4; ++m) span |= top[m] - best[m];
            // bit length of the widest bracket in the wavefront: brackets are at most 1 wide where the
            // bracket's derivation holds, which two ballots establish; else bit by bit from the top
            int bits;
            if (__builtin_amdgcn_ballot_w64(span > 1u) == 0) {
                bits = __builtin_amdgcn_ballot_w64(span != 0u) != 0 ? 1 : 0;
            } else {
                bits = 32;
                while (bits > 2 && __builtin_amdgcn_ballot_w64((span >> (bits - 1)) != 0u) == 0) --bits;
            }
            for (int bit = bits - 1; bit >= 0; --bit) {                   // best + 2^bit, 2^bit above what is left of the span
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const u32 cand = best[m] + (1u << bit);
                    const bool ok = cand <= top[m] && fits(m, cand);
                    best[m] = ok ? cand : best[m];
                }
            }
        };
        if (page_form) {
            // the bracket in pages: growth per sample G = (c_out + c_logits + 2 c_shifted + c_back / t) / cu_p,
            // room R = floor((m_total - fixed) / cu_p); b * G <= pages(b) <= b * G + 6, so every b that
            // fits is at most R / G and every b up to (R - 6) / G fits
            const float per_page = __builtin_ldexpf(1.0f, -cu_shift);
            const float slope = (float)plain_whole + ((float)r_out + (float)r_logits + 2.0f * (float)r_shifted) * per_page;
            u32 room_pages[4];
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const i64 room = a.m_total - (i64)q.fixed[m];
                const u64 p = room < 0 ? 0ull : (u64)room >> cu_shift;
                room_pages[m] = p > 0x7fffffffull ? 0x7fffffffu : (u32)p;     // no estimate here has more pages
                float growth = slope;
                if (m == LLMEM_METHOD_TP)
                    growth += ((float)back_whole_tp + (float)r_back_tp * per_page) * __builtin_amdgcn_rcpf((float)(g ? g : 1u));
                if (m == LLMEM_METHOD_HYBRID)
                    growth += ((float)back_whole_hy + (float)r_back_hy * per_page) * __builtin_amdgcn_rcpf((float)tp1);
                u32 hi = cap, lo = 0;
                if (room < 0) {
                    hi = 0;                                               // not even the fixed part fits
                } else if (growth > 0.0f) {
                    // Single precision: G, 1 / G and the products are each within a few units of the last
                    // place; the computed quotient is within 16 * 2^-24 = 1e-6 of R / G relatively.
                    // Upper end: used for quotients under the cap (at most 65535), where that is below
                    // 0.07; moved out by 0.25.  Lower end: (R - 6) / G computed as quotient - 6.5 / G - 0.25;
                    // its error is at most (1e-6 * R + 1e-5) / G, which the extra 0.5 / G covers while
                    // R < 2^18 pages - then every batch size up to the lower end fits without being
                    // probed.  A wave with a query of more room confirms its lower ends by a probe.
                    const float inv = __builtin_amdgcn_rcpf(growth);
                    const float upper = (float)room_pages[m] * inv;
                    if (upper < (float)cap) { const u32 u = (u32)(upper + 0.25f); hi = u < cap ? u : cap; }
                    const float lower = upper - 6.5f * inv - 0.25f;
                    if (lower > 0.0f) lo = lower < (float)hi ? (u32)lower : hi;
                }
                best[m] = lo; top[m] = hi;
            }
            const bool much_room = ((room_pages[0] | room_pages[1] | room_pages[2] | room_pages[3]) >> 18) != 0;
            search([&](int m, u32 b) -> bool {
                u32 p = plain_pages(b);
                if (m == LLMEM_METHOD_TP) p += back_pages(b, back_whole_tp, r_back_tp, g, div_g);
                if (m == LLMEM_METHOD_HYBRID) p += back_pages(b, back_whole_hy, r_back_hy, tp1, div_t);
                return p <= room_pages[m];
            }, __builtin_amdgcn_ballot_w64(valid && much_room) != 0);
        } else {
            // the same bracket in bytes
            const float slope = (float)(q.c_out + q.c_logits + 2 * q.c_shifted);
            const float six_pages = (float)(6ull << cu_shift);
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const i64 room = a.m_total - (i64)q.fixed[m];
                const float back = m == LLMEM_METHOD_TP ? (float)q.c_back_tp / (float)(g ? g : 1u)
                                   : m == LLMEM_METHOD_HYBRID ? (float)q.c_back_hy / (float)tp1 : 0.0f;
                u32 hi = cap, lo = 0;
                if (room < 0) {
                    hi = 0;
                } else if (slope + back > 0.0f) {
                    const float growth = slope + back;
                    const float upper = __fdividef((float)room, growth);
                    if (upper < (float)cap) hi = (u32)upper + 2u < cap ? (u32)upper + 2u : cap;
                    const float lower = __fdividef((float)room - six_pages, growth) - 1.0f;
                    if (lower > 0.0f) lo = lower < (float)hi ? (u32)lower : hi;
                }
                best[m] = lo; top[m] = hi;
            }
            search([&](int m, u32 b) -> bool { return peak_at(q, m, b) <= a.m_total; }, true);
        }
        if (tp == 0) best[LLMEM_METHOD_HYBRID] = 0;
        // scores (doubled) and the choice
        const u32 dp_n = tp ? (u32)d_div(g, tp, div_t) : 0u;
        u32 score2[4];                                 // batch sizes are below 2^16 and gpu_n below 2^8: 32 bits hold them
        score2[0] = 3u * best[0] * g; score2[1] = 2u * best[1] * g; score2[2] = 2u * best[2];
        score2[3] = 2u * best[3] * dp_n;
        int idx = 0;
#pragma unroll
        for (int m = 1; m < 4; ++m) idx = score2[m] > score2[idx] ? m : idx;
        int method = idx;
        u32 chosen_bs = idx == 0 ? best[0] : idx == 1 ? best[1] : idx == 2 ? best[2] : best[3];
        // the chosen method's estimate at its batch size: one evaluation with that method's terms
        const u64 fixed_chosen = idx == 0 ? q.fixed[0] : idx == 1 ? q.fixed[1] : idx == 2 ? q.fixed[2] : q.fixed[3];
        const bool hybrid = idx == LLMEM_METHOD_HYBRID, gathers = idx >= LLMEM_METHOD_TP;
        const u32 t_chosen = hybrid ? tp1 : g;
        const DivMagic div_chosen = hybrid ? div_t : div_g;
        i64 peak;
        if (page_form) {
            const u32 whole = !gathers ? 0u : hybrid ? back_whole_hy : back_whole_tp;
            const u32 r = !gathers ? 0u : hybrid ? r_back_hy : r_back_tp;
            const u32 pages = plain_pages(chosen_bs) + back_pages(chosen_bs, whole, r, t_chosen, div_chosen);
            peak = (i64)(fixed_chosen + ((u64)pages << cu_shift));
        } else {
            const u64 b = chosen_bs;
            const u64 c_back = !gathers ? 0ull : hybrid ? q.c_back_hy : q.c_back_tp;
            peak = (i64)(fixed_chosen + d_up(b * q.c_out, cu_shift) + d_up(b * q.c_logits, cu_shift)
                         + 2 * d_up(b * q.c_shifted, cu_shift) + pages_over(b * c_back, t_chosen, div_chosen, cu_shift));
        }
        if (score2[2] == 0) {
            method = LLMEM_METHOD_OFFLOAD; chosen_bs = 0; peak = 0;
            if (score2[0] | score2[1] | score2[3]) flags |= LLMEM_F_FALLBACK_READINGS_DIFFER;
        }
        if (in_range) {
            // An invalid query considers no batch size (its cap is 0): every batch size, score and the
            // estimate are 0 already and the fallback has been taken; its method and flags are replaced.
            const bool bad = err != 0;
            const int method_out = bad ? -1 : method;
            const i64 flags_out = bad ? (i64)err : (i64)flags;
            // the batch's position is wave-uniform; the lane is a 32-bit offset from it
            const u32 at = (u32)lane;
            if (a.out_method) put(&(a.out_method + first)[at], method_out);
            if (a.out_bs) put(&(a.out_bs + first)[at], (int)chosen_bs);
            if (a.out_detail) {
                long long *o = a.out_detail + first;
                put(&(o + LLMEM_C_METHOD * n)[at], method_out);
                put(&(o + LLMEM_C_BS * n)[at], (i64)chosen_bs);
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    put(&(o + (LLMEM_C_BS_CDP + m) * n)[at], (i64)best[m]);
                    put(&(o + (LLMEM_C_SCORE2_CDP + m) * n)[at], (i64)score2[m]);
                }
                put(&(o + LLMEM_C_PEAK * n)[at], peak);
                put(&(o + LLMEM_C_FLAGS * n)[at], flags_out);
            }
        }
    }
}

int launch(bool decide, const llmem_configs *cfg, const uint8_t *tp_n, int64_t n, const llmem_tables *tables,
           DecideArgs &a, hipStream_t stream)
{
    if (!cfg || !tables) return LLMEM_EINVAL_NULL;
    if (n < 0) return LLMEM_EINVAL_N;
    EstimateArgs plan;
    const int rc = check_tables(tables, &plan);
    if (rc != LLMEM_OK) return rc;
    if (decide) {
        // a parameter size that depends on bs would make the estimates' fixed parts vary with bs
        for (int ar = 0; ar < tables->n_arch; ++ar)
            for (int j = 0; j < tables->arch[ar].n_param; ++j) {
                const llmem_param_entry &p = tables->params_host[tables->arch[ar].param_first + j];
                for (int q = 0; q < 4; ++q) if (p.dim[q] == LLMEM_DIM_BS) return LLMEM_EINVAL_TABLE;
            }
    }
    if (n == 0) return LLMEM_OK;
    if (!cfg->arch_id || !cfg->h || !cfg->L || !cfg->n_heads || !cfg->n_kv || !cfg->ffn || !cfg->V
        || !cfg->P || !cfg->bs || !cfg->sl || !cfg->d || !cfg->chunk_k || !cfg->flags)
        return LLMEM_EINVAL_NULL;
    a.cfg = *cfg;
    a.tp_n = tp_n;
    a.n = n;
    a.m_base = plan.m_base;
    a.cu_shift = plan.cu_shift;
    a.align_shift = plan.align_shift;
    a.n_arch = plan.n_arch;
    for (int ar = 0; ar < LLMEM_MAX_ARCH; ++ar) {
        a.param_first[ar] = ar < plan.n_arch ? plan.arch[ar].param_first : 0;
        a.n_param[ar] = ar < plan.n_arch ? plan.arch[ar].n_param : 0;
    }
    a.params_dev = reinterpret_cast<const uint4 *>(tables->params_dev);
    // the entries grouped by size expression, if the groups of all architectures fit the arguments
    a.use_groups = 1;
    int n_group_total = 0;
    for (int ar = 0; ar < plan.n_arch && a.use_groups; ++ar) {
        uint32_t e_n = 0;
        const int got = compile_param_groups(tables->params_host + plan.arch[ar].param_first, plan.arch[ar].n_param,
                                             a.groups + 4 * n_group_total, DC_GROUPS_MAX - n_group_total, &e_n);
        if (got < 0) { a.use_groups = 0; break; }
        a.group_first[ar] = 4 * n_group_total;
        a.n_groups[ar] = got;
        a.e_n[ar] = (int)e_n;
        n_group_total += got;
    }
    const int64_t n_batch = (n + 63) / 64;
    int64_t blocks = (n_batch + DC_WAVES - 1) / DC_WAVES;
    const int64_t max_blocks = 256 * 40;                // 256 CUs; 5 to 160 workgroups per CU measured, 40 to 80 are the fastest
    if (blocks > max_blocks) blocks = max_blocks;
    if (decide)
        hipLaunchKernelGGL(decide_kernel<true>, dim3((unsigned)blocks), dim3(DC_BLOCK), 0, stream, a);
    else
        hipLaunchKernelGGL(decide_kernel<false>, dim3((unsigned)blocks), dim3(DC_BLOCK), 0, stream, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e); return LLMEM_EHIP; }
    return LLMEM_OK;
}

}  // namespace

}  // namespace llmem

extern "C" int llmem_estimate_methods(const llmem_configs *cfg, const uint8_t *tp_n, int64_t n,
                                      const llmem_tables *method_tables, int64_t *out_peaks, int64_t *out_flags,
                                      void *hip_stream)
{
    using namespace llmem;
    if (!out_peaks) return LLMEM_EINVAL_NULL;
    DecideArgs a = {};
    a.out_peaks = reinterpret_cast<long long *>(out_peaks);
    a.out_flags = reinterpret_cast<long long *>(out_flags);
    return launch(false, cfg, tp_n, n, method_tables, a, reinterpret_cast<hipStream_t>(hip_stream));
}

extern "C" int llmem_decide(const llmem_configs *queries, const uint8_t *tp_n, int64_t n,
                            const llmem_tables *method_tables, int64_t m_total, int32_t *out_method,
                            int32_t *out_bs, int64_t *out_detail, void *hip_stream)
{
    using namespace llmem;
    if (!out_detail && (!out_method || !out_bs)) return LLMEM_EINVAL_NULL;
    DecideArgs a = {};
    a.m_total = m_total;
    a.out_method = out_method;
    a.out_bs = out_bs;
    a.out_detail = reinterpret_cast<long long *>(out_detail);
    return launch(true, queries, tp_n, n, method_tables, a, reinterpret_cast<hipStream_t>(hip_stream));
}
