// Batched peak-GPU-memory estimator, throughput kernel: one lane per
// configuration, 64 configurations per wavefront.
//
// The lanes of a wave hold 64 consecutive configurations (coalesced column
// loads).  Table entries are wave-uniform, so the wave walks the parameter table
// and the timeline of the architecture entry by entry while every lane evaluates
// the entry for its own configuration: no cross-lane reduction is needed, the
// prefix sum and running maximum of the timeline live in registers, and results
// are already one per lane for a coalesced store.
//
// Workgroup set-up (once, in LDS): the timeline events of each architecture are
// grouped into size classes - events whose byte size is the same expression
// (coefficient, dimensions, element width, scaling, method mask).  Every event
// becomes a 16-bit code: the value slot of its class, whether it releases, and
// whether the live total can peak there (an allocation followed by a release or
// by the end of its segment).  Per batch a lane evaluates each class once and
// stores the rounded size in a wave-private LDS array [slot][lane]; an event is
// then one LDS read and one 64-bit add or subtract.
//
// Compiled form (EstimateArgs::use_program): the host has already reduced every
// segment to the peak points no other point dominates, each a short list of
// (class, count) terms, and passes classes and terms in the kernel arguments;
// they arrive through scalar loads and the set-up above is skipped.  A peak
// point costs its terms (count * value) instead of every event before it.
//
// Direct form (EstimateArgs::direct): for tables with more distinct sizes than class slots fit,
// every event's size is evaluated where it stands, from the lane's dimension vector kept in
// wave-private LDS rows.
//
// Closed form: Sec. 4.2 (m_p, m_os, m_out, m_lm, m_peak^s) and Sec. 5 (m_peak^dp,
// m_peak^tp, m_back^tp) of arXiv 2404.10933; chunk size per Sec. 4.1; timeline
// traversal per Sec. 2.1 / Sec. 3.1.
//
// Specialized form (LLMEM_SPECIALIZED, see specialize.hip): this file is compiled again with the
// compiled tables of one set of architecture tables as constants - when the library is built,
// for the table sets it ships with, and at run time (specialized_prog.h) for any other.  The
// loops over parameter groups, classes and terms then have constant bounds and are unrolled;
// every word, offset and count becomes an immediate and every flag test disappears.  Only the
// path for sizes of 2^31 blocks and more keeps reading the words in loops.
#ifndef __HIPCC_RTC__
#include <hip/hip_runtime.h>
#include <stdint.h>
#else
// the run-time compiler has no C library headers: the fixed-width types the headers below use
typedef unsigned char uint8_t;
typedef signed char int8_t;
typedef unsigned short uint16_t;
typedef unsigned int uint32_t;
typedef int int32_t;
typedef unsigned long long uint64_t;
typedef long long int64_t;
#define INT64_MAX 0x7fffffffffffffffll
#endif

#ifdef __HIPCC_RTC__
#include "llmem.h"                 // the run-time compiler gets every file by its bare name
#else
#include "../../include/llmem.h"
#endif
#include "estimate_args.h"
#include "grid_draws.h"
#include "wave.h"

#ifdef LLMEM_SPECIALIZED
// The constants of this build, as macros: LLMEM_SPEC_WAVES (waves per SIMD to aim at),
// LLMEM_SPEC_ARCHS, LLMEM_SPEC_FIRSTS (first word of each of eight architectures) and
// LLMEM_SPEC_WORDS (the compiled tables).  A build ahead of time names its own file.
#ifndef LLMEM_SPEC_HEADER
#define LLMEM_SPEC_HEADER "specialized_prog.h"
#endif
#include LLMEM_SPEC_HEADER
namespace llmem {
namespace {
constexpr int SPEC_WAVES = LLMEM_SPEC_WAVES;
constexpr int SPEC_ARCHS = LLMEM_SPEC_ARCHS;
constexpr int SPEC_FIRST[8] = {LLMEM_SPEC_FIRSTS};
__device__ constexpr unsigned SPEC_PROG[] = {LLMEM_SPEC_WORDS};      // every read folds to an immediate
__constant__ unsigned SPEC_PROG_MEM[] = {LLMEM_SPEC_WORDS};          // the same words in memory, for the loops
}  // namespace
}  // namespace llmem
#define LLMEM_PROG(i) SPEC_PROG[i]
#define LLMEM_PROG_LOOP(i) SPEC_PROG_MEM[i]
#define LLMEM_UNROLL_IF(flag) _Pragma("unroll")
#define LLMEM_UNROLL_NARROW _Pragma("unroll NARROW ? 4096 : 1")
// The value is the same afterwards, but the compiler cannot know: work that depends on it stays
// behind this point instead of being hoisted to the start of the batch (registers).
#define LLMEM_ANCHOR(x) asm volatile("" : "+v"(x))
#define LLMEM_WAVES_PER_SIMD SPEC_WAVES
#define LLMEM_TERM_IS_PADDING(word) ((word) == 0u)            // known when compiling: the term vanishes
#else
#define LLMEM_PROG(i) a.prog[i]
#define LLMEM_PROG_LOOP(i) a.prog[i]
#define LLMEM_UNROLL_IF(flag)
#define LLMEM_UNROLL_NARROW
#define LLMEM_ANCHOR(x)
#define LLMEM_WAVES_PER_SIMD 5
#define LLMEM_TERM_IS_PADDING(word) false                     // a wave-uniform test would cost more than the term
#endif

namespace llmem {

namespace {

struct Narrow { static constexpr bool value = true; };
struct Wide { static constexpr bool value = false; };
// where an architecture's compiled tables start: read from the kernel arguments, or a constant
struct WordsFromArguments { static constexpr bool from_arguments = true; static constexpr int first = 0; };
template <int FIRST> struct WordsAt { static constexpr bool from_arguments = false; static constexpr int first = FIRST; };
static_assert(LLMEM_MAX_ARCH == 8, "the architecture switch of the specialized build lists eight cases");

constexpr int BB_WAVES = BATCH_WAVES;
constexpr int BB_BLOCK = 64 * BB_WAVES;
constexpr i64 LOWEST = (i64)0x8000000000000000ull;

__device__ __forceinline__ u64 b_div(u64 x, u32 d, u64 mul, u32 shift)
{
    return d == 1 ? x : (__umul64hi(x, mul) >> shift);
}
__device__ __forceinline__ u64 b_cdiv(u64 x, u32 d, u64 mul, u32 shift) { return b_div(x + (d - 1), d, mul, shift); }
// ceil(x / d) for x + d - 1 < 2^32: the multiply-high of the same 64-bit constant with a 32-bit dividend
__device__ __forceinline__ u32 b_cdiv32(u32 x, u32 d, u64 mul, u32 shift)
{
    const u32 dividend = x + (d - 1);
    const u64 low = (u64)dividend * (u32)mul;
    const u64 high = (u64)dividend * (u32)(mul >> 32) + (low >> 32);
    return d == 1 ? x : (u32)(high >> 32) >> shift;
}
__device__ __forceinline__ u64 b_up(u64 x, int shift) { return ((x + ((1ull << shift) - 1)) >> shift) << shift; }
// x * m (mod 2^64) in three instructions: the 64-bit product of the low half, the low 32 bits of
// the high half's product (kept as one v_mul_lo_u32, which issues at full rate on gfx950), one add
__device__ __forceinline__ u64 mul_64x32(u64 x, u32 m)
{
    const u64 lo = (u64)(u32)x * (u64)m;
    u32 hi_part;
    asm("v_mul_lo_u32 %0, %1, %2" : "=v"(hi_part) : "v"((u32)(x >> 32)), "v"(m));
    return ((u64)(hi_part + (u32)(lo >> 32)) << 32) | (u64)(u32)lo;
}
// acc + value * factor with value and the wave-uniform factor sign-extended from 32 bits, in one instruction
__device__ __forceinline__ i64 mad_i64_i32(int value, int factor, i64 acc)
{
    i64 sum;
    asm("v_mad_i64_i32 %0, vcc, %1, %2, %3" : "=v"(sum) : "v"(value), "s"(factor), "v"(acc) : "vcc");
    return sum;
}
// The larger of two 64-bit integers, each of them 0 or in [2^59, 2^61]: read as doubles such bit
// patterns are +0 or positive normal numbers, and doubles of one sign are ordered like their bit
// patterns, so one v_max_f64 does what takes a compare and two selects on integers (it returns one of
// its operands unchanged; no NaN, infinity or denormal is among them, so no mode bit matters).
__device__ __forceinline__ i64 max_of_positive(i64 x, i64 y)
{
    i64 larger;
    asm("v_max_f64 %0, %1, %2" : "=v"(larger) : "v"(x), "v"(y));
    return larger;
}
__device__ __forceinline__ u32 uni(u32 v) { return (u32)__builtin_amdgcn_readfirstlane((int)v); }
// Results are written once and not read again: streaming stores, which do not keep the lines in
// the L2 at the expense of what the kernel still reads.
__device__ __forceinline__ void put(long long *p, i64 v) { __builtin_nontemporal_store((long long)v, p); }

}  // namespace

// FORM_COMPILED: the tables come compiled in the kernel arguments.  FORM_EVENTS: the kernel reads the
// entries from memory, groups the events into size classes (values in LDS slots) and walks every
// event as an add or subtract of its class's value.  FORM_DIRECT: the same walk with every event's
// size evaluated where it stands - no classes, any number of distinct sizes (LDS holds the
// dimension vectors of the wave's 64 configurations only).
// SWEEP: the configurations are drawn here instead of loaded,
// and their results are folded into statistics per (method, d) instead of stored: LDS atomics per
// configuration into the workgroup's copy, one global atomic per statistic when the workgroup ends.
template <bool DETAIL, int FORM, bool SWEEP>
__device__ __forceinline__ void estimate_batch_body(const EstimateArgs &a)
{
    constexpr bool COMPILED = FORM == FORM_COMPILED, DIRECT = FORM == FORM_DIRECT;
    extern __shared__ uint4 lds[];
    const int block = a.waves * 64;                       // threads of this workgroup (a.waves wavefronts)
    constexpr int SWEEP_WORDS = LLMEM_NSWEEP * LLMEM_SWEEP_GROUPS;
    __shared__ u64 sweep_acc[SWEEP ? SWEEP_WORDS : 1];
    if (SWEEP) {
        for (int t = threadIdx.x; t < SWEEP_WORDS; t += block)
            sweep_acc[t] = t / LLMEM_SWEEP_GROUPS == LLMEM_S_MIN_PEAK ? (u64)INT64_MAX : 0ull;
    }
    // LDS: class table | event codes | per-architecture counts | value slots of the waves
    // (the set-up's scratch shares the space of the value slots)
    uint4 *cls_tab = lds;                                                       // n_arch * CLS_MAX
    unsigned short *codes = reinterpret_cast<unsigned short *>(lds + a.n_arch * CLS_MAX);
    int *n_class = reinterpret_cast<int *>(codes + a.code_count);                // code_count is a multiple of 8
    uint4 *dyn = (COMPILED || DIRECT) ? lds : reinterpret_cast<uint4 *>(n_class + LLMEM_MAX_ARCH);
    uint4 *tmp_key = dyn;                                                        // max_events
    unsigned short *tmp_rep = reinterpret_cast<unsigned short *>(tmp_key + a.max_events);
    unsigned short *tmp_cid = tmp_rep + a.max_events;

    // ---- set-up: size classes, value slots and event codes of every architecture -----
    if (DETAIL && FORM == FORM_EVENTS) {
        for (int t = threadIdx.x; t < a.code_count; t += block) codes[t] = 0;  // padding: slot 0, no check
        for (int ar = 0; ar < a.n_arch; ++ar) {
            const ArchLayout &al = a.arch[ar];
            const int n = al.seg_first[LLMEM_NSEG];
            if (threadIdx.x == 0) n_class[ar] = 0;
            for (int e = threadIdx.x; e < n; e += block) {
                const uint4 raw = a.events_dev[al.event_first + e];
                const ClassKey k = make_class_key(raw.x, raw.y, raw.z);
                tmp_key[e] = make_uint4(k.coef, k.dims, k.meta, raw.z);
            }
            __syncthreads();
            for (int e = threadIdx.x; e < n; e += block) {        // first event with the same key
                const uint4 me = tmp_key[e];
                int rep = e;
                for (int j = 0; j < e; ++j) {
                    const uint4 o = tmp_key[j];
                    if (o.x == me.x && o.y == me.y && o.z == me.z) { rep = j; break; }
                }
                tmp_rep[e] = (unsigned short)rep;
            }
            __syncthreads();
            for (int e = threadIdx.x; e < n; e += block) {        // class id = rank of its first event
                if (tmp_rep[e] != e) continue;
                int cid = 0;
                for (int j = 0; j < e; ++j) cid += tmp_rep[j] == j ? 1 : 0;
                tmp_cid[e] = (unsigned short)cid;
                if (cid < CLS_MAX) cls_tab[ar * CLS_MAX + cid] = tmp_key[e];
                atomicMax(&n_class[ar], cid + 1);
            }
            __syncthreads();
            for (int e = threadIdx.x; e < n; e += block) {
                const u32 z = tmp_key[e].w;
                const u32 seg = (z >> 8) & 255u, fl = (z >> 16) & 255u;
                const bool is_free = fl & LLMEM_EV_FREE;
                bool check = !is_free;
                if (check && e + 1 < n) {
                    const u32 zn = tmp_key[e + 1].w;
                    check = (((zn >> 8) & 255u) != seg) || (((zn >> 16) & 255u) & LLMEM_EV_FREE);
                }
                const int cid = tmp_cid[tmp_rep[e]];
                const u32 slot = cid + 1 < a.s_slots ? (u32)cid + 1u : 0u;
                const u32 sg = seg < LLMEM_NSEG ? seg : LLMEM_NSEG - 1;
                const int at = al.code_first + al.seg_code[sg] + (e - al.seg_first[sg]);
                if (at >= 0 && at < a.code_count) codes[at] = (unsigned short)((slot << 9) | (is_free ? CODE_FREE : 0u) | (check ? CODE_CHECK : 0u));
            }
            __syncthreads();
        }
    }

    __syncthreads();
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const long long n = a.n;
    const long long n_batch = (n + 63) >> 6;
    const int cu_shift = a.cu_shift, align_shift = a.align_shift;
    const u64 m_base = (u64)a.m_base;
    // value slots of this wave.  Events form: slot s of lane l at byte s * 512 + l * 8; an event
    // code is the slot's byte offset with the check flag in bit 0.  Compiled form: a slot is a row
    // of SLOT_ROW bytes holding either 64 values of 32 bits (minus the sizes in allocator blocks, lane
    // l at l * 4) or the 64-bit byte sizes of one half of the wave (lane l at (l % 32) * 8).
    char *vals = reinterpret_cast<char *>(dyn) + (COMPILED ? (size_t)wave * a.p_slots * SLOT_ROW
                                                  : DIRECT ? (size_t)wave * DIRECT_ROWS * 256    // rows of the dimension vector
                                                           : ((size_t)wave * a.s_slots * 64 + lane) * sizeof(i64));
    if (DETAIL && !DIRECT) {
        if (COMPILED) *reinterpret_cast<u32 *>(vals + lane * 4) = 0;
        else *reinterpret_cast<i64 *>(vals) = 0;
    }

    // the columns of one configuration as loaded
    struct Raw { u32 h, ffn, V, P, arch_id, method, d, cflags, L, n_heads, n_kv, bs, sl; int chunk_k; };
    // The 64 configurations of a batch start at a wave-uniform position: every column is read at
    // that position plus the lane (a 32-bit offset), lanes past the end of the grid read its last
    // configuration again and are masked afterwards.
    auto fetch = [&](long long batch) -> Raw {
        Raw r = {1, 0, 0, 0, 0, 0, 1, 0, 0, 1, 0, 0, 0, 0};
        const long long first = batch << 6;
        if (SWEEP) {
            const long long i = first + lane;
            if (i < n) {
                const DrawnConfig g = draw_config(a.sweep_grid, a.sweep_seed, (u64)(a.sweep_first + i));
                r.h = g.h; r.ffn = g.ffn; r.V = g.V; r.P = g.P; r.arch_id = g.arch_id; r.method = g.method; r.d = g.d;
                r.cflags = g.flags; r.L = g.L; r.n_heads = g.n_heads; r.n_kv = g.n_kv; r.chunk_k = g.chunk_k;
                r.bs = g.bs; r.sl = g.sl;
            }
        } else {
            const long long left = n - first;
            const u32 last = left < 64 ? (u32)left - 1u : 63u;
            const u32 at = (u32)lane < last ? (u32)lane : last;
#ifdef LLMEM_SPECIALIZED
            // the fourteen column pointers are read from the argument segment again for every batch
            // (scalar loads) instead of occupying 28 scalar registers through all of it
            const char __attribute__((address_space(4))) *segment =
                (const char __attribute__((address_space(4))) *)__builtin_amdgcn_kernarg_segment_ptr();
            asm volatile("" : "+s"(segment));
#define LLMEM_COLUMN(field) (*(decltype(a.cfg.field) const __attribute__((address_space(4))) *)( \
            segment + __builtin_offsetof(EstimateArgs, cfg) + __builtin_offsetof(llmem_configs, field)))
            llmem_configs c;
            c.h = LLMEM_COLUMN(h); c.ffn = LLMEM_COLUMN(ffn); c.V = LLMEM_COLUMN(V); c.P = LLMEM_COLUMN(P);
            c.arch_id = LLMEM_COLUMN(arch_id); c.method = LLMEM_COLUMN(method); c.d = LLMEM_COLUMN(d);
            c.flags = LLMEM_COLUMN(flags); c.L = LLMEM_COLUMN(L); c.n_heads = LLMEM_COLUMN(n_heads);
            c.n_kv = LLMEM_COLUMN(n_kv); c.chunk_k = LLMEM_COLUMN(chunk_k); c.bs = LLMEM_COLUMN(bs); c.sl = LLMEM_COLUMN(sl);
#undef LLMEM_COLUMN
#else
            const llmem_configs &c = a.cfg;
#endif
            r.h = (c.h + first)[at]; r.ffn = (c.ffn + first)[at]; r.V = (c.V + first)[at]; r.P = (c.P + first)[at];
            r.arch_id = (c.arch_id + first)[at]; r.method = (c.method + first)[at]; r.d = (c.d + first)[at];
            r.cflags = (c.flags + first)[at]; r.L = (c.L + first)[at]; r.n_heads = (c.n_heads + first)[at];
            r.n_kv = (c.n_kv + first)[at]; r.chunk_k = (c.chunk_k + first)[at]; r.bs = (c.bs + first)[at];
            r.sl = (c.sl + first)[at];
        }
        return r;
    };
    const long long b_step = (long long)gridDim.x * a.waves;
    long long b = (long long)blockIdx.x * a.waves + wave;
    for (; b < n_batch; b += b_step) {
        const long long i = (b << 6) + lane;                       // only the sweep uses it as a value
        const bool in_range = (long long)lane < n - (b << 6);
        const Raw now = fetch(b);
        const u32 h = now.h, ffn = now.ffn, V = now.V, P = now.P, arch_id = now.arch_id, method = now.method, d = now.d,
                  cflags = now.cflags, L = now.L, n_heads = now.n_heads, n_kv = now.n_kv, bs = now.bs, sl = now.sl;
        const int chunk_k = now.chunk_k;
        // every column is requested before the first is looked at: left alone, the compiler moves the
        // loads that only valid configurations need behind the validity test, a second round trip
        if (!SWEEP) asm volatile("" :: "v"(h), "v"(ffn), "v"(V), "v"(P), "v"(cflags), "v"(L), "v"(n_kv), "v"(bs), "v"(sl));
        u32 err = 0;
        if (arch_id >= (u32)a.n_arch) err |= LLMEM_F_ERR_ARCH;
        if (method > 2) err |= LLMEM_F_ERR_METHOD;
        if (d == 0) err |= LLMEM_F_ERR_D;
        if (n_heads == 0) err |= LLMEM_F_ERR_HEADS;
        if (!(chunk_k == -1 || (chunk_k >= 0 && chunk_k <= K_FIXED_MAX))) err |= LLMEM_F_ERR_CHUNK;
        const bool valid = in_range && err == 0;

        // dimension vector of this lane's configuration
        const u32 head_dim = h / (n_heads ? n_heads : 1u);
        u32 D[16];
        D[LLMEM_DIM_ONE] = 1; D[LLMEM_DIM_BS] = bs; D[LLMEM_DIM_SL] = sl; D[LLMEM_DIM_SL_M1] = sl ? sl - 1 : 0;
        D[LLMEM_DIM_H] = h; D[LLMEM_DIM_FFN] = ffn; D[LLMEM_DIM_N_HEADS] = n_heads; D[LLMEM_DIM_N_KV] = n_kv;
        D[LLMEM_DIM_HEAD_DIM] = head_dim; D[LLMEM_DIM_KV_DIM] = n_kv * head_dim; D[LLMEM_DIM_V] = V;
        D[LLMEM_DIM_P] = P; D[LLMEM_DIM_L] = L;
        const u32 Blog = (cflags & LLMEM_CFG_LOGITS_FP32) ? B32 : B16;
        D[LLMEM_DIM_B_LOGITS] = Blog; D[LLMEM_DIM_D] = d; D[DIM_BS_SL] = bs * sl;        // both below 2^16
        // multiplier of the divisions by the partition degree: a lane looks its own d up in the table in
        // constant memory (4 KB, in the caches).  A copy of it in LDS, filled by every workgroup, made no
        // difference to a batch and cost launches of many short-lived workgroups their set-up.
        const u64 div_mul = c_div.t[d & 255u].mul;
        const u32 div_shift = d > 1 ? 31u - (u32)__builtin_clz(d - 1) : 0u;        // ceil(log2 d) - 1

        i64 r_peak = err ? -1 : 0, r_live = 0;
#ifndef LLMEM_SPECIALIZED
        i64 r_param = 0, r_grad = 0, r_os = 0, r_out = 0, r_lm = 0, r_back = 0, r_k = 0, r_np = 0, r_tmax = 0, r_flags = err;
#endif

        // The lanes of architecture `ar` (the active ones) estimate their configurations.
        // `words`: where the architecture's compiled tables start, WordsFromArguments or WordsAt<N>.
        auto for_architecture = [&](const u32 ar, auto words) {
            const ArchLayout &al = a.arch[ar];

            // size of a compiled expression for this lane's configuration (descriptor: see estimate_args.h)
            auto expression = [&](u32 coef, u32 desc) -> u64 {
                const u32 nd = desc & 7u;
#ifdef LLMEM_SPECIALIZED
                // the dimensions first, the coefficient last: here it is a constant, and a power of two
                // more often than not - a shift
                if (nd == 0) return coef;
                if (nd == 1) return (u64)coef * D[(desc >> 4) & 15u];
                u64 x = (u64)D[(desc >> 4) & 15u] * D[(desc >> 8) & 15u];
                if (nd > 2) x = mul_64x32(x, D[(desc >> 12) & 15u]);
                if (nd > 3) x = mul_64x32(x, D[(desc >> 16) & 15u]);
                return x * (u64)coef;
#else
                u64 x = coef;
                if (nd > 0) x = (u64)coef * D[(desc >> 4) & 15u];
                if (nd > 1) x = mul_64x32(x, D[(desc >> 8) & 15u]);
                if (nd > 2) x = mul_64x32(x, D[(desc >> 12) & 15u]);
                if (nd > 3) x = mul_64x32(x, D[(desc >> 16) & 15u]);
                return x;
#endif
            };
            // A table entry names its dimensions by wave-uniform numbers.  Registers cannot be indexed
            // so; the direct form keeps the dimension vector in LDS as well, one row of 64 lanes per
            // dimension, and a number selects a row (the other forms index a copy in scratch memory
            // for the few entries of the parameter table).
            char *const drow = vals + lane * 4;
            if (DIRECT) {
#pragma unroll
                for (int q = 0; q < 16; ++q) *reinterpret_cast<u32 *>(drow + q * 256) = D[q];
            }
            auto dim_at = [&](u32 sel) -> u32 {
                if (DIRECT) return *reinterpret_cast<const u32 *>(drow + sel * 256);
                return D[sel];
            };
            // ---- parameter table (Notation table; Sec. 4.2, equation for m_os) ---------
            u64 embed_p = 0, lm_p = 0, other_p = 0, t_max = 0, m_os = 0;
            u32 e_n = 0;
            int pc = 0;                                                    // read position in the compiled tables
            u32 head = 0, seg_at[LLMEM_NSEG + 1] = {0, 0, 0, 0, 0, 0};     // header of the compiled tables
            if (COMPILED) {
                // entries with the same size expression arrive as one group with the number of
                // entries that count towards each sum, once and once per block
                // start of the architecture's words: selected from reads at constant positions, so that
                // every read of the compiled tables is a scalar load
                if constexpr (decltype(words)::from_arguments) {
                    pc = a.arch[0].prog_first;
#pragma unroll
                    for (int q = 1; q < LLMEM_MAX_ARCH; ++q) pc = ar == (u32)q ? a.arch[q].prog_first : pc;
                    pc = (int)uni((u32)pc);
                } else {
                    pc = decltype(words)::first;
                }
                head = LLMEM_PROG(pc);
#pragma unroll
                for (int q = 0; q <= LLMEM_NSEG; ++q) seg_at[q] = LLMEM_PROG(pc + 1 + q);
                pc += PROG_HEADER;
                e_n = (head >> 8) & 255u;
                const int n_groups = (int)(head & 255u);
                LLMEM_UNROLL_IF(true)
                for (int g = 0; g < n_groups; ++g, pc += 4) {
#pragma unroll
                    for (int q = 0; q < 16; ++q) LLMEM_ANCHOR(D[q]);
                    const u32 w2 = LLMEM_PROG(pc + 2), w3 = LLMEM_PROG(pc + 3);
                    const u64 t_p = expression(LLMEM_PROG(pc), LLMEM_PROG(pc + 1));
                    if (w2 & 0xffffu) embed_p += t_p * (u64)((w2 & 255u) + ((w2 >> 8) & 255u) * L);
                    if (w2 >> 16) lm_p += t_p * (u64)(((w2 >> 16) & 255u) + (w2 >> 24) * L);
                    if (w3 & 0xffffu) {
                        other_p += t_p * (u64)((w3 & 255u) + ((w3 >> 8) & 255u) * L);
                        t_max = t_p > t_max ? t_p : t_max;
                    }
                    if (w3 >> 16) m_os += b_up(t_p * (u64)(B32 + B32), cu_shift) * (u64)(((w3 >> 16) & 255u) + (w3 >> 24) * L);
                }
            } else {
                const int n_param = (int)uni((u32)al.n_param), param_first = (int)uni((u32)al.param_first);
                for (int j = 0; j < n_param; ++j) {
                    const uint4 pe = a.params_dev[param_first + j];           // wave-uniform
                    const u32 cls = pe.z & 255u, role = (pe.z >> 8) & 255u, per_layer = (pe.z >> 16) & 255u;
                    u64 t_p = (u64)pe.x * dim_at(pe.y & 15u);
                    t_p *= dim_at((pe.y >> 8) & 15u);
                    t_p *= dim_at((pe.y >> 16) & 15u);
                    t_p *= dim_at((pe.y >> 24) & 15u);
                    const u64 copies = per_layer ? (u64)L : 1ull;
                    const u64 tot = t_p * copies;
                    if (role == LLMEM_ROLE_EMBED_TOK) embed_p += tot;
                    else if (role == LLMEM_ROLE_LM_HEAD) lm_p += tot;
                    else { other_p += tot; t_max = t_p > t_max ? t_p : t_max; }
                    if (cls <= LLMEM_CLS_LINEAR && role != LLMEM_ROLE_LM_HEAD)
                        m_os += b_up(t_p * (u64)(B32 + B32), cu_shift) * copies;
                    if (cls == LLMEM_CLS_EMBEDDING && role != LLMEM_ROLE_LM_HEAD) ++e_n;
                }
            }
            const u64 n_params = embed_p + other_p + ((cflags & LLMEM_CFG_TIED_LM_HEAD) ? 0ull : lm_p);

            // ---- Sec. 4.2: m_out, m_lm; Sec. 5: m_back^tp -----------------------------------
            // (the batch size goes through an empty asm: what follows is then formed here, after the
            // parameter table, instead of being hoisted in front of it and kept in registers across it)
            u32 bs_here = bs;
            asm volatile("" : "+v"(bs_here));
            const u64 A = (u64)bs_here * sl * h;
            const u64 m_out = b_up(((u64)e_n + L) * A * B16, cu_shift);
            const u64 row = (u64)bs_here * V * Blog;
            const u64 m_lm = b_up(row * sl, cu_shift) + 2 * b_up(row * D[LLMEM_DIM_SL_M1], cu_shift) + lm_p * B16;
            u64 m_back = 0;
#ifdef LLMEM_SPECIALIZED
            {
                // ceil(x / (d * cu_p)) = ceil(ceil(x / cu_p) / d); the page count is divided in 32 bits
                // when that of every lane fits
                u64 pages = 0;
                if (method == LLMEM_METHOD_TP) pages = ((u64)L * A * (d - 1) * B16 + ((1ull << cu_shift) - 1)) >> cu_shift;
                if (__builtin_amdgcn_ballot_w64(((pages + 255) >> 32) != 0) == 0)
                    m_back = (u64)b_cdiv32((u32)pages, d, div_mul, div_shift) << cu_shift;
                else
                    m_back = b_cdiv(pages, d, div_mul, div_shift) << cu_shift;
            }
#else
            if (method == LLMEM_METHOD_TP) {
                const u64 pages = ((u64)L * A * (d - 1) * B16 + ((1ull << cu_shift) - 1)) >> cu_shift;
                m_back = b_cdiv(pages, d, div_mul, div_shift) << cu_shift;
            }
#endif
            // ---- Sec. 4.1: gradients alias param fp16 unless switched off -------------------
            const u64 grad_bytes = (embed_p + other_p) * B16;
            const u64 grad_logical = method == LLMEM_METHOD_CDP ? grad_bytes : b_cdiv(grad_bytes, d, div_mul, div_shift);
            u64 grad_extra = 0;
            if (!(cflags & LLMEM_CFG_GRAD_ALIAS)) {
                const u64 g = b_up(grad_bytes, cu_shift);
                grad_extra = method == LLMEM_METHOD_CDP ? g : b_up(b_cdiv(g, d, div_mul, div_shift), align_shift);
            }

#ifdef LLMEM_SPECIALIZED
            // the columns known by now are stored now, so that they do not occupy registers any longer
            // (the built-in forms, whose batch is a loop over architectures, store everything at the end:
            // stores inside that loop cost them more registers than they free)
            if (DETAIL && !SWEEP) {
                const u32 at = (u32)lane;
                long long *o = a.out_detail + (b << 6);                 // wave-uniform; the lane is a 32-bit offset
                put(&(o + (long long)LLMEM_D_GRAD_GPU * n)[at], (i64)grad_logical);
                put(&(o + (long long)LLMEM_D_OUT * n)[at], (i64)m_out);
                put(&(o + (long long)LLMEM_D_LM * n)[at], (i64)m_lm);
                put(&(o + (long long)LLMEM_D_BACK * n)[at], (i64)m_back);
                put(&(o + (long long)LLMEM_D_NPARAMS * n)[at], (i64)n_params);
                put(&(o + (long long)LLMEM_D_TMAX * n)[at], (i64)t_max);
            }
#endif
            // ---- chunk size (Sec. 4.1), m_p and the method's peak ----------------------------
            // Every candidate k = 2..10 is estimated; the feasible one with the least padding
            // waste wins, ties to the smaller chunk.  A lane with a given chunk size estimates
            // that one.
            const bool search = chunk_k == -1;
            const bool any_search = __builtin_amdgcn_ballot_w64(search) != 0;
            const bool zero3 = method == LLMEM_METHOD_ZERO3;
            u64 m_peak = 0;
            int k_used = search ? K_SEARCH_MAX : chunk_k;
            bool found = !search;
            const u64 rest = m_base + m_out + m_lm + grad_extra;               // the same for every candidate
            // Page form of the candidates.  A chunk of 2^(k+19) elements is a whole number of pages
            // (cu_p bytes) at 2, 4 and 6 bytes per element once k + 20 >= log2 cu_p; then the
            // chunked part of m_p, m_p16, m_p32 needs no rounding, the embedding's part is rounded
            // once, before the loop, and every size of a candidate is a count of pages or allocator
            // blocks that fits 32 bits (checked through an upper bound in bytes): the division by d
            // becomes a 32-bit one.  The same values as the byte form below, which waves with a
            // lane outside these conditions take.  Only the specialized build has it: there the
            // vector instructions are the bound, while the built-in forms would pay for the second
            // loop with registers.
#ifdef LLMEM_SPECIALIZED
            const int k_low = search ? K_SEARCH_MIN : chunk_k, k_high = search ? K_SEARCH_MAX : chunk_k;
            const u64 bytes_bound = 6 * (other_p + embed_p + (1ull << (k_high + 19))) + m_os + m_back + (4ull << cu_shift);
            const bool pages_ok = cu_shift >= 1 && k_low + 20 >= cu_shift && ((other_p | embed_p) >> 50) == 0
                                  && (bytes_bound >> (align_shift + 31)) == 0;
            const bool page_form = __builtin_amdgcn_ballot_w64(!pages_ok) == 0;
#else
            const bool page_form = false;
#endif
            // the page form's per-lane constants: also used for the detail columns below
            const int half_shift = cu_shift - 1, page_shift = cu_shift - align_shift;
            const u32 fw_half = zero3 ? 2u : 3u;                              // m_p32 or m_p: bytes per element / 2
            u32 embed_wide_pages = 0, embed_p16_pages = 0, os_blocks = 0;
            if (page_form) {
#ifdef LLMEM_SPECIALIZED
                // every size is a 32-bit count of allocator blocks
                const u64 half_round = (1ull << half_shift) - 1;
                embed_wide_pages = (u32)((embed_p * fw_half + half_round) >> half_shift);
                embed_p16_pages = (u32)((embed_p + half_round) >> half_shift);
                os_blocks = (u32)(m_os >> align_shift);
                const u32 need_shift = t_max > 1 ? 64u - (u32)__builtin_clzll(t_max - 1) : 0u;   // least s with t_max <= 2^s
                const u32 base_blocks = (embed_wide_pages << page_shift) + os_blocks;            // shared out besides the chunks
                const bool whole = method == LLMEM_METHOD_CDP || d == 1;                        // nothing is divided
                const u32 kept_blocks = method == LLMEM_METHOD_CDP ? 0u : zero3 ? embed_p16_pages << page_shift
                                                                                : (u32)(m_back >> align_shift);
                const u32 div_low = (u32)div_mul, div_high = (u32)(div_mul >> 32);
                // the model states of candidate k in blocks, its padding waste and whether the largest tensor fits
                auto candidate = [&](const int k, u32 &state_blocks, u32 &waste, bool &feasible) {
                    const int cs_shift = k + 19;                                                 // 2^k MiB of fp16 values
                    const u32 chunks = (u32)((other_p + ((1ull << cs_shift) - 1)) >> cs_shift);  // ceil(other_p / cs)
                    const u32 chunk_blocks = chunks << (cs_shift - half_shift + page_shift);     // at 2 bytes per element
                    const u32 to_shard = chunk_blocks * fw_half + base_blocks;                   // m_p32 (or m_p) + m_os
                    const u32 dividend = to_shard + (d - 1);
                    const u64 low = (u64)dividend * div_low;
                    const u64 high = (u64)dividend * div_high + (low >> 32);
                    const u32 shard = whole ? to_shard : (u32)(high >> 32) >> div_shift;
                    state_blocks = shard + kept_blocks + (zero3 ? chunk_blocks : 0u);            // ZeRO-3 keeps m_p16 whole
                    waste = (chunks << cs_shift) - (u32)other_p;       // below the chunk size: exact modulo 2^32 for k <= 10
                    feasible = need_shift <= (u32)cs_shift;
                };
                u32 best_state = 0, best_waste = ~0u;
                if (__builtin_amdgcn_ballot_w64(!search) != 0) {
                    // lanes with a given chunk size estimate that one
                    u32 state, waste;
                    bool feasible;
                    candidate(search ? K_SEARCH_MIN : chunk_k, state, waste, feasible);
                    best_state = state;
                }
                if (any_search) {
                    // the others: strictly smaller waste among feasible candidates; the last one stands in
                    // when none is feasible
#pragma unroll
                    for (int j = 0; j <= K_SEARCH_MAX - K_SEARCH_MIN; ++j) {
                        u32 state, waste;
                        bool feasible;
                        candidate(K_SEARCH_MIN + j, state, waste, feasible);
                        const bool better = feasible && waste < best_waste;
                        const bool take = search && (better || (!found && j == K_SEARCH_MAX - K_SEARCH_MIN));
                        best_state = take ? state : best_state;
                        k_used = take ? K_SEARCH_MIN + j : k_used;
                        best_waste = (search && better) ? waste : best_waste;
                        found = found || (search && better);
                    }
                }
                m_peak = rest + ((u64)best_state << align_shift);
#endif
            } else {
                u64 best_waste = ~0ull;
#ifdef LLMEM_SPECIALIZED
#pragma nounroll
#endif
                for (int j = 0; j <= K_SEARCH_MAX - K_SEARCH_MIN; ++j) {
                    if (j > 0 && !any_search) break;
                    const int k = search ? K_SEARCH_MIN + j : chunk_k;
                    const int cs_shift = k + 19;                              // 2^k MiB of fp16 values
                    const u64 cs_mask = (1ull << cs_shift) - 1;
                    const u64 other_chunked = (other_p + cs_mask) & ~cs_mask; // ceil(other_p / cs) * cs
                    const u64 chunked = embed_p + other_chunked;
                    // ZeRO-3 shards m_p32 and keeps m_p16 whole; the other two methods use m_p = 6 bytes per element
                    const u64 wide_part = b_up((chunked << 2) + (zero3 ? 0ull : chunked << 1), cu_shift);   // m_p32 or m_p
                    const u64 c_p16 = b_up(chunked << 1, cu_shift);
                    const u64 to_shard = wide_part + m_os;
                    const u64 shard = b_up(b_cdiv(to_shard, d, div_mul, div_shift), align_shift);
                    u64 states;
                    if (method == LLMEM_METHOD_CDP) states = to_shard;
                    else if (zero3) states = c_p16 + shard;
                    else states = shard + m_back;
                    const u64 c_peak = rest + states;
                    const u64 waste = other_chunked - other_p;
                    const bool feasible = t_max <= (1ull << cs_shift);
                    // search lanes: strictly smaller waste among feasible candidates; the last candidate
                    // stands in when none is feasible.  Other lanes: iteration 0 is their estimate.
                    const bool take = search ? ((feasible && waste < best_waste) || (!found && j == K_SEARCH_MAX - K_SEARCH_MIN))
                                             : j == 0;
                    if (take) {
                        m_peak = c_peak; k_used = k;
                        if (feasible) { best_waste = waste; found = true; }
                    }
                }
            }
            const u32 flags = t_max > (1ull << (k_used + 19)) ? LLMEM_F_CHUNK_INFEASIBLE : 0;
            r_peak = (i64)m_peak;
            if (SWEEP) {
                // everything but the timeline's peak is known: folded into the group's statistics now (a
                // group: method and d <= 16), so that it occupies no registers during the timeline
                if (d - 1u < 16u) {
                    u64 *at = sweep_acc + (method * 16u + (d - 1u));
                    auto add = [&](int col, u64 v) {
                        __hip_atomic_fetch_add(at + col * LLMEM_SWEEP_GROUPS, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    };
                    auto raise = [&](int col, u64 v) {
                        __hip_atomic_fetch_max(at + col * LLMEM_SWEEP_GROUPS, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    };
                    add(LLMEM_S_COUNT, 1);
                    add(LLMEM_S_K_SUM, (u64)k_used);
                    raise(LLMEM_S_MAX_PEAK, m_peak);
                    __hip_atomic_fetch_min(at + LLMEM_S_MIN_PEAK * LLMEM_SWEEP_GROUPS, m_peak, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_WORKGROUP);
                    if ((i64)m_peak <= a.m_total) {
                        // Sec. 6, Algorithm 1: the batch per step over all GPUs, times 1.5 for conventional
                        // DP, one batch for a TP group; doubled.  Higher score first, then the lower index.
                        const u32 score2 = method == LLMEM_METHOD_CDP ? 3u * bs * d : method == LLMEM_METHOD_ZERO3 ? 2u * bs * d : 2u * bs;
                        const u64 index_mask = (1ull << SWEEP_INDEX_BITS) - 1;
                        add(LLMEM_S_FIT, 1);
                        raise(LLMEM_S_MAX_NPARAMS_FIT, n_params);
                        raise(LLMEM_S_BEST, ((u64)score2 << SWEEP_INDEX_BITS) | (index_mask - (u64)(a.sweep_first + i)));
                    }
                }
            }

            if (DETAIL) {
                // m_p, m_p16, m_p32 of the chunk size used (formed again here rather than carried
                // through the candidates: fewer live registers)
                u64 param_gpu, os_gpu;
                if (page_form) {
                    // in pages and blocks, as the candidates above: the chunked part is whole pages at
                    // 2, 4 and 6 bytes per element, the shards are 32-bit divisions
                    const int used_shift = k_used + 19;
                    const u32 used_chunks = (u32)((other_p + ((1ull << used_shift) - 1)) >> used_shift);
                    const u32 chunk_pages = used_chunks << (used_shift - half_shift);            // at 2 bytes per element
                    const u32 wide_pages = chunk_pages * fw_half + embed_wide_pages;             // m_p32 (ZeRO-3) or m_p
                    const u64 p_sh = (u64)b_cdiv32(wide_pages << page_shift, d, div_mul, div_shift) << align_shift;
                    param_gpu = method == LLMEM_METHOD_CDP ? (u64)wide_pages << cu_shift
                                : zero3 ? ((u64)(chunk_pages + embed_p16_pages) << cu_shift) + p_sh : p_sh;
                    os_gpu = method == LLMEM_METHOD_CDP ? m_os : (u64)b_cdiv32(os_blocks, d, div_mul, div_shift) << align_shift;
                } else {
                    const u64 used_mask = (1ull << (k_used + 19)) - 1;
                    const u64 used_chunked = embed_p + ((other_p + used_mask) & ~used_mask);
                    const u64 mp = b_up(used_chunked * (B16 + B32), cu_shift), mp16 = b_up(used_chunked * B16, cu_shift),
                              mp32 = b_up(used_chunked * B32, cu_shift);
                    if (method == LLMEM_METHOD_CDP) {
                        param_gpu = mp; os_gpu = m_os;
                    } else {
                        const u64 os_sh = b_up(b_cdiv(m_os, d, div_mul, div_shift), align_shift);
                        const u64 p_sh = b_up(b_cdiv(method == LLMEM_METHOD_ZERO3 ? mp32 : mp, d, div_mul, div_shift), align_shift);
                        param_gpu = method == LLMEM_METHOD_ZERO3 ? mp16 + p_sh : p_sh;
                        os_gpu = os_sh;
                    }
                }

#ifdef LLMEM_SPECIALIZED
                // every remaining column but the timeline peak is known: stored now, so that none of
                // them occupies registers during the timeline
                if (!SWEEP) {
                    const u32 at = (u32)lane;
                    if (a.out_peaks) put(&(a.out_peaks + (b << 6))[at], (i64)m_peak);
                    long long *o = a.out_detail + (b << 6);             // wave-uniform; the lane is a 32-bit offset
                    put(&(o + (long long)LLMEM_D_PEAK * n)[at], (i64)m_peak);
                    put(&(o + (long long)LLMEM_D_PARAM_GPU * n)[at], (i64)param_gpu);
                    put(&(o + (long long)LLMEM_D_OS_GPU * n)[at], (i64)os_gpu);
                    put(&(o + (long long)LLMEM_D_K * n)[at], (i64)k_used);
                    put(&(o + (long long)LLMEM_D_FLAGS * n)[at], (i64)flags);
                }
#endif
                // what is resident before the iteration starts (one value instead of five during the timeline)
                const i64 prelude = (i64)(m_base + param_gpu + os_gpu + lm_p * B16 + grad_extra);
                i64 at = 0, best = 0;                                         // the empty prefix counts
                // value of one size class for this lane's configuration: rounded bytes
                auto class_value = [&](u32 coef, u32 dims, u32 meta) -> u64 {
                    u64 x = (u64)coef * (meta & 255u);
                    x *= D[dims & 15u];
                    x *= D[(dims >> 8) & 15u];
                    x *= D[(dims >> 16) & 15u];
                    x *= D[(dims >> 24) & 15u];
                    const u32 fl = (meta >> 8) & 255u, mask = (meta >> 16) & 7u;
                    if (fl & LLMEM_EV_TP_GATHER) x = b_cdiv(x * (u64)(d - 1), d, div_mul, div_shift);
                    u64 r = b_up(x, align_shift);
                    if (fl & LLMEM_EV_TIMES_L) r *= (u64)L;
                    if (mask != 7u) r = ((mask >> method) & 1u) ? r : 0ull;
                    return r;
                };
                // after a segment: `at` is the live total at its start relative to the resident state,
                // `run` its net change, `top` its highest prefix.  The L equal blocks shift the prefix
                // linearly, so the maximum over the repetitions of F (or B) is at the first or last one.
                // `has_point`: the segment has a prefix that can be a peak (`top` is meaningful)
                auto close_segment = [&](int s, i64 run, i64 top, bool has_point) {
                    const bool repeated = s == LLMEM_SEG_F || s == LLMEM_SEG_B;
                    if (repeated) {
                        const i64 shift = ((i64)L - 1) * run;
                        const i64 cand = at + top + (shift > 0 ? shift : 0);
                        if (has_point && L != 0) best = cand > best ? cand : best;
                        at += (i64)L * run;
                    } else {
                        const i64 cand = at + top;
                        if (has_point) best = cand > best ? cand : best;
                        at += run;
                    }
                };
                if (COMPILED) {
                    // ---- compiled timeline: classes and terms come from the kernel arguments ----
                    const int nc = (int)((head >> 16) & 255u);
                    const int pc_classes = pc;
                    // Classes: four per fetch (the host pads the list with empty classes).  NARROW: sizes
                    // in allocator blocks, negated, as signed 32-bit values, all 64 lanes; else 64-bit byte
                    // sizes of the lanes of one half of the wave.  Returns 0 if every size is at most
                    // 2^31 blocks.
                    auto store_classes = [&](auto narrow) -> u32 {
                        constexpr bool NARROW = decltype(narrow)::value;
                        char *row = vals + (NARROW ? lane * 4 : (lane & 31) * 8);
                        u64 raw_before = 0;
                        u32 beyond = 0;                           // stays 0 while every size is at most 2^31 blocks
                        int at_word = pc_classes;
                        LLMEM_UNROLL_NARROW
                        for (int c0 = 0; c0 < nc; c0 += PROG_CLASS_FETCH, at_word += 2 * PROG_CLASS_FETCH) {
#pragma unroll
                            for (int q = 0; q < 16; ++q) LLMEM_ANCHOR(D[q]);
                            u32 cw[2 * PROG_CLASS_FETCH];
#pragma unroll
                            for (int q = 0; q < 2 * PROG_CLASS_FETCH; ++q)
                                cw[q] = NARROW ? LLMEM_PROG(at_word + q) : LLMEM_PROG_LOOP(at_word + q);
#pragma unroll
                            for (int u = 0; u < PROG_CLASS_FETCH; ++u) {
                                const int c = c0 + u;
                                const u32 desc = cw[2 * u + 1];
                                u64 x;
                                if ((desc & 7u) == DESC_FROM_PREVIOUS) {
                                    asm volatile("" ::: "memory");
                                    x = raw_before << cw[2 * u];              // same dimensions, 2^k times the coefficient
                                } else {
                                    x = expression(cw[2 * u], desc);
                                }
                                raw_before = x;
                                u64 r;                                                        // blocks
                                if ((desc & DESC_TP_GATHER) && NARROW) {
                                    // ceil(ceil(x (d - 1) / d) / block) = ceil(ceil(x (d - 1) / block) / d): the division
                                    // in 32 bits, on blocks (a count of 2^31 and more sends the wave to the wide walk)
                                    const u64 scaled = (mul_64x32(x, d - 1) + ((1ull << align_shift) - 1)) >> align_shift;
                                    beyond |= (u32)(scaled >> 31);
                                    r = b_cdiv32((u32)scaled, d, div_mul, div_shift);
                                } else {
                                    if (desc & DESC_TP_GATHER) x = b_cdiv(mul_64x32(x, d - 1), d, div_mul, div_shift);
                                    r = (x + ((1ull << align_shift) - 1)) >> align_shift;
                                }
                                // the rare descriptor flags are wave-uniform: real branches, no selects
                                if (desc & DESC_TIMES_L) {
                                    asm volatile("" ::: "memory");
                                    r = mul_64x32(r, L);
                                }
                                const u32 mask = (desc >> DESC_MASK_SHIFT) & 7u;
                                if (mask != 7u) {
                                    asm volatile("" ::: "memory");
                                    r = ((mask >> method) & 1u) ? r : 0ull;
                                }
                                if (NARROW) {
                                    // minus the size in blocks: sizes up to 2^31 blocks inclusive fit
                                    beyond |= (u32)((r + 0x7fffffffull) >> 32);
                                    if (c < nc) *reinterpret_cast<u32 *>(row + (c + 1) * SLOT_ROW) = 0u - (u32)r;
                                } else {
                                    if (c < nc) *reinterpret_cast<u64 *>(row + (c + 1) * SLOT_ROW) = r << align_shift;
                                }
                            }
                        }
                        return beyond;
                    };
                    // Sums of count * value, PROG_FETCH terms per fetch in groups of four.  A group flagged as
                    // a point's end lets its sum compete for the segment's maximum; the group that ends a
                    // segment's net change closes the segment.  The flags are wave-uniform: groups inside a
                    // sum cost their multiply-adds only.
                    auto walk_terms = [&](auto narrow) {
                        constexpr bool NARROW = decltype(narrow)::value;
                        const char *row = vals + (NARROW ? lane * 4 : (lane & 31) * 8);
                        int seg = 0;
                        u32 has_point = 0;                                                // wave-uniform, kept scalar
                        // The narrow sums start at 2^60 instead of 0.  A sum is below 2^53 in magnitude (at most
                        // 100 values of at most 2^31 blocks, factors below 2^15), so its bit pattern is that
                        // of a positive double and a point's maximum is one max_of_positive(), against 0
                        // before the segment's first point.  2^60 is in the high word only: taking it off
                        // again at the segment's end is one 32-bit add.
                        constexpr u64 NARROW_ZERO = 1ull << 60;
                        i64 zero = NARROW ? (i64)NARROW_ZERO : 0;
                        if (NARROW) asm volatile("" : "+v"(zero));                      // one register pair, not an immediate per sum
                        i64 acc = zero, top = NARROW ? 0 : LOWEST;
                        const int w_begin = (int)seg_at[0], w_end = (int)seg_at[LLMEM_NSEG];
                        LLMEM_UNROLL_NARROW
                        for (int w = w_begin; w < w_end; w += PROG_FETCH) {
                            u32 t[PROG_FETCH];
#pragma unroll
                            for (int q = 0; q < PROG_FETCH; ++q) t[q] = NARROW ? LLMEM_PROG(w + q) : LLMEM_PROG_LOOP(w + q);
                            int v32[NARROW ? PROG_FETCH : 1];
                            if (NARROW) {
#pragma unroll
                                for (int q = 0; q < PROG_FETCH; ++q)
                                    v32[q] = *reinterpret_cast<const int *>(row + (t[q] & PROG_OFFSET_MASK));
                            }
#pragma unroll
                            for (int g = 0; g < PROG_FETCH; g += PROG_GROUP) {
                                if (NARROW) {
                                    // signed 32-bit blocks times a signed 16-bit factor: one multiply-add each
                                    // (written out: left to itself the compiler replaces the products by the
                                    // small constant factors of a specialized build with sign extensions, shifts
                                    // and 64-bit adds, two to three instructions per term)
#pragma unroll
                                    for (int q = g; q < g + PROG_GROUP; ++q) {
                                        if (LLMEM_TERM_IS_PADDING(t[q])) continue;
                                        acc = mad_i64_i32(v32[q], (int)t[q] >> 16, acc);
                                    }
                                } else {
                                    // the rows hold the byte sizes themselves; the factor is minus the count.
                                    // |count| * value from the low and the high half of the value (each
                                    // product is below 2^48), added or subtracted by the factor's sign
#pragma unroll
                                    for (int q = g; q < g + PROG_GROUP; ++q) {
                                        const u64 v = *reinterpret_cast<const u64 *>(row + (t[q] & PROG_OFFSET_MASK));
                                        const int factor = (int)t[q] >> 16;
                                        const u32 mag = (u32)(factor < 0 ? -factor : factor);
                                        const u64 prod = (u64)(u32)v * mag + (((u64)(u32)(v >> 32) * mag) << 32);
                                        acc = factor < 0 ? (i64)((u64)acc + prod) : (i64)((u64)acc - prod);
                                    }
                                }
                                // a sum ends with this group (wave-uniform): a point competes for the
                                // segment's maximum, the net change closes the segment
                                if (t[g] & (PROG_END_POINT | PROG_END_SEGMENT)) {
#ifndef LLMEM_SPECIALIZED
                                    // (keeps the next sum's reads behind this point: fewer live registers.  A
                                    // specialized build knows every slot a term names and, left free, reads
                                    // each class value once for all the sums that use it)
                                    asm volatile("" ::: "memory");
#endif
                                    if (t[g] & PROG_END_SEGMENT) {
                                        // the narrow sums are in blocks
                                        const i64 run = NARROW ? (i64)(((u64)acc - NARROW_ZERO) << align_shift) : acc;
                                        const i64 peak = NARROW ? (i64)(((u64)top - NARROW_ZERO) << align_shift) : top;
                                        close_segment(seg, run, peak, has_point != 0);
                                        ++seg;
                                        top = NARROW ? 0 : LOWEST;
                                        has_point = 0;
                                    } else {
#ifdef LLMEM_SPECIALIZED
                                        // (a segment's first point needs no comparison, and this build knows which it is)
                                        if (NARROW) top = has_point ? max_of_positive(acc, top) : acc;
#else
                                        if (NARROW) top = max_of_positive(acc, top);
#endif
                                        else top = acc > top ? acc : top;
                                        has_point = 1;
                                    }
                                    acc = zero;
                                }
                            }
                        }
                    };
                    const u32 beyond = store_classes(Narrow());
                    // every size of every lane at most 2^31 blocks: the 32-bit walk is exact
                    if (__builtin_amdgcn_ballot_w64(beyond != 0) == 0) {
                        walk_terms(Narrow());
                    } else {
                        // the halves of the wave take turns with the same rows (lane l and lane l + 32
                        // share a slot): the second half's stores stay behind the first half's reads
                        for (u32 half = 0; half < 2; ++half) {
                            if ((u32)(lane >> 5) == half) {
                                store_classes(Wide());
                                walk_terms(Wide());
                            }
                            wave_lds_fence();
                        }
                    }
                } else if (DIRECT) {
                    // ---- timeline (Sec. 2.1 / Sec. 3.1): A, F x L, H, B x L, Z, every event's size evaluated
                    // where it stands; the live total can only peak right after an allocation
                    // Events are fetched four at a time (wave-uniform scalar loads, the next four requested
                    // before these are evaluated; reads stay inside the architecture's entries) and a
                    // dimension that is LLMEM_DIM_ONE costs nothing (wave-uniform branches).
                    const int event_first = (int)uni((u32)al.event_first);
                    const int event_last = event_first + (int)uni((u32)al.seg_first[LLMEM_NSEG]) - 1;
                    auto fetch_four = [&](int e, uint4 (&four)[4]) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) four[q] = a.events_dev[e + q < event_last ? e + q : event_last];
                    };
                    auto event_value = [&](u32 coef, u32 dims, u32 z) -> u64 {
                        u32 dv[4];
#pragma unroll
                        for (int q = 0; q < 4; ++q) dv[q] = dim_at((dims >> (8 * q)) & 15u);
                        u64 x = (u64)coef * (z & 255u);                                   // wave-uniform
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            if (((dims >> (8 * q)) & 15u) != LLMEM_DIM_ONE) {
                                asm volatile("" ::: "memory");
                                x = mul_64x32(x, dv[q]);
                            }
                        }
                        const u32 fl = (z >> 16) & 255u, mask = (z >> 24) & 7u;
                        if (fl & LLMEM_EV_TP_GATHER) x = b_cdiv(x * (u64)(d - 1), d, div_mul, div_shift);
                        u64 r = b_up(x, align_shift);
                        if (fl & LLMEM_EV_TIMES_L) r *= (u64)L;
                        if (mask != 7u) r = ((mask >> method) & 1u) ? r : 0ull;
                        return r;
                    };
                    for (int s = 0; s < LLMEM_NSEG; ++s) {
                        i64 run = 0, top = LOWEST;
                        const int e_begin = event_first + (int)uni((u32)al.seg_first[s]);
                        const int e_end = event_first + (int)uni((u32)al.seg_first[s + 1]);
                        for (int e = e_begin; e < e_end; ++e) {
                            const uint4 raw = a.events_dev[e];                  // wave-uniform
                            const u32 z = uni(raw.z);
                            const i64 v = (i64)event_value(uni(raw.x), uni(raw.y), z);
                            if ((z >> 16) & LLMEM_EV_FREE) {
                                asm volatile("" ::: "memory");
                                run -= v;
                            } else {
                                run += v;
                                top = run > top ? run : top;
                            }
                        }
                        close_segment(s, run, top, top != LOWEST);
                    }
                } else {
                // ---- size classes of the timeline: rounded bytes into the value slots ----
                const int nc_raw = (int)uni((u32)n_class[ar]);
                const int nc = nc_raw < CLS_MAX ? nc_raw : CLS_MAX;
                for (int c = 0; c < nc; ++c) {
                    const uint4 ce = cls_tab[ar * CLS_MAX + c];                // wave-uniform
                    const u64 r = class_value(uni(ce.x), uni(ce.y), uni(ce.z));
                    if (c + 1 < a.s_slots) *reinterpret_cast<i64 *>(vals + (c + 1) * 512) = (i64)r;
                }
                // ---- timeline (Sec. 2.1 / Sec. 3.1): A, F x L, H, B x L, Z, event by event ---------
                const int code_first = (int)uni((u32)al.code_first);
                for (int s = 0; s < LLMEM_NSEG; ++s) {
                    i64 run = 0, top = LOWEST;
                    const int e_begin = code_first + (int)uni((u32)al.seg_code[s]);
                    const int e_end = code_first + (int)uni((u32)al.seg_code[s + 1]);
                    for (int e = e_begin; e < e_end; e += CODE_GROUP) {
                        const uint4 cq = *reinterpret_cast<const uint4 *>(codes + e);   // 8 codes, wave-uniform
                        const u32 w0 = uni(cq.x), w1 = uni(cq.y), w2 = uni(cq.z), w3 = uni(cq.w);
                        const u32 c0 = w0 & 0xffffu, c1 = w0 >> 16, c2 = w1 & 0xffffu, c3 = w1 >> 16,
                                  c4 = w2 & 0xffffu, c5 = w2 >> 16, c6 = w3 & 0xffffu, c7 = w3 >> 16;
#define LLMEM_VAL(c) (*reinterpret_cast<const i64 *>(vals + (c & CODE_OFFSET_MASK)))
                        const i64 v0 = LLMEM_VAL(c0), v1 = LLMEM_VAL(c1), v2 = LLMEM_VAL(c2), v3 = LLMEM_VAL(c3),
                                  v4 = LLMEM_VAL(c4), v5 = LLMEM_VAL(c5), v6 = LLMEM_VAL(c6), v7 = LLMEM_VAL(c7);
#undef LLMEM_VAL
                        // the flags are wave-uniform: scalar branches pick add or subtract and skip the
                        // compare and selects where the total cannot peak
#define LLMEM_STEP(v, c) if (c & CODE_FREE) { asm volatile("" ::: "memory"); run -= v; } else { run += v; } \
                         if (c & CODE_CHECK) { asm volatile("" ::: "memory"); top = run > top ? run : top; }
                        LLMEM_STEP(v0, c0) LLMEM_STEP(v1, c1) LLMEM_STEP(v2, c2) LLMEM_STEP(v3, c3)
                        LLMEM_STEP(v4, c4) LLMEM_STEP(v5, c5) LLMEM_STEP(v6, c6) LLMEM_STEP(v7, c7)
#undef LLMEM_STEP
                    }
                    close_segment(s, run, top, top != LOWEST);
                }
                }
                r_live = prelude + best;
#ifndef LLMEM_SPECIALIZED
                r_k = (i64)k_used; r_np = (i64)n_params;
#endif
#ifndef LLMEM_SPECIALIZED
                r_param = (i64)param_gpu; r_grad = (i64)grad_logical; r_os = (i64)os_gpu; r_out = (i64)m_out;
                r_lm = (i64)m_lm; r_back = (i64)m_back; r_tmax = (i64)t_max; r_flags = (i64)flags;
#endif
            }
        };
#ifdef LLMEM_SPECIALIZED
        if (SPEC_ARCHS == 1) {
            // one architecture: every valid lane at once, and no loop for the compiler to hoist out of
            if (valid) for_architecture(0u, WordsAt<SPEC_FIRST[0]>());
        } else
#endif
        {
            // architecture by architecture: the lanes of the first remaining one together
            unsigned long long todo = __builtin_amdgcn_ballot_w64(valid);
            while (todo) {
                const int first = __builtin_ctzll(todo);
                const u32 ar = read_lane(arch_id, first);
                const bool mine = valid && arch_id == ar;
                todo &= ~__builtin_amdgcn_ballot_w64(mine);
                if (mine) {
#ifdef LLMEM_SPECIALIZED
#define LLMEM_ARCH_CASE(q) case q: if (q < SPEC_ARCHS) for_architecture(ar, WordsAt<SPEC_FIRST[q < SPEC_ARCHS ? q : 0]>()); break;
                    switch (ar) {
                    LLMEM_ARCH_CASE(0) LLMEM_ARCH_CASE(1) LLMEM_ARCH_CASE(2) LLMEM_ARCH_CASE(3)
                    LLMEM_ARCH_CASE(4) LLMEM_ARCH_CASE(5) LLMEM_ARCH_CASE(6) LLMEM_ARCH_CASE(7)
                    }
#undef LLMEM_ARCH_CASE
#else
                    for_architecture(ar, WordsFromArguments());
#endif
                }
            }
        }

        if (SWEEP) {
            // the timeline's peak joins the statistics that were folded when the estimate was known
            if (valid && d - 1u < 16u)
                __hip_atomic_fetch_max(sweep_acc + (method * 16u + (d - 1u)) + LLMEM_S_MAX_LIVE * LLMEM_SWEEP_GROUPS, (u64)r_live,
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
#ifdef LLMEM_SPECIALIZED
        } else if (DETAIL) {
            // valid configurations have stored the other columns already; invalid ones store them all
            if (in_range) {
                const u32 at = (u32)lane;
                long long *o = a.out_detail + (b << 6);                 // wave-uniform; the lane is a 32-bit offset
                if (valid) {
                    put(&(o + (long long)LLMEM_D_PEAK_LIVE * n)[at], r_live);
                } else {
                    if (a.out_peaks) put(&(a.out_peaks + (b << 6))[at], -1);
#pragma unroll
                    for (int c = 0; c < LLMEM_NDETAIL; ++c)
                        put(&(o + (long long)c * n)[at], c == LLMEM_D_PEAK ? -1 : c == LLMEM_D_FLAGS ? (i64)err : 0);
                }
            }
#endif
        } else if (in_range) {
            // the batch's position is wave-uniform; the lane is a 32-bit offset from it
            const u32 at = (u32)lane;
            if (a.out_peaks) put(&(a.out_peaks + (b << 6))[at], r_peak);
#ifndef LLMEM_SPECIALIZED
            if (DETAIL) {
                long long *o = a.out_detail + (b << 6);
                put(&(o + (long long)LLMEM_D_PEAK * n)[at], r_peak);
                put(&(o + (long long)LLMEM_D_PARAM_GPU * n)[at], r_param);
                put(&(o + (long long)LLMEM_D_GRAD_GPU * n)[at], r_grad);
                put(&(o + (long long)LLMEM_D_OS_GPU * n)[at], r_os);
                put(&(o + (long long)LLMEM_D_OUT * n)[at], r_out);
                put(&(o + (long long)LLMEM_D_LM * n)[at], r_lm);
                put(&(o + (long long)LLMEM_D_BACK * n)[at], r_back);
                put(&(o + (long long)LLMEM_D_K * n)[at], r_k);
                put(&(o + (long long)LLMEM_D_PEAK_LIVE * n)[at], r_live);
                put(&(o + (long long)LLMEM_D_NPARAMS * n)[at], r_np);
                put(&(o + (long long)LLMEM_D_TMAX * n)[at], r_tmax);
                put(&(o + (long long)LLMEM_D_FLAGS * n)[at], r_flags);
            }
#endif
        }
    }
    if (SWEEP) {
        // the workgroup's statistics join the caller's: sums add, extremes combine
        __syncthreads();
        for (int t = threadIdx.x; t < SWEEP_WORDS; t += block) {
            const int col = t / LLMEM_SWEEP_GROUPS;
            const u64 v = sweep_acc[t];
            u64 *to = a.sweep_stats + t;
            if (col == LLMEM_S_MIN_PEAK) {
                if (v != (u64)INT64_MAX) __hip_atomic_fetch_min(to, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else if (v != 0) {
                if (col == LLMEM_S_COUNT || col == LLMEM_S_FIT || col == LLMEM_S_K_SUM)
                    __hip_atomic_fetch_add(to, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                else
                    __hip_atomic_fetch_max(to, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

#ifdef LLMEM_SPECIALIZED

// the flavour this build was asked for (LLMEM_SPEC_FLAVOUR: 0 m_peak only, 1 with the detail
// columns, 2 sweep); a build ahead of time names its kernel itself (LLMEM_SPEC_KERNEL)
#ifndef LLMEM_SPEC_KERNEL
#if LLMEM_SPEC_FLAVOUR == 0
#define LLMEM_SPEC_KERNEL llmem_specialized_peaks
#elif LLMEM_SPEC_FLAVOUR == 1
#define LLMEM_SPEC_KERNEL llmem_specialized_detail
#else
#define LLMEM_SPEC_KERNEL llmem_specialized_sweep
#endif
#endif
extern "C" __global__ __launch_bounds__(BB_BLOCK) __attribute__((amdgpu_waves_per_eu(LLMEM_WAVES_PER_SIMD)))
void LLMEM_SPEC_KERNEL(const EstimateArgs a)
{
    estimate_batch_body<LLMEM_SPEC_FLAVOUR != 0, FORM_COMPILED, LLMEM_SPEC_FLAVOUR == 2>(a);
}

#ifdef LLMEM_SPEC_ENTRY
// built into the library: the host side reaches the kernel through this function
extern "C" __attribute__((visibility("hidden"))) const void *LLMEM_SPEC_ENTRY()
{
    return reinterpret_cast<const void *>(&LLMEM_SPEC_KERNEL);
}
#endif

}  // namespace llmem

#else

template <bool DETAIL, int FORM, bool SWEEP>
__global__ __launch_bounds__(BB_BLOCK) __attribute__((amdgpu_waves_per_eu(LLMEM_WAVES_PER_SIMD)))
void estimate_batch_kernel(const EstimateArgs a)
{
    estimate_batch_body<DETAIL, FORM, SWEEP>(a);
}

// empty statistics: 0, and the largest value where a minimum is kept
__global__ __launch_bounds__(256) void sweep_reset_kernel(long long *stats)
{
    for (int t = threadIdx.x; t < LLMEM_NSWEEP * LLMEM_SWEEP_GROUPS; t += 256)
        stats[t] = t / LLMEM_SWEEP_GROUPS == LLMEM_S_MIN_PEAK ? INT64_MAX : 0;
}

void launch_sweep_reset(long long *stats, hipStream_t stream)
{
    hipLaunchKernelGGL(sweep_reset_kernel, dim3(1), dim3(256), 0, stream, stats);
}

size_t batch_kernel_lds_bytes(const EstimateArgs &a)
{
    if (a.use_program)                                                // compiled form: value slots only
        return ((size_t)SLOT_ROW * (size_t)a.p_slots * a.waves + 15) & ~(size_t)15;
    if (a.direct) return (size_t)DIRECT_ROWS * 256 * a.waves;         // direct form: the dimension vectors of 64 lanes
    const size_t values = sizeof(long long) * 64 * (size_t)a.s_slots * a.waves;
    size_t fixed = sizeof(uint4) * (size_t)a.n_arch * CLS_MAX;        // class table
    fixed += sizeof(unsigned short) * (size_t)a.code_count;            // event codes
    fixed += sizeof(int) * LLMEM_MAX_ARCH;                             // class counts
    size_t scratch = sizeof(uint4) * (size_t)a.max_events;             // set-up scratch: keys
    scratch += 2 * sizeof(unsigned short) * (size_t)(a.max_events + 1); // representatives, class ids
    return ((fixed + (scratch > values ? scratch : values)) + 15) & ~(size_t)15;
}

int batch_kernel_waves(EstimateArgs a)
{
    for (a.waves = BATCH_WAVES; a.waves >= 1; a.waves /= 2)
        if (batch_kernel_lds_bytes(a) <= BATCH_LDS_LIMIT) return a.waves;
    return 0;
}

static void launch_lane_kernel(const EstimateArgs &args, bool detail, bool sweep, long long n_batch, hipStream_t stream)
{
    const size_t lds_bytes = batch_kernel_lds_bytes(args);
    // as many workgroups as stay resident at once; each strides over the batches
    static int cu_count = 0;
    if (cu_count == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess
            && hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            cu_count = v;
        else
            cu_count = 256;
    }
    typedef void (*Kernel)(const EstimateArgs);
    const Kernel kernels[3][3] = {
        {estimate_batch_kernel<false, FORM_EVENTS, false>, estimate_batch_kernel<false, FORM_COMPILED, false>,
         estimate_batch_kernel<false, FORM_EVENTS, false>},            // without the timeline the direct form is the events form
        {estimate_batch_kernel<true, FORM_EVENTS, false>, estimate_batch_kernel<true, FORM_COMPILED, false>,
         estimate_batch_kernel<true, FORM_DIRECT, false>},
        {estimate_batch_kernel<true, FORM_EVENTS, true>, estimate_batch_kernel<true, FORM_COMPILED, true>,
         estimate_batch_kernel<true, FORM_DIRECT, true>}};
    const Kernel kernel = kernels[sweep ? 2 : detail ? 1 : 0][args.use_program ? FORM_COMPILED : args.direct ? FORM_DIRECT : FORM_EVENTS];
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(kernel), 64 * args.waves, lds_bytes)
            != hipSuccess || per_cu < 1)
        per_cu = 1;
    // the compiled form has next to no set-up per workgroup: several times more workgroups than
    // stay resident at once; the others stage their tables per workgroup
    const long long blocks = lane_kernel_blocks(n_batch, args.waves, (long long)per_cu * cu_count, args.use_program ? 16 : 1, sweep);
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(64 * args.waves), lds_bytes, stream, args);
}

void launch_batch_kernel(const EstimateArgs &args, bool detail, long long n_batch, hipStream_t stream)
{
    launch_lane_kernel(args, detail, false, n_batch, stream);
}

void launch_sweep_kernel(const EstimateArgs &args, long long n_batch, hipStream_t stream)
{
    launch_lane_kernel(args, true, true, n_batch, stream);
}

}  // namespace llmem

#endif  // LLMEM_SPECIALIZED
