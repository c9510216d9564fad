// Kernel arguments and table planning shared by the two estimator kernels
// (one wavefront per configuration; one lane per configuration).
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

constexpr int K_SEARCH_MIN = 2, K_SEARCH_MAX = 10, K_FIXED_MAX = 16;
// forms of the lane-per-configuration kernel (see estimate_batch.hip)
constexpr int FORM_EVENTS = 0, FORM_COMPILED = 1, FORM_DIRECT = 2;
constexpr int DIRECT_ROWS = 16;                // direct form: LDS rows (256 bytes) per wavefront, one per dimension
constexpr int B16 = 2, B32 = 4;

// lane-per-configuration kernel: at most CLS_MAX size classes per architecture; class c
// keeps its value in slot c + 1 of the wave's LDS array, slot 0 holds 0 (padding events).
// An event code is the slot's byte offset (slot * 512, below 2^16) with two flags in the low
// bits; codes are fetched CODE_GROUP at a time.
constexpr int CLS_MAX = 120;
constexpr int CODE_GROUP = 8;
constexpr unsigned CODE_CHECK = 1, CODE_FREE = 2, CODE_OFFSET_MASK = 0xfe00;
constexpr int BATCH_WAVES = 4;                 // wavefronts per workgroup: this many, or 2 or 1 when the value
                                               // slots of four wavefronts do not fit the workgroup's LDS
// lane-per-configuration kernel, compiled form of the tables: the host groups parameter entries
// with the same size expression, groups events into size classes, reduces the events of every
// segment to the peak points no other point dominates (class-count vectors compared
// component-wise) and passes the result in the kernel arguments.  Stream of 32-bit words per
// architecture:
//   header     PROG_HEADER words: n_groups | e_n << 8 | n_class << 16; the first word of each
//              segment's terms and the word after the last segment (absolute); padding
//   per group  coefficient; descriptor; E_once | E_layer << 8 | LM_once << 16 | LM_layer << 24;
//              OTHER_once | OTHER_layer << 8 | OS_once << 16 | OS_layer << 24
//              (how many entries of the group count towards embed_p, lm_p, other_p, m_os, once or
//              once per block)
//   per class  coefficient * element bytes; descriptor (padded with empty classes, 0 0, to a
//              multiple of PROG_CLASS_FETCH)
//   the sums of the segments A F H B Z one after the other, each sum in groups of PROG_GROUP
//              terms: a segment's peak points, then its net change.  A term is
//              slot * SLOT_ROW | factor << 16 with a signed 16-bit factor: the partial sum gains
//              factor * slot value.  A flag in
//              the first term of a sum's last group closes it: PROG_END_POINT (the sum competes
//              for the segment's maximum and the partial sum restarts) or PROG_END_SEGMENT (the
//              sum is the segment's net change; the next segment starts).  Padding terms are 0
//              (slot 0 holds 0); whole groups of them pad the list to PROG_FETCH words.
//              Slot c + 1 holds MINUS the value of class c and the factor is minus the count, so
//              that a value of exactly 2^31 allocator blocks still fits a signed 32-bit slot.
// Descriptor: number of dimensions (bits 0-2), their selectors (4 bits each from bit 4),
// DESC_TP_GATHER, DESC_TIMES_L, method mask (3 bits from DESC_MASK_SHIFT).
constexpr unsigned DESC_TP_GATHER = 1u << 20, DESC_TIMES_L = 1u << 21;
constexpr unsigned DESC_FROM_PREVIOUS = 7;     // in place of the number of dimensions: the previous class's raw
                                               // size shifted left by the first word
constexpr int DESC_MASK_SHIFT = 22;
constexpr int PROG_SLOT_MAX = 100;
constexpr int PROG_WORDS = 704;
constexpr int DIM_BS_SL = 15;                  // selector of bs * sl in the compiled descriptors (after the LLMEM_DIM_* ones)
static_assert(LLMEM_NDIM == DIM_BS_SL, "the product's selector follows the public ones");
constexpr int PROG_HEADER = 8;
constexpr int PROG_GROUP = 4;
constexpr int PROG_CLASS_FETCH = 4;            // classes the list is padded to and read by
constexpr int PROG_FETCH = 8;                   // words a segment's term list is padded to and read by
constexpr int SLOT_ROW = 256;                   // bytes of LDS per value slot and wavefront in the compiled form
constexpr unsigned PROG_OFFSET_MASK = 0xff00, PROG_END_POINT = 0x1, PROG_END_SEGMENT = 0x2;
constexpr size_t BATCH_LDS_LIMIT = 62 * 1024;  // dynamic LDS a launch may ask for (the kernel has 2 KB of its own)

struct ArchLayout {
    int param_first, n_param;
    int event_first;                 // first entry of the architecture in events_dev
    int seg_first[LLMEM_NSEG + 1];   // segment boundaries relative to event_first
    // wavefront-per-configuration kernel: every lane owns `per_lane` consecutive events of a
    // single segment; segment s occupies lanes lane0[s] .. lane0[s+1]-1; LDS slot
    // slot_first + j*64 + lane holds the lane's j-th event
    int per_lane;
    int lane0[LLMEM_NSEG + 1];
    int slot_first;
    // lane-per-configuration kernel: the architecture's event codes start at code_first; the
    // codes of segment s occupy [seg_code[s], seg_code[s+1]) relative to that, each segment
    // padded to a multiple of CODE_GROUP
    int code_first;
    int seg_code[LLMEM_NSEG + 1];
    // compiled timeline: first word of the architecture in EstimateArgs::prog; the terms of
    // segment s start at word prog_seg[s] (absolute) and end at prog_seg[s + 1]
    int prog_first;
    int prog_seg[LLMEM_NSEG + 1];
};

struct EstimateArgs {
    llmem_configs cfg;
    long long n;
    long long m_base;
    int cu_shift, align_shift;
    int n_arch, n_param_total, n_slot_total;
    int code_count, max_events, s_slots;
    int p_slots;                     // value slots per wave in the compiled form
    int waves;                       // wavefronts per workgroup of this launch (4, 2 or 1)
    int direct;                      // 1 (with use_program 0): every event evaluated where it stands, no size classes
    ArchLayout arch[LLMEM_MAX_ARCH];
    const uint4 *params_dev;
    const uint4 *events_dev;
    long long *out_peaks;
    long long *out_detail;
    int use_program;                 // 1: the compiled timeline below is valid and used
    // sweep: configurations sweep_first .. sweep_first + n - 1 of grid sweep_grid are drawn in the
    // kernel (cfg is not read) and folded into sweep_stats (nothing is stored per configuration)
    int sweep_grid;
    unsigned long long sweep_seed;
    long long sweep_first;
    long long m_total;
    unsigned long long *sweep_stats;
    uint32_t prog[PROG_WORDS];
};

static_assert(sizeof(EstimateArgs) <= 4096, "kernel arguments are limited to 4 KB");

// Events with equal keys have equal byte sizes for every configuration: same
// coefficient, same multiset of dimensions, same element width, scaling flags
// and method mask.  x, y, z are the first three dwords of an llmem_event_entry.
struct ClassKey { uint32_t coef, dims, meta; };

__host__ __device__ inline ClassKey make_class_key(uint32_t x, uint32_t y, uint32_t z)
{
    uint32_t d0 = y & 15u, d1 = (y >> 8) & 15u, d2 = (y >> 16) & 15u, d3 = (y >> 24) & 15u, t;
#define LLMEM_CSWAP(p, q) if (p > q) { t = p; p = q; q = t; }
    LLMEM_CSWAP(d0, d1) LLMEM_CSWAP(d2, d3) LLMEM_CSWAP(d0, d2) LLMEM_CSWAP(d1, d3) LLMEM_CSWAP(d1, d2)
#undef LLMEM_CSWAP
    const uint32_t elem_bytes = z & 255u, flags = (z >> 16) & 255u, mask = (z >> 24) & 7u;
    ClassKey k;
    k.coef = x;
    k.dims = d0 | (d1 << 8) | (d2 << 16) | (d3 << 24);
    k.meta = elem_bytes | ((flags & (LLMEM_EV_TIMES_L | LLMEM_EV_TP_GATHER)) << 8) | (mask << 16);
    return k;
}

// Validates the host copy of the tables exactly as the estimator does and fills the constants
// and per-architecture ranges of `out`; LLMEM_OK or LLMEM_EINVAL_*.
#ifndef __HIPCC_RTC__
int check_tables(const llmem_tables *tables, EstimateArgs *out);
// unloads every kernel built at run time (specialize.hip); returns how many
int release_built();
// Parameter entries of one architecture grouped by size expression: four words per group as in
// the compiled tables above, into `words` (room for max_groups groups).  Returns the number of
// groups, -1 if there are more than max_groups; *e_n = embedding tables whose outputs are kept.
int compile_param_groups(const llmem_param_entry *pe, int n_param, uint32_t *words, int max_groups, uint32_t *e_n);
// dynamic LDS of a lane-kernel launch with a.waves wavefronts per workgroup
size_t batch_kernel_lds_bytes(const EstimateArgs &a);
// the most wavefronts per workgroup (4, 2, 1) whose LDS fits, 0 if not even one does; a.use_program picks the form
int batch_kernel_waves(EstimateArgs a);
void launch_batch_kernel(const EstimateArgs &args, bool detail, long long n_batch, hipStream_t stream);
void launch_sweep_kernel(const EstimateArgs &args, long long n_batch, hipStream_t stream);
void launch_sweep_reset(long long *stats, hipStream_t stream);
// Specialized form: the lane kernel compiled with the compiled tables of `args` as constants:
// a kernel built into the library when the tables are those of a set it ships with
// (has_prebuilt), else, or when at_run_time is set, one built at run time (one build per set of
// tables, flavour and device, kept until the process ends).  flavour: 0 m_peak only, 1 with the
// detail columns, 2 sweep.  LLMEM_OK, or LLMEM_EHIP with the compiler's or the loader's message
// as the error text.
// Workgroups of a lane-kernel launch over n_batch batches of 64 configurations, `waves` wavefronts
// each striding over the batches.  `resident`: workgroups the device holds at once; `spread`: how
// many times that number the launch may have (forms with next to no set-up per workgroup take 16:
// the dispatcher then evens out the compute units; measured 2 to 48).  Every workgroup of a sweep ends with one
// global atomic per statistic and group (384), which all workgroups aim at the same addresses: they
// stay few against its own work from six batches per wavefront on (10^7 configurations: 0.40 ms
// with 16 x resident workgroups, 0.26 ms with 6 x; 10^6: 0.092 ms with one batch per wavefront,
// 0.038 ms with as many workgroups as are resident).
inline long long lane_kernel_blocks(long long n_batch, int waves, long long resident, int spread, bool sweep)
{
    const long long blocks = (n_batch + waves - 1) / waves;
    long long cap = resident * spread;
    if (sweep) {
        const long long by_work = (n_batch + waves * 6 - 1) / (waves * 6);
        if (by_work < cap) cap = by_work > resident ? by_work : resident;
    }
    return blocks < cap ? blocks : cap;
}
bool has_prebuilt(const EstimateArgs &args, int flavour);
int launch_specialized(const EstimateArgs &args, int flavour, long long n_batch, hipStream_t stream, bool at_run_time);
#endif
constexpr int SWEEP_INDEX_BITS = 40;             // LLMEM_S_BEST: score2 << 40 | (2^40 - 1 - index)

}  // namespace llmem
