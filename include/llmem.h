/* llmem.h - C ABI of the batched peak-GPU-memory estimator (gfx950).
 *
 * The library evaluates, for n independent fine-tuning configurations, the
 * estimator of "LLMem: Estimating GPU Memory Usage for Fine-Tuning Pre-Trained
 * LLMs" (arXiv 2404.10933): the closed-form peak of Sec. 4.2 (single GPU /
 * conventional data parallelism) and Sec. 5 (ZeRO-3 "advanced DP", 1-D tensor
 * parallelism), the chunk-size choice of Sec. 4.1, and a traversal of the
 * operator timeline with live tensors and 512-byte allocator blocks (Sec. 2.1,
 * Sec. 3.1); further the estimate for combined DP+TP (Sec. 5) and the choice of
 * the fine-tuning method with its largest batch size (Sec. 6, Algorithm 1), and
 * the same estimates for whole seeded grids that are drawn, estimated and reduced
 * to statistics inside one kernel.  All arithmetic is exact int64 byte arithmetic.
 *
 * Conventions
 *   DEV   pointer to device memory, owned by the caller; the library never
 *         allocates, frees or retains it.  (The one exception to "never allocates" is the
 *         kernel built at run time, see LLMEM_KERNEL_LANE_SPECIALIZED: its first call with a
 *         set of tables allocates host memory for the build and device memory for the code.)
 *   HOST  pointer to host memory, read during the call only.
 *   Every call enqueues its kernels on `hip_stream` (a hipStream_t passed as
 *   void*; NULL = the default stream) and returns without synchronising.
 *   A call only validates on the host and launches kernels, so it may be recorded
 *   while its stream is capturing into a HIP graph; a kernel built at run time
 *   (LLMEM_KERNEL_LANE_SPECIALIZED with tables the library has no built-in specialization for,
 *   LLMEM_KERNEL_LANE_RUNTIME) must have been built by a call outside the capture first.
 *   Return value: LLMEM_OK or a negative error code; on an error nothing has been
 *   enqueued and no output is written.
 */
#ifndef LLMEM_H
#define LLMEM_H

#ifndef __HIPCC_RTC__            /* the run-time compiler brings the fixed-width types itself */
#include <stddef.h>
#include <stdint.h>
#endif

#ifdef __cplusplus
extern "C" {
#endif

#define LLMEM_ABI_VERSION 5

/* ---- error codes --------------------------------------------------------- */
#define LLMEM_OK            0
#define LLMEM_EINVAL_NULL  (-1)   /* a required pointer is NULL                          */
#define LLMEM_EINVAL_N     (-2)   /* n < 0 (n == 0 is a valid no-op)                     */
#define LLMEM_EINVAL_TABLE (-3)   /* malformed tables / constants (see llmem_tables)     */
#define LLMEM_EHIP         (-4)   /* a HIP call failed; llmem_strerror gives the text    */
#define LLMEM_EINVAL_ARG   (-5)   /* any other bad argument (unknown grid id, ...)       */

/* ---- limits --------------------------------------------------------------- */
#define LLMEM_MAX_ARCH          8     /* architecture tables per call                   */
#define LLMEM_MAX_PARAM_ENTRIES 64    /* parameter-table entries per architecture       */
#define LLMEM_MAX_EVENT_ENTRIES 1024  /* timeline events per architecture               */
#define LLMEM_MAX_EVENT_SLOTS   3072  /* LDS slots for all architectures of one call    */

/* ---- configurations (structure of arrays) --------------------------------- */
/* One fine-tuning configuration = the inputs of the paper's problem statement
 * (Notation table; Algorithm 1 inputs): decoder shape, bs, sl, method, gpu_n (d),
 * chunk size.  Each member is a DEV array of n values.  The order of the
 * configurations never changes a result; it does change the time: 64 consecutive
 * configurations share a wavefront, which takes the architectures they name one
 * after the other, so arrays grouped by arch_id run fastest.                   */
typedef struct llmem_configs {
    uint8_t  *arch_id;   /* index into llmem_tables.arch                                   */
    uint32_t *h;         /* hidden width (o_n)                                             */
    uint16_t *L;         /* number of transformer blocks (l_n)                             */
    uint16_t *n_heads;   /* attention heads; head_dim = h / n_heads                        */
    uint16_t *n_kv;      /* key/value heads; kv_dim = n_kv * head_dim                      */
    uint32_t *ffn;       /* feed-forward width                                             */
    uint32_t *V;         /* dictionary size (dict_n)                                       */
    uint32_t *P;         /* rows of a learned position table (0 if none)                   */
    uint16_t *bs;        /* batch size                                                     */
    uint16_t *sl;        /* sequence length                                                */
    uint8_t  *method;    /* LLMEM_METHOD_*                                                 */
    uint8_t  *d;         /* partition degree gpu_n, >= 1 (ignored by conventional DP)      */
    int8_t   *chunk_k;   /* chunk of 2^k MiB of fp16 values, 0..16; LLMEM_CHUNK_SEARCH     */
    uint8_t  *flags;     /* LLMEM_CFG_* bits                                               */
} llmem_configs;

#define LLMEM_METHOD_CDP   0   /* conventional data parallelism = single-GPU peak (Sec. 5) */
#define LLMEM_METHOD_ZERO3 1   /* advanced data parallelism, ZeRO-3 (Sec. 5)              */
#define LLMEM_METHOD_TP    2   /* 1-D tensor parallelism (Sec. 5)                         */
/* results of llmem_decide only (llmem_estimate takes methods 0..2): */
#define LLMEM_METHOD_HYBRID  3 /* DP+TP: tp_n GPUs per tensor-parallel group (Sec. 5)      */
#define LLMEM_METHOD_OFFLOAD 4 /* "4, 0": no method fits, train with CPU memory (Sec. 6)   */

#define LLMEM_CHUNK_SEARCH (-1) /* search k = 2..10: least padding waste among the chunk
                                   sizes that hold the largest tensor, ties to the smaller */

#define LLMEM_CFG_LOGITS_FP32 1 /* B = 4 bytes per logit in m_lm, else 2 (Sec. 4.2)        */
#define LLMEM_CFG_TIED_LM_HEAD 2 /* lm_head shares the input embedding: n_params only      */
#define LLMEM_CFG_GRAD_ALIAS  4 /* gradient fp16 shares the param fp16 space (Sec. 4.1);
                                   when clear a gradient term is added to the peak         */

/* ---- architecture tables --------------------------------------------------- */
/* Every size is  coef * D[dim[0]] * D[dim[1]] * D[dim[2]] * D[dim[3]]  over the
 * per-configuration dimension vector D; unused selectors are LLMEM_DIM_ONE.   */
enum llmem_dim {
    LLMEM_DIM_ONE = 0, LLMEM_DIM_BS, LLMEM_DIM_SL, LLMEM_DIM_SL_M1 /* max(sl-1,0) */, LLMEM_DIM_H,
    LLMEM_DIM_FFN, LLMEM_DIM_N_HEADS, LLMEM_DIM_N_KV, LLMEM_DIM_HEAD_DIM, LLMEM_DIM_KV_DIM,
    LLMEM_DIM_V, LLMEM_DIM_P, LLMEM_DIM_L, LLMEM_DIM_B_LOGITS /* 2 or 4 */, LLMEM_DIM_D,
    LLMEM_NDIM
};

/* A parameter tensor (element count).  Classes and roles follow Sec. 4.2: only
 * Embedding and Linear tensors carry optimizer-state pages (m_os); the token
 * embedding is embed_p, the lm_head is lm_p, everything else other_p.          */
typedef struct llmem_param_entry {
    uint32_t coef;
    uint8_t  dim[4];
    uint8_t  cls;        /* LLMEM_CLS_*                                                   */
    uint8_t  role;       /* LLMEM_ROLE_*                                                  */
    uint8_t  per_layer;  /* 1: one such tensor in each of the L blocks                    */
    uint8_t  reserved[5];
} llmem_param_entry;     /* 16 bytes */

#define LLMEM_CLS_EMBEDDING 0
#define LLMEM_CLS_LINEAR    1
#define LLMEM_CLS_BIAS      2
#define LLMEM_CLS_NORM      3
#define LLMEM_ROLE_EMBED_TOK 0
#define LLMEM_ROLE_LM_HEAD   1
#define LLMEM_ROLE_OTHER     2

/* One allocator event of the fine-tuning iteration (bytes = monomial * elem_bytes,
 * optionally scaled, rounded up to the allocator block, optionally times L).
 * Events of one architecture must be grouped by segment in the order A F H B Z:
 * A once, F once per block, H once, B once per block, Z once.                  */
typedef struct llmem_event_entry {
    uint32_t coef;
    uint8_t  dim[4];
    uint8_t  elem_bytes;
    uint8_t  seg;          /* LLMEM_SEG_*                                                 */
    uint8_t  flags;        /* LLMEM_EV_* bits                                             */
    uint8_t  method_mask;  /* bit m set: the event exists under method m                  */
    uint32_t reserved;
} llmem_event_entry;       /* 16 bytes */

#define LLMEM_SEG_A 0
#define LLMEM_SEG_F 1
#define LLMEM_SEG_H 2
#define LLMEM_SEG_B 3
#define LLMEM_SEG_Z 4
#define LLMEM_NSEG  5
#define LLMEM_EV_FREE      1   /* release (negative) instead of allocation                 */
#define LLMEM_EV_TIMES_L   2   /* rounded size multiplied by L (L equal tensors at once)   */
#define LLMEM_EV_TP_GATHER 4   /* raw bytes -> ceil(raw * (d-1) / d): the backward
                                  all-gather buffer of Sec. 5 (m_back^tp)                  */

typedef struct llmem_arch_desc {
    int32_t param_first, n_param;   /* range in params_host / params_dev                   */
    int32_t event_first, n_event;   /* range in events_host / events_dev                   */
} llmem_arch_desc;

/* HOST struct.  The entry arrays are given twice with identical contents: a HOST
 * copy, validated on every call, and a DEV copy the kernels read.  (Each host thread
 * keeps what the library derived from the last four table sets it was called with and
 * reuses it when constants, ranges and entries compare equal byte for byte, which makes a
 * repeated call cost microseconds; the caller may change the contents between calls.)
 * LLMEM_EINVAL_TABLE is returned when: n_arch is outside 1..LLMEM_MAX_ARCH; a
 * range is negative, exceeds the limits above or the array lengths (the slot limit
 * only binds the kernel that uses slots, see LLMEM_KERNEL_*); a selector
 * is >= LLMEM_NDIM; cls / role / seg are out of range; events are not grouped
 * A F H B Z; cu_p or align is not a power of two, align > cu_p, align < 1,
 * or m_base < 0.                                                               */
typedef struct llmem_tables {
    int64_t m_base;     /* initially used GPU memory (Notation table), bytes               */
    int64_t cu_p;       /* CUDA page size of Sec. 4.2, typically 2 MiB; power of two       */
    int64_t align;      /* allocator block, 512 bytes (Sec. 3.1); power of two             */
    int32_t n_arch;
    int32_t n_param_total, n_event_total;   /* lengths of the entry arrays                 */
    int32_t kernel;                         /* LLMEM_KERNEL_*; 0 lets the library choose   */
    llmem_arch_desc arch[LLMEM_MAX_ARCH];
    const llmem_param_entry *params_host;   /* HOST */
    const llmem_event_entry *events_host;   /* HOST */
    const llmem_param_entry *params_dev;    /* DEV  */
    const llmem_event_entry *events_dev;    /* DEV  */
} llmem_tables;

/* Two kernels compute the same results.  LLMEM_KERNEL_LANE holds one configuration
 * per lane (64 per wavefront) and walks the tables entry by entry.  Its timeline
 * walk has three forms.  The host reduces each segment to the peak points that no other
 * point dominates and hands them to the kernel in its arguments
 * (LLMEM_KERNEL_LANE_COMPILED, when that fits the argument space); or the kernel groups the
 * events into size classes, keeps each class's value in LDS and walks every event as an add
 * or subtract (LLMEM_KERNEL_LANE_EVENTS; at most 120 distinct size expressions among the events
 * of each architecture, fewer when the LDS of a workgroup does not hold the slots of even one
 * wavefront); or it evaluates every event's size where it stands (LLMEM_KERNEL_LANE_DIRECT:
 * any tables, no LDS, slower per event).  LLMEM_KERNEL_WAVE gives a whole
 * wavefront to each configuration with the lanes spread over table entries; it needs
 * the events of all architectures, dealt to lanes, to fit LLMEM_MAX_EVENT_SLOTS, and is only
 * used when asked for (it is several times slower than any lane form).
 * LLMEM_KERNEL_LANE_SPECIALIZED is the compiled form taken one step further: the lane kernel's
 * own source compiled once more with the compiled tables as constants, so that every table word
 * becomes an immediate and every loop over table entries straight-line code.  Results are the
 * same bit for bit.  Such kernels exist in two ways.
 *   Built into the library, for the table sets it ships with (the GPT-, OPT- and Llama-style
 *   tables of its workloads module, with and without gradient checkpointing, each alone, and the
 *   three checkpointed ones together): a call whose tables compile to exactly the same words
 *   launches the built-in kernel; nothing is compiled, loaded or allocated.
 *   Built at run time (hiprtc) for any other tables the compiled form admits: the first call with
 *   a given set of tables takes a fraction of a second to a few seconds to build and load the
 *   kernel and allocates host memory for the build and device memory for the loaded code object;
 *   the build is kept, per device, until llmem_kernels_release or the end of the process, and also
 *   between processes when the environment variable LLMEM_KERNEL_CACHE names a writable directory
 *   (one file per build, used only if its recorded identity matches in full).  At most 64 such
 *   kernels stay loaded per device (LLMEM_KERNELS_KEPT changes the number): a call that has to
 *   build one more first waits for the device (hipDeviceSynchronize) and unloads the less recently
 *   used half of those no call is using; a later call with their tables builds them again.  A failure of the run-time compiler or loader
 *   is LLMEM_EHIP with its message in llmem_strerror.  The run-time compiler is not started in a
 *   process that a profiler has been loaded into (ROCP_TOOL_LIBRARIES set, or LD_PRELOAD /
 *   HSA_TOOLS_LIB naming a rocprofiler library): without a kept code object such a call is
 *   LLMEM_EHIP; fill LLMEM_KERNEL_CACHE in an unprofiled run first.  A call recorded into a HIP
 *   graph must not be the one that builds.
 * LLMEM_KERNEL_AUTO and LLMEM_KERNEL_LANE take a built-in specialization when one matches, else
 * the first of compiled, events, direct that the tables allow; they never build at run time.  LLMEM_KERNEL_LANE_SPECIALIZED takes a built-in specialization when
 * one matches and builds at run time otherwise; LLMEM_KERNEL_LANE_RUNTIME always builds at run
 * time.  A forced choice the tables do not allow is LLMEM_EINVAL_TABLE.  llmem_estimate(_ex) and
 * llmem_sweep honour all of these.                                                          */
#define LLMEM_KERNEL_AUTO 0
#define LLMEM_KERNEL_WAVE 1
#define LLMEM_KERNEL_LANE 2
#define LLMEM_KERNEL_LANE_EVENTS 3
#define LLMEM_KERNEL_LANE_COMPILED 4
#define LLMEM_KERNEL_LANE_SPECIALIZED 5
#define LLMEM_KERNEL_LANE_RUNTIME 6
#define LLMEM_KERNEL_LANE_DIRECT 7

/* ---- outputs --------------------------------------------------------------- */
/* Detail columns: out_detail is DEV, LLMEM_NDETAIL columns of n int64 each
 * (column c of configuration i at out_detail[c * n + i]).                      */
enum llmem_detail {
    LLMEM_D_PEAK = 0,     /* m_peak of the configuration's method (Sec. 4.2 / Sec. 5)      */
    LLMEM_D_PARAM_GPU,    /* parameter bytes resident per GPU                              */
    LLMEM_D_GRAD_GPU,     /* logical fp16 gradient bytes per GPU                           */
    LLMEM_D_OS_GPU,       /* momentum + variance bytes per GPU                             */
    LLMEM_D_OUT,          /* m_out                                                         */
    LLMEM_D_LM,           /* m_lm                                                          */
    LLMEM_D_BACK,         /* m_back^tp (0 unless TP)                                       */
    LLMEM_D_K,            /* chunk exponent used                                           */
    LLMEM_D_PEAK_LIVE,    /* largest live bytes over the event timeline                    */
    LLMEM_D_NPARAMS,      /* parameter count                                               */
    LLMEM_D_TMAX,         /* largest single tensor outside embedding / lm_head (elements)  */
    LLMEM_D_FLAGS,        /* LLMEM_F_* bits                                                */
    LLMEM_NDETAIL
};

/* Per-configuration data errors are reported in band: m_peak = -1, every other
 * detail column 0 except the flags.                                            */
#define LLMEM_F_ERR_ARCH    1   /* arch_id >= n_arch                                       */
#define LLMEM_F_ERR_METHOD  2   /* method > 2                                              */
#define LLMEM_F_ERR_D       4   /* d == 0                                                  */
#define LLMEM_F_ERR_HEADS   8   /* n_heads == 0                                            */
#define LLMEM_F_ERR_CHUNK   16  /* chunk_k outside {-1} U [0, 16]                          */
#define LLMEM_F_CHUNK_INFEASIBLE 32 /* the largest tensor exceeds the chunk used (a search
                                       without a feasible candidate falls back to k = 10) */
/* llmem_estimate_methods / llmem_decide only: */
#define LLMEM_F_ERR_TP      64  /* tp_n > 0 does not divide gpu_n                          */
#define LLMEM_F_HYBRID_READINGS_DIFFER 128   /* m_p16 * tp_n / gpu_n (as printed, used) and
                                       m_p16 * (tp_n - 1) / tp_n give different DP+TP estimates */
#define LLMEM_F_FALLBACK_READINGS_DIFFER 256 /* the TP score is 0 (so the result is "4, 0" as
                                       Algorithm 1 prints it) but another score is not    */

/* ---- entry points ---------------------------------------------------------- */

/* m_peak of n configurations (Sec. 4.2 equation for m_peak^s; Sec. 5 equations
 * for m_peak^dp and m_peak^tp; chunk search per Sec. 4.1).
 *   cfg            HOST struct of DEV columns, n values each
 *   method_tables  HOST struct (see llmem_tables)
 *   out_peaks      DEV, n int64
 * Runs on the default stream.  Intermediate values must fit int64 (they do for
 * any decoder up to ~10^12 parameters at bs*sl <= 2^20); overflow wraps.      */
int llmem_estimate(const llmem_configs *cfg, int64_t n, const llmem_tables *method_tables,
                   int64_t *out_peaks);

/* As llmem_estimate, plus the detail columns (component sizes of the same
 * sections, and the timeline peak of Sec. 2.1 / Sec. 3.1) when out_detail is not
 * NULL; out_peaks may be NULL when out_detail is given.                        */
int llmem_estimate_ex(const llmem_configs *cfg, int64_t n, const llmem_tables *method_tables,
                      int64_t *out_peaks, int64_t *out_detail, void *hip_stream);

/* m_peak of all four methods for n configurations: out_peaks[m * n + i] for m = 0..3 is
 * m_peak^s, m_peak^dp, m_peak^tp (Sec. 4.2, Sec. 5) and m_peak^{dp+tp} = m_peak^dp -
 * m_p16 * tp_n / gpu_n + m_back^tp (Sec. 5, "Combination of DP+TP"), where m_peak^dp is taken
 * over all gpu_n = cfg.d GPUs, the division is the same ceiling-then-block rule as everywhere
 * and m_back^tp is the buffer of a tensor-parallel group of tp_n GPUs.
 *   cfg        as for llmem_estimate; the method column is not read
 *   tp_n       DEV, n uint8: tensor-parallel degree of the DP+TP set-up; 0 = none (that
 *              estimate is -1); NULL = none anywhere; otherwise it must divide gpu_n
 *              (else LLMEM_F_ERR_TP: all four estimates -1)
 *   out_peaks  DEV, 4 * n int64
 *   out_flags  DEV, n int64 of LLMEM_F_* bits, or NULL
 * The closed forms only: no timeline is walked.                                           */
int llmem_estimate_methods(const llmem_configs *cfg, const uint8_t *tp_n, int64_t n,
                           const llmem_tables *method_tables, int64_t *out_peaks, int64_t *out_flags,
                           void *hip_stream);

/* Decision columns: out_detail of llmem_decide is DEV, LLMEM_NDECIDE columns of n int64 each
 * (column c of query i at out_detail[c * n + i]).  Scores are stored doubled so that CDP's
 * factor 1.5 stays an integer.                                                            */
enum llmem_decision {
    LLMEM_C_METHOD = 0,     /* LLMEM_METHOD_* chosen (0..4); -1 for an invalid query        */
    LLMEM_C_BS,             /* its batch size (0 with LLMEM_METHOD_OFFLOAD)                 */
    LLMEM_C_BS_CDP, LLMEM_C_BS_ADP, LLMEM_C_BS_TP, LLMEM_C_BS_HYBRID,     /* bs_list       */
    LLMEM_C_SCORE2_CDP, LLMEM_C_SCORE2_ADP, LLMEM_C_SCORE2_TP, LLMEM_C_SCORE2_HYBRID, /* 2 * eval */
    LLMEM_C_PEAK,           /* the chosen method's estimate at the chosen batch size        */
    LLMEM_C_FLAGS,          /* LLMEM_F_* bits                                               */
    LLMEM_NDECIDE
};

/* Algorithm 1 (Sec. 6) for n queries (model, gpu_n, sl): for CDP, ADP (ZeRO-3), TP and DP+TP
 * the largest batch size whose estimate does not exceed m_total; eval = bs * gpu_n * 1.5,
 * bs * gpu_n, bs, bs * dp_n (dp_n = gpu_n / tp_n); the first highest score wins (ties in the
 * order CDP, ADP, TP, DP+TP) unless the TP score is 0, which selects LLMEM_METHOD_OFFLOAD with
 * batch size 0.  A method that does not fit even at bs = 1 has batch size and score 0.  The
 * batch sizes are found by bisection inside a bracket derived from the estimates' linear growth
 * with bs, which equals the algorithm's one-by-one search because the estimates never decrease
 * with bs.
 *   queries    configurations whose bs column holds the largest batch size to consider and
 *              whose method column is not read; d = gpu_n
 *   tp_n       as for llmem_estimate_methods; 0 / NULL: DP+TP takes no part (score 0)
 *   m_total    GPU memory capacity in bytes
 *   out_method DEV, n int32 (LLMEM_C_METHOD), out_bs DEV, n int32 (LLMEM_C_BS); either may
 *              be NULL when out_detail is given
 *   out_detail DEV, LLMEM_NDECIDE * n int64, or NULL
 * Invalid queries: method -1, all other columns 0 except the flags.  LLMEM_EINVAL_TABLE also
 * when a parameter entry's size refers to LLMEM_DIM_BS.  Intermediate values at the largest
 * batch size considered must fit int64.                                                   */
int llmem_decide(const llmem_configs *queries, const uint8_t *tp_n, int64_t n,
                 const llmem_tables *method_tables, int64_t m_total, int32_t *out_method,
                 int32_t *out_bs, int64_t *out_detail, void *hip_stream);

/* Peaks of explicit allocator timelines (Sec. 2.1 / Sec. 3.1: sequential
 * traversal with live tensors, sizes rounded to 512-byte blocks).
 *   events   DEV, signed raw byte counts: > 0 allocation, < 0 release, 0 no-op
 *   offsets  DEV, n + 1 ascending offsets; list i is events[offsets[i] .. offsets[i+1])
 *   out_allocated DEV n int64: max over prefixes of the live rounded bytes
 *   out_reserved  DEV n int64: two pools split at LLMEM_POOL_SPLIT of rounded size
 *                 (a release goes to the pool of its own size); each pool's largest
 *                 live total rounded up to LLMEM_SEGMENT, summed
 * The empty prefix counts, so both outputs are >= 0.                          */
int llmem_timeline_peaks(const int64_t *events, const int64_t *offsets, int64_t n,
                         int64_t *out_allocated, int64_t *out_reserved, void *hip_stream);

#define LLMEM_BLOCK      512
#define LLMEM_POOL_SPLIT (2 * 1024 * 1024)
#define LLMEM_SEGMENT    (2 * 1024 * 1024)

/* Seeded synthetic inputs, generated on the device.  Every draw is
 * lo + mix64(seed, index, field) mod span with splitmix64's finaliser over
 * seed + 0x9E3779B97F4A7C15*(index+1) + 0xD1B54A32D192ED03*(field+1).
 * grid_id 1..4: the tiny Cartesian grid (432 configurations), the OPT/GPT-style
 * grid, the Llama-style grid, and the Llama-style grid with chunk search.
 * cfg_out columns are DEV arrays of n values receiving configurations
 * first .. first+n-1 (grid 1: first + n <= 432, else LLMEM_EINVAL_ARG).       */
int llmem_grid_generate(int grid_id, uint64_t seed, int64_t first, int64_t n,
                        const llmem_configs *cfg_out, void *hip_stream);

/* Queries first .. first+n-1 of the decision grid: the model shapes and sequence lengths of
 * grid 4, gpu_n in {1, 2, 4, 8, 16} in column d, tp_n = 2^j with j uniform in [0, log2 gpu_n]
 * in tp_n_out (DEV, n uint8), LLMEM_QUERY_BS_CAP in column bs.                            */
#define LLMEM_QUERY_BS_CAP 4096
int llmem_queries_generate(uint64_t seed, int64_t first, int64_t n, const llmem_configs *cfg_out,
                           uint8_t *tp_n_out, void *hip_stream);

/* Sweep of a seeded grid without storing a configuration or an estimate: each
 * configuration first .. first+n-1 of grid grid_id (1..4, as for llmem_grid_generate) is drawn in
 * registers, estimated exactly as llmem_estimate_ex does (closed forms of Sec. 4.2 and Sec. 5,
 * chunk search of Sec. 4.1, timeline of Sec. 2.1 / Sec. 3.1) and folded into statistics per
 * group = method * 16 + (gpu_n - 1), the questions Algorithm 1 (Sec. 6) asks of one
 * configuration asked of the whole grid.  stats is DEV, LLMEM_NSWEEP columns of
 * LLMEM_SWEEP_GROUPS int64 (column c of group g at stats[c * LLMEM_SWEEP_GROUPS + g]).
 * llmem_sweep ADDS to what stats holds (counts are added, extremes combined), so that the
 * statistics of several index ranges, seeds or devices can share one array or be merged
 * column by column afterwards; llmem_sweep_reset writes the empty statistics (0 everywhere,
 * INT64_MAX in LLMEM_S_MIN_PEAK).  Both are asynchronous on hip_stream; neither allocates.
 * Runs a lane form (LLMEM_KERNEL_LANE_*; LLMEM_KERNEL_WAVE is LLMEM_EINVAL_TABLE here);
 * first + n <= 2^40, else LLMEM_EINVAL_ARG.                                               */
#define LLMEM_SWEEP_GROUPS 48
enum llmem_sweep_column {
    LLMEM_S_COUNT = 0,          /* configurations of the group                                 */
    LLMEM_S_FIT,                /* those with m_peak <= m_total                                */
    LLMEM_S_MAX_PEAK,           /* largest m_peak                                              */
    LLMEM_S_MIN_PEAK,           /* smallest m_peak (INT64_MAX: the group is empty)             */
    LLMEM_S_MAX_LIVE,           /* largest timeline peak (LLMEM_D_PEAK_LIVE)                   */
    LLMEM_S_BEST,               /* best-scoring configuration that fits: score2 << 40 |
                                 * (2^40 - 1 - index); score2 is Algorithm 1's score doubled,
                                 * 3 * bs * gpu_n (CDP), 2 * bs * gpu_n (ZeRO-3), 2 * bs (TP);
                                 * equal scores: the lowest index; 0: nothing fits             */
    LLMEM_S_K_SUM,              /* sum of the chunk exponents used (LLMEM_D_K)                 */
    LLMEM_S_MAX_NPARAMS_FIT,    /* largest parameter count among those that fit                */
    LLMEM_NSWEEP
};
int llmem_sweep_reset(int64_t *stats, void *hip_stream);
int llmem_sweep(int grid_id, uint64_t seed, int64_t first, int64_t n, const llmem_tables *method_tables,
                int64_t m_total, int64_t *stats, void *hip_stream);

/* Event lists of configurations first .. first+n-1 of the explicit-timeline
 * grid.  Two steps, both asynchronous: llmem_events_count writes the n list
 * lengths (DEV int64); the caller turns them into n + 1 offsets (exclusive
 * prefix sum) and passes those to llmem_events_generate, which fills
 * events[offsets[i] .. offsets[i+1]).                                         */
int llmem_events_count(uint64_t seed, int64_t first, int64_t n, int64_t *counts, void *hip_stream);
int llmem_events_generate(uint64_t seed, int64_t first, int64_t n, const int64_t *offsets,
                          int64_t *events, void *hip_stream);

/* Bytes of device memory n configurations occupy over all 14 columns. */
size_t llmem_config_bytes(int64_t n);
/* Upper bound of the bytes of n event lists (events only, not the offsets). */
size_t llmem_events_bytes(int64_t n);

/* Host-only: which kernel forms these tables allow and what they cost.  info[0] = bit mask
 * (bit k set: LLMEM_KERNEL_k is allowed, k = 1..7; LLMEM_FORMS_PREBUILT_*: the library holds a
 * built-in specialization for these tables, for m_peak only / with the detail columns / for
 * llmem_sweep), info[1] = 32-bit words of the compiled
 * tables (of LLMEM_PROGRAM_WORDS available), info[2] = value slots per wavefront in the
 * compiled form, info[3] = value slots per wavefront in the events form, info[4] = LDS slots
 * of the wavefront-per-configuration form; when the compiled form is allowed also info[5] =
 * parameter groups | size classes << 16, info[6] = (class, count) terms, info[7] = peak points
 * kept, summed over the architectures (else 0).  Returns LLMEM_OK or the error the estimator
 * would return for these tables.                                                          */
#define LLMEM_PROGRAM_WORDS 704
#define LLMEM_FORMS_PREBUILT_PEAKS  (1 << 8)
#define LLMEM_FORMS_PREBUILT_DETAIL (1 << 9)
#define LLMEM_FORMS_PREBUILT_SWEEP  (1 << 10)
int llmem_kernel_forms(const llmem_tables *method_tables, int32_t info[8]);

/* Host-only: the compiled form of these tables, the 32-bit words a specialized kernel holds as
 * constants (parameter groups, size classes, peak points and net changes of the timeline
 * segments of every architecture; the library's build step makes its built-in specializations
 * from them, and a built-in one is used when a call's tables compile to the same words).
 *   words      HOST, room for max_words values
 *   first      HOST, LLMEM_MAX_ARCH values: the first word of each architecture (0 beyond n_arch)
 * Returns the number of words (>= 0), LLMEM_EINVAL_ARG if max_words is too small,
 * LLMEM_EINVAL_TABLE if the tables do not admit the compiled form, or the estimator's error
 * for these tables.  The device pointers of method_tables are not dereferenced.            */
int llmem_compiled_tables(const llmem_tables *method_tables, uint32_t *words, int32_t max_words,
                          int32_t first[LLMEM_MAX_ARCH]);

/* Host-only diagnostic, not part of the estimator: floor(x / d) computed by the
 * multiply-high constants the kernels use for their divisions by the partition degree
 * (0 <= x < 2^63, 1 <= d <= 255; returns 0 for d outside that range).  Lets a host test
 * compare the constants with integer division without a GPU.                              */
uint64_t llmem_selftest_divide(uint64_t x, uint32_t d);

/* Unloads every kernel that was built at run time (LLMEM_KERNEL_LANE_SPECIALIZED without a
 * built-in match, LLMEM_KERNEL_LANE_RUNTIME) and frees the host and device memory of its code
 * object: for a process that goes through many table sets.  Built-in kernels are not
 * affected.  Every device that has such kernels is synchronized first (launches still pending
 * there have ended before their code goes), so the call may block and must not be made while a
 * stream is being captured.  A kernel that a call of another thread holds at that moment (being
 * built, or found and about to be launched) is left alone.  A later call with the same tables
 * builds again (or loads from LLMEM_KERNEL_CACHE).  Returns the number of kernels released; 0 -
 * and no device call - when there are none.                                                  */
int llmem_kernels_release(void);

const char *llmem_strerror(int code);
int llmem_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LLMEM_H */
