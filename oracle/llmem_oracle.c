/* CPU oracle B: the peak-GPU-memory estimator in plain C, int64 with 128-bit
 * overflow checks.
 *
 * TEST INFRASTRUCTURE ONLY: the parity tests, the smoke check and the benchmark's
 * CPU-baseline leg call this; the product never does, and this file shares no
 * code, header or table with the HIP path.  It restates oracle A
 * (llmem_oracle.py) for speed; the two are compared on whole grids by the tests,
 * and oracle A carries the pins against the paper.
 *
 * Passages followed (same as oracle A):
 *   Sec. 4.2  m_peak^s, m_p, m_os, m_out, m_lm
 *   Sec. 5    m_peak^dp (ZeRO-3), m_peak^tp, m_back^tp
 *   Sec. 4.1  chunk size chosen to minimise waste (search over 2^k MiB, k = 2..10)
 *   Sec. 2.1 / Sec. 3.1  timeline traversal with live tensors, 512-byte blocks
 *   Sec. 5    m_peak^{dp+tp}
 *   Sec. 6    Algorithm 1 (largest batch size per method, scores, choice)
 *   Sec. 6    the statistics of a whole grid per (method, gpu_n): llmem_oracle_sweep
 *
 * The timeline is walked event by event, block by block; no closed form over the
 * L equal blocks is used here.
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>

typedef __int128 i128;

enum { B16 = 2, B32 = 4 };
enum { NDIM = 15 };
enum { DIM_ONE, DIM_BS, DIM_SL, DIM_SLM1, DIM_H, DIM_FFN, DIM_NHEADS, DIM_NKV, DIM_HEADDIM,
       DIM_KVDIM, DIM_V, DIM_P, DIM_L, DIM_BLOGITS, DIM_D };
enum { CLS_E, CLS_L, CLS_B, CLS_N };
enum { ROLE_EMBED_TOK, ROLE_LM_HEAD, ROLE_OTHER };
enum { SEG_A, SEG_F, SEG_H, SEG_B, SEG_Z, NSEG };
enum { NDETAIL = 12 };
enum { D_PEAK, D_PARAM, D_GRAD, D_OS, D_OUT, D_LM, D_BACK, D_K, D_LIVE, D_NPARAMS, D_TMAX, D_FLAGS };
enum { ERR_ARCH = 1, ERR_METHOD = 2, ERR_D = 4, ERR_HEADS = 8, ERR_CHUNK = 16, CHUNK_INFEASIBLE = 32,
       ERR_TP = 64, HYBRID_READINGS_DIFFER = 128, FALLBACK_READINGS_DIFFER = 256 };
enum { NDECIDE = 12 };
enum { C_METHOD, C_BS, C_BS_LIST, C_SCORE2 = C_BS_LIST + 4, C_PEAK = C_SCORE2 + 4, C_FLAGS };
enum { CFG_LOGITS_FP32 = 1, CFG_TIED = 2, CFG_GRAD_ALIAS = 4 };
enum { K_MIN = 2, K_MAX = 10, K_FIXED_MAX = 16 };

typedef struct {
    int64_t coef;
    int32_t ndims, dims[4];
    int32_t cls, role, per_layer;
} o_param;

typedef struct {
    int64_t coef;
    int32_t ndims, dims[4];
    int32_t elem_bytes, seg, sign, method_mask, scale, times_L;
} o_event;

typedef struct {
    int32_t n_params, n_events;
    const o_param *params;
    const o_event *events;
} o_table;

typedef struct {
    const uint8_t *arch_id; const uint32_t *h; const uint16_t *L; const uint16_t *n_heads;
    const uint16_t *n_kv; const uint32_t *ffn; const uint32_t *V; const uint32_t *P;
    const uint16_t *bs; const uint16_t *sl; const uint8_t *method; const uint8_t *d;
    const int8_t *chunk_k; const uint8_t *flags;
} o_configs;

/* every intermediate goes through fit(): overflow of int64 is recorded, not ignored */
static int64_t fit(i128 v, int *ovf)
{
    if (v > (i128)INT64_MAX || v < (i128)INT64_MIN) { *ovf = 1; return 0; }
    return (int64_t)v;
}
static int64_t cdiv(int64_t a, int64_t b) { return (int64_t)(((i128)a + b - 1) / b); }
static int64_t up(int64_t a, int64_t unit, int *ovf) { return fit((i128)cdiv(a, unit) * unit, ovf); }

static int64_t monomial(int64_t coef, int ndims, const int32_t *dims, const int64_t *D, int *ovf)
{
    int64_t x = coef;
    for (int j = 0; j < ndims; ++j) x = fit((i128)x * D[dims[j]], ovf);
    return x;
}

static int64_t chunk_elems(int k) { return ((int64_t)1 << k) * 1024 * 1024 / B16; }

static void param_memory(int64_t embed_p, int64_t other_p, int64_t cs, int64_t cu_p,
                         int64_t *m_p, int64_t *m_p16, int64_t *m_p32, int *ovf)
{
    int64_t chunked = fit((i128)embed_p + (i128)cdiv(other_p, cs) * cs, ovf);
    *m_p = up(fit((i128)chunked * (B16 + B32), ovf), cu_p, ovf);
    *m_p16 = up(fit((i128)chunked * B16, ovf), cu_p, ovf);
    *m_p32 = up(fit((i128)chunked * B32, ovf), cu_p, ovf);
}

static int64_t compose(int method, int64_t d, int64_t m_base, int64_t m_p, int64_t m_p16,
                       int64_t m_p32, int64_t m_os, int64_t m_out, int64_t m_lm, int64_t m_back,
                       int64_t align, int *ovf)
{
    if (method == 0) return fit((i128)m_base + m_p + m_os + m_out + m_lm, ovf);
    if (method == 1)
        return fit((i128)m_base + m_p16 + up(cdiv(fit((i128)m_p32 + m_os, ovf), d), align, ovf)
                   + m_out + m_lm, ovf);
    return fit((i128)m_base + up(cdiv(fit((i128)m_p + m_os, ovf), d), align, ovf)
               + m_out + m_lm + m_back, ovf);
}

static void estimate_one(const o_configs *c, int64_t i, const o_table *tables, int n_tables,
                         int64_t m_base, int64_t cu_p, int64_t align, int want_timeline,
                         int64_t *out, int64_t *scratch, int *ovf, int64_t *m_p16_out)
{
    for (int j = 0; j < NDETAIL; ++j) out[j] = 0;
    int err = 0;
    int method = c->method[i], k_in = c->chunk_k[i], cflags = c->flags[i];
    int64_t d = c->d[i];
    if (c->arch_id[i] >= n_tables) err |= ERR_ARCH;
    if (method > 2) err |= ERR_METHOD;
    if (d == 0) err |= ERR_D;
    if (c->n_heads[i] == 0) err |= ERR_HEADS;
    if (!(k_in == -1 || (k_in >= 0 && k_in <= K_FIXED_MAX))) err |= ERR_CHUNK;
    if (err) { out[D_PEAK] = -1; out[D_FLAGS] = err; return; }

    const o_table *t = &tables[c->arch_id[i]];
    int64_t D[NDIM];
    int64_t L = c->L[i], bs = c->bs[i], sl = c->sl[i], h = c->h[i], V = c->V[i];
    int64_t head_dim = h / c->n_heads[i];
    D[DIM_ONE] = 1; D[DIM_BS] = bs; D[DIM_SL] = sl; D[DIM_SLM1] = sl > 0 ? sl - 1 : 0;
    D[DIM_H] = h; D[DIM_FFN] = c->ffn[i]; D[DIM_NHEADS] = c->n_heads[i]; D[DIM_NKV] = c->n_kv[i];
    D[DIM_HEADDIM] = head_dim; D[DIM_KVDIM] = (int64_t)c->n_kv[i] * head_dim; D[DIM_V] = V;
    D[DIM_P] = c->P[i]; D[DIM_L] = L; D[DIM_BLOGITS] = (cflags & CFG_LOGITS_FP32) ? B32 : B16;
    D[DIM_D] = d;

    /* Notation table: embed_p, lm_p, other_p; Sec. 4.2: m_os summed tensor by tensor */
    int64_t embed_p = 0, lm_p = 0, other_p = 0, t_max = 0, e_n = 0, m_os = 0;
    for (int j = 0; j < t->n_params; ++j) {
        const o_param *p = &t->params[j];
        int64_t t_p = monomial(p->coef, p->ndims, p->dims, D, ovf);
        int64_t count = p->per_layer ? L : 1;
        if (p->role == ROLE_EMBED_TOK) embed_p = fit((i128)embed_p + (i128)t_p * count, ovf);
        else if (p->role == ROLE_LM_HEAD) lm_p = fit((i128)lm_p + (i128)t_p * count, ovf);
        else {
            other_p = fit((i128)other_p + (i128)t_p * count, ovf);
            if (t_p > t_max) t_max = t_p;
        }
        if (p->cls == CLS_E && p->role != ROLE_LM_HEAD) e_n += 1;
        if ((p->cls == CLS_E || p->cls == CLS_L) && p->role != ROLE_LM_HEAD) {
            int64_t one = up(fit((i128)t_p * (B32 + B32), ovf), cu_p, ovf);
            for (int64_t l = 0; l < count; ++l) m_os = fit((i128)m_os + one, ovf);
        }
    }
    int64_t n_params = fit((i128)embed_p + other_p + ((cflags & CFG_TIED) ? 0 : lm_p), ovf);

    /* Sec. 4.2: m_out, m_lm; Sec. 5: m_back^tp */
    int64_t A = fit((i128)bs * sl * h, ovf);
    int64_t m_out = up(fit((i128)(e_n + L) * A * B16, ovf), cu_p, ovf);
    int64_t B = D[DIM_BLOGITS];
    int64_t m_lm = fit((i128)up(fit((i128)bs * sl * V * B, ovf), cu_p, ovf)
                       + 2 * (i128)up(fit((i128)bs * D[DIM_SLM1] * V * B, ovf), cu_p, ovf)
                       + (i128)lm_p * B16, ovf);
    int64_t m_back = 0;
    if (method == 2)
        m_back = fit((i128)cdiv(fit((i128)L * A * (d - 1) * B16, ovf), d * cu_p) * cu_p, ovf);

    /* Sec. 4.1: gradient fp16 aliases param fp16 unless switched off */
    int64_t trainable = fit((i128)embed_p + other_p, ovf);
    int64_t grad_bytes = fit((i128)trainable * B16, ovf);
    int64_t grad_logical = method == 0 ? grad_bytes : cdiv(grad_bytes, d);
    int64_t grad_extra = 0;
    if (!(cflags & CFG_GRAD_ALIAS))
        grad_extra = method == 0 ? up(grad_bytes, cu_p, ovf)
                                 : up(cdiv(up(grad_bytes, cu_p, ovf), d), align, ovf);

    /* chunk size: given, or searched over 2^k MiB (every candidate is estimated) */
    int k = k_in;
    int64_t m_p = 0, m_p16 = 0, m_p32 = 0, m_peak = 0;
    if (k_in == -1) {
        int best_k = -1; int64_t best_waste = 0;
        int64_t cand_peak[K_MAX + 1], cand_p[K_MAX + 1], cand_p16[K_MAX + 1], cand_p32[K_MAX + 1];
        for (int kk = K_MIN; kk <= K_MAX; ++kk) {
            int64_t cs = chunk_elems(kk);
            param_memory(embed_p, other_p, cs, cu_p, &cand_p[kk], &cand_p16[kk], &cand_p32[kk], ovf);
            cand_peak[kk] = fit((i128)compose(method, d, m_base, cand_p[kk], cand_p16[kk], cand_p32[kk],
                                              m_os, m_out, m_lm, m_back, align, ovf) + grad_extra, ovf);
            if (t_max > cs) continue;
            int64_t waste = fit((i128)cdiv(other_p, cs) * cs - other_p, ovf);
            if (best_k < 0 || waste < best_waste) { best_k = kk; best_waste = waste; }
        }
        k = best_k < 0 ? K_MAX : best_k;
        m_peak = cand_peak[k]; m_p = cand_p[k]; m_p16 = cand_p16[k]; m_p32 = cand_p32[k];
    } else {
        param_memory(embed_p, other_p, chunk_elems(k), cu_p, &m_p, &m_p16, &m_p32, ovf);
        m_peak = fit((i128)compose(method, d, m_base, m_p, m_p16, m_p32, m_os, m_out, m_lm, m_back,
                                   align, ovf) + grad_extra, ovf);
    }
    int flags = t_max > chunk_elems(k) ? CHUNK_INFEASIBLE : 0;
    if (m_p16_out) *m_p16_out = m_p16;

    int64_t param_gpu, os_gpu;
    if (method == 0) { param_gpu = m_p; os_gpu = m_os; }
    else if (method == 1) {
        param_gpu = fit((i128)m_p16 + up(cdiv(m_p32, d), align, ovf), ovf);
        os_gpu = up(cdiv(m_os, d), align, ovf);
    } else {
        param_gpu = up(cdiv(m_p, d), align, ovf);
        os_gpu = up(cdiv(m_os, d), align, ovf);
    }

    int64_t peak_live = 0;
    if (want_timeline) {
        /* value of every table event under this configuration ... */
        int seg_first[NSEG + 1];
        for (int s = 0, j = 0; s < NSEG; ++s) {          /* table events are grouped by segment */
            while (j < t->n_events && t->events[j].seg < s) ++j;
            seg_first[s] = j;
        }
        seg_first[NSEG] = t->n_events;
        for (int j = 0; j < t->n_events; ++j) {
            const o_event *e = &t->events[j];
            int64_t v = 0;
            if (e->method_mask & (1 << method)) {
                int64_t raw = fit((i128)monomial(e->coef, e->ndims, e->dims, D, ovf) * e->elem_bytes, ovf);
                if (e->scale == 1) raw = cdiv(fit((i128)raw * (d - 1), ovf), d);
                v = up(raw, align, ovf);
                if (e->times_L) v = fit((i128)v * L, ovf);
                v *= e->sign;
            }
            scratch[j] = v;
        }
        /* ... then the walk: resident state, A, F x L, H, B x L, Z */
        int64_t live = fit((i128)m_base + param_gpu + os_gpu + (i128)lm_p * B16 + grad_extra, ovf);
        int64_t peak = live;
        for (int s = 0; s < NSEG; ++s) {
            int64_t reps = (s == SEG_F || s == SEG_B) ? L : 1;
            for (int64_t r = 0; r < reps; ++r)
                for (int j = seg_first[s]; j < seg_first[s + 1]; ++j) {
                    live = fit((i128)live + scratch[j], ovf);
                    if (live > peak) peak = live;
                }
        }
        peak_live = peak;
    }

    out[D_PEAK] = m_peak; out[D_PARAM] = param_gpu; out[D_GRAD] = grad_logical; out[D_OS] = os_gpu;
    out[D_OUT] = m_out; out[D_LM] = m_lm; out[D_BACK] = m_back; out[D_K] = k; out[D_LIVE] = peak_live;
    out[D_NPARAMS] = n_params; out[D_TMAX] = t_max; out[D_FLAGS] = flags;
}

/* detail: n rows of NDETAIL int64 (row-major), may be NULL; peaks: n int64, may be NULL.
 * Returns 0, or 1 if any intermediate overflowed int64 (results then meaningless),
 * or 2 on a malformed table (segments out of order, selector out of range). */
int llmem_oracle_estimate(const o_configs *cfg, int64_t n, const o_table *tables, int n_tables,
                          int64_t m_base, int64_t cu_p, int64_t align, int want_timeline,
                          int64_t *peaks, int64_t *detail, int threads)
{
    int max_events = 0;
    for (int a = 0; a < n_tables; ++a) {
        const o_table *t = &tables[a];
        if (t->n_events > max_events) max_events = t->n_events;
        for (int j = 0; j < t->n_events; ++j) {
            const o_event *e = &t->events[j];
            if (e->seg < 0 || e->seg >= NSEG || (j > 0 && e->seg < t->events[j - 1].seg)) return 2;
            for (int q = 0; q < e->ndims; ++q) if (e->dims[q] < 0 || e->dims[q] >= NDIM) return 2;
        }
        for (int j = 0; j < t->n_params; ++j)
            for (int q = 0; q < t->params[j].ndims; ++q)
                if (t->params[j].dims[q] < 0 || t->params[j].dims[q] >= NDIM) return 2;
    }
    int any_ovf = 0;
    #pragma omp parallel num_threads(threads > 0 ? threads : 1) reduction(|:any_ovf)
    {
        int64_t *scratch = (int64_t *)malloc(sizeof(int64_t) * (size_t)(max_events + 1));
        int ovf = 0;
        #pragma omp for schedule(dynamic, 256)
        for (int64_t i = 0; i < n; ++i) {
            int64_t row[NDETAIL];
            estimate_one(cfg, i, tables, n_tables, m_base, cu_p, align, want_timeline, row, scratch, &ovf, NULL);
            if (peaks) peaks[i] = row[D_PEAK];
            if (detail) for (int j = 0; j < NDETAIL; ++j) detail[i * NDETAIL + j] = row[j];
        }
        free(scratch);
        any_ovf |= ovf;
    }
    return any_ovf;
}

/* ---- DP+TP and the method decision ------------------------------------------------- */

/* One configuration given by value, so that method and batch size can be varied. */
typedef struct {
    uint8_t arch_id; uint32_t h; uint16_t L, n_heads, n_kv; uint32_t ffn, V, P; uint16_t bs, sl;
    uint8_t method, d; int8_t chunk_k; uint8_t flags;
} one_config;

static one_config pick(const o_configs *c, int64_t i)
{
    one_config q = { c->arch_id[i], c->h[i], c->L[i], c->n_heads[i], c->n_kv[i], c->ffn[i], c->V[i],
                     c->P[i], c->bs[i], c->sl[i], c->method[i], c->d[i], c->chunk_k[i], c->flags[i] };
    return q;
}

static void estimate_value(const one_config *q, const o_table *tables, int n_tables, int64_t m_base,
                           int64_t cu_p, int64_t align, int64_t *row, int *ovf, int64_t *m_p16)
{
    o_configs c = { &q->arch_id, &q->h, &q->L, &q->n_heads, &q->n_kv, &q->ffn, &q->V, &q->P, &q->bs,
                    &q->sl, &q->method, &q->d, &q->chunk_k, &q->flags };
    estimate_one(&c, 0, tables, n_tables, m_base, cu_p, align, 0, row, NULL, ovf, m_p16);
}

static int query_errors(const one_config *q, int tp_n, int n_tables)
{
    int err = 0;
    if (q->arch_id >= n_tables) err |= ERR_ARCH;
    if (q->d == 0) err |= ERR_D;
    if (q->n_heads == 0) err |= ERR_HEADS;
    if (!(q->chunk_k == -1 || (q->chunk_k >= 0 && q->chunk_k <= K_FIXED_MAX))) err |= ERR_CHUNK;
    if (tp_n > 0 && q->d > 0 && q->d % tp_n != 0) err |= ERR_TP;
    return err;
}

/* out[0..3] = m_peak^s, m_peak^dp, m_peak^tp, m_peak^{dp+tp}; out[4] = flags */
static void method_peaks(const one_config *q0, int tp_n, const o_table *tables, int n_tables,
                         int64_t m_base, int64_t cu_p, int64_t align, int64_t *out, int *ovf)
{
    int err = query_errors(q0, tp_n, n_tables);
    if (err) { out[0] = out[1] = out[2] = out[3] = -1; out[4] = err; return; }
    one_config q = *q0;
    int64_t row[NDETAIL], m_p16 = 0, flags = 0;
    for (int m = 0; m < 3; ++m) {
        q.method = (uint8_t)m;
        estimate_value(&q, tables, n_tables, m_base, cu_p, align, row, ovf, m == 1 ? &m_p16 : NULL);
        out[m] = row[D_PEAK];
        flags |= row[D_FLAGS];
    }
    if (tp_n > 0) {
        /* Sec. 5: m_peak^dp - m_p16 * tp_n / gpu_n + m_back^tp of a group of tp_n GPUs */
        int64_t gpu_n = q.d;
        int64_t printed = up(cdiv(fit((i128)m_p16 * tp_n, ovf), gpu_n), align, ovf);
        int64_t other = up(cdiv(fit((i128)m_p16 * (tp_n - 1), ovf), tp_n), align, ovf);
        int64_t A = fit((i128)q.bs * q.sl * q.h, ovf);
        int64_t m_back = fit((i128)cdiv(fit((i128)q.L * A * (tp_n - 1) * B16, ovf), (int64_t)tp_n * cu_p) * cu_p, ovf);
        out[3] = fit((i128)out[1] - printed + m_back, ovf);
        if (printed != other) flags |= HYBRID_READINGS_DIFFER;
    } else {
        out[3] = -1;
    }
    out[4] = flags;
}

/* peaks: n rows of 4 int64; flags: n int64.  Returns 0, 1 (overflow) or 2 (malformed table). */
int llmem_oracle_methods(const o_configs *cfg, const uint8_t *tp_n, int64_t n, const o_table *tables,
                         int n_tables, int64_t m_base, int64_t cu_p, int64_t align,
                         int64_t *peaks, int64_t *flags, int threads)
{
    int any_ovf = 0;
    #pragma omp parallel for schedule(dynamic, 256) num_threads(threads > 0 ? threads : 1) reduction(|:any_ovf)
    for (int64_t i = 0; i < n; ++i) {
        int ovf = 0;
        int64_t out[5];
        one_config q = pick(cfg, i);
        method_peaks(&q, tp_n[i], tables, n_tables, m_base, cu_p, align, out, &ovf);
        for (int j = 0; j < 4; ++j) peaks[i * 4 + j] = out[j];
        flags[i] = out[4];
        any_ovf |= ovf;
    }
    return any_ovf;
}

/* Algorithm 1 for n queries; rows: n rows of NDECIDE int64.  The batch size of a method is raised
 * one by one from 1 until its estimate exceeds m_total or the query's bs (the cap) is passed. */
int llmem_oracle_decide(const o_configs *cfg, const uint8_t *tp_n, int64_t n, const o_table *tables,
                        int n_tables, int64_t m_base, int64_t cu_p, int64_t align, int64_t m_total,
                        int64_t *rows, int threads)
{
    for (int a = 0; a < n_tables; ++a)
        for (int j = 0; j < tables[a].n_params; ++j)
            for (int q = 0; q < tables[a].params[j].ndims; ++q)
                if (tables[a].params[j].dims[q] == DIM_BS) return 2;     /* parameter sizes must not depend on bs */
    int any_ovf = 0;
    #pragma omp parallel for schedule(dynamic, 16) num_threads(threads > 0 ? threads : 1) reduction(|:any_ovf)
    for (int64_t i = 0; i < n; ++i) {
        int ovf = 0;
        int64_t *row = rows + i * NDECIDE;
        for (int j = 0; j < NDECIDE; ++j) row[j] = 0;
        one_config q = pick(cfg, i);
        int tp = tp_n[i];
        int err = query_errors(&q, tp, n_tables);
        if (err) { row[C_METHOD] = -1; row[C_FLAGS] = err; continue; }
        int64_t gpu_n = q.d, cap = q.bs, out[5];
        q.bs = 1;
        method_peaks(&q, tp, tables, n_tables, m_base, cu_p, align, out, &ovf);
        int64_t flags = out[4];
        int64_t bs_list[4] = {0, 0, 0, 0}, peak_at[4] = {0, 0, 0, 0};
        for (int m = 0; m < (tp > 0 ? 4 : 3); ++m) {
            int64_t bs = 1;
            while (bs <= cap) {
                q.bs = (uint16_t)bs;
                method_peaks(&q, tp, tables, n_tables, m_base, cu_p, align, out, &ovf);
                if (out[m] > m_total) break;
                peak_at[m] = out[m];
                ++bs;
            }
            bs_list[m] = bs - 1;
        }
        int64_t dp_n = tp > 0 ? gpu_n / tp : 0;
        int64_t score2[4] = { 3 * bs_list[0] * gpu_n, 2 * bs_list[1] * gpu_n, 2 * bs_list[2], 2 * bs_list[3] * dp_n };
        int idx = 0;
        for (int m = 1; m < 4; ++m) if (score2[m] > score2[idx]) idx = m;
        if (score2[2] != 0) {
            row[C_METHOD] = idx; row[C_BS] = bs_list[idx]; row[C_PEAK] = peak_at[idx];
        } else {
            row[C_METHOD] = 4; row[C_BS] = 0; row[C_PEAK] = 0;
            if (score2[0] | score2[1] | score2[3]) flags |= FALLBACK_READINGS_DIFFER;
        }
        for (int m = 0; m < 4; ++m) { row[C_BS_LIST + m] = bs_list[m]; row[C_SCORE2 + m] = score2[m]; }
        row[C_FLAGS] = flags;
        any_ovf |= ovf;
    }
    return any_ovf;
}

/* ---- sweep: statistics of estimated configurations per (method, gpu_n) ---------------- */

enum { SWEEP_D_MAX = 16, SWEEP_GROUPS = 48, NSWEEP = 8, SWEEP_INDEX_BITS = 40 };
enum { S_COUNT, S_FIT, S_MAX_PEAK, S_MIN_PEAK, S_MAX_LIVE, S_BEST, S_K_SUM, S_MAX_NPARAMS_FIT };

/* detail: the n rows that llmem_oracle_estimate wrote for cfg; configuration j has index
 * first + j in its grid.  stats: NSWEEP columns of SWEEP_GROUPS values, column-major
 * (stats[column * SWEEP_GROUPS + group]).  Returns 0, or 2 if an index does not fit 40 bits. */
int llmem_oracle_sweep(const o_configs *cfg, int64_t n, int64_t first, const int64_t *detail,
                       int64_t m_total, int64_t *stats)
{
    int64_t best_score[SWEEP_GROUPS], best_index[SWEEP_GROUPS];
    if (first < 0 || first + n > ((int64_t)1 << SWEEP_INDEX_BITS)) return 2;
    for (int q = 0; q < NSWEEP * SWEEP_GROUPS; ++q) stats[q] = 0;
    for (int g = 0; g < SWEEP_GROUPS; ++g) {
        stats[S_MIN_PEAK * SWEEP_GROUPS + g] = INT64_MAX;
        best_score[g] = -1;
        best_index[g] = 0;
    }
    for (int64_t j = 0; j < n; ++j) {
        const int64_t *row = detail + j * NDETAIL;
        const int method = cfg->method[j], d = cfg->d[j];
        const int err_mask = ERR_ARCH | ERR_METHOD | ERR_D | ERR_HEADS | ERR_CHUNK | ERR_TP;
        if (row[D_PEAK] < 0 || (row[D_FLAGS] & err_mask) || d > SWEEP_D_MAX) continue;
        const int g = method * SWEEP_D_MAX + (d - 1);
        int64_t *at = stats + g;
        at[S_COUNT * SWEEP_GROUPS] += 1;
        if (row[D_PEAK] > at[S_MAX_PEAK * SWEEP_GROUPS]) at[S_MAX_PEAK * SWEEP_GROUPS] = row[D_PEAK];
        if (row[D_PEAK] < at[S_MIN_PEAK * SWEEP_GROUPS]) at[S_MIN_PEAK * SWEEP_GROUPS] = row[D_PEAK];
        if (row[D_LIVE] > at[S_MAX_LIVE * SWEEP_GROUPS]) at[S_MAX_LIVE * SWEEP_GROUPS] = row[D_LIVE];
        at[S_K_SUM * SWEEP_GROUPS] += row[D_K];
        if (row[D_PEAK] > m_total) continue;
        at[S_FIT * SWEEP_GROUPS] += 1;
        if (row[D_NPARAMS] > at[S_MAX_NPARAMS_FIT * SWEEP_GROUPS]) at[S_MAX_NPARAMS_FIT * SWEEP_GROUPS] = row[D_NPARAMS];
        const int64_t bs = cfg->bs[j];
        const int64_t score2 = method == 0 ? 3 * bs * d : method == 1 ? 2 * bs * d : 2 * bs;
        if (score2 > best_score[g]) { best_score[g] = score2; best_index[g] = first + j; }   /* j ascends: ties keep the lower index */
    }
    for (int g = 0; g < SWEEP_GROUPS; ++g)
        if (best_score[g] >= 0)
            stats[S_BEST * SWEEP_GROUPS + g] = (best_score[g] << SWEEP_INDEX_BITS)
                                               | ((((int64_t)1 << SWEEP_INDEX_BITS) - 1) - best_index[g]);
    return 0;
}

/* Explicit event lists: signed raw sizes, CSR offsets.  512-byte blocks; two
 * pools split at 2 MiB of rounded size; reserved memory in 2 MiB segments. */
int llmem_oracle_event_lists(const int64_t *events, const int64_t *offsets, int64_t n,
                             int64_t *allocated, int64_t *reserved, int threads)
{
    const int64_t ALIGN = 512, SPLIT = 2 * 1024 * 1024, SEGMENT = 2 * 1024 * 1024;
    int any_ovf = 0;
    #pragma omp parallel for schedule(dynamic, 64) num_threads(threads > 0 ? threads : 1) reduction(|:any_ovf)
    for (int64_t i = 0; i < n; ++i) {
        int ovf = 0;
        int64_t live_s = 0, live_l = 0, peak_s = 0, peak_l = 0, peak_t = 0;
        for (int64_t e = offsets[i]; e < offsets[i + 1]; ++e) {
            int64_t raw = events[e];
            int64_t mag = raw >= 0 ? raw : fit(-(i128)raw, &ovf);
            int64_t r = up(mag, ALIGN, &ovf);
            int64_t delta = raw >= 0 ? r : -r;
            if (r < SPLIT) live_s = fit((i128)live_s + delta, &ovf);
            else live_l = fit((i128)live_l + delta, &ovf);
            if (live_s > peak_s) peak_s = live_s;
            if (live_l > peak_l) peak_l = live_l;
            int64_t tot = fit((i128)live_s + live_l, &ovf);
            if (tot > peak_t) peak_t = tot;
        }
        allocated[i] = peak_t;
        reserved[i] = fit((i128)up(peak_s, SEGMENT, &ovf) + up(peak_l, SEGMENT, &ovf), &ovf);
        any_ovf |= ovf;
    }
    return any_ovf;
}
