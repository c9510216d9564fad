/* Seeded allocator event lists for the explicit-timeline workload.
 *
 * One configuration = one training iteration written as signed raw byte counts
 * (+ allocation, - release), about 10^4 events.  The shape follows what the paper
 * describes for a graph traversal with live tensors (Sec. 2.1 and Sec. 3.1):
 * forward operators whose outputs are transient or saved for the backward, a
 * backward pass that walks the saved tensors in reverse producing gradients, and
 * an optimizer phase with short-lived temporaries.  Sizes are log-uniform in
 * [2^5, 2^28) bytes and deliberately not multiples of the allocator block.
 *
 * This file holds no estimator arithmetic: no rounding, no pools, no peaks.
 * Every draw is  mix64(seed, index, field)  with the same mixer as the
 * configuration grids; index = config * 8192 + op  for per-operator draws.
 */
#include <stdint.h>
#include <stddef.h>

static uint64_t mix64(uint64_t seed, uint64_t index, uint64_t field)
{
    uint64_t x = seed + 0x9E3779B97F4A7C15ull * (index + 1) + 0xD1B54A32D192ED03ull * (field + 1);
    x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27; x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

enum { F_NFWD = 100, F_EXP = 101, F_MANT = 102, F_SAVED = 103 };
enum { NFWD_LO = 2800, NFWD_SPAN = 651, OPS_STRIDE = 8192 };

static int64_t n_forward(uint64_t seed, int64_t c)
{
    return NFWD_LO + (int64_t)(mix64(seed, (uint64_t)c, F_NFWD) % NFWD_SPAN);
}
static int64_t op_size(uint64_t seed, int64_t c, int64_t j)
{
    uint64_t idx = (uint64_t)c * OPS_STRIDE + (uint64_t)j;
    unsigned e = 5 + (unsigned)(mix64(seed, idx, F_EXP) % 23);
    return (int64_t)((1ull << e) + (mix64(seed, idx, F_MANT) & ((1ull << e) - 1)));
}
static int op_saved(uint64_t seed, int64_t c, int64_t j)
{
    uint64_t idx = (uint64_t)c * OPS_STRIDE + (uint64_t)j;
    return (mix64(seed, idx, F_SAVED) % 10) < 3;
}

/* counts[i] = number of events of configuration first + i */
void llmem_events_count(uint64_t seed, int64_t first, int64_t n, int64_t *counts, int threads)
{
    (void)threads;
    #pragma omp parallel for schedule(static) num_threads(threads > 0 ? threads : 1)
    for (int64_t i = 0; i < n; ++i) {
        int64_t c = first + i, nf = n_forward(seed, c), ns = 0;
        for (int64_t j = 0; j < nf; ++j) ns += op_saved(seed, c, j);
        counts[i] = 2 * nf + 4 * ns;
    }
}

/* events[offsets[i] .. offsets[i+1]) = the list of configuration first + i */
void llmem_events_fill(uint64_t seed, int64_t first, int64_t n, const int64_t *offsets,
                       int64_t *events, int threads)
{
    (void)threads;
    #pragma omp parallel for schedule(static) num_threads(threads > 0 ? threads : 1)
    for (int64_t i = 0; i < n; ++i) {
        int64_t c = first + i, nf = n_forward(seed, c);
        int64_t *out = events + offsets[i];
        /* forward: allocate each output; a transient output dies after the next allocation */
        for (int64_t j = 0; j < nf; ++j) {
            *out++ = op_size(seed, c, j);
            if (j > 0 && !op_saved(seed, c, j - 1)) *out++ = -op_size(seed, c, j - 1);
        }
        if (!op_saved(seed, c, nf - 1)) *out++ = -op_size(seed, c, nf - 1);
        /* backward over the saved tensors in reverse: gradient, drop saved, drop previous gradient */
        int64_t prev = 0;
        for (int64_t j = nf - 1; j >= 0; --j) {
            if (!op_saved(seed, c, j)) continue;
            int64_t s = op_size(seed, c, j);
            *out++ = s; *out++ = -s;
            if (prev) *out++ = -prev;
            prev = s;
        }
        if (prev) *out++ = -prev;
        /* optimizer: one short-lived temporary per saved tensor */
        for (int64_t j = 0; j < nf; ++j) {
            if (!op_saved(seed, c, j)) continue;
            int64_t s = op_size(seed, c, j);
            *out++ = s; *out++ = -s;
        }
    }
}
