/*
 * TEST INFRASTRUCTURE ONLY - part of the CPU oracle, not of the product.
 *
 * Byte execution of a broadcast schedule on the host, the rows of a step spread
 * over the host's cores.  The schedule itself (which rank sends which extent to
 * which rank in which step) is computed by the Python oracle and handed over as
 * plain arrays; this file only copies bytes, so that the benchmark can set an
 * all-cores CPU figure beside the GPU's.
 *
 * A row means: copy `len` bytes at offset `off` from rank `src`'s buffer to the
 * same offset in rank `dst`'s buffer [Sec. IV, listing: a send and its matching
 * receive use the same displacement].  All rows of a step read the state from
 * before the step [Sec. III-A: the exchanges of a step happen together]; steps
 * run in order.
 *
 *   staged != 0  literal form: every payload of the step is first copied aside,
 *                then every payload is delivered (what the Python oracle does).
 *   staged == 0  direct form: one memcpy per row.  Equal to the literal form
 *                whenever no row of a step reads bytes another row of the same
 *                step writes; oracle_rows_independent() checks exactly that.
 *
 * Returns 0, or -1 for bad arguments / failed allocation.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <omp.h>

int oracle_run_rows(uint8_t *const *bufs, int64_t n_steps, const uint64_t *step_ptr,
                    const uint32_t *src, const uint32_t *dst, const uint64_t *off,
                    const uint64_t *len, int staged, int threads)
{
    if (!bufs || !step_ptr || n_steps < 0 || threads < 1) return -1;
    uint8_t *stage = NULL;
    uint64_t *at = NULL;
    if (staged) {
        uint64_t most = 0, most_rows = 0;
        for (int64_t s = 0; s < n_steps; ++s) {
            uint64_t b = 0;
            for (uint64_t k = step_ptr[s]; k < step_ptr[s + 1]; ++k) b += len[k];
            if (b > most) most = b;
            if (step_ptr[s + 1] - step_ptr[s] > most_rows) most_rows = step_ptr[s + 1] - step_ptr[s];
        }
        stage = (uint8_t *)malloc(most ? most : 1);
        at = (uint64_t *)malloc(sizeof(uint64_t) * (most_rows ? most_rows : 1));
        if (!stage || !at) { free(stage); free(at); return -1; }
    }
    for (int64_t s = 0; s < n_steps; ++s) {
        const int64_t a = (int64_t)step_ptr[s], b = (int64_t)step_ptr[s + 1];
        if (staged) {
            uint64_t run = 0;
            for (int64_t k = a; k < b; ++k) { at[k - a] = run; run += len[k]; }
#pragma omp parallel for schedule(static) num_threads(threads)
            for (int64_t k = a; k < b; ++k) memcpy(stage + at[k - a], bufs[src[k]] + off[k], len[k]);
#pragma omp parallel for schedule(static) num_threads(threads)
            for (int64_t k = a; k < b; ++k) memcpy(bufs[dst[k]] + off[k], stage + at[k - a], len[k]);
        } else {
#pragma omp parallel for schedule(static) num_threads(threads)
            for (int64_t k = a; k < b; ++k) memcpy(bufs[dst[k]] + off[k], bufs[src[k]] + off[k], len[k]);
        }
    }
    free(stage);
    free(at);
    return 0;
}

/* 1 if in every step no row's source extent overlaps another row's destination
 * extent in the same buffer (and no two rows write overlapping extents of one
 * buffer), 0 if some pair does, -1 for bad arguments.  Quadratic in the rows of
 * a step: for checks, not for timing. */
int oracle_rows_independent(int64_t n_steps, const uint64_t *step_ptr, const uint32_t *src,
                            const uint32_t *dst, const uint64_t *off, const uint64_t *len)
{
    if (!step_ptr || n_steps < 0) return -1;
    for (int64_t s = 0; s < n_steps; ++s)
        for (uint64_t i = step_ptr[s]; i < step_ptr[s + 1]; ++i)
            for (uint64_t j = step_ptr[s]; j < step_ptr[s + 1]; ++j) {
                if (i == j || len[i] == 0 || len[j] == 0) continue;
                const int overlap = off[i] < off[j] + len[j] && off[j] < off[i] + len[i];
                if (overlap && (src[i] == dst[j] || (dst[i] == dst[j] && i < j))) return 0;
            }
    return 1;
}

int oracle_host_threads(void) { return omp_get_max_threads(); }
