/* Host build of the counter-based row generator (see synth_core.h). */
#include "synth_core.h"

/* rows[count][2][d] for flattened pairs first .. first+count-1 (host memory). */
int synth_fill_pairs_host(const synth_params *p, int64_t first_pair, int64_t count, float *rows) {
    if (!p || !rows || first_pair < 0 || count < 0) return -1;
    uint64_t sm = syn_seed_mixed(p->seed);
    for (int64_t q = 0; q < count; ++q)
        for (int which = 0; which < 2; ++which) {
            int64_t row = syn_row_of_pair(p, first_pair + q, which);
            float *out = rows + (2 * q + which) * p->d;
            for (int64_t e = 0; e < p->d; ++e) out[e] = syn_element(p, sm, row, e);
        }
    return 0;
}

/* out[r][c] = element elems[c] of row rows_ids[r] (row id = worker*n + position). */
int synth_sample_host(const synth_params *p, const int64_t *row_ids, int64_t nrows,
                      const int64_t *elems, int64_t nelems, float *out) {
    if (!p || !row_ids || !elems || !out) return -1;
    uint64_t sm = syn_seed_mixed(p->seed);
    for (int64_t r = 0; r < nrows; ++r)
        for (int64_t c = 0; c < nelems; ++c) {
            if (row_ids[r] < 0 || row_ids[r] >= p->m * p->n || elems[c] < 0 || elems[c] >= p->d) return -1;
            out[r * nelems + c] = syn_element(p, sm, row_ids[r], elems[c]);
        }
    return 0;
}

uint64_t synth_mix_host(uint64_t x) { return syn_mix(x); }
