/*
 * Host build of the synthetic-input generator (see synth_gen.h).
 * gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC
 */
#include "synth_gen.h"

/* Fill out[0..n) with elements first .. first+n-1 of the stream. Returns 0, or 1 on a bad argument. */
int synth_fill_host(void *out, int dtype, uint64_t n, uint64_t first, const synth_spec *spec)
{
    if (n == 0) return 0;
    if (!out || !spec || dtype < SYNTH_F32 || dtype > SYNTH_F16) return 1;
    synth_spec sp = *spec;
#pragma omp parallel for schedule(static) if (n > 65536)
    for (int64_t i = 0; i < (int64_t)n; ++i)
        synth_store(out, dtype, (uint64_t)i, synth_value(&sp, first + (uint64_t)i));
    return 0;
}

uint64_t synth_mix64_host(uint64_t z) { return synth_mix64(z); }
