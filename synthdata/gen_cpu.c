/* CPU half of the synthetic model-data generator (see gen_core.h). */
#include "gen_core.h"

uint64_t synth_cpu_key(uint64_t seed, uint32_t stream, uint64_t step) { return synth_key(seed, stream, step); }

void synth_cpu_fill(void *out, uint64_t count, const synth_spec *spec)
{
    const synth_spec s = *spec; /* local copy: lets the compiler hoist the kind/dtype tests */
    for (uint64_t i = 0; i < count; ++i) synth_store(&s, out, s.first_index + i);
}
