/* CPU half of the synthetic model-data generator (see gen_core.h).  The fill loop is compiled
 * in three versions (AVX-512, AVX2, baseline) and the loader picks one for the CPU at run time;
 * all versions perform the same integer operations and the one fp32 multiply per element. */
#include "gen_core.h"

uint64_t synth_cpu_key(uint64_t seed, uint32_t stream, uint64_t step) { return synth_key(seed, stream, step); }

#define SYNTH_CLONES __attribute__((target_clones("arch=skylake-avx512", "avx2", "default")))

SYNTH_CLONES static void fill_f32(float *out, uint64_t count, const synth_spec s)
{
    for (uint64_t i = 0; i < count; ++i) out[i] = synth_value(&s, s.first_index + i);
}

SYNTH_CLONES static void fill_bf16(uint16_t *out, uint64_t count, const synth_spec s)
{
    for (uint64_t i = 0; i < count; ++i) out[i] = synth_to_bf16(synth_value(&s, s.first_index + i));
}

SYNTH_CLONES static void fill_f32_of_bf16(float *out, uint64_t count, const synth_spec s)
{
    for (uint64_t i = 0; i < count; ++i) out[i] = synth_from_bf16(synth_to_bf16(synth_value(&s, s.first_index + i)));
}

void synth_cpu_fill(void *out, uint64_t count, const synth_spec *spec)
{
    const synth_spec s = *spec;
    if (s.out_kind == SYNTH_OUT_F32) fill_f32((float *)out, count, s);
    else if (s.dtype == SYNTH_BF16 && s.out_kind == SYNTH_OUT_LOWP) fill_bf16((uint16_t *)out, count, s);
    else if (s.dtype == SYNTH_BF16) fill_f32_of_bf16((float *)out, count, s);
    else
        for (uint64_t i = 0; i < count; ++i) synth_store(&s, out, s.first_index + i); /* fp16: scalar */
}
