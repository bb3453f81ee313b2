/*
 * gen_core.h -- seeded, counter-based synthetic model data.  Shared by the CPU
 * (gen_cpu.c, gcc) and GPU (gen_gpu.hip, hipcc) halves of the input generator so
 * that both produce bit-identical streams.  It is a test/benchmark fixture: it
 * defines INPUTS only and contains none of the optimizer's arithmetic.  Neither
 * the GPU library nor the CPU oracle includes this file.
 *
 * value(seed, stream, step, i):
 *   key = mix(mix(seed + GOLD*(stream+1)) + GOLD2*step)
 *   h1 = mix(key + GOLD*i), h2 = mix(h1 + GOLD2)
 *   z  = (sum of the eight 16-bit fields of h1,h2) - 262140        (Irwin-Hall(8), an
 *        integer in [-262140, 262140]: bell-shaped, variance 8*(65536^2-1)/12, |z| <= 4.9 sd)
 *   x  = float(z) * scale            one fp32 multiply, scale = float(sigma / sd)
 * An element is an "outlier" (uses scale_outlier instead) when the top 32 bits of
 * mix(h2 + GOLD) fall below outlier_thresh = round(prob * 2^32).
 * Only integer operations, one int->float conversion and one fp32 multiply are
 * used, so host and device agree bit for bit.  Elements with flat index >=
 * n_valid are padding and are exactly +0.
 *
 * The 16-bit roundings below (nearest-even) only decide which 16-bit inputs are
 * generated; they are this fixture's own.
 */
#ifndef SYNTH_GEN_CORE_H
#define SYNTH_GEN_CORE_H
#include <stdint.h>

#ifndef SYNTH_HD
#define SYNTH_HD static inline __attribute__((always_inline))
#endif

#define SYNTH_GOLD 0x9E3779B97F4A7C15ull
#define SYNTH_GOLD2 0xD1B54A32D192ED03ull

enum { SYNTH_BF16 = 0, SYNTH_FP16 = 1 };
enum { SYNTH_OUT_F32 = 0, SYNTH_OUT_LOWP = 1, SYNTH_OUT_F32_OF_LOWP = 2 };

typedef struct {
    uint64_t key;            /* synth_key(seed, stream, step) */
    uint64_t first_index;    /* flat index of out[0] */
    uint64_t n_valid;        /* flat indices >= n_valid are padding (zero) */
    float scale;             /* sigma / sd(Irwin-Hall 8) */
    float scale_outlier;
    uint32_t outlier_thresh; /* 0 = no outliers */
    int take_abs;
    int out_kind;            /* SYNTH_OUT_* */
    int dtype;               /* SYNTH_BF16 / SYNTH_FP16 for the LOWP kinds */
} synth_spec;

SYNTH_HD uint64_t synth_mix64(uint64_t x)
{
    x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27; x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

SYNTH_HD uint64_t synth_key(uint64_t seed, uint32_t stream, uint64_t step)
{
    return synth_mix64(synth_mix64(seed + SYNTH_GOLD * (uint64_t)(stream + 1u)) + SYNTH_GOLD2 * step);
}

SYNTH_HD uint32_t synth_f32_bits(float f) { union { float f; uint32_t u; } c; c.f = f; return c.u; }
SYNTH_HD float synth_bits_f32(uint32_t u) { union { float f; uint32_t u; } c; c.u = u; return c.f; }

SYNTH_HD uint16_t synth_to_bf16(float f)
{
    uint32_t u = synth_f32_bits(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

SYNTH_HD float synth_from_bf16(uint16_t h) { return synth_bits_f32((uint32_t)h << 16); }

SYNTH_HD uint16_t synth_to_fp16(float f)
{
    uint32_t u = synth_f32_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    u &= 0x7FFFFFFFu;
    if (u > 0x7F800000u) return (uint16_t)(sign | 0x7E00u);
    if (u >= 0x477FF000u) return (uint16_t)(sign | 0x7C00u);          /* >= 65520 -> inf */
    if (u < 0x38800000u) {                                            /* < 2^-14: subnormal */
        float a = synth_bits_f32(u) + 0.5f;                           /* ulp(0.5) = 2^-24: the add rounds */
        return (uint16_t)(sign | (uint16_t)(synth_f32_bits(a) - 0x3F000000u));
    }
    u += 0xC8000000u + 0x0FFFu + ((u >> 13) & 1u);                    /* rebias 127->15, round */
    return (uint16_t)(sign | (uint16_t)(u >> 13));
}

SYNTH_HD float synth_from_fp16(uint16_t h)
{
    uint32_t sign = ((uint32_t)h & 0x8000u) << 16, e = (h >> 10) & 0x1Fu, f = h & 0x3FFu;
    if (e == 0) return synth_bits_f32(sign | synth_f32_bits((float)f * 5.9604644775390625e-8f));
    if (e == 31) return synth_bits_f32(sign | 0x7F800000u | (f << 13));
    return synth_bits_f32(sign | ((e + 112u) << 23) | (f << 13));
}

/* Branch-free on purpose (selects only), so that the CPU fill loops vectorise. */
SYNTH_HD float synth_value(const synth_spec *s, uint64_t idx)
{
    uint64_t h1 = synth_mix64(s->key + SYNTH_GOLD * idx);
    uint64_t h2 = synth_mix64(h1 + SYNTH_GOLD2);
    uint64_t h3 = synth_mix64(h2 + SYNTH_GOLD);
    int32_t z = (int32_t)((h1 & 0xFFFF) + ((h1 >> 16) & 0xFFFF) + ((h1 >> 32) & 0xFFFF) + (h1 >> 48) +
                          (h2 & 0xFFFF) + ((h2 >> 16) & 0xFFFF) + ((h2 >> 32) & 0xFFFF) + (h2 >> 48)) - 262140;
    int outlier = (uint32_t)(h3 >> 32) < s->outlier_thresh; /* thresh 0: never */
    float sc = outlier ? s->scale_outlier : s->scale;
    float x = (float)z * sc;
    float ax = (s->take_abs && z < 0) ? -x : x;
    return idx >= s->n_valid ? 0.0f : ax;
}

/* Writes element idx of the stream at out[idx - first_index]. */
SYNTH_HD void synth_store(const synth_spec *s, void *out, uint64_t idx)
{
    float x = synth_value(s, idx);
    uint64_t j = idx - s->first_index;
    if (s->out_kind == SYNTH_OUT_F32) { ((float *)out)[j] = x; return; }
    uint16_t h = s->dtype == SYNTH_FP16 ? synth_to_fp16(x) : synth_to_bf16(x);
    if (s->out_kind == SYNTH_OUT_LOWP) ((uint16_t *)out)[j] = h;
    else ((float *)out)[j] = s->dtype == SYNTH_FP16 ? synth_from_fp16(h) : synth_from_bf16(h);
}

#endif
