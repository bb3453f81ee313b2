/*
 * adamw_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, scalar CPU statement of what the chunked mixed-precision AdamW
 * update computes.  Only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the GPU library never does, and this file
 * shares no code, header, table or constant with the GPU path.
 *
 * What the paper fixes (AutoHete, section 2.1 "Transformer-based LLM
 * Training"): model data = parameters + gradients + optimizer states;
 * parameters and gradients are 16-bit, the optimizer states are fp32 and are
 * {momentum, variance, fp32 parameter copy}: 2 + 2 + 12 = 16 bytes per
 * parameter.  Section 3.2.2 (footnote on memory) fixes the direction of the
 * cast: the 16-bit parameters are derived from the fp32 copy.  The footnote to
 * Eq. 5 says the optimizer is invoked per group of tensors (one optimizer per
 * transformer block), so every function here works on one chunk at a time and
 * the result must not depend on how chunks are grouped into calls.  Appendix
 * "memory allocation": optimizer states are touched exactly once per update.
 *
 * What the paper does not fix (it names "ADAM" and gives no equations): the
 * update rule itself.  It is taken as textbook Adam with decoupled weight
 * decay (AdamW; weight_decay = 0 is plain Adam), preceded by loss-scale
 * removal, a finite check and global-L2-norm clipping.  Every such reading is
 * marked READING below.
 *
 * Arithmetic: state is stored in fp32; every new value is computed in fp64
 * from the stored fp32/16-bit inputs and rounded once when stored.  The norm
 * is accumulated in fp64 in index order.  Compile with -ffp-contract=off so
 * each written operation is one IEEE operation.
 *
 * Parity pins (tests/test_oracle_pins.py, all CPU): step-1 sign form,
 * zero-gradient pure decay, constant-gradient closed form for every t,
 * non-finite skip, hand-worked 16-element example (tests/golden/), norm closed
 * forms, clip invariant, scale invariance, partition invariance, padding
 * invariant, fp64 torch.optim.AdamW cross-check, exhaustive 16-bit
 * round-trips and RNE against numpy/torch conversions.  No function is
 * "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

enum { ORACLE_BF16 = 0, ORACLE_FP16 = 1 };

typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    float max_grad_norm; /* <= 0 : clipping off */
    float loss_scale;    /* > 0 */
} oracle_hparams;

/* ------------------------------------------------------------------------ */
/* 16-bit formats, written from their definitions (IEEE binary16; bfloat16 = */
/* the upper half of binary32).  READING: round-to-nearest-even, subnormals  */
/* kept (the paper only says "FP16").                                        */
/* ------------------------------------------------------------------------ */

static double bf16_value(uint16_t b)
{
    int sign = b >> 15, e = (b >> 7) & 0xff, f = b & 0x7f;
    double mag;
    if (e == 0xff) mag = f ? NAN : INFINITY;
    else if (e == 0) mag = ldexp((double)f, -126 - 7);
    else mag = ldexp(128.0 + f, e - 127 - 7);
    return sign ? -mag : mag;
}

static double fp16_value(uint16_t b)
{
    int sign = b >> 15, e = (b >> 10) & 0x1f, f = b & 0x3ff;
    double mag;
    if (e == 0x1f) mag = f ? NAN : INFINITY;
    else if (e == 0) mag = ldexp((double)f, -14 - 10);
    else mag = ldexp(1024.0 + f, e - 15 - 10);
    return sign ? -mag : mag;
}

/* Nearest value on a binary floating grid with `pbits` fraction bits, minimum
 * normal exponent emin and maximum exponent emax; ties to the even grid point.
 * Returns sign/biased-exponent/fraction fields. rint() rounds to even in the
 * default rounding mode, which is never changed here. */
static uint16_t encode_grid(double x, int pbits, int emin, int emax, int bias)
{
    uint16_t sign = signbit(x) ? 1 : 0;
    int ebits_all1 = emax + 1 + bias;
    if (isnan(x)) return (uint16_t)((sign << 15) | (ebits_all1 << pbits) | (1 << (pbits - 1)));
    double a = fabs(x);
    uint16_t inf = (uint16_t)((sign << 15) | (ebits_all1 << pbits));
    if (isinf(a)) return inf;
    if (a == 0.0) return (uint16_t)(sign << 15);
    int e;
    (void)frexp(a, &e); /* a = f * 2^e, f in [0.5,1)  ->  floor(log2 a) = e-1 */
    e -= 1;
    if (e < emin) e = emin;                     /* subnormal range shares emin's spacing */
    double q = ldexp(1.0, e - pbits);           /* grid spacing at this exponent */
    double n = rint(a / q);                     /* a/q is exact: division by a power of two */
    double r = n * q;                           /* rounded magnitude, exact */
    if (r >= ldexp(1.0, emax + 1)) return inf;  /* rounded past the largest finite value */
    if (r < ldexp(1.0, emin)) return (uint16_t)((sign << 15) | (uint16_t)n); /* subnormal or 0 */
    (void)frexp(r, &e);
    e -= 1;
    uint16_t frac = (uint16_t)(r / ldexp(1.0, e - pbits) - ldexp(1.0, pbits));
    return (uint16_t)((sign << 15) | ((e + bias) << pbits) | frac);
}

float oracle_lowp_decode(uint16_t bits, int dtype)
{
    return (float)(dtype == ORACLE_FP16 ? fp16_value(bits) : bf16_value(bits));
}

uint16_t oracle_lowp_encode(float x, int dtype)
{
    if (dtype == ORACLE_FP16) return encode_grid((double)x, 10, -14, 15, 15);
    return encode_grid((double)x, 7, -126, 127, 127);
}

/* ------------------------------------------------------------------------ */
/* Chunk layout.  Tensors are packed back to back into one flat element      */
/* space cut into chunks of chunk_elems; a tensor may straddle chunks; only  */
/* the last chunk is padded.  (Section 3.1: transfers aggregate tensors;     */
/* section 3.4: parameters are mapped to device memory in advance.)          */
/* ------------------------------------------------------------------------ */

int oracle_chunk_layout(const uint64_t *tensor_numel, uint64_t n_tensors, uint64_t chunk_elems,
                        uint64_t *tensor_offset, uint64_t *n_chunks, uint64_t *total_elems,
                        uint64_t *padded_elems)
{
    if (chunk_elems == 0) return -1;
    uint64_t off = 0;
    for (uint64_t t = 0; t < n_tensors; ++t) {
        tensor_offset[t] = off;
        off += tensor_numel[t];
    }
    uint64_t nc = 0;
    while (nc * chunk_elems < off) ++nc; /* smallest nc with nc*C >= total */
    *n_chunks = nc;
    *total_elems = off;
    *padded_elems = nc * chunk_elems - off;
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Gradient preparation: remove the loss scale, look for non-finite values,  */
/* accumulate the squared L2 norm.  READING (paper silent): the finite check */
/* is on the unscaled value; a non-finite element contributes nothing to the */
/* sum and raises the flag.  Call once per chunk, in chunk order; *sumsq     */
/* starts at the caller's extra_sumsq (sum of squares of unscaled gradients  */
/* held elsewhere, e.g. host-resident chunks), *found_inf at 0.              */
/* ------------------------------------------------------------------------ */

void oracle_grad_accumulate(const uint16_t *grad, uint64_t numel, int dtype, float loss_scale,
                            double *sumsq, uint32_t *found_inf)
{
    double inv = 1.0 / (double)loss_scale;
    double s = *sumsq;
    uint32_t flag = *found_inf;
    for (uint64_t i = 0; i < numel; ++i) {
        double x = (double)oracle_lowp_decode(grad[i], dtype) * inv;
        if (!isfinite(x)) flag = 1;
        else s += x * x;
    }
    *sumsq = s;
    *found_inf = flag;
}

/* Finish: a non-finite carried-in partial sum also raises the flag.  norm is
 * NaN when the flag is raised (READING: only the flag is defined then). */
void oracle_grad_finish(double sumsq, uint32_t found_inf_in, double *norm, uint32_t *found_inf)
{
    uint32_t flag = found_inf_in || !isfinite(sumsq);
    *found_inf = flag;
    *norm = flag ? NAN : sqrt(sumsq);
}

/* READING: clip coefficient = min(1, max_norm / (norm + 1e-6)); off when
 * max_norm <= 0. */
double oracle_clip_coef(double norm, float max_grad_norm)
{
    if (!(max_grad_norm > 0.0f)) return 1.0;
    double c = (double)max_grad_norm / (norm + 1e-6);
    return c < 1.0 ? c : 1.0;
}

/* ------------------------------------------------------------------------ */
/* One AdamW step over one chunk.  `step` is the 1-based t.  If found_inf    */
/* is set nothing is touched (READING: skip-on-overflow; the caller does not */
/* advance t).  READING of the rule:                                         */
/*   g  = decode(grad) / loss_scale * coef                                   */
/*   m' = b1 m + (1-b1) g          v' = b2 v + (1-b2) g^2                     */
/*   p' = p - lr ( (m'/(1-b1^t)) / (sqrt(v'/(1-b2^t)) + eps) + wd p )         */
/* eps is outside the root and after bias correction; decay uses the old p.  */
/* ------------------------------------------------------------------------ */

void oracle_adamw_chunk(const uint16_t *grad, uint16_t *param_lp, float *master, float *exp_avg,
                        float *exp_avg_sq, uint64_t numel, int dtype, uint64_t step,
                        const oracle_hparams *hp, double norm, uint32_t found_inf)
{
    if (found_inf) return;
    double inv = 1.0 / (double)hp->loss_scale;
    double coef = oracle_clip_coef(norm, hp->max_grad_norm);
    double b1 = (double)hp->beta1, b2 = (double)hp->beta2;
    double lr = (double)hp->lr, eps = (double)hp->eps, wd = (double)hp->weight_decay;
    double bc1 = 1.0 - pow(b1, (double)step);
    double bc2 = 1.0 - pow(b2, (double)step);
    for (uint64_t i = 0; i < numel; ++i) {
        double g = (double)oracle_lowp_decode(grad[i], dtype) * inv * coef;
        double p = (double)master[i];
        double mn = b1 * (double)exp_avg[i] + (1.0 - b1) * g;
        double vn = b2 * (double)exp_avg_sq[i] + (1.0 - b2) * (g * g);
        double pn = p - lr * ((mn / bc1) / (sqrt(vn / bc2) + eps) + wd * p);
        exp_avg[i] = (float)mn;
        exp_avg_sq[i] = (float)vn;
        master[i] = (float)pn;
        if (param_lp) param_lp[i] = oracle_lowp_encode((float)pn, dtype);
    }
}

/* The 16-bit parameters of a chunk produced on demand from the fp32 copy (section 3.2.2,
 * footnote: blocks whose optimizer states stay on the GPU keep no 16-bit parameters).
 * oracle_adamw_chunk with param_lp == NULL is the matching update without write-back. */
void oracle_cast_chunk(const float *master, uint16_t *param_lp, uint64_t numel, int dtype)
{
    for (uint64_t i = 0; i < numel; ++i) param_lp[i] = oracle_lowp_encode(master[i], dtype);
}

/* Vector forms of the 16-bit conversions, for tests. */
void oracle_lowp_decode_array(const uint16_t *in, float *out, uint64_t n, int dtype)
{
    for (uint64_t i = 0; i < n; ++i) out[i] = oracle_lowp_decode(in[i], dtype);
}

void oracle_lowp_encode_array(const float *in, uint16_t *out, uint64_t n, int dtype)
{
    for (uint64_t i = 0; i < n; ++i) out[i] = oracle_lowp_encode(in[i], dtype);
}
