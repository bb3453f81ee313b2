/*
 * parity_check.c -- the element-by-element comparison rules of the GPU parity tests, in C so that
 * billions of element-steps can be judged in seconds.  TEST INFRASTRUCTURE: it holds neither the
 * oracle's nor the library's arithmetic, only the yardsticks their results are held against.
 * Loaded through ctypes by tests/_harness.py (gcc -O2 -ffp-contract=off).
 *
 * Streams: m = first moment (exp_avg), v = second moment (exp_avg_sq), p = fp32 master weights.
 * "ora" = the CPU oracle's values, "gpu" = what the HIP path left in device memory.
 * ulp32(x) = spacing of fp32 numbers at |x| (2^-149 at and below the smallest normal number).
 *
 * Two rules.
 *
 * parity_strict -- both sides started this step from IDENTICAL inputs.  An element passes if
 *     |gpu - ora| <= max(2 ulp32(ora), 1e-6 |ora|, 2 ulp32(T))
 * where T is the largest-magnitude term that feeds the value (never taken below |ora| itself):
 *     m: max(beta1 |m_old|, (1 - beta1) |g'|)   (the two terms can cancel)
 *     p: |p_old|                                (the update is a small correction to it)
 *     v: v itself                               (all terms are >= 0: no cancellation, no third arm)
 * The first two arms are the tolerance as stated (2 fp32 ulp, relative 1e-6).  The third arm exists
 * because the two sides sum the 10^9 squares of the gradient norm in different orders, so their
 * clip factors differ in the last bits of fp64; where the terms cancel to a result much smaller
 * than T, that difference can flip a rounding that is many ulps OF THE TINY RESULT.  Every use of
 * the third arm is counted and reported.
 *
 * parity_free -- the GPU state has NOT been re-synchronised with the oracle's for some steps.  A
 * last-bit difference after step k is an input difference at step k+1, so no fixed number of
 * ulps of the result is a valid bar.  But the input difference is KNOWN: D = |gpu - ora| of each
 * stream after the previous step (observed then, carried here; 0 at the start).  The element is
 * held to what the update rule makes of that known difference, plus one rounding on each side:
 * with
 *     rho   = relative difference of the two sides' clip factors (from their two sums S),
 *     kappa = 2^-48, allowance for the fp64 evaluation error of either side (relative to the
 *             largest term; the fp64 roundings and the Newton root/quotient stay below it),
 *     sp(x) = ulp32(x): a value rounded to fp32 moves by at most sp/2,
 * and g' the oracle's unscaled, clipped gradient, x_t / x~_t the oracle's / the GPU's stored
 * value after this step, the bounds E on |x~_t - x_t| are
 *     E_m = b1 D_m + (1-b1) |g'| rho + kappa (b1 (|m_old| + D_m) + (1-b1) |g'|) + sp(m_t)/2 + sp(m~_t)/2
 *     E_v = b2 D_v + (1-b2) g'^2 (2 rho + rho^2) + kappa v_t                    + sp(v_t)/2 + sp(v~_t)/2
 *     E_p = (1 + lr wd) D_p + lr (U_hi - U_lo) (1 + kappa) + kappa |p_old|      + sp(p_t)/2 + sp(p~_t)/2
 * where [U_lo, U_hi] is the image of the box  M in [m_t - E_m, m_t + E_m],
 * V in [max(v_t - E_v, 0), v_t + E_v]  (both sides' unrounded moments lie in it) under
 * U = (M / bc1) / (sqrt(V / bc2) + eps).  Each line is the triangle inequality applied to the
 * update rule plus |round(a) - round(b)| <= |a - b| + sp(a)/2 + sp(b)/2.  The element passes if
 * |gpu - ora| <= E, and D is then replaced by the |gpu - ora| just observed.  While the two sides
 * agree (D = 0) this bar is about one ulp32; it widens only by what an actual earlier difference
 * explains.  On a skipped step nothing changes on either side and D is left alone (no call).
 */
#include <math.h>
#include <stdint.h>

static inline double ulp32(float x)
{
    uint32_t b;
    __builtin_memcpy(&b, &x, 4);
    const uint32_t e = (b >> 23) & 0xFFu;
    if (e == 0xFFu) return INFINITY;                 /* inf / NaN: no spacing */
    if (e <= 1u) return 0x1p-149;                    /* subnormals and the first normal binade */
    const uint64_t d = (uint64_t)(e - 127u - 23u + 1023u) << 52; /* 2^(e - 127 - 23) */
    double r;
    __builtin_memcpy(&r, &d, 8);
    return r;
}

static inline double dmax(double a, double b) { return a > b ? a : b; }

/* Value of a 16-bit gradient pattern, from the definition of the two formats (dtype 0: bfloat16, the
 * upper half of an fp32 word; 1: IEEE binary16).  Only called for the rare elements that differ. */
static double lowp_value(uint16_t b, int dtype)
{
    if (dtype == 0) {
        const uint32_t w = (uint32_t)b << 16;
        float f;
        __builtin_memcpy(&f, &w, 4);
        return (double)f;
    }
    const int sign = b >> 15, e = (b >> 10) & 0x1F, frac = b & 0x3FF;
    double mag;
    if (e == 0x1F) mag = frac ? NAN : INFINITY;
    else if (e == 0) mag = ldexp((double)frac, -24);
    else mag = ldexp(1024.0 + frac, e - 25);
    return sign ? -mag : mag;
}

enum { /* per-stream statistics; index = stream * PS_N + field; streams in the order m, v, p */
    PS_MISMATCH = 0, /* elements whose bits differ */
    PS_BEYOND,       /* elements beyond max(2 ulp32(ora), 1e-6 |ora|): judged by the third arm / by E */
    PS_FAIL,         /* elements that fail the rule */
    PS_FIRST_FAIL,   /* index of the first failing element (as a double), -1 if none */
    PS_MAX_ULP_RES,  /* worst |err| / ulp32(ora) among the elements NOT counted in PS_BEYOND */
    PS_MAX_ULP_T,    /* worst |err| / ulp32(T) over all elements */
    PS_MAX_E_FRAC,   /* parity_free: worst |err| / E (<= 1 means inside the bound) */
    PS_MAX_E_ULP_T,  /* parity_free: largest E / ulp32(T): how wide the bar became */
    PS_MAX_ABS,      /* largest |err| */
    PS_SUMSQ_ORA,    /* parity_free: sum of ora^2 over all elements (for the stream's r.m.s. magnitude) */
    PS_N
};

typedef struct {
    double grad_scale;   /* g' = gf * grad_scale: (1 / loss_scale) * oracle's clip factor */
    double beta1, beta2, lr, eps, wd, bc1, bc2;
    double rho;          /* parity_free only */
} parity_consts;

static inline int same_bits(float a, float b)
{
    uint32_t x, y;
    __builtin_memcpy(&x, &a, 4);
    __builtin_memcpy(&y, &b, 4);
    return x == y;
}

static void stats_init(double *st)
{
    for (int i = 0; i < 3 * PS_N; ++i) st[i] = 0.0;
    for (int s = 0; s < 3; ++s) st[s * PS_N + PS_FIRST_FAIL] = -1.0;
}

static inline void judge(double *st, uint64_t i, float gpu, float ora, double T, double tol_extra, int use_E)
{
    const double err = fabs((double)gpu - (double)ora);
    if (!(T >= fabs((double)ora))) T = fabs((double)ora); /* the result itself is never larger than ~2 T */
    const double u = ulp32(ora), uT = ulp32((float)T);
    const double base = dmax(2.0 * u, 1e-6 * fabs((double)ora));
    uint32_t gb, ob;
    __builtin_memcpy(&gb, &gpu, 4);
    __builtin_memcpy(&ob, &ora, 4);
    if (gb != ob) st[PS_MISMATCH] += 1.0;
    const int finite = isfinite(gpu) && isfinite(ora);
    int fail;
    if (!finite) {
        fail = gb != ob; /* a non-finite value must be reproduced exactly */
    } else {
        if (err > base) st[PS_BEYOND] += 1.0;
        else st[PS_MAX_ULP_RES] = dmax(st[PS_MAX_ULP_RES], err / u);
        st[PS_MAX_ULP_T] = dmax(st[PS_MAX_ULP_T], err / uT);
        st[PS_MAX_ABS] = dmax(st[PS_MAX_ABS], err);
        if (use_E) {
            fail = !(err <= tol_extra);
            if (err > 0.0) st[PS_MAX_E_FRAC] = dmax(st[PS_MAX_E_FRAC], tol_extra > 0.0 ? err / tol_extra : INFINITY);
            st[PS_MAX_E_ULP_T] = dmax(st[PS_MAX_E_ULP_T], tol_extra / uT);
        } else {
            fail = !(err <= dmax(base, tol_extra));
        }
    }
    if (fail) {
        if (st[PS_FAIL] == 0.0) st[PS_FIRST_FAIL] = (double)i;
        st[PS_FAIL] += 1.0;
    }
}

/* g16: the 16-bit gradients (still multiplied by the loss scale) in format `dtype`.  *_old: the
 * state both sides started from (may be NULL: then only the first two arms apply). */
void parity_strict(uint64_t n, const uint16_t *g16, int dtype, const float *m_old, const float *p_old, const float *m_ora,
                   const float *v_ora, const float *p_ora, const float *m_gpu, const float *v_gpu, const float *p_gpu,
                   const parity_consts *k, double *stats /* [3 * PS_N] */)
{
    stats_init(stats);
    for (uint64_t i = 0; i < n; ++i) {
        /* bit-identical in all three streams (nearly every element): passes any rule, nothing to measure */
        if (same_bits(m_gpu[i], m_ora[i]) && same_bits(v_gpu[i], v_ora[i]) && same_bits(p_gpu[i], p_ora[i])) continue;
        double Tm = fabs((double)m_ora[i]), Tp = fabs((double)p_ora[i]);
        double arm_m = 0.0, arm_p = 0.0;
        if (m_old && p_old && g16) {
            const double g = fabs(lowp_value(g16[i], dtype) * k->grad_scale);
            Tm = dmax(k->beta1 * fabs((double)m_old[i]), (1.0 - k->beta1) * g);
            Tp = fabs((double)p_old[i]);
            arm_m = 2.0 * ulp32((float)Tm);
            arm_p = 2.0 * ulp32((float)Tp);
        }
        judge(stats + 0 * PS_N, i, m_gpu[i], m_ora[i], Tm, arm_m, 0);
        judge(stats + 1 * PS_N, i, v_gpu[i], v_ora[i], fabs((double)v_ora[i]), 0.0, 0);
        judge(stats + 2 * PS_N, i, p_gpu[i], p_ora[i], Tp, arm_p, 0);
    }
}

/* D_m, D_v, D_p: |gpu - ora| observed after the previous step (0 at the start); read, and
 * overwritten with the differences observed now (fp32 storage, rounded up). */
void parity_free(uint64_t n, const uint16_t *g16, int dtype, const float *m_old, const float *p_old, const float *m_ora,
                 const float *v_ora, const float *p_ora, const float *m_gpu, const float *v_gpu, const float *p_gpu,
                 float *D_m, float *D_v, float *D_p, const parity_consts *k, double *stats)
{
    const double kappa = 0x1p-48, up = 1.0 + 0x1p-20; /* `up`: fp32 storage of D, rounded up */
    const double b1 = k->beta1, b2 = k->beta2, rho = k->rho;
    stats_init(stats);
    for (uint64_t i = 0; i < n; ++i) {
        const double mo = (double)m_ora[i], vo = (double)v_ora[i];
        stats[0 * PS_N + PS_SUMSQ_ORA] += mo * mo;
        stats[1 * PS_N + PS_SUMSQ_ORA] += vo * vo;
        stats[2 * PS_N + PS_SUMSQ_ORA] += (double)p_ora[i] * (double)p_ora[i];
        /* bit-identical in all three streams (nearly every element): the error is zero, which is inside
         * any bound, and the difference carried to the next step is zero whatever it was before */
        if (same_bits(m_gpu[i], m_ora[i]) && same_bits(v_gpu[i], v_ora[i]) && same_bits(p_gpu[i], p_ora[i])) {
            D_m[i] = D_v[i] = D_p[i] = 0.0f;
            continue;
        }
        const double g = fabs(lowp_value(g16[i], dtype) * k->grad_scale);
        const double Em = b1 * D_m[i] + (1.0 - b1) * g * rho +
                          kappa * (b1 * (fabs((double)m_old[i]) + D_m[i]) + (1.0 - b1) * g) +
                          0.5 * ulp32(m_ora[i]) + 0.5 * ulp32(m_gpu[i]);
        const double Ev = b2 * D_v[i] + (1.0 - b2) * g * g * (2.0 * rho + rho * rho) + kappa * vo +
                          0.5 * ulp32(v_ora[i]) + 0.5 * ulp32(v_gpu[i]);
        /* image of the box under U = (M / bc1) / (sqrt(V / bc2) + eps) */
        const double m_lo = (mo - Em) / k->bc1, m_hi = (mo + Em) / k->bc1;
        const double v_lo = vo - Ev > 0.0 ? vo - Ev : 0.0;
        const double den_lo = sqrt(v_lo / k->bc2) + k->eps, den_hi = sqrt((vo + Ev) / k->bc2) + k->eps;
        const double U_hi = m_hi >= 0.0 ? m_hi / den_lo : m_hi / den_hi;
        const double U_lo = m_lo >= 0.0 ? m_lo / den_hi : m_lo / den_lo;
        double dU = U_hi - U_lo;
        if (!(dU >= 0.0)) dU = INFINITY; /* den_lo = 0 (eps = 0, no second moment): no bound */
        const double Ep = (1.0 + k->lr * k->wd) * D_p[i] + k->lr * dU * (1.0 + kappa) +
                          kappa * fabs((double)p_old[i]) + 0.5 * ulp32(p_ora[i]) + 0.5 * ulp32(p_gpu[i]);
        const double Tm = dmax(b1 * fabs((double)m_old[i]), (1.0 - b1) * g);
        judge(stats + 0 * PS_N, i, m_gpu[i], m_ora[i], Tm, Em, 1);
        judge(stats + 1 * PS_N, i, v_gpu[i], v_ora[i], fabs(vo), Ev, 1);
        judge(stats + 2 * PS_N, i, p_gpu[i], p_ora[i], fabs((double)p_old[i]), Ep, 1);
        D_m[i] = (float)(fabs((double)m_gpu[i] - mo) * up);
        D_v[i] = (float)(fabs((double)v_gpu[i] - vo) * up);
        D_p[i] = (float)(fabs((double)p_gpu[i] - (double)p_ora[i]) * up);
    }
}

/* 16-bit parameters: distance in representable values (sign-magnitude patterns ordered like the
 * values).  Returns the largest distance; *n_diff = elements that differ. */
uint32_t parity_lowp(uint64_t n, const uint16_t *gpu, const uint16_t *ora, uint64_t *n_diff)
{
    uint32_t worst = 0;
    uint64_t diff = 0;
    for (uint64_t i = 0; i < n; ++i) {
        if (gpu[i] == ora[i]) continue;
        ++diff;
        const int32_t a = gpu[i] & 0x8000 ? -(int32_t)(gpu[i] & 0x7FFF) : (int32_t)(gpu[i] & 0x7FFF);
        const int32_t b = ora[i] & 0x8000 ? -(int32_t)(ora[i] & 0x7FFF) : (int32_t)(ora[i] & 0x7FFF);
        const uint32_t d = (uint32_t)(a > b ? a - b : b - a);
        if (d > worst) worst = d;
    }
    *n_diff = diff;
    return worst;
}
