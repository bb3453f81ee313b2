/*
 * autohete_host.cpp -- the host half of a hybrid placement: the same AdamW chunk update for chunks
 * whose optimizer states live in host memory (paper section 3.2.1: placing a block's optimizer
 * states on the CPU means prefetching its 16-bit parameters, offloading its 16-bit gradients and
 * updating the fp32 parameters on the CPU; cost t_optim^cpu, Eq. 5, second arm).
 *
 * Same rule, same arithmetic as the GPU kernel: every new value is computed in fp64 from the stored
 * fp32 / 16-bit inputs, in the operation order of the rule in autohete.h, without contraction, and
 * rounded once -- so a chunk may move between the two placements from one step to the next without
 * a visible seam.  AVX-512 (8 fp64 lanes) where the CPU has it, plain scalar code otherwise; the
 * element range is cut into contiguous slices, one per thread.  This file shares nothing with the
 * test oracle.
 */
#include <immintrin.h>
#include <math.h>
#include <string.h>

#include <algorithm>
#include <thread>
#include <vector>

#include "../../include/autohete.h"

#pragma clang fp contract(off)

namespace {

struct Consts {
    double inv, coef, b1, b2, omb1, omb2, bc1, bc2, lr, eps, wd;
    double rbc1, rbc2;   /* correctly rounded reciprocals of bc1, bc2 */
    bool recip_exact;    /* the quotients by bc1 / bc2 may be formed from them (see div_by_const) */
};

/* ---------------------------------------------------------------- scalar 16-bit conversions */

inline float bits_f32(uint32_t u)
{
    float f;
    memcpy(&f, &u, 4);
    return f;
}
inline uint32_t f32_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    return u;
}

inline float lowp_to_f32(uint16_t h, int dtype)
{
    if (dtype == AH_BF16) return bits_f32((uint32_t)h << 16);
    const uint32_t sign = ((uint32_t)h & 0x8000u) << 16, e = (h >> 10) & 0x1Fu, f = h & 0x3FFu;
    if (e == 0) return bits_f32(sign | f32_bits((float)f * 0x1p-24f));      /* zero and subnormals */
    if (e == 31) return bits_f32(sign | 0x7F800000u | (f << 13));            /* inf, NaN */
    return bits_f32(sign | ((e + 112u) << 23) | (f << 13));
}

inline uint16_t f32_to_lowp(float x, int dtype)
{
    uint32_t u = f32_bits(x);
    if (dtype == AH_BF16) {
        if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
        return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
    }
    const uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    u &= 0x7FFFFFFFu;
    if (u > 0x7F800000u) return (uint16_t)(sign | 0x7E00u);
    if (u >= 0x477FF000u) return (uint16_t)(sign | 0x7C00u); /* rounds to infinity */
    if (u < 0x38800000u) {                                   /* subnormal half: let one fp32 add round */
        const float a = bits_f32(u) + 0.5f;
        return (uint16_t)(sign | (uint16_t)(f32_bits(a) - 0x3F000000u));
    }
    u += 0xC8000000u + 0x0FFFu + ((u >> 13) & 1u);
    return (uint16_t)(sign | (uint16_t)(u >> 13));
}

/* ---------------------------------------------------------------- scalar update and norm */

inline void step_scalar(const uint16_t *g, uint16_t *q, float *p, float *m, float *v, size_t lo, size_t hi,
                        int dtype, const Consts &k)
{
    for (size_t i = lo; i < hi; ++i) {
        const double gd = (double)lowp_to_f32(g[i], dtype) * k.inv * k.coef;
        const double pd = (double)p[i];
        const double mn = k.b1 * (double)m[i] + k.omb1 * gd;
        const double vn = k.b2 * (double)v[i] + k.omb2 * (gd * gd);
        const double pn = pd - k.lr * ((mn / k.bc1) / (sqrt(vn / k.bc2) + k.eps) + k.wd * pd);
        m[i] = (float)mn;
        v[i] = (float)vn;
        p[i] = (float)pn;
        if (q) q[i] = f32_to_lowp((float)pn, dtype);
    }
}

inline double sumsq_scalar(const uint16_t *g, size_t lo, size_t hi, int dtype)
{
    double s = 0.0;
    for (size_t i = lo; i < hi; ++i) {
        const double x = (double)lowp_to_f32(g[i], dtype);
        s += x * x;
    }
    return s;
}

/* ---------------------------------------------------------------- AVX-512 (8 elements per step) */

#define AH_AVX512 __attribute__((target("avx512f,avx512dq,avx512bw,avx512vl,f16c,fma")))

/* a / b, correctly rounded, for a divisor b that is the same for every element, without a division
 * instruction: with y = RN(1 / b) computed once, q = RN(a y) is within one ulp of the quotient, the
 * residual r = a - b q is exact in a fused multiply-add, and RN(q + r y) is the correctly rounded
 * quotient (Markstein's theorem on division by fused multiply-add; it needs y within half an ulp of
 * 1 / b, which fails only for a divisor whose significand is all ones -- checked once per call by
 * recip_is_safe -- and no zero, infinity, NaN or subnormal a, for which the vector falls back to the
 * division instruction).  The two bias-correction quotients are two thirds of the divisions of the
 * update; a 512-bit division costs as much as a dozen multiplications. */
AH_AVX512 inline __m512d div_by_const(__m512d a, __m512d b, __m512d y)
{
    /* classes: QNaN 0x01, +0 0x02, -0 0x04, +inf 0x08, -inf 0x10, denormal 0x20, SNaN 0x80 */
    if (__builtin_expect(_mm512_fpclass_pd_mask(a, 0xBF) != 0, 0)) return _mm512_div_pd(a, b);
    const __m512d q = _mm512_mul_pd(a, y);
    const __m512d r = _mm512_fnmadd_pd(b, q, a);
    return _mm512_fmadd_pd(r, y, q);
}

AH_AVX512 inline __m512d load8_lowp(const uint16_t *g, int dtype)
{
    const __m128i h = _mm_loadu_si128(reinterpret_cast<const __m128i *>(g));
    const __m256 f = dtype == AH_BF16 ? _mm256_castsi256_ps(_mm256_slli_epi32(_mm256_cvtepu16_epi32(h), 16))
                                      : _mm256_cvtph_ps(h);
    return _mm512_cvtps_pd(f);
}

AH_AVX512 inline void store8_lowp(uint16_t *q, __m256 f, int dtype)
{
    __m128i h;
    if (dtype == AH_BF16) {
        const __m256i u = _mm256_castps_si256(f);
        const __m256i lsb = _mm256_and_si256(_mm256_srli_epi32(u, 16), _mm256_set1_epi32(1));
        const __m256i r = _mm256_srli_epi32(_mm256_add_epi32(_mm256_add_epi32(u, _mm256_set1_epi32(0x7FFF)), lsb), 16);
        const __m256i quiet = _mm256_or_si256(_mm256_srli_epi32(u, 16), _mm256_set1_epi32(0x40));
        const __mmask8 nan = _mm256_cmp_ps_mask(f, f, _CMP_UNORD_Q);
        h = _mm256_cvtepi32_epi16(_mm256_mask_blend_epi32(nan, r, quiet));
    } else {
        h = _mm256_cvtps_ph(f, _MM_FROUND_TO_NEAREST_INT | _MM_FROUND_NO_EXC);
    }
    _mm_storeu_si128(reinterpret_cast<__m128i *>(q), h);
}

/* Software prefetch distance in elements (8 KB of each fp32 stream).  One core's demand misses alone
 * do not keep enough lines in flight for five streams: on the 16 threads of the GPU machine's host the
 * update runs at 10.4 G parameters/s without prefetches, 10.9 / 11.4 / 11.7 / 11.8 / 11.3 / 11.0 with
 * 256 / 512 / 1024 / 2048 / 4096 / 8192 elements ahead.  A prefetch beyond the end of an array is harmless. */
constexpr size_t kPrefetch = 2048;

AH_AVX512 void step_avx512(const uint16_t *g, uint16_t *q, float *p, float *m, float *v, size_t lo, size_t hi,
                           int dtype, const Consts &k)
{
    const __m512d inv = _mm512_set1_pd(k.inv), coef = _mm512_set1_pd(k.coef), b1 = _mm512_set1_pd(k.b1),
                  b2 = _mm512_set1_pd(k.b2), omb1 = _mm512_set1_pd(k.omb1), omb2 = _mm512_set1_pd(k.omb2),
                  bc1 = _mm512_set1_pd(k.bc1), bc2 = _mm512_set1_pd(k.bc2), lr = _mm512_set1_pd(k.lr),
                  eps = _mm512_set1_pd(k.eps), wd = _mm512_set1_pd(k.wd), rbc1 = _mm512_set1_pd(k.rbc1),
                  rbc2 = _mm512_set1_pd(k.rbc2);
    const bool recip = k.recip_exact;
    size_t i = lo;
    for (; i + 8 <= hi; i += 8) {
        if ((i & 8) == 0) { /* once per 64-byte line of the fp32 streams: ask for the lines kPrefetch elements ahead */
            _mm_prefetch(reinterpret_cast<const char *>(p + i + kPrefetch), _MM_HINT_T0);
            _mm_prefetch(reinterpret_cast<const char *>(m + i + kPrefetch), _MM_HINT_T0);
            _mm_prefetch(reinterpret_cast<const char *>(v + i + kPrefetch), _MM_HINT_T0);
            if ((i & 16) == 0) _mm_prefetch(reinterpret_cast<const char *>(g + i + kPrefetch), _MM_HINT_T0);
        }
        const __m512d gd = _mm512_mul_pd(_mm512_mul_pd(load8_lowp(g + i, dtype), inv), coef);
        const __m512d pd = _mm512_cvtps_pd(_mm256_loadu_ps(p + i));
        const __m512d md = _mm512_cvtps_pd(_mm256_loadu_ps(m + i));
        const __m512d vd = _mm512_cvtps_pd(_mm256_loadu_ps(v + i));
        const __m512d mn = _mm512_add_pd(_mm512_mul_pd(b1, md), _mm512_mul_pd(omb1, gd));
        const __m512d vn = _mm512_add_pd(_mm512_mul_pd(b2, vd), _mm512_mul_pd(omb2, _mm512_mul_pd(gd, gd)));
        const __m512d vh = recip ? div_by_const(vn, bc2, rbc2) : _mm512_div_pd(vn, bc2);
        const __m512d mh = recip ? div_by_const(mn, bc1, rbc1) : _mm512_div_pd(mn, bc1);
        const __m512d den = _mm512_add_pd(_mm512_sqrt_pd(vh), eps);
        const __m512d upd = _mm512_div_pd(mh, den);
        const __m512d pn = _mm512_sub_pd(pd, _mm512_mul_pd(lr, _mm512_add_pd(upd, _mm512_mul_pd(wd, pd))));
        const __m256 pf = _mm512_cvtpd_ps(pn);
        _mm256_storeu_ps(m + i, _mm512_cvtpd_ps(mn));
        _mm256_storeu_ps(v + i, _mm512_cvtpd_ps(vn));
        _mm256_storeu_ps(p + i, pf);
        if (q) store8_lowp(q + i, pf, dtype);
    }
    step_scalar(g, q, p, m, v, i, hi, dtype, k);
}

AH_AVX512 double sumsq_avx512(const uint16_t *g, size_t lo, size_t hi, int dtype)
{
    __m512d a0 = _mm512_setzero_pd(), a1 = _mm512_setzero_pd();
    size_t i = lo;
    for (; i + 16 <= hi; i += 16) {
        const __m512d x0 = load8_lowp(g + i, dtype), x1 = load8_lowp(g + i + 8, dtype);
        a0 = _mm512_add_pd(a0, _mm512_mul_pd(x0, x0));
        a1 = _mm512_add_pd(a1, _mm512_mul_pd(x1, x1));
    }
    double lanes[8];
    _mm512_storeu_pd(lanes, _mm512_add_pd(a0, a1));
    double s = 0.0;
    for (double x : lanes) s += x;
    return s + sumsq_scalar(g, i, hi, dtype);
}

bool g_force_scalar = false;

bool have_avx512()
{
    if (g_force_scalar) return false;
    static const bool ok = __builtin_cpu_supports("avx512f") && __builtin_cpu_supports("avx512dq") &&
                           __builtin_cpu_supports("avx512bw") && __builtin_cpu_supports("avx512vl") &&
                           __builtin_cpu_supports("f16c") && __builtin_cpu_supports("fma");
    return ok;
}

/* ---------------------------------------------------------------- threading */

/* Cuts the concatenated element space of the chunks into n_threads contiguous slices of a multiple
 * of 16 elements each and runs fn(chunk index, lo, hi, thread) for every piece.  A piece starts
 * wherever its slice meets the chunk: with ragged chunk sizes that is any element, so fn must not
 * assume alignment (the vector paths use unaligned loads and stores). */
template <typename F>
void for_slices(const autohete_chunk *chunks, uint64_t n, int n_threads, F fn)
{
    uint64_t total = 0;
    for (uint64_t c = 0; c < n; ++c) total += chunks[c].numel;
    const uint64_t per = ((total + n_threads - 1) / n_threads + 15) / 16 * 16;
    auto work = [&](int t) {
        uint64_t begin = (uint64_t)t * per, end = std::min(total, begin + per), base = 0;
        for (uint64_t c = 0; c < n && base < end; ++c) {
            const uint64_t cn = chunks[c].numel;
            if (base + cn > begin) {
                const uint64_t lo = begin > base ? begin - base : 0, hi = std::min(cn, end - base);
                if (lo < hi) fn(c, (size_t)lo, (size_t)hi, t);
            }
            base += cn;
        }
    };
    std::vector<std::thread> pool;
    pool.reserve((size_t)n_threads);
    try {
        for (int t = 1; t < n_threads; ++t) pool.emplace_back(work, t);
    } catch (...) { /* could not start a thread: finish what was started, then report */
        for (std::thread &th : pool) th.join();
        throw;
    }
    work(0);
    for (std::thread &th : pool) th.join();
}

/* Is RN(1 / b) within half an ulp of 1 / b in the sense div_by_const needs?  Always, except for a
 * divisor whose significand is all ones; b must also be a normal number. */
bool recip_is_safe(double b)
{
    uint64_t u;
    memcpy(&u, &b, 8);
    const uint64_t frac = u & 0x000FFFFFFFFFFFFFull, e = (u >> 52) & 0x7FFull;
    return b > 0.0 && e != 0 && e != 0x7FF && frac != 0x000FFFFFFFFFFFFFull;
}

int check_host_args(const autohete_chunk *chunks, uint64_t n, int dtype, int n_threads, unsigned need)
{
    if ((n && !chunks) || (dtype != AH_BF16 && dtype != AH_FP16) || n_threads < 1 || n_threads > 1024)
        return AH_EINVAL;
    for (uint64_t c = 0; c < n; ++c) {
        const autohete_chunk &k = chunks[c];
        const void *ptr[5] = {k.grad, k.param_lp, k.master, k.exp_avg, k.exp_avg_sq};
        if (k.numel == 0) return AH_EINVAL;
        for (int i = 0; i < 5; ++i)
            if ((need >> i & 1u) && !ptr[i]) return AH_EINVAL;
    }
    return AH_OK;
}

}  // namespace

extern "C" {

int autohete_host_force_scalar(int on)
{
    g_force_scalar = on != 0;
    return AH_OK;
}

int autohete_host_grad_sumsq(const autohete_chunk *chunks, uint64_t n_chunks, int lowp_dtype, float loss_scale,
                             int n_threads, double *sumsq, uint32_t *found_inf)
{
    if (!sumsq || !found_inf || !(loss_scale > 0.0f) || !isfinite(loss_scale)) return AH_EINVAL;
    int rc = check_host_args(chunks, n_chunks, lowp_dtype, n_threads, 1u);
    if (rc != AH_OK) return rc;
    try {
        std::vector<double> part((size_t)n_threads, 0.0);
        const bool vec = have_avx512();
        for_slices(chunks, n_chunks, n_threads, [&](uint64_t c, size_t lo, size_t hi, int t) {
            const uint16_t *g = static_cast<const uint16_t *>(chunks[c].grad);
            part[(size_t)t] += vec ? sumsq_avx512(g, lo, hi, lowp_dtype) : sumsq_scalar(g, lo, hi, lowp_dtype);
        });
        double s = 0.0;
        for (double x : part) s += x; /* thread order: reproducible for a given n_threads */
        const double inv = 1.0 / (double)loss_scale;
        s = s * inv * inv;
        *sumsq = s;
        *found_inf = isfinite(s) ? 0u : 1u; /* fp64 cannot overflow on finite 16-bit inputs */
    } catch (...) {
        return AH_ENOMEM;
    }
    return AH_OK;
}

int autohete_host_adamw_step(const autohete_chunk *chunks, uint64_t n_chunks, int lowp_dtype, uint64_t step,
                             const autohete_hparams *hp, double sumsq, uint32_t found_inf, int n_threads)
{
    if (!hp || step == 0) return AH_EINVAL;
    auto nonneg = [](float x) { return isfinite(x) && x >= 0.0f; };
    if (!nonneg(hp->lr) || !nonneg(hp->eps) || !nonneg(hp->weight_decay) || !isfinite(hp->max_grad_norm) ||
        !(hp->beta1 >= 0.0f && hp->beta1 < 1.0f) || !(hp->beta2 >= 0.0f && hp->beta2 < 1.0f) ||
        !(hp->loss_scale > 0.0f) || !isfinite(hp->loss_scale))
        return AH_EINVAL;
    int rc = check_host_args(chunks, n_chunks, lowp_dtype, n_threads, 1u | 4u | 8u | 16u);
    if (rc != AH_OK) return rc;
    if (found_inf || !isfinite(sumsq)) return AH_OK; /* skip-on-overflow: nothing is touched */
    Consts k;
    k.inv = 1.0 / (double)hp->loss_scale;
    k.coef = 1.0;
    if (hp->max_grad_norm > 0.0f) {
        const double c = (double)hp->max_grad_norm / (sqrt(sumsq) + 1e-6);
        k.coef = c < 1.0 ? c : 1.0;
    }
    k.b1 = (double)hp->beta1;
    k.b2 = (double)hp->beta2;
    k.omb1 = 1.0 - k.b1;
    k.omb2 = 1.0 - k.b2;
    k.bc1 = 1.0 - pow(k.b1, (double)step);
    k.bc2 = 1.0 - pow(k.b2, (double)step);
    k.lr = (double)hp->lr;
    k.eps = (double)hp->eps;
    k.wd = (double)hp->weight_decay;
    k.rbc1 = 1.0 / k.bc1;
    k.rbc2 = 1.0 / k.bc2;
    k.recip_exact = recip_is_safe(k.bc1) && recip_is_safe(k.bc2);
    try {
        const bool vec = have_avx512();
        for_slices(chunks, n_chunks, n_threads, [&](uint64_t c, size_t lo, size_t hi, int) {
            const autohete_chunk &ch = chunks[c];
            const uint16_t *g = static_cast<const uint16_t *>(ch.grad);
            uint16_t *q = static_cast<uint16_t *>(ch.param_lp);
            if (vec) step_avx512(g, q, ch.master, ch.exp_avg, ch.exp_avg_sq, lo, hi, lowp_dtype, k);
            else step_scalar(g, q, ch.master, ch.exp_avg, ch.exp_avg_sq, lo, hi, lowp_dtype, k);
        });
    } catch (...) {
        return AH_ENOMEM;
    }
    return AH_OK;
}

}  // extern "C"
