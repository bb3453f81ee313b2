/*
 * autohete_kernels.hip -- the two streaming kernels of the chunked mixed-precision AdamW
 * update for gfx950 (MI355X), and their launchers.
 *
 *   grad_prep_kernel   2 B/element read.   Sum of squares of the raw 16-bit gradients in
 *                      fp64 (per lane -> wavefront shuffle -> LDS -> one partial per block ->
 *                      ticket counter; the last block to arrive folds the partials in index
 *                      order), finite check, loss-scale removal on the scalar result.
 *   adamw_step_kernel  14 B/element read + 14 B/element written.  Fused unscale, clip,
 *                      moments, bias correction, decoupled decay, fp32 and 16-bit write-back.
 *
 * Both are HBM-bound (about 0.7 flop/byte), so there is no MFMA here: the design goal is
 * that every byte moves once, in full-width coalesced vector accesses, with enough loads in
 * flight per CU.  Model data layout: section 2.1 of the paper (16-bit parameters and
 * gradients, fp32 momentum / variance / parameter copy).  The arithmetic of the update is
 * kept in fp64 (full rate on CDNA, hidden under the memory time) so that stored values are
 * the correctly rounded results of the rule stated in autohete.h.
 */
#include "autohete_internal.h"

namespace ah {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBF16 = 0, kFP16 = 1;

/* Pointers in the chunk table come out of memory as generic addresses; the streams are known
 * to be in global memory, so accesses are made through address-space-1 pointers (global_load /
 * global_store rather than flat_*). */
#define AH_GLOBAL __attribute__((address_space(1)))
template <typename V, typename T>
__device__ __forceinline__ AH_GLOBAL V *gptr(T *p)
{
    return (AH_GLOBAL V *)(p);
}
template <typename V, typename T>
__device__ __forceinline__ const AH_GLOBAL V *gptr(const T *p)
{
    return (const AH_GLOBAL V *)(p);
}

template <bool NT, typename T>
__device__ __forceinline__ T ld(const AH_GLOBAL T *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT, typename T>
__device__ __forceinline__ void st(AH_GLOBAL T *p, T v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

/* 16-bit <-> fp32.  bf16 is the upper half of an fp32 word; fp16 uses the hardware converts.
 * Both encodes round to nearest even and keep subnormals. */
template <int DT>
__device__ __forceinline__ float lowp_to_f32(uint32_t h16)
{
    if constexpr (DT == kBF16) return __uint_as_float(h16 << 16);
    else return (float)__builtin_bit_cast(_Float16, (uint16_t)h16);
}
template <int DT>
__device__ __forceinline__ uint32_t f32_to_lowp(float x)
{
    if constexpr (DT == kBF16) return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)x);
    else return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)x);
}
/* Both halves of one 32-bit word holding two 16-bit values. */
template <int DT>
__device__ __forceinline__ void unpack2(uint32_t w, float &lo, float &hi)
{
    if constexpr (DT == kBF16) {
        lo = __uint_as_float(w << 16);
        hi = __uint_as_float(w & 0xFFFF0000u);
    } else {
        lo = lowp_to_f32<DT>(w & 0xFFFFu);
        hi = lowp_to_f32<DT>(w >> 16);
    }
}

/* ------------------------------------------------------------------------------------- */
/* One element of the update.  Each written operation is one IEEE fp64 operation (no      */
/* contraction), in the order of the rule in autohete.h.                                  */
/* ------------------------------------------------------------------------------------- */
template <int MODE>
__device__ __forceinline__ void adamw_elem(float gf, float &p, float &m, float &v, const StepConsts &k,
                                           double coef)
{
#pragma clang fp contract(off)
    const double g = (double)gf * k.inv_scale * coef;
    const double mn = k.b1 * (double)m + k.omb1 * g;
    const double vn = k.b2 * (double)v + k.omb2 * (g * g);
    const double pd = (double)p;
    double upd;
    if constexpr (MODE == 1) {
        upd = (mn / k.bc1) / (sqrt(vn / k.bc2) + k.eps);
    } else {
        /* The quotient only has to be good to ~1e-7 relative: it is scaled by lr before it
         * meets p.  fp32 root and division are correctly rounded. */
        const float mh = (float)(mn * k.rbc1);
        const float vh = (float)(vn * k.rbc2);
        upd = (double)(mh / (sqrtf(vh) + (float)k.eps));
    }
    const double pn = pd - k.lr * (upd + k.wd * pd);
    m = (float)mn;
    v = (float)vn;
    p = (float)pn;
}

template <int DT, int U, int MODE, bool NT>
__device__ __forceinline__ void step_full_tile(const DevChunk &ch, uint64_t e0, const StepConsts &k, double coef)
{
    const uint32_t lane_off = threadIdx.x * kStepVec;
    u32x2 g[U];
    f32x4 p[U], m[U], v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint64_t off = e0 + (uint64_t)u * (kThreads * kStepVec) + lane_off;
        g[u] = ld<NT>(gptr<u32x2>(ch.grad + off));
        p[u] = ld<NT>(gptr<f32x4>((const float *)ch.master + off));
        m[u] = ld<NT>(gptr<f32x4>((const float *)ch.exp_avg + off));
        v[u] = ld<NT>(gptr<f32x4>((const float *)ch.exp_avg_sq + off));
    }
    /* Keep every load of the tile ahead of the arithmetic: 4*U requests in flight per lane. */
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint64_t off = e0 + (uint64_t)u * (kThreads * kStepVec) + lane_off;
        float gf[4], pp[4], mm[4], vv[4];
        unpack2<DT>(g[u].x, gf[0], gf[1]);
        unpack2<DT>(g[u].y, gf[2], gf[3]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            pp[j] = p[u][j];
            mm[j] = m[u][j];
            vv[j] = v[u][j];
            adamw_elem<MODE>(gf[j], pp[j], mm[j], vv[j], k, coef);
        }
        u32x2 o16;
        o16.x = f32_to_lowp<DT>(pp[0]) | (f32_to_lowp<DT>(pp[1]) << 16);
        o16.y = f32_to_lowp<DT>(pp[2]) | (f32_to_lowp<DT>(pp[3]) << 16);
        f32x4 po = {pp[0], pp[1], pp[2], pp[3]}, mo = {mm[0], mm[1], mm[2], mm[3]},
              vo = {vv[0], vv[1], vv[2], vv[3]};
        st<NT>(gptr<f32x4>(ch.master + off), po);
        st<NT>(gptr<f32x4>(ch.exp_avg + off), mo);
        st<NT>(gptr<f32x4>(ch.exp_avg_sq + off), vo);
        st<NT>(gptr<u32x2>(ch.param_lp + off), o16);
    }
}

/* The last, partial tile of a chunk: element-wise, bounds-checked. */
template <int DT, int U, int MODE>
__device__ __forceinline__ void step_tail_tile(const DevChunk &ch, uint64_t e0, const StepConsts &k, double coef)
{
    const uint64_t full = e0 + (uint64_t)U * (kThreads * kStepVec);
    const uint64_t end = full < ch.numel ? full : ch.numel;
    AH_GLOBAL float *master = gptr<float>(ch.master), *exp_avg = gptr<float>(ch.exp_avg),
                    *exp_avg_sq = gptr<float>(ch.exp_avg_sq);
    const AH_GLOBAL uint16_t *grad = gptr<uint16_t>(ch.grad);
    AH_GLOBAL uint16_t *param_lp = gptr<uint16_t>(ch.param_lp);
    for (uint64_t i = e0 + threadIdx.x; i < end; i += kThreads) {
        float p = master[i], m = exp_avg[i], v = exp_avg_sq[i];
        adamw_elem<MODE>(lowp_to_f32<DT>(grad[i]), p, m, v, k, coef);
        master[i] = p;
        exp_avg[i] = m;
        exp_avg_sq[i] = v;
        param_lp[i] = (uint16_t)f32_to_lowp<DT>(p);
    }
}

template <int DT, int U, int MODE, bool NT>
__global__ void __launch_bounds__(kThreads)
adamw_step_kernel(const DevChunk *__restrict__ tab, uint32_t n_chunks, uint64_t total_tiles,
                  const GradResult *__restrict__ res, StepConsts k)
{
    /* Skip-on-overflow: leave before the first load; no stream is touched. */
    if (res->found_inf) return;
    double coef = 1.0;
    if (k.max_norm > 0.0) {
        const double c = k.max_norm / (sqrt(res->sumsq) + 1e-6);
        coef = c < 1.0 ? c : 1.0;
    }
    constexpr uint32_t kTile = kThreads * kStepVec * U;
    uint32_t c = 0;
    /* Grid-stride over tiles: at any moment the resident blocks cover one contiguous window
     * of every stream.  The chunk cursor only moves forward (wave-uniform, scalar). */
    for (uint64_t w = blockIdx.x; w < total_tiles; w += gridDim.x) {
        while (w >= tab[c + 1].tile_begin) ++c; /* sentinel entry n_chunks ends the search */
        const DevChunk ch = tab[c];
        const uint64_t e0 = (w - ch.tile_begin) * kTile;
        if (e0 + kTile <= ch.numel) step_full_tile<DT, U, MODE, NT>(ch, e0, k, coef);
        else step_tail_tile<DT, U, MODE>(ch, e0, k, coef);
    }
    (void)n_chunks;
}

/* ------------------------------------------------------------------------------------- */
/* Gradient preparation                                                                    */
/* ------------------------------------------------------------------------------------- */

/* Sum over the block in a fixed order: lanes by shuffle-down tree, then waves 0..3. */
__device__ __forceinline__ double block_sum(double x, double *lds4)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_down(x, o, 64);
    if ((threadIdx.x & 63) == 0) lds4[threadIdx.x >> 6] = x;
    __syncthreads();
    const double s = ((lds4[0] + lds4[1]) + lds4[2]) + lds4[3];
    __syncthreads();
    return s;
}

template <int DT>
__global__ void __launch_bounds__(kThreads)
grad_prep_kernel(const DevChunk *__restrict__ tab, uint32_t n_chunks, uint64_t total_tiles, double inv_scale,
                 double extra_sumsq, double *partials, uint32_t *ticket, GradResult *res)
{
    constexpr int U = kPrepUnroll;
    constexpr uint32_t kSub = kThreads * kPrepVec;
    constexpr uint32_t kTile = kSub * U;
    __shared__ double lds4[4];
    __shared__ uint32_t is_last;

    /* Squares of the RAW gradients are summed; the loss scale is removed from the scalar at
     * the end.  fp64 cannot overflow on finite 16-bit inputs, so a non-finite total means a
     * non-finite gradient: the finite check costs no extra instruction per element. */
    double acc0 = 0.0, acc1 = 0.0;
    uint32_t c = 0;
    for (uint64_t w = blockIdx.x; w < total_tiles; w += gridDim.x) {
        while (w >= tab[c + 1].tile_begin) ++c;
        const AH_GLOBAL uint16_t *grad = gptr<uint16_t>(tab[c].grad);
        const uint64_t numel = tab[c].numel;
        const uint64_t e0 = (w - tab[c].tile_begin) * kTile;
        if (e0 + kTile <= numel) {
            u32x4 g[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                g[u] = ld<true>((const AH_GLOBAL u32x4 *)(grad + e0 + (uint64_t)u * kSub + threadIdx.x * kPrepVec));
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float lo, hi;
                    unpack2<DT>(g[u][j], lo, hi);
                    acc0 += (double)lo * (double)lo;
                    acc1 += (double)hi * (double)hi;
                }
            }
        } else {
            const uint64_t end = e0 + kTile < numel ? e0 + kTile : numel;
            for (uint64_t i = e0 + threadIdx.x; i < end; i += kThreads) {
                const double x = (double)lowp_to_f32<DT>(grad[i]);
                acc0 += x * x;
            }
        }
    }
    const double bsum = block_sum(acc0 + acc1, lds4);

    /* Single pass across blocks: publish the partial, take a ticket; the last block folds. */
    if (threadIdx.x == 0) {
        __hip_atomic_store(&partials[blockIdx.x], bsum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t t = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        is_last = (t == gridDim.x - 1) ? 1u : 0u;
    }
    __syncthreads();
    if (!is_last) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    double s = 0.0;
    for (uint32_t i = threadIdx.x; i < gridDim.x; i += kThreads)
        s += __hip_atomic_load(&partials[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s = block_sum(s, lds4);
    if (threadIdx.x == 0) {
        const double total = s * inv_scale * inv_scale + extra_sumsq;
        const bool bad = !__builtin_isfinite(total);
        res->sumsq = total;
        res->norm = bad ? __builtin_nanf("") : (float)sqrt(total);
        res->found_inf = bad ? 1u : 0u;
        __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); /* re-arm */
    }
    (void)n_chunks;
}

__global__ void set_result_kernel(GradResult *res, double sumsq, uint32_t found_inf)
{
    const bool bad = found_inf || !__builtin_isfinite(sumsq);
    res->sumsq = sumsq;
    res->norm = bad ? __builtin_nanf("") : (float)sqrt(sumsq);
    res->found_inf = bad ? 1u : 0u;
}

/* ------------------------------------------------------------------------------------- */
/* Launchers                                                                               */
/* ------------------------------------------------------------------------------------- */

typedef void (*step_fn)(const DevChunk *, uint32_t, uint64_t, const GradResult *, StepConsts);

template <int DT>
static step_fn pick_step(StepVariant s)
{
#define AH_CASE(U, M, N) \
    if (s.unroll == U && s.mode == M && s.nt == N) return adamw_step_kernel<DT, U, M, (N != 0)>;
    AH_CASE(1, 0, 0) AH_CASE(2, 0, 0) AH_CASE(4, 0, 0)
    AH_CASE(1, 1, 0) AH_CASE(2, 1, 0) AH_CASE(4, 1, 0)
    AH_CASE(1, 0, 1) AH_CASE(2, 0, 1) AH_CASE(4, 0, 1)
    AH_CASE(1, 1, 1) AH_CASE(2, 1, 1) AH_CASE(4, 1, 1)
#undef AH_CASE
    return nullptr;
}

static step_fn pick_step(int dtype, StepVariant s)
{
    return dtype == kFP16 ? pick_step<kFP16>(s) : pick_step<kBF16>(s);
}

hipError_t launch_step(int dtype, StepVariant var, unsigned blocks, hipStream_t stream, const DevChunk *tab,
                       uint32_t n_chunks, uint64_t total_tiles, const GradResult *res, const StepConsts &k)
{
    step_fn fn = pick_step(dtype, var);
    if (!fn) return hipErrorInvalidValue;
    if (total_tiles == 0) return hipSuccess;
    hipLaunchKernelGGL(fn, dim3(blocks), dim3(kThreads), 0, stream, tab, n_chunks, total_tiles, res, k);
    return hipGetLastError();
}

hipError_t launch_prep(int dtype, unsigned blocks, hipStream_t stream, const DevChunk *tab, uint32_t n_chunks,
                       uint64_t total_tiles, double inv_scale, double extra_sumsq, double *partials,
                       uint32_t *ticket, GradResult *res)
{
    if (blocks == 0) blocks = 1; /* no chunks: one block still publishes S = extra_sumsq */
    if (dtype == kFP16)
        hipLaunchKernelGGL(grad_prep_kernel<kFP16>, dim3(blocks), dim3(kThreads), 0, stream, tab, n_chunks,
                           total_tiles, inv_scale, extra_sumsq, partials, ticket, res);
    else
        hipLaunchKernelGGL(grad_prep_kernel<kBF16>, dim3(blocks), dim3(kThreads), 0, stream, tab, n_chunks,
                           total_tiles, inv_scale, extra_sumsq, partials, ticket, res);
    return hipGetLastError();
}

hipError_t launch_set_result(hipStream_t stream, GradResult *res, double sumsq, uint32_t found_inf)
{
    hipLaunchKernelGGL(set_result_kernel, dim3(1), dim3(1), 0, stream, res, sumsq, found_inf);
    return hipGetLastError();
}

int step_occupancy(int dtype, StepVariant var)
{
    step_fn fn = pick_step(dtype, var);
    int n = 0;
    if (!fn || hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, fn, kThreads, 0) != hipSuccess) return -1;
    return n;
}

int prep_occupancy(int dtype)
{
    int n = 0;
    hipError_t e = dtype == kFP16
                       ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, grad_prep_kernel<kFP16>, kThreads, 0)
                       : hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, grad_prep_kernel<kBF16>, kThreads, 0);
    return e == hipSuccess ? n : -1;
}

}  // namespace ah
