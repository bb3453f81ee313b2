/*
 * autohete_kernels.hip -- the streaming kernels of the chunked mixed-precision AdamW update for
 * gfx950 (MI355X), and their launchers.
 *
 *   grad_prep_kernel         2 B/element read.  Sum of squares of the raw 16-bit gradients in
 *                            fp64 (per lane -> wavefront shuffle -> LDS -> one partial per block ->
 *                            ticket counter; the last block to arrive folds the partials in index
 *                            order), finite check, loss-scale removal on the scalar result.
 *   adamw_step_kernel        14 B/element read + 14 B/element written.  Fused unscale, clip,
 *                            moments, bias correction, decoupled decay, fp32 and 16-bit write-back
 *                            (or without the 16-bit write-back: 26 B/element).
 *   cast_params_kernel       4 B read + 2 B written: 16-bit parameters from the fp32 copy on demand.
 *   adamw_step_carry_kernel  the update plus the squares of the gradients it reads, for the norm of
 *                            the next iteration (per-block stepping); fold_partials_kernel sums them.
 *
 * All are HBM-bound (about 0.7 flop/byte), so there is no MFMA here: the design goal is that
 * every byte moves once, in full-width coalesced vector accesses, with the right amount of loads
 * in flight per CU.  Model data layout: section 2.1 of the paper (16-bit parameters and
 * gradients, fp32 momentum / variance / parameter copy).  The arithmetic of the update is
 * kept in fp64 (full rate on CDNA, hidden under the memory time) so that stored values are
 * the correctly rounded results of the rule stated in autohete.h.
 */
#include <algorithm>
#include <mutex>

#include "autohete_internal.h"

namespace ah {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
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

/* Streaming store of the update kernels: non-temporal AND system-scope write-through
 * ("sc1 nt").  Measured against every combination of the sc0/sc1/nt bits on this access
 * pattern, stores with sc1+nt are ~1 % faster than nt alone (and nt alone ~13 % faster than
 * plain stores when the loads are nt); the load policy makes no difference beyond nt.  The
 * compiler has no builtin for this combination on vector types, hence the inline assembly; the
 * stored lines are never read again by this kernel, so no wait is needed after them.
 * The trailing s_nop supplies, by hand, the wait states the ISA requires between a VMEM store of
 * more than 64 bits and a VALU write to its data registers: the compiler inserts them for its own
 * stores but cannot see into an asm statement.  gfx940 and later need TWO wait states there
 * ("s_nop 1"); with one, a wave now and then stored a later value of the register instead --
 * seen as a 16-bit intermediate of the parameter packing in 16 elements of the first moment. */
template <typename T>
__device__ __forceinline__ void st_stream(AH_GLOBAL T *p, T v)
{
    static_assert(sizeof(T) == 16 || sizeof(T) == 8 || sizeof(T) == 4 || sizeof(T) == 2, "store width");
    if constexpr (sizeof(T) == 16) asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
    else if constexpr (sizeof(T) == 8) asm volatile("global_store_dwordx2 %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
    else if constexpr (sizeof(T) == 4) asm volatile("global_store_dword %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
    else asm volatile("global_store_short %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p), "v"((uint32_t)v) : "memory");
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
/* MODE 0: root and quotient by Newton iteration in fp64 from the hardware's reciprocal   */
/*         (square-root) estimates -- a few ulp of fp64, far below one fp32 rounding.      */
/* MODE 1: correctly rounded fp64 root and divisions (reference variant, more ALU work).   */
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
        const double vh = vn * k.rbc2, mh = mn * k.rbc1;
        /* sqrt(vh): y ~ 1/sqrt(vh) from v_rsq_f64 (about 2^-23 relative), s = vh*y, then two
         * steps s <- s + (vh - s*s) * y/2, each squaring the error.  vh = 0 gives s = 0. */
        const double y = vh > 0.0 ? __builtin_amdgcn_rsq(vh) : 0.0;
        const double hy = 0.5 * y;
        double s = vh * y;
        s = __builtin_fma(__builtin_fma(-s, s, vh), hy, s);
        s = __builtin_fma(__builtin_fma(-s, s, vh), hy, s);
        /* 1/den: q from v_rcp_f64, two steps q <- q + q*(1 - den*q). */
        const double den = s + k.eps;
        const double q0 = __builtin_amdgcn_rcp(den);
        double q = __builtin_fma(q0, __builtin_fma(-den, q0, 1.0), q0);
        q = __builtin_fma(q, __builtin_fma(-den, q, 1.0), q);
        /* The iterations turn three reachable states into NaN where the exact operations do not:
         * a second moment that overflowed to +inf (a huge but finite gradient, no clipping; then
         * s = inf * 0), and den = 0 (eps = 0, no second moment yet) or den = +inf.  One class test
         * per element (den is NaN, +-inf or +-0), and only a wave that sees such an element takes
         * the branch: there the root of +inf is +inf and the hardware's reciprocal of 0 or inf is
         * already exact. */
        const bool odd = __builtin_amdgcn_class(den, 0x267);
        if (__builtin_amdgcn_ballot_w64(odd) != 0) {
            asm volatile("" ::: "memory"); /* keeps this a branch: as straight-line selects it costs 0.7 % */
            const double s_exact = vh < __builtin_huge_val() ? s : vh;
            q = odd ? __builtin_amdgcn_rcp(s_exact + k.eps) : q;
        }
        upd = mh * q;
    }
    const double pn = pd - k.lr * (upd + k.wd * pd);
    m = (float)mn;
    v = (float)vn;
    p = (float)pn;
}

/* Clip coefficient min(1, max_norm / (norm + 1e-6)); 1 when clipping is off. */
__device__ __forceinline__ double clip_coef(double max_norm, double norm)
{
    if (!(max_norm > 0.0)) return 1.0;
    const double c = max_norm / (norm + 1e-6);
    return c < 1.0 ? c : 1.0;
}

template <int VEC> struct VecTypes;
template <> struct VecTypes<4> { typedef f32x4 f32; typedef u32x2 lowp; };
template <> struct VecTypes<2> { typedef f32x2 f32; typedef uint32_t lowp; };
template <> struct VecTypes<1> { typedef float f32; typedef uint16_t lowp; };

template <int DT, int VEC>
__device__ __forceinline__ void unpack_lowp(typename VecTypes<VEC>::lowp raw, float *gf)
{
    if constexpr (VEC == 4) {
        unpack2<DT>(raw.x, gf[0], gf[1]);
        unpack2<DT>(raw.y, gf[2], gf[3]);
    } else if constexpr (VEC == 2) {
        unpack2<DT>(raw, gf[0], gf[1]);
    } else {
        gf[0] = lowp_to_f32<DT>(raw);
    }
}
template <int DT, int VEC>
__device__ __forceinline__ typename VecTypes<VEC>::lowp pack_lowp(const float *pp)
{
    if constexpr (VEC == 4) {
        u32x2 o;
        o.x = f32_to_lowp<DT>(pp[0]) | (f32_to_lowp<DT>(pp[1]) << 16);
        o.y = f32_to_lowp<DT>(pp[2]) | (f32_to_lowp<DT>(pp[3]) << 16);
        return o;
    } else if constexpr (VEC == 2) {
        return f32_to_lowp<DT>(pp[0]) | (f32_to_lowp<DT>(pp[1]) << 16);
    } else {
        return (uint16_t)f32_to_lowp<DT>(pp[0]);
    }
}
template <int VEC>
__device__ __forceinline__ void split(const typename VecTypes<VEC>::f32 &x, float *out)
{
    if constexpr (VEC == 1) out[0] = x;
    else
#pragma unroll
        for (int j = 0; j < VEC; ++j) out[j] = x[j];
}
template <int VEC>
__device__ __forceinline__ typename VecTypes<VEC>::f32 join(const float *in)
{
    if constexpr (VEC == 1) return in[0];
    else {
        typename VecTypes<VEC>::f32 r;
#pragma unroll
        for (int j = 0; j < VEC; ++j) r[j] = in[j];
        return r;
    }
}

/*
 * The update kernel.  No loop: one thread block per tile of BS*VEC elements, blockIdx.y = the
 * chunk (row of the table), blockIdx.x = the tile inside it.  The hardware dispatches blocks
 * in order, so the blocks in flight always cover one narrow, advancing window of each of the
 * five streams -- which is what keeps HBM pages open; a persistent grid-stride loop lets waves
 * drift apart and measured 10-20 % slower.  The number of blocks resident per CU is capped by
 * the launcher (through the dynamic LDS size): about 30 KB of loads in flight per CU is the
 * measured optimum, more in flight widens the window and costs bandwidth.
 * All accesses are non-temporal: every byte is touched exactly once per step.
 * WB = false leaves out the 16-bit write-back (26 B/element): the variant for blocks whose
 * 16-bit parameters are only materialised on demand (cast_params_kernel; paper section 3.2.2,
 * footnote on GPU-resident optimizer states).
 */
template <int DT, int VEC, int BS, int MODE, bool WB>
__device__ __forceinline__ void step_tile(const GradResult &r, const DevChunk &ch, const StepConsts &k, uint32_t tile)
{
    const uint64_t off = (uint64_t)tile * (BS * VEC) + threadIdx.x * VEC;
    /* Skip-on-overflow: leave before the first load, no stream is touched.  Also leave if this
     * tile lies beyond the chunk (grid.x is the largest tile count of the launch group). */
    if (r.found_inf | (uint32_t)(off >= ch.numel)) return;
    typedef typename VecTypes<VEC>::f32 fvec;
    typedef typename VecTypes<VEC>::lowp hvec;
    if (off + VEC <= ch.numel) {
        const hvec graw = ld<true>(gptr<hvec>(ch.grad + off));
        const fvec pv = ld<true>(gptr<fvec>((const float *)ch.master + off));
        const fvec mv = ld<true>(gptr<fvec>((const float *)ch.exp_avg + off));
        const fvec vv = ld<true>(gptr<fvec>((const float *)ch.exp_avg_sq + off));
        __builtin_amdgcn_sched_barrier(0); /* loads first; the clip factor is computed under them */
        const double coef = clip_coef(k.max_norm, r.norm_d);
        float gf[VEC], pp[VEC], mm[VEC], vs[VEC];
        unpack_lowp<DT, VEC>(graw, gf);
        split<VEC>(pv, pp);
        split<VEC>(mv, mm);
        split<VEC>(vv, vs);
#pragma unroll
        for (int j = 0; j < VEC; ++j) adamw_elem<MODE>(gf[j], pp[j], mm[j], vs[j], k, coef);
        st_stream(gptr<fvec>(ch.master + off), join<VEC>(pp));
        st_stream(gptr<fvec>(ch.exp_avg + off), join<VEC>(mm));
        st_stream(gptr<fvec>(ch.exp_avg_sq + off), join<VEC>(vs));
        if constexpr (WB) st_stream(gptr<hvec>(ch.param_lp + off), pack_lowp<DT, VEC>(pp));
    } else {
        /* ragged end of a chunk: fewer than VEC elements left for this lane */
        const double coef = clip_coef(k.max_norm, r.norm_d);
        for (uint64_t i = off; i < ch.numel; ++i) {
            float p = gptr<float>(ch.master)[i], m = gptr<float>(ch.exp_avg)[i], v = gptr<float>(ch.exp_avg_sq)[i];
            adamw_elem<MODE>(lowp_to_f32<DT>(gptr<uint16_t>(ch.grad)[i]), p, m, v, k, coef);
            gptr<float>(ch.master)[i] = p;
            gptr<float>(ch.exp_avg)[i] = m;
            gptr<float>(ch.exp_avg_sq)[i] = v;
            if constexpr (WB) gptr<uint16_t>(ch.param_lp)[i] = (uint16_t)f32_to_lowp<DT>(p);
        }
    }
}

template <int DT, int VEC, int BS, int MODE, bool WB>
__global__ void __launch_bounds__(BS)
adamw_step_kernel(const DevChunk *__restrict__ tab, const GradResult *__restrict__ res, StepConsts k)
{
    /* Both scalar fetches (the 32-byte result, the 64-byte table row) are issued together and
     * feed ONE exit test, so a wave pays two dependent scalar round trips (kernel arguments,
     * then these) before its vector loads instead of six. */
    const GradResult r = *res;
    const DevChunk ch = tab[blockIdx.y];
    step_tile<DT, VEC, BS, MODE, WB>(r, ch, k, blockIdx.x);
}

/* Sum of x over the 64 lanes of a wavefront, returned in every lane, in a fixed order and
 * without LDS traffic: four butterfly steps inside each row of 16 lanes through DPP lane
 * permutations (neighbour, pair, mirrored half-row, mirrored row), then the four row sums are
 * read as scalars and added in row order. */
template <int CTRL>
__device__ __forceinline__ double dpp_move(double x)
{
    const uint64_t b = __builtin_bit_cast(uint64_t, x);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_mov_dpp((int)(uint32_t)b, CTRL, 0xF, 0xF, true);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_mov_dpp((int)(uint32_t)(b >> 32), CTRL, 0xF, 0xF, true);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ double lane_value(double x, int lane)
{
    const uint64_t b = __builtin_bit_cast(uint64_t, x);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b, lane);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(b >> 32), lane);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ double wave_sum(double x)
{
    x += dpp_move<0xB1>(x);  /* quad_perm [1,0,3,2]: lane ^ 1 */
    x += dpp_move<0x4E>(x);  /* quad_perm [2,3,0,1]: lane ^ 2 */
    x += dpp_move<0x141>(x); /* row_half_mirror: the other quad of the 8 */
    x += dpp_move<0x140>(x); /* row_mirror: the other half of the 16 */
    return ((lane_value(x, 0) + lane_value(x, 16)) + lane_value(x, 32)) + lane_value(x, 48);
}

/*
 * The update kernel that also carries the gradient norm forward: the same update, clipped with
 * the norm in `res` (gathered earlier), while the squares of the gradients it reads anyway are
 * summed for the NEXT norm -- 28 B/element where grad_prep + adamw_step move 30.  Used when
 * blocks are stepped as their gradients appear (paper section 3.2.2, footnote to Eq. 5), where a
 * block's update cannot wait for the norm over gradients that do not exist yet.
 * Every wavefront leaves one fp64 partial at a slot fixed by its position in the launch:
 * slot = slot_base + (tile_begin of the row + blockIdx.x) * waves per block + wave.
 * fold_partials_kernel later sums the slots in a fixed order, so the sum is reproducible.  On
 * skip (res->found_inf) the streams are left alone but the squares are still gathered.
 */
template <int DT, int VEC, int BS, int MODE>
__device__ __forceinline__ void carry_tile(const GradResult &r, const DevChunk &ch, const StepConsts &k, uint32_t tile,
                                           double *__restrict__ wave_partials, uint64_t slot_base)
{
    const uint64_t tile0 = (uint64_t)tile * (BS * VEC);
    /* A whole block beyond the chunk owns no slot and leaves.  The flag (0 or 1) takes part in the
     * test only so that the result is fetched together with the table row, ahead of the branch,
     * as in adamw_step_kernel: one dependent scalar round trip fewer before the vector loads. */
    if ((uint32_t)(tile0 >= ch.numel) | (r.found_inf >> 1)) return;
    const uint64_t off = tile0 + threadIdx.x * VEC;
    typedef typename VecTypes<VEC>::f32 fvec;
    typedef typename VecTypes<VEC>::lowp hvec;
    double sq = 0.0;
    if (!r.found_inf && off + VEC <= ch.numel) {
        const hvec graw = ld<true>(gptr<hvec>(ch.grad + off));
        const fvec pv = ld<true>(gptr<fvec>((const float *)ch.master + off));
        const fvec mv = ld<true>(gptr<fvec>((const float *)ch.exp_avg + off));
        const fvec vv = ld<true>(gptr<fvec>((const float *)ch.exp_avg_sq + off));
        __builtin_amdgcn_sched_barrier(0);
        const double coef = clip_coef(k.max_norm, r.norm_d);
        float gf[VEC], pp[VEC], mm[VEC], vs[VEC];
        unpack_lowp<DT, VEC>(graw, gf);
        split<VEC>(pv, pp);
        split<VEC>(mv, mm);
        split<VEC>(vv, vs);
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            sq += (double)gf[j] * (double)gf[j];
            adamw_elem<MODE>(gf[j], pp[j], mm[j], vs[j], k, coef);
        }
        st_stream(gptr<fvec>(ch.master + off), join<VEC>(pp));
        st_stream(gptr<fvec>(ch.exp_avg + off), join<VEC>(mm));
        st_stream(gptr<fvec>(ch.exp_avg_sq + off), join<VEC>(vs));
        st_stream(gptr<hvec>(ch.param_lp + off), pack_lowp<DT, VEC>(pp));
    } else if (off < ch.numel) {
        /* element by element: the ragged end of a chunk, and every lane of a skipped step (which
         * only gathers squares; kept apart from the path above so that its gradient load is not
         * merged with that one and waited for ahead of the other three) */
        const double coef = clip_coef(k.max_norm, r.norm_d);
        const uint64_t end = off + VEC < ch.numel ? off + VEC : ch.numel;
        for (uint64_t i = off; i < end; ++i) {
            const float g = lowp_to_f32<DT>(gptr<uint16_t>(ch.grad)[i]);
            sq += (double)g * (double)g;
            if (r.found_inf) continue;
            float p = gptr<float>(ch.master)[i], m = gptr<float>(ch.exp_avg)[i], v = gptr<float>(ch.exp_avg_sq)[i];
            adamw_elem<MODE>(g, p, m, v, k, coef);
            gptr<float>(ch.master)[i] = p;
            gptr<float>(ch.exp_avg)[i] = m;
            gptr<float>(ch.exp_avg_sq)[i] = v;
            gptr<uint16_t>(ch.param_lp)[i] = (uint16_t)f32_to_lowp<DT>(p);
        }
    }
    /* all 64 lanes of every wave of the block arrive here (lanes beyond the chunk carry 0) */
    sq = wave_sum(sq);
    if ((threadIdx.x & 63) == 0)
        wave_partials[slot_base + (ch.tile_begin + tile) * (BS / 64) + (threadIdx.x >> 6)] = sq;
}

template <int DT, int VEC, int BS, int MODE>
__global__ void __launch_bounds__(BS)
adamw_step_carry_kernel(const DevChunk *__restrict__ tab, const GradResult *__restrict__ res, StepConsts k,
                        double *__restrict__ wave_partials, uint64_t slot_base)
{
    const GradResult r = *res;
    const DevChunk ch = tab[blockIdx.y];
    carry_tile<DT, VEC, BS, MODE>(r, ch, k, blockIdx.x, wave_partials, slot_base);
}

/*
 * On-demand materialisation of the 16-bit parameters from the fp32 master copy (paper section
 * 3.2.2, footnote: blocks whose optimizer states stay on the GPU keep no 16-bit parameters; they
 * are converted from the fp32 ones just before the block's forward / backward pass and released
 * afterwards).  4 B read + 2 B written per element, round-to-nearest-even.  One wavefront per
 * 512-element tile: lane l converts elements [4l, 4l+4) and [256+4l, 256+4l+4), so both loads
 * and both stores of a wave are contiguous.
 */
template <int DT>
__global__ void __launch_bounds__(64) cast_params_kernel(const DevChunk *__restrict__ tab)
{
    const DevChunk ch = tab[blockIdx.y];
    const uint64_t base = (uint64_t)blockIdx.x * 512 + threadIdx.x * 4;
    if (base >= ch.numel) return;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const uint64_t off = base + (uint64_t)h * 256;
        if (off + 4 <= ch.numel) {
            const f32x4 pv = ld<true>(gptr<f32x4>((const float *)ch.master + off));
            float pp[4] = {pv[0], pv[1], pv[2], pv[3]};
            st_stream(gptr<u32x2>(ch.param_lp + off), pack_lowp<DT, 4>(pp));
        } else {
            for (uint64_t i = off; i < ch.numel; ++i)
                gptr<uint16_t>(ch.param_lp)[i] = (uint16_t)f32_to_lowp<DT>(gptr<float>(ch.master)[i]);
        }
    }
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

/* Final scalar step of a norm pass (one thread): S = raw_sum / loss_scale^2 + extra, folded into
 * the result already there when `accumulate` (gradient norm gathered block by block while the
 * backward pass still runs); a non-finite S or a carried flag means skip. */
__device__ __forceinline__ void publish_total(GradResult *res, double raw_sum, double inv_scale, double extra_sumsq,
                                              uint32_t accumulate)
{
    double total = raw_sum * inv_scale * inv_scale + extra_sumsq;
    bool carried_flag = false;
    if (accumulate) {
        total += res->sumsq;
        carried_flag = res->found_inf != 0;
    }
    const bool bad = carried_flag || !__builtin_isfinite(total);
    const double nd = bad ? __builtin_nan("") : sqrt(total);
    res->sumsq = total;
    res->norm_d = nd;
    res->norm = (float)nd;
    res->found_inf = bad ? 1u : 0u;
}

/* Where the norm pass finds its chunk list: rows of the table in device memory (the workspace's
 * copy), or rows passed by value in the kernel arguments (the allocation-free entry point; read
 * through the scalar unit either way).  Row n_chunks is the sentinel. */
struct TableInMemory {
    const DevChunk *__restrict__ rows;
    __device__ __forceinline__ const uint16_t *grad(uint32_t c) const { return rows[c].grad; }
    __device__ __forceinline__ uint64_t numel(uint32_t c) const { return rows[c].numel; }
    __device__ __forceinline__ uint64_t tile_begin(uint32_t c) const { return rows[c].tile_begin; }
};
struct TableInArgs {
    const PrepRows &r;
    __device__ __forceinline__ const uint16_t *grad(uint32_t c) const { return r.grad[c]; }
    __device__ __forceinline__ uint64_t numel(uint32_t c) const { return r.numel[c]; }
    __device__ __forceinline__ uint64_t tile_begin(uint32_t c) const { return r.tile_begin[c]; }
};

template <int DT, typename Table>
__device__ __forceinline__ void
grad_prep_body(const Table tab, uint64_t total_tiles, double inv_scale, double extra_sumsq, uint32_t accumulate,
               double *partials, uint32_t *ticket, GradResult *res)
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
    /* Chunk cursor: the row of a tile's chunk is looked up (wave-uniform, scalar) only when the
     * tile index leaves the current chunk, and always one tile AHEAD: the lookup for the next tile
     * is issued right behind the current tile's vector loads and completes under them, so no
     * iteration waits for a scalar fetch before it can issue its loads.  (With chunks of 256 tiles
     * and 256 blocks every iteration changes chunk: looked up in line, that cost about a third of
     * the pass on the 124M-parameter model.) */
    struct Row {
        const AH_GLOBAL uint16_t *grad;
        uint64_t numel, begin, end;
    };
    uint32_t c = 0;
    auto lookup = [&](uint64_t w) {
        while (w >= tab.tile_begin(c + 1)) ++c; /* sentinel row n_chunks ends the search */
        return Row{gptr<uint16_t>(tab.grad(c)), tab.numel(c), tab.tile_begin(c), tab.tile_begin(c + 1)};
    };
    Row cur{nullptr, 0, 0, 0};
    if (blockIdx.x < total_tiles) cur = lookup(blockIdx.x);
    for (uint64_t w = blockIdx.x; w < total_tiles; w += gridDim.x) {
        const uint64_t e0 = (w - cur.begin) * kTile;
        const uint64_t w_next = w + gridDim.x;
        Row next = cur;
        if (e0 + kTile <= cur.numel) {
            /* All U loads are issued, in order, before the first square; the squares then follow in
             * the same order, each group waiting only for its own load (vmcnt U-1, U-2, ...), so the
             * arithmetic runs under the arrival of the later loads.  The barriers pin that order:
             * left alone, the scheduler starts with a late load and waits for nearly all of them. */
            u32x4 g[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                g[u] = ld<true>((const AH_GLOBAL u32x4 *)(cur.grad + e0 + (uint64_t)u * kSub + threadIdx.x * kPrepVec));
                __builtin_amdgcn_sched_barrier(0);
            }
            if (w_next < total_tiles && w_next >= cur.end) next = lookup(w_next);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float lo, hi;
                    unpack2<DT>(g[u][j], lo, hi);
                    acc0 += (double)lo * (double)lo;
                    acc1 += (double)hi * (double)hi;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            const uint64_t end = e0 + kTile < cur.numel ? e0 + kTile : cur.numel;
            for (uint64_t i = e0 + threadIdx.x; i < end; i += kThreads) {
                const double x = (double)lowp_to_f32<DT>(cur.grad[i]);
                acc0 += x * x;
            }
            if (w_next < total_tiles && w_next >= cur.end) next = lookup(w_next);
        }
        cur = next;
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
        publish_total(res, s, inv_scale, extra_sumsq, accumulate);
        __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); /* re-arm */
    }
}

template <int DT>
__global__ void __launch_bounds__(kThreads)
grad_prep_kernel(const DevChunk *__restrict__ tab, uint32_t n_chunks, uint64_t total_tiles, double inv_scale,
                 double extra_sumsq, uint32_t accumulate, double *partials, uint32_t *ticket, GradResult *res)
{
    grad_prep_body<DT>(TableInMemory{tab}, total_tiles, inv_scale, extra_sumsq, accumulate, partials, ticket, res);
    (void)n_chunks;
}

/* The same pass with the chunk list in the kernel arguments and the cross-block scratch (block
 * partials, ticket) handed in by the launcher: nothing here was allocated for the call. */
template <int DT>
__global__ void __launch_bounds__(kThreads)
grad_prep_args_kernel(const PrepRows rows, uint64_t total_tiles, double inv_scale, double extra_sumsq,
                      double *partials, uint32_t *ticket, GradResult *res)
{
    grad_prep_body<DT>(TableInArgs{rows}, total_tiles, inv_scale, extra_sumsq, 0u, partials, ticket, res);
}

__global__ void clear_word_kernel(uint32_t *word) { *word = 0u; }

/*
 * Second half of the norm carried by adamw_step_carry_kernel: sums the n wave partials in a
 * fixed order (each block a strided share, then the blocks in index order by the same ticket
 * scheme as above) and folds the total into `res`.  8 bytes per 64*VEC elements.
 */
__global__ void __launch_bounds__(kThreads)
fold_partials_kernel(const double *__restrict__ wave_partials, uint64_t n, double inv_scale, double *partials,
                     uint32_t *ticket, GradResult *res)
{
    __shared__ double lds4[4];
    __shared__ uint32_t is_last;
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    const uint64_t stride = (uint64_t)gridDim.x * kThreads;
    uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    for (; i + 3 * stride < n; i += 4 * stride) {
        const double x0 = wave_partials[i], x1 = wave_partials[i + stride];
        const double x2 = wave_partials[i + 2 * stride], x3 = wave_partials[i + 3 * stride];
        a0 += x0;
        a1 += x1;
        a2 += x2;
        a3 += x3;
    }
    for (; i < n; i += stride) a0 += wave_partials[i];
    const double bsum = block_sum((a0 + a1) + (a2 + a3), lds4);
    if (threadIdx.x == 0) {
        __hip_atomic_store(&partials[blockIdx.x], bsum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t t = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        is_last = (t == gridDim.x - 1) ? 1u : 0u;
    }
    __syncthreads();
    if (!is_last) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    double s = 0.0;
    for (uint32_t j = threadIdx.x; j < gridDim.x; j += kThreads)
        s += __hip_atomic_load(&partials[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s = block_sum(s, lds4);
    if (threadIdx.x == 0) {
        publish_total(res, s, inv_scale, 0.0, 1u);
        __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

__global__ void set_result_kernel(GradResult *res, double sumsq, uint32_t found_inf)
{
    const bool bad = found_inf || !__builtin_isfinite(sumsq);
    const double nd = bad ? __builtin_nan("") : sqrt(sumsq);
    res->sumsq = sumsq;
    res->norm_d = nd;
    res->norm = (float)nd;
    res->found_inf = bad ? 1u : 0u;
}

/* ------------------------------------------------------------------------------------- */
/* Launchers                                                                               */
/* ------------------------------------------------------------------------------------- */

typedef void (*step_fn)(const DevChunk *, const GradResult *, StepConsts);

template <int DT>
static step_fn pick_step(StepVariant s)
{
#define AH_CASE(V, B, M) \
    if (s.vec == V && s.block == B && s.mode == M) \
        return s.write_back ? adamw_step_kernel<DT, V, B, M, true> : adamw_step_kernel<DT, V, B, M, false>;
#define AH_CASES(V, B) AH_CASE(V, B, 0) AH_CASE(V, B, 1)
    AH_CASES(4, 64) AH_CASES(4, 128) AH_CASES(4, 256)
    AH_CASES(2, 64) AH_CASES(2, 128) AH_CASES(2, 256)
    AH_CASES(1, 128) AH_CASES(1, 256) AH_CASES(1, 512)
#undef AH_CASES
#undef AH_CASE
    return nullptr;
}

static step_fn pick_step(int dtype, StepVariant s)
{
    return dtype == kFP16 ? pick_step<kFP16>(s) : pick_step<kBF16>(s);
}

bool step_variant_valid(StepVariant s) { return pick_step(kBF16, s) != nullptr; }

typedef void (*carry_fn)(const DevChunk *, const GradResult *, StepConsts, double *, uint64_t);

template <int DT>
static carry_fn pick_carry(StepVariant s)
{
#define AH_CASE(V, B, M) \
    if (s.vec == V && s.block == B && s.mode == M) return adamw_step_carry_kernel<DT, V, B, M>;
#define AH_CASES(V, B) AH_CASE(V, B, 0) AH_CASE(V, B, 1)
    AH_CASES(4, 64) AH_CASES(4, 128) AH_CASES(4, 256)
    AH_CASES(2, 64) AH_CASES(2, 128) AH_CASES(2, 256)
    AH_CASES(1, 128) AH_CASES(1, 256) AH_CASES(1, 512)
#undef AH_CASES
#undef AH_CASE
    return nullptr;
}

hipError_t launch_step_carry(int dtype, StepVariant var, unsigned grid_x, unsigned grid_y, unsigned lds_bytes,
                             hipStream_t stream, const DevChunk *tab, const GradResult *res, const StepConsts &k,
                             double *wave_partials, uint64_t slot_base)
{
    carry_fn fn = dtype == kFP16 ? pick_carry<kFP16>(var) : pick_carry<kBF16>(var);
    if (!fn) return hipErrorInvalidValue;
    if (grid_x == 0 || grid_y == 0) return hipSuccess;
    hipLaunchKernelGGL(fn, dim3(grid_x, grid_y), dim3(var.block), lds_bytes, stream, tab, res, k, wave_partials,
                       slot_base);
    return hipGetLastError();
}

hipError_t launch_fold(unsigned blocks, hipStream_t stream, const double *wave_partials, uint64_t n,
                       double inv_scale, double *partials, uint32_t *ticket, GradResult *res)
{
    if (blocks == 0) blocks = 1;
    hipLaunchKernelGGL(fold_partials_kernel, dim3(blocks), dim3(kThreads), 0, stream, wave_partials, n, inv_scale,
                       partials, ticket, res);
    return hipGetLastError();
}

hipError_t launch_cast(int dtype, unsigned grid_x, unsigned grid_y, unsigned lds_bytes, hipStream_t stream,
                       const DevChunk *tab)
{
    if (grid_x == 0 || grid_y == 0) return hipSuccess;
    if (dtype == kFP16)
        hipLaunchKernelGGL(cast_params_kernel<kFP16>, dim3(grid_x, grid_y), dim3(64), lds_bytes, stream, tab);
    else
        hipLaunchKernelGGL(cast_params_kernel<kBF16>, dim3(grid_x, grid_y), dim3(64), lds_bytes, stream, tab);
    return hipGetLastError();
}

hipError_t launch_step(int dtype, StepVariant var, unsigned grid_x, unsigned grid_y, unsigned lds_bytes,
                       hipStream_t stream, const DevChunk *tab, const GradResult *res, const StepConsts &k)
{
    step_fn fn = pick_step(dtype, var);
    if (!fn) return hipErrorInvalidValue;
    if (grid_x == 0 || grid_y == 0) return hipSuccess;
    hipLaunchKernelGGL(fn, dim3(grid_x, grid_y), dim3(var.block), lds_bytes, stream, tab, res, k);
    return hipGetLastError();
}

hipError_t launch_prep(int dtype, unsigned blocks, hipStream_t stream, const DevChunk *tab, uint32_t n_chunks,
                       uint64_t total_tiles, double inv_scale, double extra_sumsq, bool accumulate, double *partials,
                       uint32_t *ticket, GradResult *res)
{
    if (blocks == 0) blocks = 1; /* no chunks: one block still publishes S = extra_sumsq */
    if (dtype == kFP16)
        hipLaunchKernelGGL(grad_prep_kernel<kFP16>, dim3(blocks), dim3(kThreads), 0, stream, tab, n_chunks,
                           total_tiles, inv_scale, extra_sumsq, accumulate ? 1u : 0u, partials, ticket, res);
    else
        hipLaunchKernelGGL(grad_prep_kernel<kBF16>, dim3(blocks), dim3(kThreads), 0, stream, tab, n_chunks,
                           total_tiles, inv_scale, extra_sumsq, accumulate ? 1u : 0u, partials, ticket, res);
    return hipGetLastError();
}

/* ------------------------------------------------------------------------------------- */
/* The allocation-free norm pass                                                           */
/* ------------------------------------------------------------------------------------- */

/* Its cross-block scratch: kStaticMaxBlocks fp64 block partials followed by the ticket word.
 * One copy per GPU, loaded with the code object and held until the process ends; every call on
 * a GPU uses that GPU's copy, so calls that overlap on one GPU race.  In host code the name
 * below is only a handle for hipGetSymbolAddress, never an address. */
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
struct StaticSetup {
    std::mutex lock;
    void *ptr[kMaxDevices] = {};
    int n_cu[kMaxDevices] = {};
} g_static;
}  // namespace

/* Address of the current device's copy of `scratch` and that device's CU count, looked up once
 * per device (with that device current) and kept. */
static hipError_t static_scratch(void **ptr, int *n_cu)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> g(g_static.lock);
    if (!g_static.ptr[dev]) {
        void *p = nullptr;
        int cu = 0;
        if ((e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) != hipSuccess) return e;
        if ((e = hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
        if (!p || cu <= 0) return hipErrorInvalidSymbol;
        g_static.n_cu[dev] = cu;
        g_static.ptr[dev] = p;
    }
    *ptr = g_static.ptr[dev];
    *n_cu = g_static.n_cu[dev];
    return hipSuccess;
}

hipError_t launch_prep_static(int dtype, hipStream_t stream, const PrepRows &rows, uint64_t total_tiles,
                              double inv_scale, double extra_sumsq, GradResult *res)
{
    void *base = nullptr;
    int n_cu = 0;
    hipError_t e = static_scratch(&base, &n_cu);
    if (e != hipSuccess) return e;
    double *partials = static_cast<double *>(base);
    uint32_t *ticket = reinterpret_cast<uint32_t *>(static_cast<unsigned char *>(base) +
                                                    kStaticMaxBlocks * sizeof(double));
    /* same grid rule as the workspace path: one block per CU, never more blocks than tiles */
    uint64_t blocks = std::min<uint64_t>((uint64_t)std::min(n_cu, kStaticMaxBlocks), total_tiles);
    if (blocks == 0) blocks = 1;
    /* The array keeps whatever the last call left.  Only the ticket must start at zero (every
     * partial that is read is written first); a kernel clears it, not a memset, so that the call
     * can be recorded into a graph. */
    hipLaunchKernelGGL(clear_word_kernel, dim3(1), dim3(1), 0, stream, ticket);
    if (dtype == kFP16)
        hipLaunchKernelGGL(grad_prep_args_kernel<kFP16>, dim3((unsigned)blocks), dim3(kThreads), 0, stream, rows,
                           total_tiles, inv_scale, extra_sumsq, partials, ticket, res);
    else
        hipLaunchKernelGGL(grad_prep_args_kernel<kBF16>, dim3((unsigned)blocks), dim3(kThreads), 0, stream, rows,
                           total_tiles, inv_scale, extra_sumsq, partials, ticket, res);
    return hipGetLastError();
}

hipError_t launch_set_result(hipStream_t stream, GradResult *res, double sumsq, uint32_t found_inf)
{
    hipLaunchKernelGGL(set_result_kernel, dim3(1), dim3(1), 0, stream, res, sumsq, found_inf);
    return hipGetLastError();
}

}  // namespace ah
