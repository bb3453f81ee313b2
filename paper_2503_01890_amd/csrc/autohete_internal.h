/* Internal declarations shared by the host API and the kernels of libautohete.so. */
#ifndef AUTOHETE_INTERNAL_H
#define AUTOHETE_INTERNAL_H
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ah {

constexpr int kThreads = 256;        /* 4 wavefronts of 64 */
constexpr int kStepVec = 4;          /* elements per lane per load group in the step kernel */
constexpr int kPrepVec = 8;          /* elements per lane per load in the prep kernel */
constexpr int kMaxPartials = 16384;  /* upper bound on prep blocks */

/* Device-side chunk descriptor: the caller's chunk plus the index of its first tile.
 * Entry n_chunks is a sentinel whose tile_begin is the total tile count. */
struct DevChunk {
    const uint16_t *grad;
    uint16_t *param_lp;
    float *master;
    float *exp_avg;
    float *exp_avg_sq;
    uint64_t numel;
    uint64_t tile_begin;
    uint64_t reserved;
};
static_assert(sizeof(DevChunk) == 64, "DevChunk is one 64-byte line");

/* Result of the gradient preparation, kept in device memory between the two kernels. */
struct GradResult {
    double sumsq;       /* extra_sumsq + sum (grad/loss_scale)^2 */
    float norm;         /* sqrt(sumsq) rounded to fp32; NaN when found_inf */
    uint32_t found_inf; /* 1: skip the step */
};

/* Per-launch constants of the update, prepared in fp64 on the host. */
struct StepConsts {
    double inv_scale;   /* 1 / loss_scale */
    double max_norm;    /* <= 0: no clipping */
    double b1, b2;      /* beta1, beta2 widened from fp32 */
    double omb1, omb2;  /* 1 - beta */
    double bc1, bc2;    /* 1 - beta^t */
    double rbc1, rbc2;  /* 1 / bc */
    double lr, eps, wd;
};

/* Step-kernel variants: unroll U in {1,2,4}; mode 0 = fp64 moments, fp32 root and quotient;
 * mode 1 = everything in fp64; nt = non-temporal loads and stores. */
struct StepVariant { int unroll, mode, nt; };

hipError_t launch_step(int dtype, StepVariant var, unsigned blocks, hipStream_t stream, const DevChunk *tab,
                       uint32_t n_chunks, uint64_t total_tiles, const GradResult *res, const StepConsts &k);
hipError_t launch_prep(int dtype, unsigned blocks, hipStream_t stream, const DevChunk *tab, uint32_t n_chunks,
                       uint64_t total_tiles, double inv_scale, double extra_sumsq, double *partials,
                       uint32_t *ticket, GradResult *res);
hipError_t launch_set_result(hipStream_t stream, GradResult *res, double sumsq, uint32_t found_inf);
int step_occupancy(int dtype, StepVariant var);   /* resident blocks per CU, <= 0 on error */
int prep_occupancy(int dtype);

inline uint32_t step_tile_elems(int unroll) { return (uint32_t)(kThreads * kStepVec * unroll); }
constexpr int kPrepUnroll = 2;
inline uint32_t prep_tile_elems() { return (uint32_t)(kThreads * kPrepVec * kPrepUnroll); }

}  // namespace ah
#endif
