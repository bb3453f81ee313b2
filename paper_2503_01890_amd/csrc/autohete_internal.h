/* Internal declarations shared by the host API and the kernels of libautohete.so. */
#ifndef AUTOHETE_INTERNAL_H
#define AUTOHETE_INTERNAL_H
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ah {

constexpr int kThreads = 256;        /* 4 wavefronts of 64 */
constexpr int kPrepVec = 8;          /* elements per lane per load in the prep kernel */
constexpr int kMaxPartials = 16384;  /* upper bound on prep blocks (one fp64 partial each) */

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
    double norm_d;      /* sqrt(sumsq); NaN when found_inf */
    float norm;         /* norm_d rounded to fp32 */
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

/* Step-kernel variants: vec = elements per lane (1, 2, 4), block = threads per block,
 * mode 0 = fp64 with Newton root/quotient, mode 1 = fp64 with correctly rounded root/quotient. */
struct StepVariant { int vec, block, mode; bool write_back = true; };
bool step_variant_valid(StepVariant s);

/* grid_x tiles of vec*block elements for each of grid_y table rows; lds_bytes of dynamic LDS
 * per block caps the blocks resident per CU. */
hipError_t launch_step(int dtype, StepVariant var, unsigned grid_x, unsigned grid_y, unsigned lds_bytes,
                       hipStream_t stream, const DevChunk *tab, const GradResult *res, const StepConsts &k);
/* The same launch shape for the norm-carrying update: wave w of block (x, y) writes slot
 * slot_base + (tab[y].tile_begin + x) * (block / 64) + w of wave_partials; launch_fold sums n
 * slots into res (S += sum * inv_scale^2). */
hipError_t launch_step_carry(int dtype, StepVariant var, unsigned grid_x, unsigned grid_y, unsigned lds_bytes,
                             hipStream_t stream, const DevChunk *tab, const GradResult *res, const StepConsts &k,
                             double *wave_partials, uint64_t slot_base);
hipError_t launch_fold(unsigned blocks, hipStream_t stream, const double *wave_partials, uint64_t n,
                       double inv_scale, double *partials, uint32_t *ticket, GradResult *res);
/* master -> 16-bit conversion: grid_x tiles of 512 elements for each of grid_y table rows */
constexpr uint32_t kCastTileElems = 512;
hipError_t launch_cast(int dtype, unsigned grid_x, unsigned grid_y, unsigned lds_bytes, hipStream_t stream,
                       const DevChunk *tab);
hipError_t launch_prep(int dtype, unsigned blocks, hipStream_t stream, const DevChunk *tab, uint32_t n_chunks,
                       uint64_t total_tiles, double inv_scale, double extra_sumsq, bool accumulate, double *partials,
                       uint32_t *ticket, GradResult *res);
hipError_t launch_set_result(hipStream_t stream, GradResult *res, double sumsq, uint32_t found_inf);

/* Chunk list of the allocation-free norm pass, passed by value in the kernel arguments (3096 of the
 * 4096 bytes a launch may carry); entry n is the sentinel holding the total tile count. */
constexpr int kStaticMaxChunks = 128;
struct PrepRows {
    const uint16_t *grad[kStaticMaxChunks + 1];
    uint64_t numel[kStaticMaxChunks + 1];
    uint64_t tile_begin[kStaticMaxChunks + 1];
};
/* Cross-block scratch of that pass, a file-scope device array: block partials, then the ticket. */
constexpr int kStaticMaxBlocks = 2048;
constexpr size_t kStaticScratchBytes = kStaticMaxBlocks * sizeof(double) + 256;
/* Norm pass over `rows` on the current device with the static scratch; the 32-byte result goes to
 * res (device memory of the caller).  Makes no allocation. */
hipError_t launch_prep_static(int dtype, hipStream_t stream, const PrepRows &rows, uint64_t total_tiles,
                              double inv_scale, double extra_sumsq, GradResult *res);

constexpr int kPrepUnroll = 8; /* 8 x 16 B per lane in flight: 32 KB per 256-thread block */
inline uint32_t prep_tile_elems() { return (uint32_t)(kThreads * kPrepVec * kPrepUnroll); }

}  // namespace ah
#endif
