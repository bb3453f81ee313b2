/*
 * autohete.h -- C ABI of the MI355X (gfx950) chunked mixed-precision AdamW update.
 *
 * The operation is the GPU optimizer update of AutoHete (cost t_optim^gpu, charged on
 * the backward compute stream in Eq. 5, first arm) over "model data" as section 2.1
 * defines it: 16-bit parameters and gradients plus fp32 optimizer states (momentum,
 * variance, fp32 parameter copy), 16 bytes per parameter.  Model data is packed into
 * fixed-size flat chunks (section 3.1: transfers aggregate tensors; section 3.4:
 * parameters are mapped to device memory in advance).  The paper names Adam and gives
 * no equations; the rule implemented is Adam with decoupled weight decay, preceded by
 * loss-scale removal, a finite check and global-L2-norm clipping:
 *
 *     S     = extra_sumsq + sum over all chunk elements of (grad / loss_scale)^2
 *     skip  = any non-finite gradient, or S non-finite     -> nothing is modified
 *     c     = max_grad_norm > 0 ? min(1, max_grad_norm / (sqrt(S) + 1e-6)) : 1
 *     g     = grad / loss_scale * c
 *     m'    = beta1 m + (1 - beta1) g
 *     v'    = beta2 v + (1 - beta2) g^2
 *     p'    = p - lr ( (m' / (1 - beta1^t)) / (sqrt(v' / (1 - beta2^t)) + eps) + weight_decay p )
 *     p16'  = round-to-nearest-even(p') in bf16 or fp16
 *
 * Conventions
 *   - Every function returns an int status (AH_OK = 0, negative = error); nothing is
 *     thrown or printed.  autohete_strerror() names a status.
 *   - "device pointer" = address in the HBM of the current HIP device; "host pointer" =
 *     ordinary process memory.  The caller owns every buffer it passes; the library owns
 *     only the workspace object.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work and return, except where a host output is requested (stated below).
 *   - One workspace serves one stream at a time: calls that use the same workspace must
 *     be issued in stream order from one host thread.
 */
#ifndef AUTOHETE_H
#define AUTOHETE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    AH_OK = 0,
    AH_EINVAL = -1, /* null pointer, bad enum, numel == 0, step == 0, bad hyper-parameter */
    AH_EALIGN = -2, /* a device pointer is not 16-byte aligned */
    AH_ENOMEM = -3, /* allocation failed, or more chunks than the workspace was made for */
    AH_EHIP = -4,   /* a HIP runtime call failed */
    AH_EINFEASIBLE = -5, /* autohete_strategy_search: no strategy satisfies the memory constraints */
    AH_ELIMIT = -6  /* autohete_grad_prep_static: more chunks than AUTOHETE_STATIC_MAX_CHUNKS */
};

enum { AH_BF16 = 0, AH_FP16 = 1 }; /* format of the two 16-bit streams */

/*
 * Chunk layout (host only, integer only; sections 3.1 and 3.4).
 * Tensors are packed back to back, in the order given, into one flat element space that
 * is cut into chunks of chunk_elems elements.  Tensor t occupies flat elements
 * [tensor_offset[t], tensor_offset[t] + tensor_numel[t]); its first element lies in chunk
 * tensor_offset[t] / chunk_elems at position tensor_offset[t] % chunk_elems; a tensor may
 * straddle chunks.  Only the last chunk is padded.
 *   tensor_numel   host in : n_tensors sizes (elements); may be NULL iff n_tensors == 0
 *   tensor_offset  host out: n_tensors flat offsets (exclusive prefix sum); may be NULL
 *   n_chunks       host out: ceil(total / chunk_elems)
 *   total_elems    host out: sum of sizes
 *   padded_elems   host out: n_chunks * chunk_elems - total
 * Errors: AH_EINVAL if chunk_elems == 0, an out pointer (other than tensor_offset) is
 * NULL, or the total overflows 64 bits.
 */
int autohete_chunk_layout(const uint64_t *tensor_numel, uint64_t n_tensors, uint64_t chunk_elems,
                          uint64_t *tensor_offset, uint64_t *n_chunks, uint64_t *total_elems,
                          uint64_t *padded_elems);

/*
 * One chunk of model data (section 2.1): five element-aligned streams of `numel`
 * elements, all DEVICE pointers, each 16-byte aligned, none overlapping another.
 */
typedef struct {
    const void *grad; /* 16-bit gradients, still multiplied by the loss scale; read only  */
    void *param_lp;   /* 16-bit parameters; write only (derived from master)              */
    float *master;    /* fp32 parameter copy; read and written in place                   */
    float *exp_avg;   /* fp32 first moment m; read and written in place                   */
    float *exp_avg_sq;/* fp32 second moment v >= 0; read and written in place             */
    uint64_t numel;   /* elements to process, padding included; >= 1, any value           */
} autohete_chunk;

typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    float max_grad_norm; /* <= 0: no clipping */
    float loss_scale;    /* > 0 and finite */
} autohete_hparams;

/*
 * Workspace: device scratch for the cross-block norm reduction, the 32-byte reduction
 * result, and device copies of the chunk tables of recent calls (up to 128, about 8 MB at most;
 * found again by content, so a caller that cycles through a few chunk lists uploads each once;
 * a list is uploaded on the stream of the call that first brings it, and a call that finds it
 * on another stream waits there for that upload).  max_chunks bounds n_chunks of later calls.
 * Create/destroy allocate/free device memory on the current device and synchronise it; do not
 * call them inside a timed region.  One workspace serves one host thread and one stream at a
 * time: calls on different streams must be ordered by the caller.
 */
typedef struct autohete_ws autohete_ws;
int autohete_ws_create(autohete_ws **ws, uint64_t max_chunks);
int autohete_ws_destroy(autohete_ws *ws);

/*
 * Gradient preparation: loss-scale removal, finite check and global L2 norm over the
 * given chunks in one streaming pass (2 bytes read per element).  The per-element
 * gradients are not modified; the result {S, norm, skip flag} is left in the workspace
 * on the device for autohete_adamw_step.
 *   chunks        host in : n_chunks descriptors (device pointers inside); only .grad
 *                           and .numel are used here
 *   n_chunks      may be 0 (then S = extra_sumsq)
 *   lowp_dtype    AH_BF16 or AH_FP16
 *   loss_scale    > 0, finite
 *   extra_sumsq   sum of squares of UNSCALED gradients that live elsewhere (chunks kept in
 *                 host memory, other devices); 0 if none.  Non-finite raises the skip flag.
 *   norm_out, found_inf_out   host out, each may be NULL.  If either is non-NULL the call
 *                 waits for the stream and stores sqrt(S) (NaN when skipping) and the flag.
 * The sum is accumulated in fp64 and is bit-reproducible for a given chunk list and
 * workspace tuning.  Errors: AH_EINVAL, AH_EALIGN, AH_ENOMEM (n_chunks > max_chunks), AH_EHIP.
 */
int autohete_grad_prep(autohete_ws *ws, const autohete_chunk *chunks, uint64_t n_chunks,
                       int lowp_dtype, float loss_scale, double extra_sumsq, void *stream,
                       float *norm_out, uint32_t *found_inf_out);

/*
 * The same pass, folded into the result already in the workspace instead of replacing it:
 * S += sum (grad / loss_scale)^2 over the given chunks, skip flag |= non-finite.  Lets a caller
 * gather the global norm block by block as the backward pass produces gradients (the paper steps
 * each block's optimizer as soon as its gradients exist: section 3.2.2, footnote to Eq. 5), starting
 * from autohete_grad_result_set(ws, 0, 0, stream).  Chunks may be sub-ranges of larger chunks (any
 * 16-byte-aligned slice).  The result equals one autohete_grad_prep over all the chunks up to the
 * order of the fp64 additions.
 */
int autohete_grad_prep_accumulate(autohete_ws *ws, const autohete_chunk *chunks, uint64_t n_chunks,
                                  int lowp_dtype, float loss_scale, void *stream);

/*
 * autohete_grad_prep for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  It needs no workspace and makes no allocation (no
 * hipMalloc, hipFree, host-pinned memory or upload): the chunk list travels in the kernel
 * arguments, and the cross-block scratch of the reduction (2048 fp64 block partials and a ticket
 * word, 16640 bytes) is a static device array inside the library, one copy per GPU, held until the
 * process ends.  Same kernel body, grid and summation order as autohete_grad_prep with default
 * tuning, so S is bit-identical to that call's on the same chunk list.
 *   chunks      host in : n_chunks descriptors; only .grad (device, 16-byte aligned) and .numel used.
 *                         A descriptor may span several chunks that are contiguous in memory.
 *   n_chunks    0..AUTOHETE_STATIC_MAX_CHUNKS (0: S = extra_sumsq); more -> AH_ELIMIT, nothing runs
 *   result      DEVICE out, caller-owned, 8-byte aligned: {S, sqrt(S), (float)sqrt(S), skip flag},
 *               written on `stream`; sqrt(S) is NaN when the flag is set
 * The device current at the call is used; the pointers must belong to it.  Every call on a GPU
 * shares that GPU's scratch array: calls that overlap on one GPU (different streams, or threads)
 * race -- order them.  The ticket word is cleared by a small kernel ahead of the pass (no memset
 * node), so the call may be captured.  Errors: AH_EINVAL, AH_EALIGN, AH_ELIMIT, AH_EHIP.
 */
#define AUTOHETE_STATIC_MAX_CHUNKS 128
typedef struct {
    double sumsq;       /* S = extra_sumsq + sum (grad / loss_scale)^2 */
    double norm_d;      /* sqrt(S); NaN when found_inf */
    float norm;         /* the same, rounded to fp32 */
    uint32_t found_inf; /* 1: a gradient or S is not finite -- skip the step */
} autohete_grad_result;
int autohete_grad_prep_static(const autohete_chunk *chunks, uint64_t n_chunks, int lowp_dtype, float loss_scale,
                              double extra_sumsq, void *stream, autohete_grad_result *result);

/*
 * The update (rule at the top of this file) over the given chunks in one fused pass:
 * 14 bytes read and 14 bytes written per element; each optimizer state is read once and
 * written once per update (the paper's appendix on memory allocation states the same).  It consumes the workspace's
 * device-side result, so it must follow an autohete_grad_prep (or
 * autohete_grad_result_set) on the same stream.  If the skip flag is set the kernel
 * exits before its first load and every stream is left bit-identical; the caller should
 * then not advance `step`.  The chunk list may be any subset or partition of the list
 * given to autohete_grad_prep (one optimizer per transformer block: footnote to Eq. 5),
 * and per-element results do not depend on that grouping.
 *   step   the 1-based t of the bias corrections; the library keeps no counter
 *   hp     host in; loss_scale must be the value given to autohete_grad_prep
 * Errors: AH_EINVAL (also: beta outside [0,1), lr/eps/weight_decay negative or
 * non-finite), AH_EALIGN, AH_ENOMEM, AH_EHIP.
 */
int autohete_adamw_step(autohete_ws *ws, const autohete_chunk *chunks, uint64_t n_chunks,
                        int lowp_dtype, uint64_t step, const autohete_hparams *hp, void *stream);

/*
 * The same update without the 16-bit write-back: 14 bytes read and 12 bytes written per element;
 * chunk.param_lp is ignored and may be NULL.  For blocks whose optimizer states stay on the GPU
 * the paper keeps no 16-bit parameters (section 3.2.2, footnote to the peak-memory model): they
 * are produced from the fp32 copy just before the block's forward or backward pass and released
 * afterwards.  autohete_cast_params is that conversion: param_lp = round-to-nearest-even(master),
 * 4 bytes read and 2 bytes written per element; only .param_lp, .master and .numel are used.
 * autohete_adamw_step_master followed by autohete_cast_params leaves all five streams
 * bit-identical to autohete_adamw_step.  Errors as for autohete_adamw_step.
 */
int autohete_adamw_step_master(autohete_ws *ws, const autohete_chunk *chunks, uint64_t n_chunks,
                               int lowp_dtype, uint64_t step, const autohete_hparams *hp, void *stream);
int autohete_cast_params(autohete_ws *ws, const autohete_chunk *chunks, uint64_t n_chunks,
                         int lowp_dtype, void *stream);

/*
 * autohete_adamw_step that also carries the gradient norm forward.  When each block's optimizer
 * is stepped as soon as that block's gradients exist (section 3.2.2, footnote to Eq. 5), the
 * update of an early block cannot wait for a norm over gradients the backward pass has not
 * produced yet: it clips with the norm the workspace `ws` already holds (the previous
 * iteration's, or one set by autohete_grad_result_set), and the squares of the gradients it
 * reads anyway are summed for the next one.  The call leaves every stream and both workspaces
 * exactly as
 *     autohete_grad_prep_accumulate(ws_next, chunks, n_chunks, lowp_dtype, hp->loss_scale, stream);
 *     autohete_adamw_step(ws, chunks, n_chunks, lowp_dtype, step, hp, stream);
 * would, up to the order of the fp64 additions inside ws_next's S, while reading the gradients
 * once: 28 bytes per element instead of 30.  The sum is bit-reproducible for a given chunk list
 * and tuning.  If ws holds a skip flag nothing is updated but the squares are still gathered.
 * Note what any such schedule implies: a non-finite gradient is only seen in ws_next, after the
 * blocks stepped earlier in the same iteration have been written.
 *   ws_next   must differ from ws and live on the same device; its result is accumulated into,
 *             so start an iteration with autohete_grad_result_set(ws_next, 0, 0, stream)
 * The squares are kept as one fp64 partial per wavefront in a buffer of ws_next (numel / 32 bytes
 * per iteration with the default tuning) and are summed into ws_next's result, by one small
 * kernel, on the stream of the next call that uses or reads that result -- which the caller has
 * to order after these updates anyway.  The buffer grows by doubling until it holds a whole
 * iteration; growing allocates and thereby waits for the device (first iteration only), unless
 * autohete_ws_tune(ws_next, AH_TUNE_CARRY_ELEMS, elements per iteration) has sized it beforehand:
 * then no call of this function allocates or frees.
 * Errors: as autohete_adamw_step; AH_EINVAL also if ws_next is NULL or equals ws.
 */
int autohete_adamw_step_carry(autohete_ws *ws, autohete_ws *ws_next, const autohete_chunk *chunks,
                              uint64_t n_chunks, int lowp_dtype, uint64_t step,
                              const autohete_hparams *hp, void *stream);

/*
 * Read (waits for the stream) or overwrite (enqueued on the stream) the workspace's
 * gradient result.  Setting it lets a caller step a block with a norm obtained elsewhere
 * -- e.g. per-block stepping during backward with clipping off (sumsq = 0), or with the
 * previous iteration's norm.  Any out pointer may be NULL.
 */
int autohete_grad_result_get(autohete_ws *ws, void *stream, double *sumsq, float *norm,
                             uint32_t *found_inf);
int autohete_grad_result_set(autohete_ws *ws, double sumsq, uint32_t found_inf, void *stream);

/*
 * Launch tuning (optional; defaults are chosen for MI355X).  Changing a knob never
 * changes the update's results; AH_TUNE_PREP_BLOCKS changes the summation order of the
 * norm (last bits of S).
 */
enum {
    AH_TUNE_STEP_BLOCKS_PER_CU = 0, /* cap on step-kernel blocks resident per CU: 3..64 (64 = no
                                       cap; 1 and 2 cannot be enforced and are refused with
                                       AH_EINVAL); 0 = default: chosen per call from the
                                       elements it covers (10 to 12; shorter calls take more)  */
    AH_TUNE_PREP_BLOCKS = 1,        /* thread blocks of the prep kernel; 0 = default           */
    AH_TUNE_CAST_BLOCKS_PER_CU = 3, /* the same cap for the cast kernel; 0 = default           */
    AH_TUNE_CARRY_ELEMS = 4,        /* elements that autohete_adamw_step_carry calls carry INTO
                                       this workspace per iteration (the model's element count):
                                       sizes the buffer of per-wavefront partials now (allocates,
                                       waits for the device), so that no later call does.  Set
                                       the step variant first; AH_EINVAL while a carried sum is
                                       pending                                                 */
    AH_TUNE_STEP_VARIANT = 2        /* step-kernel variant: elements per lane (1, 2, 4)
                                       | mode << 4 (0 = fp64 Newton root/quotient, 1 = fp64
                                       correctly rounded) | (threads per block / 64) << 8;
                                       0 = default                                             */
};
int autohete_ws_tune(autohete_ws *ws, int knob, int64_t value);

/*
 * Host half of a hybrid placement (paper section 3.2.1: a block whose optimizer states are placed on
 * the CPU has its 16-bit gradients offloaded and its fp32 parameters updated there; cost
 * t_optim^cpu, Eq. 5 second arm).  Same rule, same fp64 arithmetic and rounding as the GPU kernels,
 * on chunks whose five pointers are HOST pointers (any alignment); multi-threaded, AVX-512 where
 * the CPU has it.  Both calls are synchronous.
 *   autohete_host_grad_sumsq   *sumsq = sum (grad / loss_scale)^2 over the chunks (only .grad and
 *                              .numel are used), *found_inf = 1 if any gradient is non-finite.
 *                              Add it to the device-side sum through extra_sumsq, or the other way.
 *   autohete_host_adamw_step   the update with the GLOBAL sum of squares `sumsq` and skip flag
 *                              given by the caller (nothing is touched when the flag is set or
 *                              sumsq is non-finite); .param_lp may be NULL (no 16-bit write-back).
 *                              .grad and .param_lp may be the SAME buffer (on the host the two never
 *                              coexist, Eq. 2: 14 bytes per parameter): each element's gradient is
 *                              read before its parameter is written.
 *   n_threads                  1..1024 worker threads; results do not depend on it except the
 *                              last bits of *sumsq.
 *   autohete_host_force_scalar test hook: non-zero disables the AVX-512 path (same results).
 * Errors: AH_EINVAL (as for the device calls), AH_ENOMEM (threads could not be started).
 */
int autohete_host_grad_sumsq(const autohete_chunk *chunks, uint64_t n_chunks, int lowp_dtype, float loss_scale,
                             int n_threads, double *sumsq, uint32_t *found_inf);
int autohete_host_adamw_step(const autohete_chunk *chunks, uint64_t n_chunks, int lowp_dtype, uint64_t step,
                             const autohete_hparams *hp, double sumsq, uint32_t found_inf, int n_threads);
int autohete_host_force_scalar(int on);

/*
 * Cost model and strategy search (host only; paper section 3.2.2, Eq. 1-6).  The planning unit is
 * the transformer block; a strategy is (c, p, o) = how many blocks use activation checkpointing
 * and parameter offloading (the first c and p blocks: Insight 1) and optimizer-state offloading
 * (the last o blocks: Insight 2).  Sizes are in ELEMENTS where the paper writes M (it multiplies
 * by 2, 12 or 14 bytes itself), capacities and constants in bytes, times per block in any one
 * unit.  t_optim_gpu is the quantity this library's benchmark measures.
 *   autohete_strategy_eval    fills every field of *out for one (c, p, o); feasible = Eq. 1 and
 *                             Eq. 2 hold and p <= o.  AH_EINVAL if a count exceeds n_blocks.
 *   autohete_strategy_search  exact minimum of t_fwd + t_bwd over the feasible points (Eq. 6);
 *                             ties go to the smallest o, then p, then c.  AH_EINFEASIBLE if none.
 * AH_EINVAL for NULL pointers, n_blocks outside 1..4096, negative or non-finite inputs, or
 * act_in_elems > act_elems.
 */
typedef struct {
    uint32_t n_blocks;          /* L */
    double act_elems;           /* M_a : activations of one block */
    double act_in_elems;        /* M_a': its input activations (what checkpointing keeps) */
    double param_elems;         /* M_p : parameters of one block */
    double gpu_const_bytes;     /* M_gc */
    double cpu_const_bytes;     /* M_cc */
    double gpu_capacity_bytes;  /* M_gpu */
    double cpu_capacity_bytes;  /* M_cpu */
    double t_fp, t_bp;          /* forward / backward compute of one block */
    double t_h2d, t_d2h;        /* 16-bit parameter prefetch / gradient (or parameter) offload of one block */
    double t_optim_cpu, t_optim_gpu; /* optimizer update of one block on the host / on the GPU */
} autohete_cost_model;

typedef struct {
    uint32_t n_ckpt, n_param_offload, n_optim_offload; /* c, p, o */
    int feasible;
    double gpu_bytes;           /* left side of Eq. 1 */
    double cpu_bytes;           /* left side of Eq. 2 */
    double t_fwd;               /* Eq. 3 */
    double t_sync;              /* Eq. 4 */
    double t_bwd;               /* Eq. 5 */
} autohete_strategy;

int autohete_strategy_eval(const autohete_cost_model *model, uint32_t n_ckpt, uint32_t n_param_offload,
                           uint32_t n_optim_offload, autohete_strategy *out);
int autohete_strategy_search(const autohete_cost_model *model, autohete_strategy *best);

const char *autohete_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* AUTOHETE_H */
