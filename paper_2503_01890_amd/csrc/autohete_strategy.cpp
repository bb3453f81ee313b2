/*
 * autohete_strategy.cpp -- host-only part of libautohete.so: the paper's cost model (Eq. 1-5)
 * and strategy search (Eq. 6) over the three decision variables (c, p, o) = numbers of
 * transformer blocks with activation checkpointing, parameter offloading and optimizer-state
 * offloading.  The paper solves Eq. 6 as an integer linear program; the space has only
 * (L+1)^3 points, so it is enumerated exactly.  t_optim_gpu is what bench.py measures.
 */
#include <math.h>

#include <algorithm>

#include "../../include/autohete.h"

namespace {

bool valid_model(const autohete_cost_model *m)
{
    if (!m || m->n_blocks == 0 || m->n_blocks > 4096) return false;
    const double v[] = {m->act_elems, m->act_in_elems, m->param_elems, m->gpu_const_bytes, m->cpu_const_bytes,
                        m->gpu_capacity_bytes, m->cpu_capacity_bytes, m->t_fp, m->t_bp, m->t_h2d, m->t_d2h,
                        m->t_optim_cpu, m->t_optim_gpu};
    for (double x : v)
        if (!isfinite(x) || x < 0.0) return false;
    return m->act_in_elems <= m->act_elems;
}

void evaluate(const autohete_cost_model &m, uint32_t c, uint32_t p, uint32_t o, autohete_strategy *s)
{
    const double L = (double)m.n_blocks;
    /* Eq. 1: peak GPU bytes, reached at the turn from forward to backward. */
    s->gpu_bytes = 2.0 * m.act_in_elems * c + 2.0 * m.act_elems * (L - c + 1.0) + 2.0 * m.param_elems * (L - p + 1.0) +
                   12.0 * m.param_elems * (L - o) + m.gpu_const_bytes;
    /* Eq. 2: host bytes (fp32 states + the shared 16-bit parameter/gradient buffer = 14 B/param). */
    s->cpu_bytes = 14.0 * m.param_elems * o + m.cpu_const_bytes;
    /* Eq. 3: forward critical path = compute stream or parameter prefetch. */
    s->t_fwd = std::max(m.t_fp * L, m.t_h2d * o + m.t_fp);
    /* Eq. 4: stalls of the backward compute stream on one-block-ahead parameter prefetch; v blocks
     * have both checkpointing and parameter offloading (both start from block 1, so v = min(c, p)). */
    const double v = (double)std::min(c, p);
    s->t_sync = v * std::max(m.t_h2d - m.t_fp - m.t_bp, 0.0) + ((double)p - v) * std::max(m.t_h2d - m.t_bp, 0.0);
    /* Eq. 5: backward critical path = compute stream (with recomputation, GPU optimizer updates and
     * stalls) or the host workflow. */
    s->t_bwd = std::max(m.t_bp * L + m.t_fp * c + m.t_optim_gpu * (L - o) + s->t_sync,
                        m.t_bp + m.t_d2h + m.t_optim_cpu * o);
    s->n_ckpt = c;
    s->n_param_offload = p;
    s->n_optim_offload = o;
    /* Constraints of Eq. 6, plus p <= o: blocks whose optimizer states stay on the GPU need no
     * parameter-offload decision (section 3.2.2, footnote to the peak-memory model). */
    s->feasible = (s->gpu_bytes <= m.gpu_capacity_bytes && s->cpu_bytes <= m.cpu_capacity_bytes && p <= o) ? 1 : 0;
}

}  // namespace

extern "C" {

int autohete_strategy_eval(const autohete_cost_model *model, uint32_t n_ckpt, uint32_t n_param_offload,
                           uint32_t n_optim_offload, autohete_strategy *out)
{
    if (!valid_model(model) || !out) return AH_EINVAL;
    if (n_ckpt > model->n_blocks || n_param_offload > model->n_blocks || n_optim_offload > model->n_blocks)
        return AH_EINVAL;
    evaluate(*model, n_ckpt, n_param_offload, n_optim_offload, out);
    return AH_OK;
}

int autohete_strategy_search(const autohete_cost_model *model, autohete_strategy *best)
{
    if (!valid_model(model) || !best) return AH_EINVAL;
    const uint32_t L = model->n_blocks;
    bool found = false;
    autohete_strategy cur;
    /* Enumeration order o, p, c ascending with a strict "<" keeps, among equal times, the least
     * optimizer offloading, then the least parameter offloading, then the least checkpointing. */
    for (uint32_t o = 0; o <= L; ++o)
        for (uint32_t p = 0; p <= o; ++p)
            for (uint32_t c = 0; c <= L; ++c) {
                evaluate(*model, c, p, o, &cur);
                if (!cur.feasible) continue;
                if (!found || cur.t_fwd + cur.t_bwd < best->t_fwd + best->t_bwd) {
                    *best = cur;
                    found = true;
                }
            }
    return found ? AH_OK : AH_EINFEASIBLE;
}

}  // extern "C"
