/* A plain C99 caller of the C ABI (host-only entry points: no GPU needed).  Built and run by
 * tests/test_abi_cpu.py against libautohete.so: proves that include/autohete.h is valid C and that
 * the library can be used without Python or C++. */
#include <math.h>
#include <stdio.h>
#include <string.h>

#include "autohete.h"

#define CHECK(cond)                                                  \
    do {                                                             \
        if (!(cond)) {                                               \
            printf("FAILED line %d: %s\n", __LINE__, #cond);         \
            return 1;                                                \
        }                                                            \
    } while (0)

int main(void)
{
    /* chunk layout: three tensors into chunks of 8 elements */
    uint64_t numel[3] = {5, 8, 4}, off[3], n_chunks, total, padded;
    CHECK(autohete_chunk_layout(numel, 3, 8, off, &n_chunks, &total, &padded) == AH_OK);
    CHECK(off[0] == 0 && off[1] == 5 && off[2] == 13 && n_chunks == 3 && total == 17 && padded == 7);
    CHECK(autohete_chunk_layout(numel, 3, 0, off, &n_chunks, &total, &padded) == AH_EINVAL);
    CHECK(strcmp(autohete_strerror(AH_OK), "ok") == 0);

    /* host optimizer: zero gradient, zero moments -> pure decay p (1 - lr wd), exactly */
    uint16_t grad[4] = {0, 0, 0, 0}, lp[4] = {0, 0, 0, 0};
    float master[4] = {1.0f, -2.0f, 0.5f, 0.0f}, m[4] = {0, 0, 0, 0}, v[4] = {0, 0, 0, 0};
    autohete_chunk c;
    autohete_hparams hp;
    double sumsq = -1.0;
    uint32_t flag = 9;
    c.grad = grad; c.param_lp = lp; c.master = master; c.exp_avg = m; c.exp_avg_sq = v; c.numel = 4;
    hp.lr = 0.25f; hp.beta1 = 0.5f; hp.beta2 = 0.5f; hp.eps = 1.0f; hp.weight_decay = 0.5f;
    hp.max_grad_norm = 1.0f; hp.loss_scale = 1.0f;
    CHECK(autohete_host_grad_sumsq(&c, 1, AH_BF16, 1.0f, 1, &sumsq, &flag) == AH_OK);
    CHECK(sumsq == 0.0 && flag == 0);
    CHECK(autohete_host_adamw_step(&c, 1, AH_BF16, 1, &hp, sumsq, flag, 1) == AH_OK);
    CHECK(master[0] == 0.875f && master[1] == -1.75f && master[2] == 0.4375f && master[3] == 0.0f);
    CHECK(lp[0] == 0x3F60 && lp[1] == 0xBFE0 && lp[2] == 0x3EE0 && lp[3] == 0); /* bf16 of the above, exact */
    CHECK(m[0] == 0.0f && v[0] == 0.0f);
    CHECK(autohete_host_adamw_step(&c, 1, 7, 1, &hp, sumsq, flag, 1) == AH_EINVAL);

    /* strategy search: memory to spare -> nothing offloaded */
    autohete_cost_model cm;
    autohete_strategy best;
    memset(&cm, 0, sizeof cm);
    cm.n_blocks = 2; cm.act_elems = 10; cm.act_in_elems = 2; cm.param_elems = 100; cm.gpu_const_bytes = 50;
    cm.cpu_const_bytes = 7; cm.gpu_capacity_bytes = 1e9; cm.cpu_capacity_bytes = 1e9; cm.t_fp = 1; cm.t_bp = 2;
    cm.t_h2d = 4; cm.t_d2h = 0.5; cm.t_optim_cpu = 3; cm.t_optim_gpu = 0.25;
    CHECK(autohete_strategy_search(&cm, &best) == AH_OK);
    CHECK(best.n_ckpt == 0 && best.n_param_offload == 0 && best.n_optim_offload == 0 && best.feasible);
    CHECK(best.t_fwd + best.t_bwd == 2 * (1 + 2 + 0.25));
    cm.gpu_capacity_bytes = 100;
    CHECK(autohete_strategy_search(&cm, &best) == AH_EINFEASIBLE);

    /* device entry points reject bad arguments before they touch a device */
    CHECK(autohete_grad_prep(NULL, NULL, 0, AH_BF16, 1.0f, 0.0, NULL, NULL, NULL) == AH_EINVAL);
    CHECK(autohete_grad_prep_static(NULL, 1, AH_BF16, 1.0f, 0.0, NULL, NULL) == AH_EINVAL);
    CHECK(sizeof(autohete_grad_result) == 24 && sizeof(autohete_chunk) == 48);
    printf("c abi host: ok\n");
    return 0;
}
