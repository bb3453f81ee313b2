#!/usr/bin/env python3
"""Hybrid placement end to end: the GPU half and the host half of one optimizer step.

Workload gpt-13b-half-resident (13B parameters, half of the chunks resident): the first half of the
chunks keeps its optimizer states in HBM, the second half keeps fp32 master / momentum / variance in host memory.
One step = global gradient norm on the GPU, the GPU update of the resident chunks, and for every
host-owned chunk: 16-bit gradients D2H, host AdamW (libautohete's AVX-512 path), 16-bit parameters
H2D, pipelined chunk by chunk (paper_2503_01890_amd/hybrid.py).  Reports the quantities the
paper's cost model takes as inputs: t_optim^gpu, t_optim^cpu, t_d2h, t_h2d (per parameter and per
transformer block), and the end-to-end step time.  Prints one JSON line.  Synthetic inputs.
"""
import argparse
import concurrent.futures as cf
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="gpt-13b-half-resident")
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--host-chunks", type=int, default=0, help="host-owned chunks to run (0 = all of the workload's)")
    ap.add_argument("--threads", type=int, default=0, help="host optimizer threads (0 = the box's CPU share)")
    args = ap.parse_args()

    import numpy as np
    import torch
    import synthdata
    from paper_2503_01890_amd import binding as B
    from paper_2503_01890_amd.hybrid import HostChunks, HybridStepper
    from paper_2503_01890_amd.modeldata import ModelData

    torch.cuda.set_device(0)
    st = torch.cuda.current_stream().cuda_stream
    w = synthdata.workload(args.workload)
    C, n_res = w.chunk_elems, w.n_resident
    n_host = args.host_chunks or (w.n_chunks - n_res)
    threads = args.threads or min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or 16)

    md = ModelData([C] * n_res)
    for c in range(n_res):
        synthdata.fill_gpu(md.ptr("param_lp", c), C, w.spec_param_lp(c), st)
        synthdata.fill_gpu(md.ptr("master", c), C, w.spec_master(c), st)
        synthdata.fill_gpu(md.ptr("exp_avg", c), C, w.spec_exp_avg(c), st)
        synthdata.fill_gpu(md.ptr("exp_avg_sq", c), C, w.spec_exp_avg_sq(c), st)
    host = HostChunks(n_host, C)

    def init_host(c):
        g = n_res + c
        synthdata.fill_cpu(host.master[c], w.spec_master(g))
        synthdata.fill_cpu(host.exp_avg[c], w.spec_exp_avg(g))
        synthdata.fill_cpu(host.exp_avg_sq[c], w.spec_exp_avg_sq(g))

    t0 = time.perf_counter()
    with cf.ThreadPoolExecutor(threads) as ex:
        list(ex.map(init_host, range(n_host)))
    for c in range(n_host):
        synthdata.fill_gpu(host.dev_view("param_lp", c).data_ptr(), C, w.spec_param_lp(n_res + c), st)
    t_init = time.perf_counter() - t0

    stepper = HybridStepper(md, host, w.dtype, threads)
    hp = B.hparams(**w.hparams, loss_scale=w.loss_scale)
    runs = []
    for it in range(1, args.warmup + args.steps + 1):
        for c in range(n_res):
            synthdata.fill_gpu(md.ptr("grad", c), C, w.spec_grad(c, it), st)
        for c in range(n_host):
            synthdata.fill_gpu(host.dev_view("grad", c).data_ptr(), C, w.spec_grad(n_res + c, it), st)
        torch.cuda.synchronize()
        r = stepper.step(it, hp)
        assert r["found_inf"] == 0
        if it > args.warmup:
            runs.append(r)
    mean = lambda k: sum(r[k] for r in runs) / len(runs)

    # PCIe legs on their own (pinned buffers, one chunk at a time, nothing else running)
    def copy_rate(to_host):
        torch.cuda.synchronize()
        a = time.perf_counter()
        for c in range(n_host):
            if to_host:
                host.stage[c].copy_(host.dev_view("grad", c), non_blocking=True)
            else:
                host.dev_view("param_lp", c).copy_(host.stage[c], non_blocking=True)
        torch.cuda.synchronize()
        return 2.0 * C * n_host / (time.perf_counter() - a)

    d2h_Bps, h2d_Bps = copy_rate(True), copy_rate(False)
    host_params = n_host * C
    block = 12 * 5120 ** 2 + 13 * 5120 if "13b" in w.name else C
    host_rate = host_params / mean("host_update_s")
    gpu_rate = n_res * C / mean("gpu_step_s")
    out = {
        "workload": w.name, "resident_chunks": n_res, "host_chunks": n_host, "chunk_elems": C,
        "host_threads": threads, "steps": args.steps, "host_init_s": t_init,
        "step_total_s": mean("total_s"),
        "gpu_share": {"params": n_res * C, "update_s": mean("gpu_step_s"), "params_per_s": gpu_rate,
                      "achieved_GBps": 28 * gpu_rate / 1e9},
        "host_share": {"params": host_params, "update_s": mean("host_update_s"), "params_per_s": host_rate,
                       "host_memory_GBps": 28 * host_rate / 1e9,
                       "waiting_for_gradients_s": mean("host_wait_for_grads_s")},
        "pcie": {"d2h_GBps": d2h_Bps / 1e9, "h2d_GBps": h2d_Bps / 1e9},
        "cost_model_inputs_per_block": {"block_params": block, "t_optim_gpu_s": block / gpu_rate,
                                        "t_optim_cpu_s": block / host_rate, "t_d2h_s": 2 * block / d2h_Bps,
                                        "t_h2d_s": 2 * block / h2d_Bps},
        "grad_norm": runs[-1]["norm"],
    }
    stepper.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
