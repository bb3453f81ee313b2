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
    ap.add_argument("--plan", action="store_true",
                    help="also time a plain streaming pass on the host threads, measure a synthetic transformer "
                         "block's GEMMs, and feed all measured costs to autohete_strategy_search")
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
    if args.plan:
        del md, host, stepper
        torch.cuda.empty_cache()
        out["host_streaming_roofline"] = host_stream_rate(threads)
        out["plan"] = plan(w, out["cost_model_inputs_per_block"], args)
    print(json.dumps(out))


def host_stream_rate(threads, log2_elems=27):
    """What the same host threads reach on a plain streaming pass with the update's traffic (per
    element: 2 + 12 bytes read, 12 + 2 written) and no arithmetic beyond copies: the roofline the
    host optimizer's rate is read against."""
    import concurrent.futures as cf
    import numpy as np
    n = 1 << log2_elems
    per = n // threads
    src = [np.ones(per, np.float32) for _ in range(threads)]
    dst = [[np.empty(per, np.float32) for _ in range(3)] for _ in range(threads)]
    g = [np.ones(per, np.uint16) for _ in range(threads)]

    def work(t):
        for k in range(3):
            np.copyto(dst[t][k], src[t])          # 4 B read + 4 B written, three streams
        np.copyto(g[t], g[t])                     # 2 B read + 2 B written
    with cf.ThreadPoolExecutor(threads) as ex:
        list(ex.map(work, range(threads)))
        t0 = time.perf_counter()
        for _ in range(3):
            list(ex.map(work, range(threads)))
        dt = (time.perf_counter() - t0) / 3
    return {"GBps": 28.0 * per * threads / dt / 1e9, "params_per_s": per * threads / dt, "threads": threads,
            "what": "numpy copies of three fp32 streams and one 16-bit stream, %d elements per thread" % per}


def plan(w, per_block, args):
    """Feeds the costs measured above into the library's cost model and strategy search (paper Eq. 1-6)
    for this workload's transformer block.  t_fp / t_bp are measured on the block's four bf16 weight
    GEMMs at the paper's batch (8 sequences of 1024 tokens; attention scores left out), activations
    are taken as 17 b s d elements per block (34 b s d bytes in 16 bits) with b s d kept by a
    checkpointed block: stand-ins for what a profiler of a real model would supply."""
    import torch
    from paper_2503_01890_amd import binding as B
    d = {"gpt-13b-half-resident": 5120, "gpt-6.7b": 4096, "gpt-1.3b": 2048, "gpt-124m": 768}[w.name]
    n_layers = (len(w.tensor_numel) - 2) // 12
    tokens = 8 * 1024
    x = torch.randn(tokens, d, device="cuda:0", dtype=torch.bfloat16)
    x4 = torch.randn(tokens, 4 * d, device="cuda:0", dtype=torch.bfloat16)
    ws_ = [torch.randn(d, k * d, device="cuda:0", dtype=torch.bfloat16) for k in (3, 1, 4)]
    w_down = torch.randn(4 * d, d, device="cuda:0", dtype=torch.bfloat16)

    def fwd():
        for m in ws_:
            torch.matmul(x, m)
        torch.matmul(x4, w_down)
    for _ in range(3):
        fwd()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(10):
        fwd()
    torch.cuda.synchronize()
    t_fp = (time.perf_counter() - t0) / 10
    host_ram = os.sysconf("SC_PAGE_SIZE") * os.sysconf("SC_PHYS_PAGES")
    block = per_block["block_params"]
    model = dict(n_blocks=n_layers, act_elems=17.0 * tokens * d, act_in_elems=1.0 * tokens * d, param_elems=float(block),
                 gpu_const_bytes=2.0 * 16 * float(w.tensor_numel[0] + w.tensor_numel[1]) + 2e9, cpu_const_bytes=2e9,
                 gpu_capacity_bytes=288e9, cpu_capacity_bytes=float(host_ram), t_fp=t_fp, t_bp=2 * t_fp,
                 t_h2d=per_block["t_h2d_s"], t_d2h=per_block["t_d2h_s"], t_optim_cpu=per_block["t_optim_cpu_s"],
                 t_optim_gpu=per_block["t_optim_gpu_s"])
    res = {"inputs": model}
    for name, cap in (("mi355x_288GB", 288e9), ("gpu_80GB", 80e9), ("gpu_40GB", 40e9)):
        cm = B.autohete_cost_model(**dict(model, gpu_capacity_bytes=cap))
        try:
            s = B.autohete_strategy_search(cm)
            res[name] = {"ckpt_blocks": s.n_ckpt, "param_offload_blocks": s.n_param_offload,
                         "optim_offload_blocks": s.n_optim_offload, "eq1_gpu_bytes": s.gpu_bytes,
                         "eq2_cpu_bytes": s.cpu_bytes, "t_fwd_s": s.t_fwd, "t_sync_s": s.t_sync, "t_bwd_s": s.t_bwd}
        except B.AutoheteError as e:
            res[name] = {"infeasible": str(e)}
    return res


if __name__ == "__main__":
    main()
