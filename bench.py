#!/usr/bin/env python3
"""Benchmark of the chunked mixed-precision AdamW update on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic gradients:
autohete_grad_prep (unscale + finite check + global L2 norm) followed by autohete_adamw_step
(fused clip / AdamW / bias correction / decay / fp32 and 16-bit write-back) over every
GPU-resident chunk of the workload.  All inputs -- the model data and one gradient slab per
step -- are generated on the device and resident in HBM before the timed region starts.

Prints ONE JSON line: metric/value (parameters per second), ms_per_step, the whole-step HBM figure, a
`roofline` object for the dominant kernel, the prep kernel's figures and `cpu_baseline`.  The CPU oracle is timed on a
bounded sample of the same workload as a reported baseline only.
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

HBM_PEAK_GBPS = 8000.0           # MI355X published peak
STEP_BYTES_PER_ELEM = 28         # 14 read (g16, p32, m, v) + 14 written (p32, m, v, p16)
PREP_BYTES_PER_ELEM = 2          # g16 read


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="gpt-6.7b")
    ap.add_argument("--path", choices=("fused", "split"), default="fused",
                    help="fused: prep + adamw_step (headline).  split: prep + adamw_step_master (no 16-bit "
                         "write-back) + cast_params, the on-demand 16-bit materialisation variant")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--grad-slabs", type=int, default=0, help="gradient sets kept resident (0 = one per step if they fit)")
    ap.add_argument("--layout", choices=("group", "slab"), default="group",
                    help="HBM layout of the model data: groups of chunks, each group holding one run per stream "
                         "(default), or one slab per stream")
    ap.add_argument("--group-chunks", type=int, default=0, help="chunks per group of the group layout (0 = by size)")
    ap.add_argument("--step-variant", type=lambda x: int(x, 0), default=0, help="AH_TUNE_STEP_VARIANT value (0 = default)")
    ap.add_argument("--blocks-per-cu", type=int, default=0, help="AH_TUNE_STEP_BLOCKS_PER_CU (0 = default)")
    ap.add_argument("--prep-blocks", type=int, default=0, help="AH_TUNE_PREP_BLOCKS (0 = default)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain device copy of 4 GiB (known traffic: 4 GiB read + 4 GiB written per "
                         "launch) so that rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE readings can be scaled")
    ap.add_argument("--cpu-sample-log2", type=int, default=26,
                    help="log2 of the elements per thread in the oracle timing sample")
    return ap.parse_args()


def measured_traffic(workload):
    """HBM bytes per adamw_step launch from the committed rocprofv3 --pmc summary, if present."""
    path = os.path.join(ROOT, "profiles", "adamw_step_kernel_%s_pmc.txt" % workload)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def cpu_baseline(w, sample_log2):
    """Times the CPU oracle (prep + step, as it stands) on a bounded sample of the workload:
    single-threaded on one sample chunk, then one sample chunk per thread on all cores."""
    import numpy as np
    import oracle
    import synthdata

    n = 1 << sample_log2
    hp = oracle.hparams(**w.hparams, loss_scale=w.loss_scale)
    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1))

    def make(i):
        mk = lambda stream, sigma, kind, **kw: synthdata.fill_cpu(
            np.empty(n, np.uint16 if kind == synthdata.OUT_LOWP else np.float32),
            synthdata.make_spec(w.seed, stream, 1, i * n, sigma, kind, w.dtype, **kw))
        return dict(grad=mk(synthdata.STREAM_GRAD, 1e-3 * w.loss_scale, synthdata.OUT_LOWP,
                            outlier_prob=w.outlier_prob, sigma_outlier=w.loss_scale),
                    param_lp=mk(synthdata.STREAM_PARAM, 0.02, synthdata.OUT_LOWP),
                    master=mk(synthdata.STREAM_PARAM, 0.02, synthdata.OUT_F32_OF_LOWP),
                    exp_avg=mk(synthdata.STREAM_EXP_AVG, 1e-4, synthdata.OUT_F32),
                    exp_avg_sq=mk(synthdata.STREAM_EXP_AVG_SQ, 1e-6, synthdata.OUT_F32, take_abs=True))

    def one_step(c):
        s, f = oracle.grad_accumulate(c["grad"], w.dtype, w.loss_scale)
        return s, f

    def update(c, norm, flag):
        oracle.adamw_chunk(c["grad"], c["param_lp"], c["master"], c["exp_avg"], c["exp_avg_sq"], w.dtype, 1,
                           hp, norm, flag)

    with cf.ThreadPoolExecutor(cores) as ex:
        chunks = list(ex.map(make, range(cores)))
        # single thread, one chunk
        t0 = time.perf_counter()
        s, f = one_step(chunks[0])
        norm, flag = oracle.grad_finish(s, f)
        update(chunks[0], norm, flag)
        t_single = time.perf_counter() - t0
        # all cores, one chunk per thread (the C calls release the GIL)
        t0 = time.perf_counter()
        parts = list(ex.map(one_step, chunks))
        norm, flag = oracle.grad_finish(sum(p[0] for p in parts), max(p[1] for p in parts))
        list(ex.map(lambda c: update(c, norm, flag), chunks))
        t_all = time.perf_counter() - t0
    return {"value": n * cores / t_all, "unit": "params/s", "cores": cores, "kind": "oracle",
            "single_thread_value": n / t_single,
            "sample": "one step (prep + update) on %d chunks of 2^%d elements of %s-distributed model data, "
                      "one chunk per thread; single_thread_value is one such chunk on one thread"
                      % (cores, sample_log2, w.name)}


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus %d is not "
                 "supported -- run with --gpus 1" % args.gpus)
    import torch
    import synthdata
    from paper_2503_01890_amd import binding as B
    from paper_2503_01890_amd.modeldata import ModelData

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.zeros(1 << 30, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4}))
        return
    stream = torch.cuda.current_stream().cuda_stream
    w = synthdata.workload(args.workload)
    nres, C = w.n_resident, w.chunk_elems
    elems = nres * C                                   # elements each launch processes (padding included)
    n_valid = min(w.n_valid, elems)                    # parameters updated per step (padding excluded)

    # gradient slabs: one per step when they fit, else as many as fit, used round-robin
    total_steps = args.warmup + args.steps
    free, _ = torch.cuda.mem_get_info()
    state_bytes = elems * 14
    grad_bytes = elems * 2
    fit = int((free - state_bytes - (6 << 30)) // grad_bytes)
    n_sets = max(1, min(total_steps, fit, args.grad_slabs or total_steps))
    md = ModelData([C] * nres, n_grad_sets=n_sets, layout=args.layout, group_chunks=args.group_chunks or None)
    for c in range(nres):
        synthdata.fill_gpu(md.ptr("param_lp", c), C, w.spec_param_lp(c), stream)
        synthdata.fill_gpu(md.ptr("master", c), C, w.spec_master(c), stream)
        synthdata.fill_gpu(md.ptr("exp_avg", c), C, w.spec_exp_avg(c), stream)
        synthdata.fill_gpu(md.ptr("exp_avg_sq", c), C, w.spec_exp_avg_sq(c), stream)
        for s in range(n_sets):
            synthdata.fill_gpu(md.ptr("grad", c, s), C, w.spec_grad(c, s + 1), stream)
    torch.cuda.synchronize()

    ws = B.Workspace(nres)
    ws.tune(B.AH_TUNE_STEP_VARIANT, args.step_variant)
    ws.tune(B.AH_TUNE_STEP_BLOCKS_PER_CU, args.blocks_per_cu)
    ws.tune(B.AH_TUNE_PREP_BLOCKS, args.prep_blocks)
    hp = B.hparams(**w.hparams, loss_scale=w.loss_scale)
    arrays = [md.chunk_array(grad_set=s) for s in range(n_sets)]
    extra = 0.0
    if nres < w.n_chunks:
        # squared norm of the gradients of the chunks that stay in host memory (a placement's
        # host share): what a caller would pass in; here the expected value of the distribution
        extra = float((w.n_valid - n_valid) * (1e-3 ** 2 * (1 - w.outlier_prob) + w.outlier_prob))

    split = args.path == "split"

    def one_step(i, t, ev=None):
        arr = arrays[i % n_sets]
        if ev:
            ev[0].record()
        ws.autohete_grad_prep(arr, nres, w.dtype, w.loss_scale, extra, stream)
        if ev:
            ev[1].record()
        if split:
            ws.autohete_adamw_step_master(arr, nres, w.dtype, t, hp, stream)
        else:
            ws.autohete_adamw_step(arr, nres, w.dtype, t, hp, stream)
        if ev:
            ev[2].record()
        if split:
            ws.autohete_cast_params(arr, nres, w.dtype, stream)
            if ev:
                ev[3].record()

    for i in range(args.warmup):
        one_step(i, i + 1)
    # Timing events are created and recorded once here, outside the timed region: the first record of
    # a timing event in a process can take tens of milliseconds on the host (runtime set-up).
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    for ev in events:
        for e in ev:
            e.record()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_step(args.warmup + k, args.warmup + k + 1, events[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sumsq, norm, flag = ws.autohete_grad_result_get(stream)
    assert flag == 0, "synthetic gradients must be finite"

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    prep_all = sorted(e[0].elapsed_time(e[1]) for e in events)
    step_all = sorted(e[1].elapsed_time(e[2]) for e in events)
    prep_ms, step_ms = sum(prep_all) / args.steps, sum(step_all) / args.steps
    median = lambda xs: 0.5 * (xs[(len(xs) - 1) // 2] + xs[len(xs) // 2])
    step_bytes = 26 if split else STEP_BYTES_PER_ELEM        # no 16-bit write-back in the split path
    total_bytes = step_bytes + PREP_BYTES_PER_ELEM + (6 if split else 0)
    step_gbps = step_bytes * elems / step_ms / 1e6
    prep_gbps = PREP_BYTES_PER_ELEM * elems / prep_ms / 1e6
    both_gbps = total_bytes * elems / ms_per_step / 1e6

    out = {
        "metric": "AdamW chunk-update params/sec",
        "value": n_valid * args.steps / (t1 - t0),
        "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64",      # arithmetic type of the update (fp32/16-bit storage, fp64 arithmetic)
        "data": "synthetic",
        "config": {"workload": w.name, "params": w.n_valid, "resident_params": n_valid,
                   "chunks": nres, "chunk_elems": C, "lowp": "bf16" if w.dtype == B.AH_BF16 else "fp16",
                   "path": args.path, "layout": args.layout if args.layout == "slab" else "groups of %d chunks" % md.group_chunks, "grad_slabs_resident": n_sets, "grad_norm": norm,
                   "hparams": dict(w.hparams, loss_scale=w.loss_scale)},
        "hbm": {"achieved_GBps": both_gbps, "frac_of_peak": both_gbps / HBM_PEAK_GBPS,
                "bytes_per_param": total_bytes,
                "note": "whole step (%s), algorithmic bytes per element, wall clock"
                        % ("prep + update without 16-bit write-back + cast" if split else "prep + update")},
        "roofline": {"kernel": "adamw_step_kernel", "bound": "hbm", "achieved": step_gbps,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": step_gbps / HBM_PEAK_GBPS,
                     "traffic": None if split else measured_traffic(w.name),
                     "algorithmic_bytes_per_launch": step_bytes * elems,
                     "avg_launch_ms": step_ms, "median_launch_ms": median(step_all), "min_launch_ms": step_all[0]},
        "prep_kernel": {"kernel": "grad_prep_kernel", "achieved": prep_gbps, "unit": "GB/s",
                        "frac": prep_gbps / HBM_PEAK_GBPS, "avg_launch_ms": prep_ms, "median_launch_ms": median(prep_all),
                        "min_launch_ms": prep_all[0]},
    }
    if split:
        cast_ms = sum(e[2].elapsed_time(e[3]) for e in events) / args.steps
        out["cast_kernel"] = {"kernel": "cast_params_kernel", "achieved": 6 * elems / cast_ms / 1e6, "unit": "GB/s",
                              "frac": 6 * elems / cast_ms / 1e6 / HBM_PEAK_GBPS, "avg_launch_ms": cast_ms}
    ws.close()
    del md
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_sample_log2)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
