#!/usr/bin/env python3
"""Benchmark of the chunked mixed-precision AdamW update on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic gradients:
autohete_grad_prep (unscale + finite check + global L2 norm) followed by autohete_adamw_step
(fused clip / AdamW / bias correction / decay / fp32 and 16-bit write-back) over every
GPU-resident chunk of the workload.  All inputs -- the model data and one gradient slab per
step -- are generated on the device and resident in HBM before the timed region starts.

Prints ONE JSON line.  Headline (metric/value/ms_per_step/roofline/...): the 6.7B configuration,
fused path.  With the default invocation the same line also carries
  "paths"      the other ways of stepping the same 6.7B model data: the split path (update
               without 16-bit write-back + on-demand cast) and per-block stepping in backward
               order through the norm-carrying update;
  "workloads"  the other four configurations (fused path), each with its whole-step and
               per-kernel figures;
  "cpu_baseline"  the CPU oracle timed on a bounded sample of the headline workload (a reported
               baseline only).
--workload X makes X the headline and leaves the extras out; --headline-only does the latter.
"""
import argparse
import concurrent.futures as cf
import gc
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
HEADLINE = "gpt-6.7b"
OTHER_WORKLOADS = ("gpt-124m", "gpt-1.3b", "gpt-13b-half-resident", "ragged-fp16")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default=None, help="headline workload (default %s, with the other "
                    "configurations and paths appended)" % HEADLINE)
    ap.add_argument("--path", choices=("fused", "split", "per_block_carry"), default="fused",
                    help="fused: prep + adamw_step (headline).  split: prep + adamw_step_master (no 16-bit "
                         "write-back) + cast_params.  per_block_carry: one autohete_adamw_step_carry per "
                         "optimizer partition, last block first")
    ap.add_argument("--headline-only", action="store_true", help="leave out the other paths and workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--grad-slabs", type=int, default=4,
                    help="gradient sets kept resident and used round-robin, one per step (default 4: at least 1 GB "
                         "of gradients for every workload, four times the chip's 256 MB last-level cache, so no "
                         "step finds its gradients cached; 0 = one per step if they fit)")
    ap.add_argument("--layout", choices=("group", "slab"), default="group",
                    help="HBM layout of the model data: groups of chunks, each group holding one run per stream "
                         "(default), or one slab per stream")
    ap.add_argument("--group-chunks", type=int, default=0, help="chunks per group of the group layout (0 = by size)")
    ap.add_argument("--step-variant", type=lambda x: int(x, 0), default=0, help="AH_TUNE_STEP_VARIANT value (0 = default)")
    ap.add_argument("--blocks-per-cu", type=int, default=0, help="AH_TUNE_STEP_BLOCKS_PER_CU (0 = default)")
    ap.add_argument("--prep-blocks", type=int, default=0, help="AH_TUNE_PREP_BLOCKS (0 = default)")
    ap.add_argument("--cast-blocks-per-cu", type=int, default=0, help="AH_TUNE_CAST_BLOCKS_PER_CU (0 = default)")
    ap.add_argument("--blocks-per-call", type=int, default=1,
                    help="per_block_carry path: optimizer partitions (transformer blocks) stepped by one call")
    ap.add_argument("--graph", action="store_true",
                    help="fused path only: record each step (prep + update) into a HIP graph once and time replays")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain device copy of 4 GiB (known traffic: 4 GiB read + 4 GiB written per "
                         "launch) so that rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE readings can be scaled")
    ap.add_argument("--cpu-sample-log2", type=int, default=26,
                    help="log2 of the elements per thread in the oracle timing sample")
    return ap.parse_args()


def measured_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` on `workload` from the committed rocprofv3 --pmc summary
    (a stored figure, measured in a profiler run of its own: counters perturb timing).
    -> (bytes or None, path of the summary relative to the repository or None)"""
    rel = os.path.join("profiles", "%s_%s_pmc.txt" % (kernel, workload))
    try:
        for line in open(os.path.join(ROOT, rel)):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1]), rel
    except OSError:
        pass
    return None, None


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


class Resident:
    """One workload's model data in HBM (state + as many gradient sets as fit, at most one per
    step), filled by the device half of the seeded generator."""

    def __init__(self, w, args, total_steps):
        import torch
        import synthdata
        from paper_2503_01890_amd.modeldata import ModelData
        self.w = w
        self.stream = stream = torch.cuda.current_stream().cuda_stream
        self.nres, self.C = nres, C = w.n_resident, w.chunk_elems
        self.elems = nres * C                                   # elements each launch processes (padding included)
        self.n_valid = min(w.n_valid, self.elems)               # parameters updated per step (padding excluded)
        free, _ = torch.cuda.mem_get_info()
        fit = int((free - self.elems * 14 - (6 << 30)) // (self.elems * 2))
        self.n_sets = max(1, min(total_steps, fit, args.grad_slabs or total_steps))
        self.md = md = ModelData([C] * nres, n_grad_sets=self.n_sets, layout=args.layout,
                                 group_chunks=args.group_chunks or None)
        for c in range(nres):
            synthdata.fill_gpu(md.ptr("param_lp", c), C, w.spec_param_lp(c), stream)
            synthdata.fill_gpu(md.ptr("master", c), C, w.spec_master(c), stream)
            synthdata.fill_gpu(md.ptr("exp_avg", c), C, w.spec_exp_avg(c), stream)
            synthdata.fill_gpu(md.ptr("exp_avg_sq", c), C, w.spec_exp_avg_sq(c), stream)
            for s in range(self.n_sets):
                synthdata.fill_gpu(md.ptr("grad", c, s), C, w.spec_grad(c, s + 1), stream)
        torch.cuda.synchronize()
        self.arrays = [md.chunk_array(grad_set=s) for s in range(self.n_sets)]
        # squared norm of the gradients of the chunks that stay in host memory (a placement's host
        # share): what a caller would pass in; here the expected value of the distribution
        self.extra = 0.0
        if nres < w.n_chunks:
            self.extra = float((w.n_valid - self.n_valid) * (1e-3 ** 2 * (1 - w.outlier_prob) + w.outlier_prob))

    def release(self):
        import torch
        self.md = self.arrays = None
        gc.collect()
        torch.cuda.empty_cache()


def measure_graph(res, steps, warmup, args):
    """The fused step recorded into HIP graphs, one per resident gradient set, after a warm-up on
    the capture stream (the chunk tables are on the device by then: each recording holds the two
    kernels and nothing else), then `steps` replays timed between two device synchronisations."""
    import torch
    from paper_2503_01890_amd import binding as B
    w, nres = res.w, res.nres
    ws = B.Workspace(nres + 2)
    ws.tune(B.AH_TUNE_STEP_VARIANT, args.step_variant)
    ws.tune(B.AH_TUNE_STEP_BLOCKS_PER_CU, args.blocks_per_cu)
    ws.tune(B.AH_TUNE_PREP_BLOCKS, args.prep_blocks)
    hp = B.hparams(**w.hparams, loss_scale=w.loss_scale)
    side = torch.cuda.Stream()                                   # default priority
    n_graphs = min(res.n_sets, steps)

    def one_step(i):
        ws.autohete_grad_prep(res.arrays[i], nres, w.dtype, w.loss_scale, res.extra, side.cuda_stream)
        ws.autohete_adamw_step(res.arrays[i], nres, w.dtype, i + 1, hp, side.cuda_stream)

    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for i in range(n_graphs):
            one_step(i)
    side.synchronize()
    graphs = []
    for i in range(n_graphs):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            one_step(i)
        graphs.append(g)
    for i in range(warmup):
        graphs[i % n_graphs].replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        graphs[k % n_graphs].replay()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    assert ws.autohete_grad_result_get(res.stream)[2] == 0
    ws.close()
    ms = (t1 - t0) * 1e3 / steps
    total_bytes = STEP_BYTES_PER_ELEM + PREP_BYTES_PER_ELEM
    return {"ms_per_step": ms, "params_per_s": res.n_valid * steps / (t1 - t0),
            "whole_step_frac": total_bytes * res.elems / ms / 1e6 / HBM_PEAK_GBPS, "graphs": n_graphs, "steps": steps}


def measure(res, path, steps, warmup, args):
    """Times `steps` steps of `path` on the resident workload (after `warmup` untimed ones) between
    two device synchronisations, with events around every kernel on the launch stream."""
    import torch
    from paper_2503_01890_amd import binding as B
    w, md, stream, nres, elems = res.w, res.md, res.stream, res.nres, res.elems
    ws = B.Workspace(nres + 2)
    ws.tune(B.AH_TUNE_STEP_VARIANT, args.step_variant)
    ws.tune(B.AH_TUNE_STEP_BLOCKS_PER_CU, args.blocks_per_cu)
    ws.tune(B.AH_TUNE_PREP_BLOCKS, args.prep_blocks)
    ws.tune(B.AH_TUNE_CAST_BLOCKS_PER_CU, getattr(args, "cast_blocks_per_cu", 0))
    hp = B.hparams(**w.hparams, loss_scale=w.loss_scale)
    n_ev = {"fused": 3, "split": 4, "per_block_carry": 2}[path]

    if path == "per_block_carry":
        # Optimizer partitions (embedding tables, then each transformer block), stepped last block
        # first: each update clips with the previous iteration's norm (workspace `cur`) while the
        # squares of the gradients it reads are gathered for the next (`nxt`); two workspaces alternate.
        assert nres == w.n_chunks, "per-block stepping is measured on a fully resident workload"
        other = B.Workspace(nres + 2)
        for x in (ws, other):
            x.tune(B.AH_TUNE_CARRY_ELEMS, elems)
        other.tune(B.AH_TUNE_STEP_BLOCKS_PER_CU, args.blocks_per_cu)
        bounds = w.partition_bounds()
        per_call = max(1, getattr(args, "blocks_per_call", 1))
        bounds = bounds[:-1][::per_call] + bounds[-1:]         # several adjacent partitions per call
        parts = []
        for s in range(res.n_sets):
            per_set = []
            for a, b in zip(bounds[:-1], bounds[1:]):
                tup = md.range_tuples(a, b, grad_set=s)
                per_set.append((B.chunk_array(tup), len(tup)))
            per_set.reverse()
            parts.append(per_set)
        ws.autohete_grad_prep(res.arrays[0], nres, w.dtype, w.loss_scale, 0.0, stream)   # a norm to start from
        pair = [ws, other]

    def one_step(i, t, ev=None):
        arr = res.arrays[i % res.n_sets]
        if ev:
            ev[0].record()
        if path == "per_block_carry":
            cur, nxt = pair[i % 2], pair[(i + 1) % 2]
            nxt.autohete_grad_result_set(0.0, 0, stream)
            for chunks, k in parts[i % res.n_sets]:
                cur.autohete_adamw_step_carry(nxt, chunks, k, w.dtype, t, hp, stream)
            if ev:
                ev[1].record()
            return
        ws.autohete_grad_prep(arr, nres, w.dtype, w.loss_scale, res.extra, stream)
        if ev:
            ev[1].record()
        if path == "split":
            ws.autohete_adamw_step_master(arr, nres, w.dtype, t, hp, stream)
        else:
            ws.autohete_adamw_step(arr, nres, w.dtype, t, hp, stream)
        if ev:
            ev[2].record()
        if path == "split":
            ws.autohete_cast_params(arr, nres, w.dtype, stream)
            ev and ev[3].record()

    for i in range(warmup):
        one_step(i, i + 1)
    # Timing events are created and recorded once here, outside the timed region: the first record of
    # a timing event in a process can take tens of milliseconds on the host (runtime set-up).
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(n_ev)] for _ in range(steps)]
    for ev in events:
        for e in ev:
            e.record()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        one_step(warmup + k, warmup + k + 1, events[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    last = pair[(warmup + steps) % 2] if path == "per_block_carry" else ws
    sumsq, norm, flag = last.autohete_grad_result_get(stream)
    assert flag == 0, "synthetic gradients must be finite"

    ms_per_step = (t1 - t0) * 1e3 / steps
    median = lambda xs: 0.5 * (xs[(len(xs) - 1) // 2] + xs[len(xs) // 2])

    def kernel(name, a, b, bytes_per_elem, launches=1):
        xs = sorted(e[a].elapsed_time(e[b]) for e in events)
        avg = sum(xs) / len(xs)
        gbps = bytes_per_elem * elems / avg / 1e6
        out = {"kernel": name, "bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
               "frac": gbps / HBM_PEAK_GBPS, "algorithmic_bytes_per_launch": bytes_per_elem * elems // launches,
               "avg_launch_ms": avg / launches, "median_launch_ms": median(xs) / launches,
               "min_launch_ms": xs[0] / launches}
        if launches > 1:
            out["launches_per_step"] = launches
        return out

    if path == "per_block_carry":
        total_bytes = STEP_BYTES_PER_ELEM
        n_launch = len(parts[0])     # whole-chunk and partial-chunk groups of a partition may be separate launches
        kernels = {"step": kernel("adamw_step_carry_kernel", 0, 1, STEP_BYTES_PER_ELEM, n_launch)}
        kernels["step"]["note"] = ("%d partitions per step, launched back to back; figures are per partition, "
                                   "achieved/frac over the whole step's kernels" % n_launch)
    elif path == "split":
        total_bytes = 26 + PREP_BYTES_PER_ELEM + 6
        kernels = {"prep": kernel("grad_prep_kernel", 0, 1, PREP_BYTES_PER_ELEM),
                   "step": kernel("adamw_step_kernel (no 16-bit write-back)", 1, 2, 26),
                   "cast": kernel("cast_params_kernel", 2, 3, 6)}
    else:
        total_bytes = STEP_BYTES_PER_ELEM + PREP_BYTES_PER_ELEM
        kernels = {"prep": kernel("grad_prep_kernel", 0, 1, PREP_BYTES_PER_ELEM),
                   "step": kernel("adamw_step_kernel", 1, 2, STEP_BYTES_PER_ELEM)}
    both_gbps = total_bytes * elems / ms_per_step / 1e6
    ws.close()
    if path == "per_block_carry":
        other.close()
    return {"value": res.n_valid * steps / (t1 - t0), "ms_per_step": ms_per_step, "steps": steps, "warmup": warmup,
            "grad_norm": norm, "kernels": kernels,
            "hbm": {"achieved_GBps": both_gbps, "frac_of_peak": both_gbps / HBM_PEAK_GBPS, "bytes_per_param": total_bytes,
                    "note": "whole step, algorithmic bytes per element, wall clock"}}


def config_of(res, path, args):
    from paper_2503_01890_amd import binding as B
    w = res.w
    return {"workload": w.name, "params": w.n_valid, "resident_params": res.n_valid, "chunks": res.nres,
            "chunk_elems": res.C, "elements_per_launch": res.elems, "lowp": "bf16" if w.dtype == B.AH_BF16 else "fp16",
            "path": path,
            "layout": args.layout if args.layout == "slab" else "groups of %d chunks" % res.md.group_chunks,
            "grad_slabs_resident": res.n_sets, "hparams": dict(w.hparams, loss_scale=w.loss_scale)}


def brief(m, res):
    """One extra leg (another workload or path) as it appears in the JSON line."""
    out = {"ms_per_step": m["ms_per_step"], "params_per_s": m["value"], "elements_per_launch": res.elems,
           "whole_step_frac": m["hbm"]["frac_of_peak"], "bytes_per_param": m["hbm"]["bytes_per_param"],
           "steps": m["steps"]}
    for k, v in m["kernels"].items():
        out[k] = {x: v[x] for x in ("kernel", "avg_launch_ms", "achieved", "frac", "launches_per_step") if x in v}
    return out


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus %d is not "
                 "supported -- run with --gpus 1" % args.gpus)
    import torch
    import synthdata

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
    extras = args.workload is None and args.path == "fused" and not args.headline_only
    w = synthdata.workload(args.workload or HEADLINE)
    res = Resident(w, args, args.warmup + args.steps)
    m = measure(res, args.path, args.steps, args.warmup, args)
    if args.graph and args.path == "fused":
        m["hip_graph"] = measure_graph(res, args.steps, args.warmup, args)

    step = m["kernels"]["step"]
    traffic, source = (measured_traffic("adamw_step_kernel", w.name) if args.path == "fused" else (None, None))
    roofline = dict(step, traffic=traffic, traffic_source=source)
    out = {
        "metric": "AdamW chunk-update params/sec",
        "value": m["value"],
        "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": m["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64",      # arithmetic type of the update (fp32/16-bit storage, fp64 arithmetic)
        "data": "synthetic",
        "config": dict(config_of(res, args.path, args), grad_norm=m["grad_norm"]),
        "hbm": m["hbm"],
        "roofline": roofline,
    }
    for k, v in m["kernels"].items():
        if k != "step":
            out[k + "_kernel"] = v
    if "hip_graph" in m:
        out["hip_graph"] = m["hip_graph"]
    if extras:
        # the same model data stepped the other two ways (fewer steps: they only need a stable mean)
        k = max(3, args.steps // 2)
        out["paths"] = {p: brief(measure(res, p, k, 2, args), res) for p in ("split", "per_block_carry")}
    res.release()
    if extras:
        out["workloads"] = {}
        for name in OTHER_WORKLOADS:
            wk = synthdata.workload(name)
            r = Resident(wk, args, 2 + 20)
            out["workloads"][name] = brief(measure(r, "fused", 20, 2, args), r)
            if r.elems < (1 << 31):       # short steps: what recording the two launches into a HIP graph changes
                out["workloads"][name]["hip_graph"] = measure_graph(r, 20, 2, args)
            r.release()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_sample_log2)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
