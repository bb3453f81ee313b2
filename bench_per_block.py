#!/usr/bin/env python3
"""Per-block optimizer stepping, alone and overlapped with a synthetic compute stream.

The paper steps each transformer block's optimizer as soon as that block's gradients exist
(section 3.2.2, footnote to Eq. 5) and charges t_optim^gpu per block on the backward critical
path (Eq. 5, first arm).  This script measures, for one workload on one MI355X:

  one_shot      one grad_prep + one adamw_step over all chunks (what bench.py times)
  per_block     the same work issued block by block in backward order: for every partition
                (embedding, then each transformer block) one autohete_grad_prep_accumulate into
                the NEXT iteration's norm and one autohete_adamw_step that clips with the
                PREVIOUS iteration's norm (a global norm cannot be known before the last block's
                gradients exist); two workspaces alternate
  per_block_carry  the same schedule through autohete_adamw_step_carry: one launch per partition
                updates it and gathers its squares for the next norm, reading the gradients once
                (28 B/element instead of 30)
  compute       a synthetic backward pass: bf16 GEMMs per block on the compute stream
  overlapped    compute on one stream, per-block optimizer work on a second stream of the same
                (default) priority, block i's optimizer work released by an event after block i's
                GEMMs -- the schedule of the paper's backward phase

Prints one JSON line.  Not the headline benchmark; inputs are synthetic and resident in HBM.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="gpt-6.7b")
    ap.add_argument("--iters", type=int, default=6)
    ap.add_argument("--gemm", type=int, default=8192, help="edge of the square bf16 GEMMs of the synthetic backward")
    ap.add_argument("--gemms-per-block", type=int, default=2)
    ap.add_argument("--blocks-per-cu", type=int, default=0, help="AH_TUNE_STEP_BLOCKS_PER_CU (0 = default)")
    args = ap.parse_args()

    import torch
    import synthdata
    from paper_2503_01890_amd import binding as B
    from paper_2503_01890_amd.modeldata import ModelData

    torch.cuda.set_device(0)
    main_stream = torch.cuda.current_stream()
    side = torch.cuda.Stream()                       # default priority
    w = synthdata.workload(args.workload)
    assert w.n_resident == w.n_chunks, "per-block stepping is measured on a fully resident workload"
    C, n = w.chunk_elems, w.n_chunks
    md = ModelData([C] * n)
    st = main_stream.cuda_stream
    for c in range(n):
        synthdata.fill_gpu(md.ptr("param_lp", c), C, w.spec_param_lp(c), st)
        synthdata.fill_gpu(md.ptr("master", c), C, w.spec_master(c), st)
        synthdata.fill_gpu(md.ptr("exp_avg", c), C, w.spec_exp_avg(c), st)
        synthdata.fill_gpu(md.ptr("exp_avg_sq", c), C, w.spec_exp_avg_sq(c), st)
        synthdata.fill_gpu(md.ptr("grad", c), C, w.spec_grad(c, 1), st)
    torch.cuda.synchronize()

    # partitions of the flat element space: embedding + positions, then 12 tensors per block
    off, _, total, _ = B.autohete_chunk_layout([int(x) for x in w.tensor_numel], C)
    n_layers = (len(off) - 2) // 12
    bounds = [0, off[2]] + [off[2 + 12 * (i + 1)] if 2 + 12 * (i + 1) < len(off) else total for i in range(n_layers)]
    bounds[-1] = n * C                               # the last partition also carries the padding
    parts = []
    for a, b in zip(bounds[:-1], bounds[1:]):
        tup = md.range_tuples(a, b)
        parts.append((B.chunk_array(tup), len(tup)))
    parts.reverse()                                  # backward order: last block first

    hp = B.hparams(**w.hparams, loss_scale=w.loss_scale)
    ws = [B.Workspace(n + 2), B.Workspace(n + 2)]
    for x in ws:
        x.tune(B.AH_TUNE_STEP_BLOCKS_PER_CU, args.blocks_per_cu)
        x.tune(B.AH_TUNE_CARRY_ELEMS, n * C)
    whole = md.chunk_array()
    a_mat = torch.randn(args.gemm, args.gemm, device="cuda:0", dtype=torch.bfloat16)
    b_mat = torch.randn(args.gemm, args.gemm, device="cuda:0", dtype=torch.bfloat16)
    c_mat = torch.empty_like(a_mat)
    step = [1]

    def one_shot():
        ws[0].autohete_grad_prep(whole, n, w.dtype, w.loss_scale, 0.0, st)
        ws[0].autohete_adamw_step(whole, n, w.dtype, step[0], hp, st)
        step[0] += 1

    def optimizer_block(i, cur, nxt, stream_handle):
        arr, k = parts[i]
        nxt.autohete_grad_prep_accumulate(arr, k, w.dtype, w.loss_scale, stream_handle)
        cur.autohete_adamw_step(arr, k, w.dtype, step[0], hp, stream_handle)

    def per_block(stream_handle=None, events=None, carry=False):
        s = st if stream_handle is None else stream_handle
        cur, nxt = ws[step[0] % 2], ws[(step[0] + 1) % 2]
        nxt.autohete_grad_result_set(0.0, 0, s)
        for i in range(len(parts)):
            if events is not None:
                side.wait_event(events[i])
            if carry:
                cur.autohete_adamw_step_carry(nxt, parts[i][0], parts[i][1], w.dtype, step[0], hp, s)
            else:
                optimizer_block(i, cur, nxt, s)
        step[0] += 1

    def per_block_carry():
        per_block(carry=True)

    def compute(events=None):
        for i in range(len(parts)):
            for _ in range(args.gemms_per_block):
                torch.matmul(a_mat, b_mat, out=c_mat)
            if events is not None:
                events[i].record(main_stream)

    def overlapped(carry=False):
        events = [torch.cuda.Event() for _ in parts]
        compute(events)
        with torch.cuda.stream(side):
            per_block(side.cuda_stream, events, carry)
        main_stream.wait_stream(side)

    def overlapped_carry():
        overlapped(True)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.iters):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.iters

    # seed both workspaces with a norm so that the first per-block iteration clips like the others
    ws[0].autohete_grad_prep(whole, n, w.dtype, w.loss_scale, 0.0, st)
    sumsq, _, _ = ws[0].autohete_grad_result_get(st)
    ws[1].autohete_grad_result_set(sumsq, 0, st)
    res = {"workload": w.name, "partitions": len(parts), "elements": n * C,
           "gemm": "%d x bf16 %d^3 per partition" % (args.gemms_per_block, args.gemm),
           "blocks_per_cu": args.blocks_per_cu or "default"}
    res["one_shot_ms"] = timed(one_shot)
    res["per_block_ms"] = timed(per_block)
    res["per_block_carry_ms"] = timed(per_block_carry)
    res["compute_ms"] = timed(compute)
    res["overlapped_ms"] = timed(overlapped)
    res["overlapped_carry_ms"] = timed(overlapped_carry)
    res["serial_sum_ms"] = res["per_block_ms"] + res["compute_ms"]
    res["ideal_overlap_ms"] = max(res["per_block_ms"], res["compute_ms"])
    res["per_block_GBps"] = 30 * n * C / res["per_block_ms"] / 1e6
    res["one_shot_GBps"] = 30 * n * C / res["one_shot_ms"] / 1e6
    res["per_block_carry_GBps"] = 28 * n * C / res["per_block_carry_ms"] / 1e6
    for x in ws:
        x.close()
    print(json.dumps(res))


if __name__ == "__main__":
    main()
