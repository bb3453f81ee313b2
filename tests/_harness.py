"""Glue for the GPU parity tests: numpy <-> device chunks, generator fills, comparisons."""
import concurrent.futures as cf

import numpy as np
import torch

import oracle
import synthdata
from paper_2503_01890_amd import binding as B
from paper_2503_01890_amd.modeldata import ModelData, STREAMS

N_THREADS = 16


def stream_handle():
    return torch.cuda.current_stream().cuda_stream


def upload(md, i, arrays, grad_set=0):
    for s in STREAMS:
        if s in arrays:
            a = arrays[s]
            t = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a)
            md.view(s, i, grad_set).copy_(t)


def download(md, i, streams=STREAMS, grad_set=0):
    out = {}
    for s in streams:
        a = md.view(s, i, grad_set).cpu().numpy()
        out[s] = a.view(np.uint16).copy() if a.dtype == np.int16 else a.copy()
    return out


def random_state(n, dtype, rng, grad_sigma=1e-3, scale=1.0):
    """Model-data-like values from numpy (small tests only)."""
    def lowp(x):
        if dtype == oracle.FP16:
            return np.asarray(x, np.float32).astype(np.float16).view(np.uint16).copy()
        return torch.tensor(np.asarray(x, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
    p16 = lowp(rng.normal(0, 0.02, n))
    return dict(grad=lowp(rng.normal(0, grad_sigma, n) * scale), param_lp=p16.copy(),
                master=oracle.decode(p16, dtype), exp_avg=rng.normal(0, 1e-4, n).astype(np.float32),
                exp_avg_sq=np.abs(rng.normal(0, 1e-6, n)).astype(np.float32))


def ordered16(bits):
    """16-bit sign-magnitude patterns -> integers ordered like the values (for ULP distance)."""
    b = bits.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)


def ulp32(x):
    x = np.abs(np.asarray(x, np.float32))
    return np.spacing(np.maximum(x, np.float32(1.1754944e-38))).astype(np.float64)


def compare_state(gpu, ora, where="", old=None, drift_steps=0):
    """The parity bar: fp32 master and moments within 2 ulp (relative 1e-6) of the oracle,
    16-bit parameters within 1 ulp of their format, when both sides start the step from
    identical inputs.

    Two effects make "ulps of the result" the wrong yardstick for a few elements, and both are
    handled explicitly and counted, never silently:
      * cancellation.  The two sides may differ in the last bits of the global gradient norm
        (the sum is taken in a different order).  Where beta1*m and (1-beta1)*g, or p and the
        update, cancel to a result orders of magnitude smaller than the operands, that shows up
        as many ulps of the tiny result.  If the caller passes the pre-step state `old`, such an
        element is judged against 2 ulp of the larger operand instead;
      * drift (drift_steps > 0: a chunk whose GPU state is never re-synchronised with the
        oracle's).  A last-bit difference after step k is an input difference at step k+1 and
        is carried on with weight beta1 / beta2 / 1; if the element then cancels, ulps of the
        result say nothing.  Such elements are only required to agree to 1e-6 of the stream's
        r.m.s. value (they are tiny in absolute terms).
    Elements that needed either allowance are counted and must stay a vanishing fraction."""
    stats = {}
    for k in ("master", "exp_avg", "exp_avg_sq"):
        g, o = gpu[k].astype(np.float64), ora[k].astype(np.float64)
        assert np.all(np.isfinite(g)), (where, k, "non-finite")
        err = np.abs(g - o)
        tol = np.maximum(2.0 * ulp32(ora[k]), 1e-6 * np.abs(o))
        strict_bad = err > tol
        stats[k + "_relaxed"] = int(strict_bad.sum())
        if strict_bad.any() and old is not None:
            big = np.maximum(np.abs(o), np.abs(old[k].astype(np.float64))) if k in old else np.abs(o)
            tol = np.maximum(tol, 2.0 * ulp32(big))
            if drift_steps:
                tol = np.maximum(tol, 1e-6 * np.sqrt(np.mean(o * o)))
            assert strict_bad.sum() <= max(2, (1e-5 if drift_steps else 1e-6) * err.size), \
                (where, k, "too many relaxed elements", int(strict_bad.sum()))
        bad = err > tol
        assert not bad.any(), (where, k, int(bad.sum()), float((err / ulp32(ora[k])).max()))
        ok = ~strict_bad
        stats[k + "_max_ulp"] = float((err[ok] / ulp32(ora[k])[ok]).max()) if ok.any() else 0.0
        stats[k + "_mismatch"] = int((gpu[k].view(np.uint32) != ora[k].view(np.uint32)).sum())
    d = np.abs(ordered16(gpu["param_lp"]) - ordered16(ora["param_lp"]))
    assert d.max(initial=0) <= 1, (where, "param_lp", int(d.max()))
    stats["param_lp_max_ulp"] = int(d.max(initial=0))
    stats["param_lp_mismatch"] = int((d != 0).sum())
    stats["n"] = int(d.size)
    return stats


def oracle_hp(hp):
    return oracle.hparams(hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, hp.max_grad_norm, hp.loss_scale)


def fill_device_chunk(md, w, c, iteration=None, grad_set=0, loss_scale=None, state=True):
    """Fill chunk c of workload w on the device with the GPU half of the generator."""
    st = stream_handle()
    n = md.numel[c]
    if state:
        synthdata.fill_gpu(md.ptr("param_lp", c), n, w.spec_param_lp(c), st)
        synthdata.fill_gpu(md.ptr("master", c), n, w.spec_master(c), st)
        synthdata.fill_gpu(md.ptr("exp_avg", c), n, w.spec_exp_avg(c), st)
        synthdata.fill_gpu(md.ptr("exp_avg_sq", c), n, w.spec_exp_avg_sq(c), st)
    if iteration is not None:
        synthdata.fill_gpu(md.ptr("grad", c, grad_set), n, w.spec_grad(c, iteration, loss_scale), st)


def cpu_chunk_state(w, c):
    """Initial state of chunk c from the CPU half of the generator."""
    n = w.chunk_elems
    return dict(param_lp=synthdata.fill_cpu(np.empty(n, np.uint16), w.spec_param_lp(c)),
                master=synthdata.fill_cpu(np.empty(n, np.float32), w.spec_master(c)),
                exp_avg=synthdata.fill_cpu(np.empty(n, np.float32), w.spec_exp_avg(c)),
                exp_avg_sq=synthdata.fill_cpu(np.empty(n, np.float32), w.spec_exp_avg_sq(c)))


def cpu_chunk_grad(w, c, iteration, loss_scale=None):
    return synthdata.fill_cpu(np.empty(w.chunk_elems, np.uint16), w.spec_grad(c, iteration, loss_scale))


def oracle_sumsq_over_chunks(w, chunks, iteration, loss_scale, patch=None):
    """Oracle sum of squares / flag over the given chunk indices, regenerating each chunk's
    gradients on the CPU (threads; the C calls release the GIL).  Per-chunk sums are added in
    chunk order.  patch: {(chunk, index): 16-bit pattern} overwrites applied before summing."""
    def one(c):
        g = cpu_chunk_grad(w, c, iteration, loss_scale)
        for (pc, pi), bits in (patch or {}).items():
            if pc == c:
                g[pi] = bits
        return oracle.grad_accumulate(g, w.dtype, loss_scale if loss_scale else w.loss_scale)
    with cf.ThreadPoolExecutor(N_THREADS) as ex:
        parts = list(ex.map(one, chunks))
    s, f = 0.0, 0
    for ps, pf in parts:
        s += ps
        f |= pf
    return s, f
