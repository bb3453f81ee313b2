"""Glue for the GPU parity tests: numpy <-> device chunks, generator fills, comparisons."""
import concurrent.futures as cf
import ctypes
import os
import subprocess
import threading

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


_tls = threading.local()


def download_pinned(md, i, streams=STREAMS, grad_set=0):
    """download() through this thread's pinned staging buffers (several times the bandwidth of a
    copy into pageable memory).  The arrays returned alias the staging buffers: they are valid
    until this thread's next call."""
    bufs = getattr(_tls, "bufs", None)
    if bufs is None:
        bufs = _tls.bufs = {}
    out = {}
    for s in streams:
        v = md.view(s, i, grad_set)
        b = bufs.get(s)
        if b is None or b.numel() < v.numel():
            b = bufs[s] = torch.empty(v.numel(), dtype=v.dtype, pin_memory=True)
        b[:v.numel()].copy_(v)
        a = b[:v.numel()].numpy()
        out[s] = a.view(np.uint16) if a.dtype == np.int16 else a
    return out


def bit_view(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a.view(np.uint16)


def resync(md, i, got, ora, streams):
    """Oracle -> device: overwrite, on the device, the elements of chunk i in which the downloaded
    device state `got` differs from the oracle's `ora` (a handful per million), so that the next
    step starts from identical inputs.  Returns the number of elements written."""
    n = 0
    for s in streams:
        idx = np.flatnonzero(bit_view(got[s]) != bit_view(ora[s]))
        if idx.size == 0:
            continue
        n += idx.size
        if idx.size > ora[s].size // 64:
            upload(md, i, {s: ora[s]})
            continue
        vals = ora[s][idx]
        vals = torch.from_numpy(vals.view(np.int16) if vals.dtype == np.uint16 else vals)
        md.view(s, i)[torch.from_numpy(idx).to(md.device)] = vals.to(md.device)
    return n


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


_HERE = os.path.dirname(os.path.abspath(__file__))
_PC_SRC, _PC_LIB = os.path.join(_HERE, "parity_check.c"), os.path.join(_HERE, "libparity_check.so")
PS_FIELDS = ("mismatch", "beyond", "fail", "first_fail", "max_ulp", "max_ulp_T", "max_E_frac", "max_E_ulp_T",
             "max_abs", "sumsq_ora")
_F32_STREAMS = ("exp_avg", "exp_avg_sq", "master")          # the order parity_check.c reports in: m, v, p


class ParityConsts(ctypes.Structure):
    _fields_ = [(k, ctypes.c_double) for k in ("grad_scale", "beta1", "beta2", "lr", "eps", "wd", "bc1", "bc2", "rho")]


def build_parity_check(force=False):
    if force or not os.path.exists(_PC_LIB) or os.path.getmtime(_PC_LIB) < os.path.getmtime(_PC_SRC):
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-o", _PC_LIB,
                               _PC_SRC, "-lm"])
    return _PC_LIB


_pc = None


def _parity_lib():
    global _pc
    if _pc is None:
        L = ctypes.CDLL(build_parity_check())
        f32p, u16p, dp = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_uint16), ctypes.POINTER(ctypes.c_double)
        L.parity_strict.restype = None
        L.parity_strict.argtypes = [ctypes.c_uint64, u16p, ctypes.c_int] + [f32p] * 8 + [ctypes.POINTER(ParityConsts), dp]
        L.parity_free.restype = None
        L.parity_free.argtypes = [ctypes.c_uint64, u16p, ctypes.c_int] + [f32p] * 11 + [ctypes.POINTER(ParityConsts), dp]
        L.parity_lowp.restype = ctypes.c_uint32
        L.parity_lowp.argtypes = [ctypes.c_uint64, u16p, u16p, ctypes.POINTER(ctypes.c_uint64)]
        _pc = L
    return _pc


def _fp(a):
    if a is None:
        return None
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


class StepCtx:
    """What the comparison rules need to know about the step that was just taken: the format, the
    hyper-parameters, the step number and the ORACLE's gradient norm (fp64)."""

    def __init__(self, dtype, hp, step, norm, sumsq_gpu=None):
        self.dtype, self.hp, self.step, self.norm = dtype, hp, int(step), float(norm)
        # rho: relative difference of the two sides' clip factors, known when the caller read the
        # GPU's sum of squares (the oracle's is norm^2).  The factor is max_norm / (sqrt(S) + 1e-6), so
        # it differs by at most half the relative difference of the sums; the full difference is taken,
        # plus 2^-50 for the few fp64 roundings (square root, sum, quotient) each side makes on the way.
        self.rho = None
        if sumsq_gpu is not None:
            s_o = self.norm * self.norm
            self.rho = (abs(sumsq_gpu - s_o) / min(sumsq_gpu, s_o) + 2.0 ** -50) if (
                hp.max_grad_norm > 0 and min(sumsq_gpu, s_o) > 0) else 0.0

    def consts(self, rho=0.0):
        hp = self.hp
        b1, b2 = float(np.float32(hp.beta1)), float(np.float32(hp.beta2))
        coef = oracle.clip_coef(self.norm, hp.max_grad_norm)
        return ParityConsts(coef / float(np.float32(hp.loss_scale)), b1, b2, float(np.float32(hp.lr)),
                            float(np.float32(hp.eps)), float(np.float32(hp.weight_decay)), 1.0 - b1 ** self.step,
                            1.0 - b2 ** self.step, rho)


def _collect(raw, where, what):
    stats = {}
    for j, s in enumerate(_F32_STREAMS):
        for f, name in enumerate(PS_FIELDS):
            stats["%s_%s" % (s, name)] = raw[j * len(PS_FIELDS) + f]
    for s in _F32_STREAMS:
        assert stats[s + "_fail"] == 0, (where, what, s, "elements outside the rule: %d, first at %d" %
                                         (stats[s + "_fail"], stats[s + "_first_fail"]), stats)
    return stats


def _lowp(gpu, ora, where, stats):
    nd = ctypes.c_uint64()
    g, o = np.ascontiguousarray(gpu["param_lp"]), np.ascontiguousarray(ora["param_lp"])
    u16p = ctypes.POINTER(ctypes.c_uint16)
    d = _parity_lib().parity_lowp(g.size, g.ctypes.data_as(u16p), o.ctypes.data_as(u16p), ctypes.byref(nd))
    assert d <= 1, (where, "param_lp", d)
    stats["param_lp_max_ulp"], stats["param_lp_mismatch"], stats["n"] = int(d), int(nd.value), int(g.size)
    return stats


def _u16p(a):
    if a is None:
        return None
    assert a.dtype == np.uint16 and a.flags.c_contiguous
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


_scratch = threading.local()


def keep_old(state):
    """Copies of the three fp32 streams of `state` in this thread's reusable buffers (valid until
    the thread's next call): the pre-step state the comparison rules need."""
    bufs = getattr(_scratch, "old", None)
    n = state["master"].size
    if bufs is None or bufs["master"].size < n:
        bufs = _scratch.old = {k: np.empty(n, np.float32) for k in _F32_STREAMS}
    out = {}
    for k in _F32_STREAMS:
        out[k] = bufs[k][:n]
        np.copyto(out[k], state[k])
    return out


def compare_state(gpu, ora, where="", old=None, ctx=None):
    """The parity bar for a step that both sides took from IDENTICAL inputs (tests/parity_check.c,
    parity_strict): fp32 master and moments within max(2 ulp32, relative 1e-6) of the oracle, or
    within 2 ulp32 of the largest term that feeds the value where the terms cancel (counted);
    16-bit parameters within 1 ulp of their format.  `old`: the state before the step, `ctx`: a
    StepCtx (default: ora["ctx"]); without them only the first two arms apply."""
    ctx = ctx or ora.get("ctx")
    third = old is not None and ctx is not None and "grad" in ora
    raw = (ctypes.c_double * (3 * len(PS_FIELDS)))()
    k = ctx.consts() if third else ParityConsts()
    _parity_lib().parity_strict(ora["master"].size, _u16p(ora["grad"]) if third else None, ctx.dtype if third else 0,
                                _fp(old["exp_avg"]) if third else None,
                                _fp(old["master"]) if third else None, _fp(ora["exp_avg"]), _fp(ora["exp_avg_sq"]),
                                _fp(ora["master"]), _fp(gpu["exp_avg"]), _fp(gpu["exp_avg_sq"]), _fp(gpu["master"]),
                                ctypes.byref(k), raw)
    stats = _collect(raw, where, "identical inputs")
    if third and ctx.rho is not None:
        # The third arm is for the rare cancelled element, not a second tolerance.  From identical
        # inputs the unrounded results differ by at most rho * T, so the rounded ones are equal or
        # adjacent (<= 1 ulp32 < 1e-6 relative) unless |result| < 1e6 * rho * T; result / T is spread
        # over [-2, 2] with a density below 1 at zero, so at most 2e6 * rho of the elements qualify.
        # Twice that plus a floor for the fluctuation of a small count is allowed.
        for s in ("exp_avg", "master"):
            assert stats[s + "_beyond"] <= 10 + 4e6 * ctx.rho * ora["master"].size, \
                (where, s, "third arm used too often", stats[s + "_beyond"], ctx.rho)
    return _lowp(gpu, ora, where, stats)


class FreeRun:
    """Parity of a chunk whose GPU state is never re-synchronised with the oracle's: keeps the
    difference |gpu - ora| observed after each step and holds every element of the next step to
    what the update rule makes of that known input difference plus one rounding on each side
    (tests/parity_check.c, parity_free)."""

    def __init__(self, n):
        self.D = {s: np.zeros(n, np.float32) for s in _F32_STREAMS}

    def step(self, gpu, ora, old, ctx, where=""):
        """After a (non-skipped) step: ora / old = the oracle's state after / before it, gpu = the
        free-running device state, ctx = a StepCtx that knows both sides' sums of squares."""
        assert ctx.rho is not None, "the bound needs the GPU's sum of squares"
        k = ctx.consts(ctx.rho)
        raw = (ctypes.c_double * (3 * len(PS_FIELDS)))()
        _parity_lib().parity_free(ora["master"].size, _u16p(ora["grad"]), ctx.dtype, _fp(old["exp_avg"]), _fp(old["master"]),
                                  _fp(ora["exp_avg"]), _fp(ora["exp_avg_sq"]), _fp(ora["master"]),
                                  _fp(gpu["exp_avg"]), _fp(gpu["exp_avg_sq"]), _fp(gpu["master"]),
                                  _fp(self.D["exp_avg"]), _fp(self.D["exp_avg_sq"]), _fp(self.D["master"]),
                                  ctypes.byref(k), raw)
        return _lowp(gpu, ora, where, _collect(raw, where, "free-running"))


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


def oracle_sumsq_over_chunks(w, chunks, iteration, loss_scale, patch=None, keep=None):
    """Oracle sum of squares / flag over the given chunk indices, regenerating each chunk's
    gradients on the CPU (threads; the C calls release the GIL).  Per-chunk sums are added in
    chunk order.  patch: {(chunk, index): 16-bit pattern} overwrites applied before summing.
    keep: a dict; the (patched) gradients of the chunks that are already keys of it are stored there
    instead of being thrown away, for the caller's element-by-element replay."""
    def one(c):
        g = cpu_chunk_grad(w, c, iteration, loss_scale)
        for (pc, pi), bits in (patch or {}).items():
            if pc == c:
                g[pi] = bits
        if keep is not None and c in keep:
            keep[c] = g
        return oracle.grad_accumulate(g, w.dtype, loss_scale if loss_scale else w.loss_scale)
    with cf.ThreadPoolExecutor(N_THREADS) as ex:
        parts = list(ex.map(one, chunks))
    s, f = 0.0, 0
    for ps, pf in parts:
        s += ps
        f |= pf
    return s, f
