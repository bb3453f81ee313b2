"""Seeded synthetic model data: GPT-shaped tensor lists, the ragged mix, and a
counter-based generator with a CPU half and a GPU half that agree bit for bit.

A fixture shared by the tests and the benchmark.  It holds workload SHAPES and
input VALUES only -- none of the optimizer's arithmetic -- and imports neither
the GPU library nor the CPU oracle.

Streams (one id each): the 16-bit parameters (the fp32 master copy is their exact
upcast), the 16-bit gradients (a fresh draw per step), and the two fp32 Adam moments.
"""
import ctypes
import math
import os
import subprocess

import numpy as np

BF16, FP16 = 0, 1
OUT_F32, OUT_LOWP, OUT_F32_OF_LOWP = 0, 1, 2
STREAM_PARAM, STREAM_GRAD, STREAM_EXP_AVG, STREAM_EXP_AVG_SQ, STREAM_MISC = 1, 2, 3, 4, 5

# standard deviation of the sum of eight independent uniform 16-bit integers
IH8_SD = math.sqrt(8.0 * (65536.0 ** 2 - 1.0) / 12.0)

_HERE = os.path.dirname(os.path.abspath(__file__))
_CPU_LIB = os.path.join(_HERE, "libsynth_cpu.so")
_GPU_LIB = os.path.join(_HERE, "libsynth_gpu.so")

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(force=False, gpu=True):
    core = os.path.join(_HERE, "gen_core.h")
    newest = lambda *fs: max(os.path.getmtime(f) for f in fs)
    src = os.path.join(_HERE, "gen_cpu.c")
    if force or not os.path.exists(_CPU_LIB) or os.path.getmtime(_CPU_LIB) < newest(src, core):
        subprocess.check_call(["gcc", "-O3", "-ffp-contract=off", "-fPIC", "-shared", "-o", _CPU_LIB, src])
    src = os.path.join(_HERE, "gen_gpu.hip")
    if gpu and (force or not os.path.exists(_GPU_LIB) or os.path.getmtime(_GPU_LIB) < newest(src, core)):
        subprocess.check_call(["/opt/rocm/bin/hipcc"] + HIPCC_FLAGS + ["-ffp-contract=off", "-o", _GPU_LIB, src])


class Spec(ctypes.Structure):
    _fields_ = [("key", ctypes.c_uint64), ("first_index", ctypes.c_uint64), ("n_valid", ctypes.c_uint64),
                ("scale", ctypes.c_float), ("scale_outlier", ctypes.c_float),
                ("outlier_thresh", ctypes.c_uint32), ("take_abs", ctypes.c_int),
                ("out_kind", ctypes.c_int), ("dtype", ctypes.c_int)]


_cpu = _gpu = None


def _cpu_lib():
    global _cpu
    if _cpu is None:
        if not os.path.exists(_CPU_LIB):
            build(gpu=False)
        _cpu = ctypes.CDLL(_CPU_LIB)
        _cpu.synth_cpu_key.restype = ctypes.c_uint64
        _cpu.synth_cpu_key.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64]
        _cpu.synth_cpu_fill.restype = None
        _cpu.synth_cpu_fill.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.POINTER(Spec)]
    return _cpu


def _gpu_lib():
    global _gpu
    if _gpu is None:
        if not os.path.exists(_GPU_LIB):
            raise RuntimeError("libsynth_gpu.so is not built: run __graft_entry__.build() first")
        try:
            import torch  # noqa: F401  (its bundled HIP runtime must be the one this library binds to)
        except ImportError:
            pass
        _gpu = ctypes.CDLL(_GPU_LIB)
        _gpu.synth_gpu_fill.restype = ctypes.c_int
        _gpu.synth_gpu_fill.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.POINTER(Spec), ctypes.c_void_p]
    return _gpu


def make_spec(seed, stream, step, first_index, sigma, out_kind, dtype=BF16, take_abs=False,
              outlier_prob=0.0, sigma_outlier=0.0, n_valid=2 ** 63):
    key = _cpu_lib().synth_cpu_key(int(seed), int(stream), int(step))
    return Spec(key, int(first_index), int(n_valid), np.float32(sigma / IH8_SD), np.float32(sigma_outlier / IH8_SD),
                int(round(outlier_prob * 2 ** 32)), int(bool(take_abs)), int(out_kind), int(dtype))


def fill_cpu(out, spec):
    """Fill a 1-d numpy array (float32 or uint16, matching spec.out_kind) in place."""
    want = np.uint16 if spec.out_kind == OUT_LOWP else np.float32
    if out.dtype != want or not out.flags.c_contiguous:
        raise TypeError("output array must be contiguous %s" % np.dtype(want).name)
    _cpu_lib().synth_cpu_fill(out.ctypes.data, out.size, ctypes.byref(spec))
    return out


def fill_gpu(dev_ptr, count, spec, hip_stream=0):
    """Fill `count` elements at device address dev_ptr on the given HIP stream (async)."""
    rc = _gpu_lib().synth_gpu_fill(ctypes.c_void_p(dev_ptr), int(count), ctypes.byref(spec),
                                   ctypes.c_void_p(hip_stream))
    if rc != 0:
        raise RuntimeError("synth_gpu_fill: HIP error %d" % rc)


# ----------------------------------------------------------------------------- workloads

def gpt_tensor_numel(d, n_layer, vocab, n_pos):
    """Tied token embedding, position table, then per layer: LN1 (gamma, beta), QKV weight and
    bias, attention out-projection weight and bias, LN2 (gamma, beta), MLP up weight and bias,
    MLP down weight and bias."""
    per_layer = [d, d, 3 * d * d, 3 * d, d * d, d, d, d, 4 * d * d, 4 * d, d * 4 * d, d]
    return np.array([vocab * d, n_pos * d] + per_layer * n_layer, dtype=np.uint64)


def ragged_tensor_numel(seed, n_tensors=2000, lo=64, hi=2 ** 24):
    """Sizes log-uniform in [lo, hi]: many bias/LayerNorm-sized tensors plus large matrices."""
    u = np.random.default_rng(seed).uniform(math.log(lo), math.log(hi), n_tensors)
    return np.minimum(np.floor(np.exp(u)), hi).astype(np.uint64)


class Workload:
    """One of the five configurations: shapes, distributions, hyper-parameters, schedule."""

    def __init__(self, name, tensor_numel, chunk_elems, dtype=BF16, steps=1, loss_scale=1.0,
                 outlier_prob=0.0, resident_fraction=1.0, inject=None, seed=0):
        self.name, self.dtype, self.steps, self.seed = name, dtype, steps, seed
        self.tensor_numel = np.asarray(tensor_numel, np.uint64)
        self.chunk_elems = int(chunk_elems)
        self.n_valid = int(self.tensor_numel.sum())
        self.n_chunks = -(-self.n_valid // self.chunk_elems)
        self.n_resident = int(math.floor(self.n_chunks * resident_fraction + 1e-9))
        self.loss_scale = float(loss_scale)
        self.outlier_prob = outlier_prob
        self.inject = inject or {}          # iteration (1-based) -> "inf" | "nan"
        self.hparams = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, max_grad_norm=1.0)

    # Specs for one chunk (flat indices [c*C, (c+1)*C)).
    def _spec(self, stream, step, chunk, sigma, kind, **kw):
        return make_spec(self.seed, stream, step, chunk * self.chunk_elems, sigma, kind, self.dtype,
                         n_valid=self.n_valid, **kw)

    def spec_param_lp(self, chunk):
        return self._spec(STREAM_PARAM, 0, chunk, 0.02, OUT_LOWP)

    def spec_master(self, chunk):
        return self._spec(STREAM_PARAM, 0, chunk, 0.02, OUT_F32_OF_LOWP)

    def spec_exp_avg(self, chunk):
        return self._spec(STREAM_EXP_AVG, 0, chunk, 1e-4, OUT_F32)

    def spec_exp_avg_sq(self, chunk):
        return self._spec(STREAM_EXP_AVG_SQ, 0, chunk, 1e-6, OUT_F32, take_abs=True)

    def spec_grad(self, chunk, iteration, loss_scale=None):
        s = self.loss_scale if loss_scale is None else loss_scale
        return self._spec(STREAM_GRAD, iteration, chunk, 1e-3 * s, OUT_LOWP,
                          outlier_prob=self.outlier_prob, sigma_outlier=1.0 * s)

    def partition_bounds(self):
        """Flat element bounds of the optimizer partitions of a GPT-shaped workload: the embedding
        tables, then one partition per transformer block (12 tensors each); the last one also
        takes the padding of the last chunk.  -> [0, b1, ..., n_chunks * chunk_elems]"""
        off = np.concatenate([[0], np.cumsum(self.tensor_numel.astype(np.int64))])
        n_layers, rest = divmod(len(self.tensor_numel) - 2, 12)
        assert rest == 0 and n_layers > 0, "not a GPT-shaped tensor list"
        bounds = [0] + [int(off[2 + 12 * i]) for i in range(n_layers)] + [self.n_chunks * self.chunk_elems]
        return bounds

    def inject_index(self, iteration):
        """Flat element (within the resident chunks) that is overwritten at `iteration`."""
        k = _cpu_lib().synth_cpu_key(self.seed, STREAM_MISC, iteration)
        return int(k % min(self.n_valid, self.n_resident * self.chunk_elems))


def workload(name, seed=0):
    V = 50257
    if name == "gpt-124m":
        return Workload(name, gpt_tensor_numel(768, 12, V, 1024), 2 ** 22, steps=1, seed=seed)
    if name == "gpt-1.3b":
        return Workload(name, gpt_tensor_numel(2048, 24, V, 2048), 2 ** 24, steps=10, seed=seed)
    if name == "gpt-6.7b":
        return Workload(name, gpt_tensor_numel(4096, 32, V, 2048), 2 ** 25, steps=10, outlier_prob=1e-3, seed=seed)
    if name == "gpt-13b-half-resident":
        return Workload(name, gpt_tensor_numel(5120, 40, V, 2048), 2 ** 25, steps=5, resident_fraction=0.5, seed=seed)
    if name == "ragged-fp16":
        return Workload(name, ragged_tensor_numel(seed), 2 ** 23, dtype=FP16, steps=10, loss_scale=2.0 ** 16,
                        inject={3: "inf", 7: "nan"}, seed=seed)
    raise KeyError(name)


WORKLOADS = ("gpt-124m", "gpt-1.3b", "gpt-6.7b", "gpt-13b-half-resident", "ragged-fp16")
