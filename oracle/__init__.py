"""ctypes access to the scalar CPU oracle (oracle/adamw_oracle.c).

TEST INFRASTRUCTURE.  Importable only from tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg.  Nothing here imports the GPU package, and the GPU
package never imports this.

The functions mirror the C ones one to one; arrays are numpy arrays that the C
code reads and writes in place (uint16 for the 16-bit streams, float32 for the
fp32 master copy and the two Adam moments).
"""
import ctypes
import os
import subprocess

import numpy as np

BF16, FP16 = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "adamw_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force=False):
    """Compile the oracle with gcc.  One IEEE operation per written operation:
    no contraction into fused multiply-adds, no fast-math."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


class HParams(ctypes.Structure):
    _fields_ = [(k, ctypes.c_float) for k in
                ("lr", "beta1", "beta2", "eps", "weight_decay", "max_grad_norm", "loss_scale")]


_lib = None


def bind(path):
    """Load an oracle shared library and declare its prototypes."""
    L = ctypes.CDLL(path)
    u16p = ctypes.POINTER(ctypes.c_uint16)
    f32p = ctypes.POINTER(ctypes.c_float)
    u64p = ctypes.POINTER(ctypes.c_uint64)
    L.oracle_lowp_decode.restype = ctypes.c_float
    L.oracle_lowp_decode.argtypes = [ctypes.c_uint16, ctypes.c_int]
    L.oracle_lowp_encode.restype = ctypes.c_uint16
    L.oracle_lowp_encode.argtypes = [ctypes.c_float, ctypes.c_int]
    L.oracle_lowp_decode_array.restype = None
    L.oracle_lowp_decode_array.argtypes = [u16p, f32p, ctypes.c_uint64, ctypes.c_int]
    L.oracle_lowp_encode_array.restype = None
    L.oracle_lowp_encode_array.argtypes = [f32p, u16p, ctypes.c_uint64, ctypes.c_int]
    L.oracle_chunk_layout.restype = ctypes.c_int
    L.oracle_chunk_layout.argtypes = [u64p, ctypes.c_uint64, ctypes.c_uint64, u64p, u64p, u64p, u64p]
    L.oracle_grad_accumulate.restype = None
    L.oracle_grad_accumulate.argtypes = [u16p, ctypes.c_uint64, ctypes.c_int, ctypes.c_float,
                                         ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_uint32)]
    L.oracle_grad_finish.restype = None
    L.oracle_grad_finish.argtypes = [ctypes.c_double, ctypes.c_uint32, ctypes.POINTER(ctypes.c_double),
                                     ctypes.POINTER(ctypes.c_uint32)]
    L.oracle_clip_coef.restype = ctypes.c_double
    L.oracle_clip_coef.argtypes = [ctypes.c_double, ctypes.c_float]
    L.oracle_adamw_chunk.restype = None
    L.oracle_adamw_chunk.argtypes = [u16p, u16p, f32p, f32p, f32p, ctypes.c_uint64, ctypes.c_int,
                                     ctypes.c_uint64, ctypes.POINTER(HParams), ctypes.c_double,
                                     ctypes.c_uint32]
    L.oracle_cast_chunk.restype = None
    L.oracle_cast_chunk.argtypes = [f32p, u16p, ctypes.c_uint64, ctypes.c_int]
    return L


def lib():
    global _lib
    if _lib is None:
        _lib = bind(build())
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _chk(a, dt):
    if not (isinstance(a, np.ndarray) and a.dtype == dt and a.flags.c_contiguous and a.ndim == 1):
        raise TypeError("oracle arrays must be 1-d C-contiguous %s" % np.dtype(dt).name)
    return a


def hparams(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, max_grad_norm=1.0,
            loss_scale=1.0):
    return HParams(lr, beta1, beta2, eps, weight_decay, max_grad_norm, loss_scale)


def decode(bits, dtype):
    bits = _chk(np.ascontiguousarray(bits, dtype=np.uint16).ravel(), np.uint16)
    out = np.empty(bits.size, np.float32)
    lib().oracle_lowp_decode_array(_p(bits, ctypes.c_uint16), _p(out, ctypes.c_float), bits.size, dtype)
    return out


def encode(x, dtype):
    x = _chk(np.ascontiguousarray(x, dtype=np.float32).ravel(), np.float32)
    out = np.empty(x.size, np.uint16)
    lib().oracle_lowp_encode_array(_p(x, ctypes.c_float), _p(out, ctypes.c_uint16), x.size, dtype)
    return out


def chunk_layout(tensor_numel, chunk_elems):
    """-> (offsets[np.uint64], n_chunks, total_elems, padded_elems)"""
    numel = np.ascontiguousarray(tensor_numel, dtype=np.uint64)
    off = np.empty(numel.size, np.uint64)
    nc, tot, pad = ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_uint64()
    rc = lib().oracle_chunk_layout(_p(numel, ctypes.c_uint64), numel.size, int(chunk_elems),
                                   _p(off, ctypes.c_uint64), ctypes.byref(nc), ctypes.byref(tot),
                                   ctypes.byref(pad))
    if rc != 0:
        raise ValueError("oracle_chunk_layout: bad chunk_elems")
    return off, nc.value, tot.value, pad.value


def grad_accumulate(grad, dtype, loss_scale, sumsq=0.0, found_inf=0):
    """Fold one chunk's gradients into (sumsq, found_inf); returns the new pair."""
    _chk(grad, np.uint16)
    s, f = ctypes.c_double(sumsq), ctypes.c_uint32(found_inf)
    lib().oracle_grad_accumulate(_p(grad, ctypes.c_uint16), grad.size, dtype, loss_scale,
                                 ctypes.byref(s), ctypes.byref(f))
    return s.value, f.value


def grad_finish(sumsq, found_inf):
    """-> (norm as double, found_inf)"""
    n, f = ctypes.c_double(), ctypes.c_uint32()
    lib().oracle_grad_finish(sumsq, found_inf, ctypes.byref(n), ctypes.byref(f))
    return n.value, f.value


def grad_prep(grads, dtype, loss_scale, extra_sumsq=0.0):
    """Whole gradient preparation over a list of chunks, in chunk order.
    -> (norm, found_inf)"""
    s, f = float(extra_sumsq), 0
    for g in grads:
        s, f = grad_accumulate(g, dtype, loss_scale, s, f)
    return grad_finish(s, f)


def clip_coef(norm, max_grad_norm):
    return lib().oracle_clip_coef(norm, max_grad_norm)


def adamw_chunk(grad, param_lp, master, exp_avg, exp_avg_sq, dtype, step, hp, norm, found_inf):
    """In-place AdamW step on one chunk's arrays.  param_lp=None: no 16-bit write-back."""
    n = _chk(grad, np.uint16).size
    _chk(master, np.float32), _chk(exp_avg, np.float32), _chk(exp_avg_sq, np.float32)
    if param_lp is not None:
        _chk(param_lp, np.uint16)
    if not ((param_lp is None or param_lp.size == n) and master.size == exp_avg.size == exp_avg_sq.size == n):
        raise ValueError("stream lengths differ")
    lib().oracle_adamw_chunk(_p(grad, ctypes.c_uint16), None if param_lp is None else _p(param_lp, ctypes.c_uint16),
                             _p(master, ctypes.c_float), _p(exp_avg, ctypes.c_float),
                             _p(exp_avg_sq, ctypes.c_float), n, dtype, int(step),
                             ctypes.byref(hp), float(norm), int(found_inf))


def cast_chunk(master, param_lp, dtype):
    """param_lp = round-to-nearest-even(master), in place."""
    _chk(master, np.float32), _chk(param_lp, np.uint16)
    if master.size != param_lp.size:
        raise ValueError("stream lengths differ")
    lib().oracle_cast_chunk(_p(master, ctypes.c_float), _p(param_lp, ctypes.c_uint16), master.size, dtype)


def full_step(chunks, dtype, step, hp, extra_sumsq=0.0):
    """grad_prep then adamw over a list of chunk dicts with keys
    grad, param_lp, master, exp_avg, exp_avg_sq.  -> (norm, found_inf)"""
    norm, flag = grad_prep([c["grad"] for c in chunks], dtype, hp.loss_scale, extra_sumsq)
    for c in chunks:
        adamw_chunk(c["grad"], c["param_lp"], c["master"], c["exp_avg"], c["exp_avg_sq"],
                    dtype, step, hp, norm, flag)
    return norm, flag
