"""One optimizer step of a hybrid placement (plumbing only: PyTorch pinned buffers, HIP streams and
events; every arithmetic step runs in libautohete.so, on the GPU or on the host).

Placement (paper section 3.2.1): the first chunks keep their optimizer states in HBM and are
updated by the GPU kernels; the others keep fp32 master/m/v in host memory.  For those the GPU
only holds the 16-bit gradients (produced by backward) and the 16-bit parameters (needed by
forward); per chunk the step is: gradients D2H -> host AdamW -> 16-bit parameters H2D, pipelined
chunk by chunk over two copy streams, earlier chunks first (the paper's priority order: the next
forward pass needs block 1 first).  On the host the 16-bit gradients and parameters of a chunk
share ONE pinned buffer (they never coexist: 14 bytes per host parameter, Eq. 2).

The global gradient norm is taken on the GPU over ALL gradients -- they are all in HBM when
backward ends -- so the host needs only the resulting scalar.
"""
import ctypes
import time

import numpy as np
import torch

from . import binding as B


class HostChunks:
    """fp32 master / exp_avg / exp_avg_sq in ordinary host memory, one pinned 16-bit staging buffer per
    chunk (gradients in, parameters out), plus the device-side 16-bit gradient and parameter slabs."""

    def __init__(self, n_chunks, chunk_elems, device="cuda:0"):
        self.n, self.C = n_chunks, chunk_elems
        self.master = [np.empty(chunk_elems, np.float32) for _ in range(n_chunks)]
        self.exp_avg = [np.empty(chunk_elems, np.float32) for _ in range(n_chunks)]
        self.exp_avg_sq = [np.empty(chunk_elems, np.float32) for _ in range(n_chunks)]
        self.stage = [torch.empty(chunk_elems, dtype=torch.int16, pin_memory=True) for _ in range(n_chunks)]
        self.dev_grad = torch.empty(n_chunks * chunk_elems, dtype=torch.int16, device=device)
        self.dev_param_lp = torch.empty(n_chunks * chunk_elems, dtype=torch.int16, device=device)

    def dev_view(self, which, c):
        t = self.dev_grad if which == "grad" else self.dev_param_lp
        return t[c * self.C:(c + 1) * self.C]

    def host_chunk_array(self, c):
        p = self.stage[c].data_ptr()
        return B.chunk_array([(p, p, self.master[c].ctypes.data, self.exp_avg[c].ctypes.data,
                               self.exp_avg_sq[c].ctypes.data, self.C)])

    def grad_only_tuples(self):
        """Descriptors of the device-side gradients (for the global norm on the GPU)."""
        return [(self.dev_view("grad", c).data_ptr(), None, None, None, None, self.C) for c in range(self.n)]


class HybridStepper:
    def __init__(self, resident, host, lowp_dtype, n_threads):
        """resident: modeldata.ModelData of the GPU-resident chunks; host: HostChunks."""
        self.md, self.host, self.dtype, self.n_threads = resident, host, lowp_dtype, n_threads
        self.ws = B.Workspace(resident.n_chunks + host.n + 1)
        self.resident_arr = resident.chunk_array()
        self.all_grads = B.chunk_array([resident.chunk_tuple(i) for i in range(resident.n_chunks)] +
                                       host.grad_only_tuples())
        self.d2h, self.h2d = torch.cuda.Stream(), torch.cuda.Stream()      # default priority
        self.host_arr = [host.host_chunk_array(c) for c in range(host.n)]

    def step(self, t, hp):
        """Returns a dict of timings (seconds) and the norm / skip flag."""
        md, host, ws = self.md, self.host, self.ws
        main = torch.cuda.current_stream()
        s = main.cuda_stream
        t0 = time.perf_counter()
        # gradients of the host-owned chunks start crossing PCIe at once, earliest chunk first
        self.d2h.wait_stream(main)
        arrived = []
        with torch.cuda.stream(self.d2h):
            for c in range(host.n):
                host.stage[c].copy_(host.dev_view("grad", c), non_blocking=True)
                ev = torch.cuda.Event()
                ev.record(self.d2h)
                arrived.append(ev)
        # global norm over every gradient, then the GPU's share of the update
        ws.autohete_grad_prep(self.all_grads, md.n_chunks + host.n, self.dtype, hp.loss_scale, 0.0, s)
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record(main)
        ws.autohete_adamw_step(self.resident_arr, md.n_chunks, self.dtype, t, hp, s)
        g1.record(main)
        sumsq, norm, flag = ws.autohete_grad_result_get(s)                   # the host needs the scalar
        t_norm = time.perf_counter() - t0
        # host share: as each chunk's gradients arrive, update it and send its 16-bit parameters back
        t_wait = t_host = 0.0
        for c in range(host.n):
            a = time.perf_counter()
            arrived[c].synchronize()
            b = time.perf_counter()
            B.autohete_host_adamw_step(self.host_arr[c], 1, self.dtype, t, hp, sumsq, flag, self.n_threads)
            e = time.perf_counter()
            t_wait += b - a
            t_host += e - b
            if not flag:
                with torch.cuda.stream(self.h2d):
                    host.dev_view("param_lp", c).copy_(host.stage[c], non_blocking=True)
        main.wait_stream(self.h2d)
        torch.cuda.synchronize()
        total = time.perf_counter() - t0
        return dict(total_s=total, until_norm_s=t_norm, host_update_s=t_host, host_wait_for_grads_s=t_wait,
                    gpu_step_s=g0.elapsed_time(g1) * 1e-3, norm=norm, found_inf=flag, sumsq=sumsq)

    def close(self):
        self.ws.close()
