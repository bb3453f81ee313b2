"""Device memory for chunked model data (plumbing only: PyTorch-ROCm allocates HBM and hands
out raw addresses; no arithmetic happens here).

Model data = the five per-element streams of section 2.1 of the paper: 16-bit gradients and
parameters, fp32 master copy, fp32 first and second Adam moments (2+2+4+4+4 = 16 B/parameter).
Each stream is one contiguous HBM slab; chunk i occupies a 256-byte-aligned slice of it.
"""
import torch

from . import binding

STREAMS = ("grad", "param_lp", "master", "exp_avg", "exp_avg_sq")
_DTYPES = dict(grad=torch.int16, param_lp=torch.int16, master=torch.float32, exp_avg=torch.float32,
               exp_avg_sq=torch.float32)
_ALIGN_ELEMS = 128  # 256 B for the 16-bit streams, 512 B for fp32


class ModelData:
    def __init__(self, chunk_numels, device="cuda:0", n_grad_sets=1):
        """chunk_numels: elements per chunk (equal sizes or ragged).  n_grad_sets > 1 keeps
        several gradient slabs resident (fresh gradients per step without regenerating)."""
        self.device = torch.device(device)
        self.numel = [int(n) for n in chunk_numels]
        self.offset, run = [], 0
        for n in self.numel:
            self.offset.append(run)
            run += -(-n // _ALIGN_ELEMS) * _ALIGN_ELEMS
        self.slab_elems = max(run, _ALIGN_ELEMS)
        self.slab = {s: torch.empty(self.slab_elems, dtype=_DTYPES[s], device=self.device)
                     for s in STREAMS if s != "grad"}
        self.grad_sets = [torch.empty(self.slab_elems, dtype=torch.int16, device=self.device)
                          for _ in range(n_grad_sets)]
        self.slab["grad"] = self.grad_sets[0]

    @property
    def n_chunks(self):
        return len(self.numel)

    def view(self, stream, i, grad_set=0):
        t = self.grad_sets[grad_set] if stream == "grad" else self.slab[stream]
        return t[self.offset[i]:self.offset[i] + self.numel[i]]

    def ptr(self, stream, i, grad_set=0):
        return self.view(stream, i, grad_set).data_ptr()

    def chunk_tuple(self, i, grad_set=0):
        return (self.ptr("grad", i, grad_set), self.ptr("param_lp", i), self.ptr("master", i),
                self.ptr("exp_avg", i), self.ptr("exp_avg_sq", i), self.numel[i])

    def chunk_array(self, indices=None, grad_set=0):
        idx = range(self.n_chunks) if indices is None else indices
        return binding.chunk_array([self.chunk_tuple(i, grad_set) for i in idx])

    def range_tuples(self, start, end, grad_set=0):
        """Descriptors covering flat elements [start, end) of equally sized chunks (element e lives in
        chunk e // C at position e % C): one sub-chunk per chunk touched.  Used to address one
        transformer block's slice of the model data; start and end must be multiples of 8 elements
        so that every slice stays 16-byte aligned."""
        C = self.numel[0]
        assert all(n == C for n in self.numel) and start % 8 == 0 and end % 8 == 0 and start <= end
        out = []
        e = start
        while e < end:
            c, pos = divmod(e, C)
            n = min(C - pos, end - e)
            out.append(tuple(self.view(s, c, grad_set)[pos:pos + n].data_ptr() for s in STREAMS) + (n,))
            e += n
        return out

    def zero_(self):
        for t in list(self.slab.values()) + self.grad_sets:
            t.zero_()
