"""Device memory for chunked model data (plumbing only: PyTorch-ROCm allocates HBM and hands
out raw addresses; no arithmetic happens here).

Model data = the five per-element streams of section 2.1 of the paper: 16-bit gradients and
parameters, fp32 master copy, fp32 first and second Adam moments (2+2+4+4+4 = 16 B/parameter).

Two layouts:
  "group" (default)  one allocation; every `group_chunks` consecutive chunks form a group laid out as
                     [master of the group | exp_avg | exp_avg_sq | param_lp | grad set 0 | grad set 1 | ...],
                     every chunk of every stream 256-byte aligned.  The update kernel touches all
                     five streams at the same element offset, so with groups its accesses in flight
                     stay within a few GB of address space: measured 1.5-3 % faster on MI355X than
                     five slabs tens of GB apart.  Runs that are too short lose it again (streams
                     16 MB apart measured 12 % slower), hence the default of 512 MB runs.
  "slab"             each stream is one contiguous slab; chunk i is a slice of each slab.
The library itself only sees pointers: either layout, or any other, is valid input.
"""
import torch

from . import binding

STREAMS = ("grad", "param_lp", "master", "exp_avg", "exp_avg_sq")
_DTYPES = dict(grad=torch.int16, param_lp=torch.int16, master=torch.float32, exp_avg=torch.float32,
               exp_avg_sq=torch.float32)
_ALIGN_ELEMS = 128  # 256 B for the 16-bit streams, 512 B for fp32
_BLOCK_ORDER = ("master", "exp_avg", "exp_avg_sq", "param_lp")   # then the gradient sets
_GROUP_RUN_ELEMS = 1 << 27


class ModelData:
    def __init__(self, chunk_numels, device="cuda:0", n_grad_sets=1, layout="group", group_chunks=None):
        """chunk_numels: elements per chunk (equal sizes or ragged).  n_grad_sets > 1 keeps
        several sets of gradients resident (fresh gradients per step without regenerating).
        group_chunks: chunks per group; None picks the smallest count that makes each stream's
        run inside a group at least 2^27 elements (512 MB of fp32)."""
        assert layout in ("group", "slab")
        self.device = torch.device(device)
        self.numel = [int(n) for n in chunk_numels]
        self.n_grad_sets = n_grad_sets
        self.layout = layout
        padded = [-(-n // _ALIGN_ELEMS) * _ALIGN_ELEMS for n in self.numel]
        if group_chunks is None:
            mean = max(1, sum(padded) // max(1, len(padded)))
            group_chunks = max(1, -(-_GROUP_RUN_ELEMS // mean))
        assert group_chunks >= 1
        self.group_chunks = group_chunks
        if layout == "group":
            # per chunk: byte offset of its group, elements in its group, elements of the group before it
            self._where, run = [], 0
            for g0 in range(0, len(padded), group_chunks):
                members = padded[g0:g0 + group_chunks]
                total, before = sum(members), 0
                for p in members:
                    self._where.append((run, total, before))
                    before += p
                run += total * (14 + 2 * n_grad_sets)
            self.block = torch.empty(max(run, 256), dtype=torch.uint8, device=self.device)
        else:
            self.offset, run = [], 0
            for p in padded:
                self.offset.append(run)
                run += p
            self.slab_elems = max(run, _ALIGN_ELEMS)
            self.slab = {s: torch.empty(self.slab_elems, dtype=_DTYPES[s], device=self.device)
                         for s in STREAMS if s != "grad"}
            self.grad_sets = [torch.empty(self.slab_elems, dtype=torch.int16, device=self.device)
                              for _ in range(n_grad_sets)]
            self.slab["grad"] = self.grad_sets[0]

    @property
    def n_chunks(self):
        return len(self.numel)

    def storages(self):
        """The underlying allocations as flat byte tensors."""
        if self.layout == "group":
            return [self.block]
        return [t.view(torch.uint8) for t in list(self.slab[s] for s in STREAMS if s != "grad") + self.grad_sets]

    def byte_span(self, stream, i, grad_set=0):
        """(index into storages(), first byte, end byte) of one stream of chunk i."""
        size = 2 if stream in ("grad", "param_lp") else 4
        if self.layout == "group":
            base, total, before = self._where[i]
            run = 14 * total + 2 * total * grad_set if stream == "grad" else 4 * total * _BLOCK_ORDER.index(stream)
            start = base + run + size * before
            return 0, start, start + size * self.numel[i]
        which = 4 + grad_set if stream == "grad" else [s for s in STREAMS if s != "grad"].index(stream)
        return which, size * self.offset[i], size * (self.offset[i] + self.numel[i])

    def view(self, stream, i, grad_set=0):
        if self.layout == "group":
            _, a, b = self.byte_span(stream, i, grad_set)
            return self.block[a:b].view(_DTYPES[stream])
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
        for t in self.storages():
            t.zero_()

    def checksums(self):
        """One integer per allocation: the wrapping sum of its 32-bit words (bit-exactness checks)."""
        return [int(t.view(torch.int32).sum(dtype=torch.int64).item()) for t in self.storages()]
