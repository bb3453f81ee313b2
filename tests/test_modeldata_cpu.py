"""Layout arithmetic of the device-memory plumbing, checked on the CPU (no kernels involved)."""
import random

import pytest

from paper_2503_01890_amd.modeldata import ModelData, STREAMS


@pytest.mark.parametrize("layout", ["group", "slab"])
def test_spans_are_aligned_disjoint_and_inside_their_allocation(layout):
    rnd = random.Random(7)
    for _ in range(100):
        n, sets, group = rnd.randint(1, 23), rnd.randint(1, 3), rnd.randint(1, 9)
        numels = [rnd.choice([1, 7, 128, 129, 1000, 4096, 5000]) for _ in range(n)]
        md = ModelData(numels, device="cpu", n_grad_sets=sets, layout=layout, group_chunks=group)
        sizes = [t.numel() for t in md.storages()]
        spans = []
        for i in range(n):
            for s in STREAMS:
                for k in (range(sets) if s == "grad" else [0]):
                    which, a, b = md.byte_span(s, i, k)
                    width = 2 if s in ("grad", "param_lp") else 4
                    assert a % 256 == 0 and b <= sizes[which] and b - a == numels[i] * width
                    v = md.view(s, i, k)
                    assert v.numel() == numels[i] and v.data_ptr() == md.storages()[which].data_ptr() + a
                    spans.append((which, a, b))
        spans.sort()
        for (w0, _, b0), (w1, a1, _) in zip(spans, spans[1:]):
            assert w0 != w1 or b0 <= a1


def test_range_tuples_cover_a_flat_element_range():
    C = 1024
    md = ModelData([C] * 5, device="cpu", layout="group", group_chunks=2)
    tup = md.range_tuples(1000, 3080)
    assert [t[5] for t in tup] == [24, 1024, 1024, 8]
    assert tup[0][2] == md.view("master", 0).data_ptr() + 4 * 1000
    assert tup[3][0] == md.view("grad", 3).data_ptr()
