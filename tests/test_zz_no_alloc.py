"""The allocation-free entry point autohete_grad_prep_static against autohete_grad_prep, through
the C ABI: same chunk list -> bit-identical S, norm and flag (same kernel body, grid and order),
and the parity bar against the oracle; two calls in a row on one GPU, the second on a smaller
input, so that whatever the first call left in the library's static scratch array is in the way;
then a non-finite gradient, an empty list, the size limit, and that no device memory is taken."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import synthdata
from paper_2503_01890_amd import binding as B

pytestmark = pytest.mark.gpu


def _result(buf):
    raw = buf.cpu().numpy().tobytes()
    r = B.autohete_grad_result.from_buffer_copy(raw)
    return r.sumsq, r.norm_d, r.norm, r.found_inf


def _grads(sizes, dtype, seed, scale):
    """One device allocation holding the given chunks back to back (256-byte aligned), and
    the same values on the host."""
    pad = [-(-n // 128) * 128 for n in sizes]
    dev = torch.zeros(sum(pad), dtype=torch.int16, device="cuda:0")
    host, tuples, at = [], [], 0
    s = torch.cuda.current_stream().cuda_stream
    for i, (n, p) in enumerate(zip(sizes, pad)):
        spec = synthdata.make_spec(seed, synthdata.STREAM_GRAD, 1, at, 1e-3 * scale, synthdata.OUT_LOWP, dtype)
        synthdata.fill_gpu(dev[at:at + n].data_ptr(), n, spec, s)
        host.append(synthdata.fill_cpu(np.empty(n, np.uint16), spec))
        tuples.append((dev[at:at + n].data_ptr(), None, None, None, None, n))
        at += p
    torch.cuda.synchronize()
    return dev, host, tuples


@pytest.mark.parametrize("dtype,scale", [(B.AH_BF16, 1.0), (B.AH_FP16, 1024.0)])
def test_static_norm_pass_equals_the_workspace_one_on_two_calls_in_a_row(dtype, scale):
    torch.cuda.set_device(0)
    s = torch.cuda.current_stream().cuda_stream
    # first call: many tiles per block and a ragged tail; second call: fewer chunks, fewer elements,
    # fewer blocks than the first (less than one tile per CU)
    big = [5 * 16384 * 40 + 777, 16384 * 300, 1, 16384 * 7 + 15]
    small = [16384 * 3 + 5, 4099]
    ws = B.Workspace(8)
    out = torch.zeros(32, dtype=torch.uint8, device="cuda:0")
    inputs = [_grads(sizes, dtype, seed=11 + k, scale=scale) for k, sizes in enumerate((big, small))]
    want = []
    for k, (dev, host, tuples) in enumerate(inputs):       # the existing entry point first
        arr = B.chunk_array(tuples)
        norm, flag = ws.autohete_grad_prep(arr, len(tuples), dtype, scale, 0.125 * k, s, want_result=True)
        want.append((ws.autohete_grad_result_get(s)[0], norm, flag))
    # a first call looks up the scratch array's address; from here on device memory must not move
    B.autohete_grad_prep_static(B.chunk_array(inputs[1][2]), len(small), dtype, scale, 0.0, s, out.data_ptr())
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    for k, (dev, host, tuples) in enumerate(inputs):       # two calls in a row, the second smaller
        arr = B.chunk_array(tuples)
        out.fill_(0xEE)
        B.autohete_grad_prep_static(arr, len(tuples), dtype, scale, 0.125 * k, s, out.data_ptr())
        torch.cuda.synchronize()
        sumsq, norm_d, norm, flag = _result(out)
        assert (sumsq, norm, flag) == want[k], (k, sumsq, want[k])
        assert norm_d == np.sqrt(sumsq)
        o_norm, o_flag = oracle.grad_prep(host, dtype, scale, 0.125 * k)
        assert flag == o_flag == 0 and abs(norm_d - o_norm) <= 1e-5 * o_norm, (norm_d, o_norm)
    assert torch.cuda.mem_get_info()[0] == free_before, "the static entry point must not take device memory"

    # a non-finite gradient in the last element of the small input: flag set, norm NaN, like the workspace path
    dev = inputs[1][0]
    dev[-(-small[0] // 128) * 128 + small[1] - 1] = int(np.array(0x7C00 if dtype == B.AH_FP16 else 0x7F80, np.uint16).view(np.int16))
    torch.cuda.synchronize()
    B.autohete_grad_prep_static(arr, len(small), dtype, scale, 0.0, s, out.data_ptr())
    torch.cuda.synchronize()
    sumsq, norm_d, norm, flag = _result(out)
    assert flag == 1 and np.isnan(norm_d) and np.isnan(norm)
    assert ws.autohete_grad_prep(arr, len(small), dtype, scale, 0.0, s, want_result=True)[1] == 1

    # and the call after a skipping one starts clean: no chunks, S = extra_sumsq
    B.autohete_grad_prep_static(arr, 0, dtype, scale, 2.25, s, out.data_ptr())
    torch.cuda.synchronize()
    assert _result(out) == (2.25, 1.5, 1.5, 0)
    ws.close()


def test_static_norm_pass_rejects_what_it_cannot_take():
    torch.cuda.set_device(0)
    s = torch.cuda.current_stream().cuda_stream
    out = torch.zeros(32, dtype=torch.uint8, device="cuda:0")
    g = torch.zeros(4096, dtype=torch.int16, device="cuda:0")
    n = B.AUTOHETE_STATIC_MAX_CHUNKS
    ok = B.chunk_array([(g.data_ptr(), None, None, None, None, 16)] * (n + 1))
    lib = B.raw()
    call = lambda arr, k, dt=B.AH_BF16, scale=1.0, res=out.data_ptr(): lib.autohete_grad_prep_static(
        arr, k, dt, scale, 0.0, ctypes.c_void_p(s), ctypes.c_void_p(res))
    assert call(ok, n + 1) == B.AH_ELIMIT
    assert call(ok, n) == B.AH_OK                      # exactly the maximum is accepted
    torch.cuda.synchronize()
    assert _result(out) == (0.0, 0.0, 0.0, 0)
    assert call(ok, 1, dt=7) == B.AH_EINVAL
    assert call(ok, 1, scale=0.0) == B.AH_EINVAL
    assert call(ok, 1, res=None) == B.AH_EINVAL
    assert call(None, 1) == B.AH_EINVAL
    assert call(ok, 1, res=out.data_ptr() + 4) == B.AH_EALIGN
    assert call(B.chunk_array([(g.data_ptr() + 2, None, None, None, None, 16)]), 1) == B.AH_EALIGN
    assert call(B.chunk_array([(g.data_ptr(), None, None, None, None, 0)]), 1) == B.AH_EINVAL
    assert B.raw().autohete_strerror(B.AH_ELIMIT).decode().startswith("more chunks")


def test_static_norm_pass_recorded_into_a_hip_graph():
    """The entry point makes no allocation and no memset node, so it can be recorded into a HIP
    graph; four replays with eager work and synchronisations between them, each against the
    workspace path on the same (changing) gradients."""
    torch.cuda.set_device(0)
    s = torch.cuda.current_stream().cuda_stream
    sizes = [16384 * 9 + 11, 70_000, 16384 * 300]
    dev, host, tuples = _grads(sizes, B.AH_BF16, seed=3, scale=1.0)
    arr = B.chunk_array(tuples)
    out = torch.zeros(32, dtype=torch.uint8, device="cuda:0")
    ws = B.Workspace(4)
    side = torch.cuda.Stream()                                     # default priority
    with torch.cuda.stream(side):                                  # first call on the capture stream: looks up the array
        B.autohete_grad_prep_static(arr, 3, B.AH_BF16, 1.0, 0.5, side.cuda_stream, out.data_ptr())
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        B.autohete_grad_prep_static(arr, 3, B.AH_BF16, 1.0, 0.5, side.cuda_stream, out.data_ptr())
    torch.cuda.synchronize()
    rng = np.random.default_rng(12)
    for rep in range(4):
        dev[:4096] = torch.from_numpy(rng.integers(0, 0x3F80, 4096).astype(np.int16)).to(dev.device)   # eager work
        out.fill_(0xEE)
        torch.cuda.synchronize()
        g.replay()
        norm, flag = ws.autohete_grad_prep(arr, 3, B.AH_BF16, 1.0, 0.5, s, want_result=True)
        torch.cuda.synchronize()
        sumsq, norm_d, norm_f, found = _result(out)
        assert (sumsq, norm_f, found) == (ws.autohete_grad_result_get(s)[0], norm, flag), rep
    ws.close()
