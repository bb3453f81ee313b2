"""The seeded input generator: shapes of the five workloads, distribution sanity (CPU),
and bit-identity of its CPU and GPU halves (GPU)."""
import numpy as np
import pytest
import torch

import synthdata


def test_workload_shapes():
    expect = {"gpt-124m": (146, 124_438_272, 30, 1_390_848), "gpt-1.3b": (290, 1_315_719_168, 79, 9_680_896),
              "gpt-6.7b": (386, 6_658_396_160, 199, 18_935_808),
              "gpt-13b-half-resident": (482, 12_853_376_000, 384, 31_525_888)}
    for name, (nt, n, nc, pad) in expect.items():
        w = synthdata.workload(name)
        assert (len(w.tensor_numel), w.n_valid, w.n_chunks, w.n_chunks * w.chunk_elems - w.n_valid) == (nt, n, nc, pad)
    assert synthdata.workload("gpt-13b-half-resident").n_resident == 192
    r = synthdata.workload("ragged-fp16")
    assert len(r.tensor_numel) == 2000 and r.tensor_numel.min() >= 64 and r.tensor_numel.max() <= 2 ** 24
    assert r.dtype == synthdata.FP16 and r.loss_scale == 65536.0 and r.inject == {3: "inf", 7: "nan"}
    assert np.array_equal(r.tensor_numel, synthdata.workload("ragged-fp16").tensor_numel)   # seeded


def test_distributions_and_determinism():
    w = synthdata.workload("gpt-6.7b")
    n = 1 << 21
    m = synthdata.fill_cpu(np.empty(n, np.float32), w.spec_exp_avg(3))
    assert abs(m.mean()) < 3e-7 and abs(m.std() / 1e-4 - 1) < 5e-3
    v = synthdata.fill_cpu(np.empty(n, np.float32), w.spec_exp_avg_sq(3))
    assert v.min() >= 0 and abs(np.sqrt((v.astype(np.float64) ** 2).mean()) / 1e-6 - 1) < 5e-3
    p16 = synthdata.fill_cpu(np.empty(n, np.uint16), w.spec_param_lp(3))
    master = synthdata.fill_cpu(np.empty(n, np.float32), w.spec_master(3))
    up = torch.tensor(p16.view(np.int16)).view(torch.bfloat16).float().numpy()
    assert np.array_equal(up, master) and abs(master.std() / 0.02 - 1) < 5e-3     # master = exact upcast
    g1 = synthdata.fill_cpu(np.empty(n, np.uint16), w.spec_grad(3, 1))
    g2 = synthdata.fill_cpu(np.empty(n, np.uint16), w.spec_grad(3, 2))
    assert not np.array_equal(g1, g2)                                             # fresh per step
    assert np.array_equal(g1, synthdata.fill_cpu(np.empty(n, np.uint16), w.spec_grad(3, 1)))
    gf = torch.tensor(g1.view(np.int16)).view(torch.bfloat16).float().numpy()
    out = np.abs(gf) > 0.02                                                        # 20 sigma of the bulk
    assert 0.0005 < out.mean() < 0.0015 and abs(gf[~out].std() / 1e-3 - 1) < 2e-2  # 0.1 % outliers ~N(0,1)
    # windows of one stream agree with the whole (counter-based addressing)
    a = synthdata.fill_cpu(np.empty(1000, np.float32), synthdata.make_spec(0, 3, 0, 5000, 1.0, synthdata.OUT_F32))
    b = synthdata.fill_cpu(np.empty(6000, np.float32), synthdata.make_spec(0, 3, 0, 0, 1.0, synthdata.OUT_F32))
    assert np.array_equal(a, b[5000:])
    # padding: flat indices past n_valid are +0 in every stream
    last = w.n_chunks - 1
    tail = synthdata.fill_cpu(np.empty(w.chunk_elems, np.uint16), w.spec_grad(last, 1))
    n_pad = w.n_chunks * w.chunk_elems - w.n_valid
    assert not tail[-n_pad:].any() and tail[:-n_pad].any()


def test_generator_fp16_rounding_is_rne():
    # the generator's own fp16 rounding agrees with numpy's (only matters for describing inputs)
    r = synthdata.workload("ragged-fp16")
    x = synthdata.fill_cpu(np.empty(1 << 18, np.float32), synthdata.make_spec(0, 1, 0, 0, 0.02, synthdata.OUT_F32))
    h = synthdata.fill_cpu(np.empty(1 << 18, np.uint16),
                           synthdata.make_spec(0, 1, 0, 0, 0.02, synthdata.OUT_LOWP, synthdata.FP16))
    assert np.array_equal(h, x.astype(np.float16).view(np.uint16))
    assert r.spec_grad(0, 1).dtype == synthdata.FP16


@pytest.mark.gpu
def test_cpu_and_gpu_halves_agree_bit_for_bit():
    st = torch.cuda.current_stream().cuda_stream
    n = (1 << 20) + 77
    for name in ("gpt-6.7b", "ragged-fp16"):
        w = synthdata.workload(name)
        c = w.n_chunks - 1
        for spec, dt in ((w.spec_param_lp(c), np.uint16), (w.spec_master(c), np.float32),
                         (w.spec_exp_avg(c), np.float32), (w.spec_exp_avg_sq(c), np.float32),
                         (w.spec_grad(c, 4), np.uint16), (w.spec_grad(0, 9), np.uint16)):
            cpu = synthdata.fill_cpu(np.empty(n, dt), spec)
            dev = torch.empty(n, dtype=torch.int16 if dt == np.uint16 else torch.float32, device="cuda:0")
            synthdata.fill_gpu(dev.data_ptr(), n, spec, st)
            torch.cuda.synchronize()
            got = dev.cpu().numpy()
            assert got.view(dt).tobytes() == cpu.tobytes(), (name, spec.out_kind)
