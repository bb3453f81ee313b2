"""GPU parity, unit scale: the HIP path through the C ABI against the CPU oracle, element by
element, on sizes that span several tiles and ragged tails; error paths; determinism."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from _golden import load_hand_worked
from _harness import (FreeRun, StepCtx, compare_state, download, oracle_hp, random_state, stream_handle, upload)
from paper_2503_01890_amd import binding as B
from paper_2503_01890_amd.modeldata import ModelData, STREAMS

pytestmark = pytest.mark.gpu

VARIANTS = [B.step_variant(v, b, m) for v, b in ((4, 64), (4, 128), (4, 256), (2, 64), (2, 128), (2, 256), (1, 128), (1, 256), (1, 512))
            for m in (0, 1)]


def run_gpu(md, ws, dtype, step, hp, extra=0.0, indices=None):
    arr = md.chunk_array(indices)
    n = md.n_chunks if indices is None else len(indices)
    norm, flag = ws.autohete_grad_prep(arr, n, dtype, hp.loss_scale, extra, stream_handle(), want_result=True)
    ws.autohete_adamw_step(arr, n, dtype, step, hp, stream_handle())
    torch.cuda.synchronize()
    return norm, flag


def run_oracle(states, dtype, step, hp, extra=0.0, ws=None):
    """Steps the oracle in place; the pre-step state is kept under "old" and what the comparison
    rules need to know about the step under "ctx" (with the GPU's sum of squares when the
    workspace that holds it is given)."""
    for st in states:
        st["old"] = dict(master=st["master"].copy(), exp_avg=st["exp_avg"].copy(),
                         exp_avg_sq=st["exp_avg_sq"].copy())
    norm, flag = oracle.full_step(states, dtype, step, oracle_hp(hp), extra)
    sumsq_gpu = ws.autohete_grad_result_get(stream_handle())[0] if (ws is not None and not flag) else None
    for st in states:
        st["ctx"] = StepCtx(dtype, hp, step, norm, sumsq_gpu)
    return norm, flag


F32_AND_LP = ("param_lp", "master", "exp_avg", "exp_avg_sq")


def resync(md, states, indices=None):
    """Oracle -> device: the next step starts from identical inputs on both sides."""
    for i, st in enumerate(states):
        upload(md, i if indices is None else indices[i], {k: st[k] for k in F32_AND_LP})


def check_norm(gn, gf, on, of):
    assert gf == of
    if not of:
        assert abs(gn - on) <= 1e-5 * on + 1e-30


@pytest.mark.parametrize("dtype", [B.AH_BF16, B.AH_FP16])
@pytest.mark.parametrize("n", [1, 3, 4, 7, 8, 9, 1023, 1024, 1025, 2047, 2048, 2049, 4101, 3 * 8192 + 17])
def test_single_chunk_odd_sizes(dtype, n):
    rng = np.random.default_rng(n * 2 + dtype)
    scale = 1.0 if dtype == B.AH_BF16 else 256.0
    st = random_state(n, dtype, rng, scale=scale)
    md = ModelData([n])
    upload(md, 0, st)
    ws = B.Workspace(4)
    hp = B.hparams(loss_scale=scale)
    for step in (1, 2, 3):
        gn, gf = run_gpu(md, ws, dtype, step, hp)
        on, of = run_oracle([st], dtype, step, hp, ws=ws)
        check_norm(gn, gf, on, of)
        compare_state(download(md, 0), st, "n=%d step=%d" % (n, step), st["old"])
        resync(md, [st])
    assert np.array_equal(download(md, 0)["grad"], st["grad"])          # gradients are read only
    ws.close()


@pytest.mark.parametrize("dtype", [B.AH_BF16, B.AH_FP16])
def test_forty_free_running_steps_stay_inside_the_carried_bound(dtype):
    """The device state is never re-synchronised with the oracle's: forty consecutive steps with
    fresh gradients and active clipping, every element held to the bound that is carried along
    with the oracle's state (tests/parity_check.c, parity_free)."""
    rng = np.random.default_rng(321 + dtype)
    n = 3 * 65536 + 77
    scale = 1.0 if dtype == B.AH_BF16 else 512.0
    st = random_state(n, dtype, rng, scale=scale)
    md = ModelData([n])
    upload(md, 0, st)
    ws = B.Workspace(1)
    hp = B.hparams(loss_scale=scale, max_grad_norm=0.3)
    bound = FreeRun(n)
    worst = {}
    for step in range(1, 41):
        st["grad"] = random_state(n, dtype, rng, scale=scale)["grad"]
        upload(md, 0, dict(grad=st["grad"]))
        gn, gf = run_gpu(md, ws, dtype, step, hp)
        on, of = run_oracle([st], dtype, step, hp, ws=ws)
        check_norm(gn, gf, on, of)
        stats = bound.step(download(md, 0), st, st["old"], st["ctx"], "free-running step %d" % step)
        for k, v in stats.items():
            worst[k] = max(worst.get(k, 0), v)
    for s in ("master", "exp_avg", "exp_avg_sq"):
        assert worst[s + "_fail"] == 0 and worst[s + "_max_E_frac"] <= 1.0
    print("free-running, 40 steps: worst error / bound E: m %.3f v %.3f p %.3f; worst error in ulp32(T): m %.2f v %.2f p %.2f"
          % tuple(worst[s + f] for f in ("_max_E_frac", "_max_ulp_T") for s in ("exp_avg", "exp_avg_sq", "master")))
    ws.close()


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("dtype", [B.AH_BF16, B.AH_FP16])
def test_every_kernel_variant_ragged_multichunk(variant, dtype):
    rng = np.random.default_rng(variant)
    numels = [int(x) for x in rng.integers(1, 40_000, 23)] + [8192, 4096, 1, 65536 + 3]
    states = [random_state(n, dtype, rng) for n in numels]
    md = ModelData(numels)
    for i, st in enumerate(states):
        upload(md, i, st)
    ws = B.Workspace(len(numels))
    ws.tune(B.AH_TUNE_STEP_VARIANT, variant)
    ws.tune(B.AH_TUNE_STEP_BLOCKS_PER_CU, [0, 3, 64][variant % 3])
    hp = B.hparams(max_grad_norm=0.05)
    for step in (1, 2):
        gn, gf = run_gpu(md, ws, dtype, step, hp, extra=1e-4)
        on, of = run_oracle(states, dtype, step, hp, extra=1e-4, ws=ws)
        check_norm(gn, gf, on, of)
        for i, st in enumerate(states):
            compare_state(download(md, i), st, "variant=%x chunk=%d" % (variant, i), st["old"])
        resync(md, states)
    ws.close()


def test_hand_worked_examples_through_hip():
    for name, c in load_hand_worked().items():
        dtype = B.AH_BF16 if c["dtype"] == "bf16" else B.AH_FP16
        hp = B.hparams(c["lr"], c["beta1"], c["beta2"], c["eps"], c["weight_decay"], c["max_grad_norm"],
                       c["loss_scale"])
        g = torch.tensor(c["grad"], dtype=torch.float32).to(torch.bfloat16 if dtype == B.AH_BF16 else torch.float16)
        g = g.view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(oracle.decode(g, dtype).astype(np.float64), c["grad"]), "fixture gradients must be exact in 16 bits"
        st = dict(grad=g.copy(), param_lp=np.zeros(16, np.uint16), master=c["master"].astype(np.float32),
                  exp_avg=c["exp_avg"].astype(np.float32), exp_avg_sq=c["exp_avg_sq"].astype(np.float32))
        md = ModelData([16])
        upload(md, 0, st)
        ws = B.Workspace(1)
        for k in range(1, int(c["steps"]) + 1):
            run_gpu(md, ws, dtype, int(c["first_step"]) + k - 1, hp)
            sumsq, norm, flag = ws.autohete_grad_result_get(stream_handle())
            assert flag == 0 and sumsq == pytest.approx(c["expect_sumsq"], rel=1e-15)
            got = download(md, 0)
            for key in ("master", "exp_avg", "exp_avg_sq"):
                assert np.array_equal(got[key], c["expect_%s_t%d" % (key, k)].astype(np.float32)), (name, key, k)
            assert np.array_equal(oracle.decode(got["param_lp"], dtype).astype(np.float64),
                                  c["expect_param_lp_t%d" % k]), (name, k)
        ws.close()


@pytest.mark.parametrize("dtype", [B.AH_BF16, B.AH_FP16])
@pytest.mark.parametrize("bad", ["inf", "-inf", "nan"])
def test_nonfinite_gradient_skips_bit_exactly(dtype, bad):
    rng = np.random.default_rng(11)
    numels = [5000, 4096, 777]
    pat = {B.AH_BF16: {"inf": 0x7F80, "-inf": 0xFF80, "nan": 0x7FC1},
           B.AH_FP16: {"inf": 0x7C00, "-inf": 0xFC00, "nan": 0x7E01}}[dtype][bad]
    for chunk, pos in ((0, 0), (0, 4999), (1, 2048), (2, 776)):
        states = [random_state(n, dtype, rng) for n in numels]
        states[chunk]["grad"][pos] = pat
        md = ModelData(numels)
        for i, st in enumerate(states):
            upload(md, i, st)
        ws = B.Workspace(8)
        gn, gf = run_gpu(md, ws, dtype, 1, B.hparams())
        on, of = run_oracle(states, dtype, 1, B.hparams())
        assert gf == 1 and of == 1 and np.isnan(gn)
        for i, st in enumerate(states):
            got = download(md, i)
            for s in STREAMS:
                assert got[s].tobytes() == st[s].tobytes(), (chunk, pos, i, s)
        # the next, clean iteration proceeds normally with the same workspace
        states[chunk]["grad"][pos] = 0
        upload(md, chunk, dict(grad=states[chunk]["grad"]))
        gn, gf = run_gpu(md, ws, dtype, 1, B.hparams())
        on, of = run_oracle(states, dtype, 1, B.hparams())
        check_norm(gn, gf, on, of)
        assert gf == 0
        for i, st in enumerate(states):
            compare_state(download(md, i), st, "after skip", st["old"])
        ws.close()


def test_nonfinite_extra_sumsq_skips():
    rng = np.random.default_rng(3)
    st = random_state(3000, B.AH_BF16, rng)
    md = ModelData([3000])
    upload(md, 0, st)
    ws = B.Workspace(1)
    for extra in (float("inf"), float("nan")):
        gn, gf = run_gpu(md, ws, B.AH_BF16, 1, B.hparams(), extra=extra)
        assert gf == 1
        got = download(md, 0)
        assert all(got[s].tobytes() == st[s].tobytes() for s in STREAMS)
    ws.close()


def test_partition_invariance_and_subsets():
    """One optimizer per block: stepping all chunks at once, one by one, or in halves gives
    bit-identical state; the norm always comes from one prep over all chunks."""
    rng = np.random.default_rng(21)
    numels = [9000, 4096, 123, 30000, 8192, 2048]
    states = [random_state(n, B.AH_BF16, rng) for n in numels]
    hp = B.hparams(max_grad_norm=0.01)
    results = []
    for groups in ([list(range(6))], [[i] for i in range(6)], [[3, 4, 5], [0, 1, 2]], [[5, 0], [2], [4, 1, 3]]):
        md = ModelData(numels)
        for i, st in enumerate(states):
            upload(md, i, st)
        ws = B.Workspace(6)
        ws.autohete_grad_prep(md.chunk_array(), 6, B.AH_BF16, 1.0, 0.0, stream_handle())
        for grp in groups:
            ws.autohete_adamw_step(md.chunk_array(grp), len(grp), B.AH_BF16, 5, hp, stream_handle())
        torch.cuda.synchronize()
        results.append([download(md, i) for i in range(6)])
        ws.close()
    for other in results[1:]:
        for a, b in zip(results[0], other):
            assert all(a[s].tobytes() == b[s].tobytes() for s in STREAMS)
    ora = [{k: v.copy() for k, v in st.items()} for st in states]
    oracle.full_step(ora, oracle.BF16, 5, oracle_hp(hp))
    for a, o in zip(results[0], ora):
        compare_state(a, o, "partition")


def test_result_set_steps_with_host_supplied_norm():
    rng = np.random.default_rng(22)
    st = random_state(10_000, B.AH_BF16, rng)
    md = ModelData([10_000])
    upload(md, 0, st)
    ws = B.Workspace(1)
    hp = B.hparams(max_grad_norm=0.5)
    ws.autohete_grad_result_set(4.0, 0, stream_handle())            # norm 2 -> coef 0.25 (minus guard)
    ws.autohete_adamw_step(md.chunk_array(), 1, B.AH_BF16, 2, hp, stream_handle())
    torch.cuda.synchronize()
    assert ws.autohete_grad_result_get(stream_handle()) == (4.0, 2.0, 0)
    oracle.adamw_chunk(st["grad"], st["param_lp"], st["master"], st["exp_avg"], st["exp_avg_sq"], oracle.BF16, 2,
                       oracle_hp(hp), 2.0, 0)
    compare_state(download(md, 0), st, "set")
    ws.autohete_grad_result_set(1.0, 1, stream_handle())            # flagged: step must not touch anything
    ws.autohete_adamw_step(md.chunk_array(), 1, B.AH_BF16, 3, hp, stream_handle())
    torch.cuda.synchronize()
    compare_state(download(md, 0), st, "flagged")
    ws.close()


def test_run_to_run_determinism_and_grid_independence():
    rng = np.random.default_rng(23)
    numels = [1 << 20, 333_333, 1 << 18]
    states = [random_state(n, B.AH_FP16, rng, scale=1024.0) for n in numels]
    hp = B.hparams(loss_scale=1024.0)
    outs, sums = [], []
    for prep_blocks in (0, 0, 1, 7, 1000):
        md = ModelData(numels)
        for i, st in enumerate(states):
            upload(md, i, st)
        ws = B.Workspace(3)
        ws.tune(B.AH_TUNE_PREP_BLOCKS, prep_blocks)
        run_gpu(md, ws, B.AH_FP16, 1, hp)
        sums.append(ws.autohete_grad_result_get(stream_handle())[0])
        outs.append([download(md, i) for i in range(3)])
        ws.close()
    assert sums[0] == sums[1]                                           # same launch: bit-identical
    for a, b in zip(outs[0], outs[1]):
        assert all(a[s].tobytes() == b[s].tobytes() for s in STREAMS)
    for s in sums[2:]:
        assert abs(s - sums[0]) <= 1e-12 * sums[0]                      # any grid: same sum to fp64 rounding
    ref = sum(float(np.sum((oracle.decode(st["grad"], oracle.FP16).astype(np.float64) / 1024.0) ** 2)) for st in states)
    assert abs(sums[0] - ref) <= 1e-12 * ref


def test_empty_chunk_list_and_extra_only():
    ws = B.Workspace(2)
    arr = B.chunk_array([])
    assert ws.autohete_grad_prep(arr, 0, B.AH_BF16, 1.0, 9.0, stream_handle(), want_result=True) == (3.0, 0)
    ws.autohete_adamw_step(arr, 0, B.AH_BF16, 1, B.hparams(), stream_handle())
    torch.cuda.synchronize()
    ws.close()


def test_error_codes():
    md = ModelData([4096, 4096])
    md.zero_()
    ws = B.Workspace(2)
    lib, h = B.raw(), ws._h
    hp = B.hparams()
    good = md.chunk_array()
    s = ctypes.c_void_p(stream_handle())

    def step(arr, n, dtype=B.AH_BF16, t=1, hp_=hp):
        return lib.autohete_adamw_step(h, arr, n, dtype, t, ctypes.byref(hp_), s)

    assert step(good, 2) == B.AH_OK
    assert step(good, 2, t=0) == B.AH_EINVAL
    assert step(good, 2, dtype=7) == B.AH_EINVAL
    assert step(good, 3) == B.AH_ENOMEM
    assert step(None, 2) == B.AH_EINVAL
    for bad in (B.hparams(beta1=1.0), B.hparams(beta2=-0.1), B.hparams(lr=float("nan")), B.hparams(loss_scale=0.0),
                B.hparams(eps=-1.0), B.hparams(weight_decay=float("inf"))):
        assert step(good, 2, hp_=bad) == B.AH_EINVAL
    t = list(md.chunk_tuple(0))
    for field in range(5):
        mis = list(t)
        mis[field] += 2
        assert step(B.chunk_array([mis]), 1) == B.AH_EALIGN, field
        nul = list(t)
        nul[field] = None
        assert step(B.chunk_array([nul]), 1) == B.AH_EINVAL, field
    zero = list(t)
    zero[5] = 0
    assert step(B.chunk_array([zero]), 1) == B.AH_EINVAL
    assert lib.autohete_grad_prep(h, good, 2, B.AH_BF16, ctypes.c_float(0.0), 0.0, s, None, None) == B.AH_EINVAL
    assert lib.autohete_grad_prep(h, good, 2, 9, ctypes.c_float(1.0), 0.0, s, None, None) == B.AH_EINVAL
    mis = list(t)
    mis[0] += 2
    assert lib.autohete_grad_prep(h, B.chunk_array([mis]), 1, B.AH_BF16, ctypes.c_float(1.0), 0.0, s, None,
                                  None) == B.AH_EALIGN
    assert lib.autohete_ws_tune(h, 99, 1) == B.AH_EINVAL
    assert lib.autohete_ws_tune(h, B.AH_TUNE_STEP_VARIANT, 3) == B.AH_EINVAL
    assert lib.autohete_ws_tune(h, B.AH_TUNE_STEP_BLOCKS_PER_CU, 65) == B.AH_EINVAL
    for knob in (B.AH_TUNE_STEP_BLOCKS_PER_CU, B.AH_TUNE_CAST_BLOCKS_PER_CU):
        for cap in (1, 2):            # the residency cap works through the LDS request: 1 and 2 cannot be enforced
            assert lib.autohete_ws_tune(h, knob, cap) == B.AH_EINVAL
        for cap in (3, 64, 0):
            assert lib.autohete_ws_tune(h, knob, cap) == B.AH_OK
    # A chunk with more tiles than one launch of the selected kernel shape can have is refused before
    # anything is launched (the pointers are never touched: no kernel runs for the call).
    huge = list(t)
    huge[5] = (1 << 33) + 16
    assert lib.autohete_ws_tune(h, B.AH_TUNE_STEP_VARIANT, B.step_variant(1, 128, 0)) == B.AH_OK
    assert step(B.chunk_array([huge]), 1) == B.AH_EINVAL              # 2^26 blocks of 128 threads: 2^33 threads along x
    assert step(B.chunk_array([t, huge]), 2) == B.AH_EINVAL           # ... also behind a chunk that would be fine
    assert lib.autohete_ws_tune(h, B.AH_TUNE_STEP_VARIANT, 0) == B.AH_OK
    huge[5] = 1 << 40
    assert step(B.chunk_array([huge]), 1) == B.AH_EINVAL              # 2^32 tiles of the default shape
    assert lib.autohete_cast_params(h, B.chunk_array([huge]), 1, B.AH_BF16, s) == B.AH_EINVAL
    torch.cuda.synchronize()
    got = download(md, 0)
    assert not got["exp_avg"].any()                                   # rejected calls launched nothing harmful
    ws.close()


def test_presized_carry_buffer_means_no_allocation_in_any_iteration():
    """autohete_adamw_step_carry appends one fp64 slot per wavefront to a buffer of the receiving
    workspace.  Sized beforehand (AH_TUNE_CARRY_ELEMS), no call allocates or frees: the device's
    free memory is the same after every iteration, the first included, and the results are those
    of a workspace that grew its buffer on demand."""
    rng = np.random.default_rng(4242)
    C, n_chunks = 1 << 20, 6
    states = [random_state(C, B.AH_BF16, rng) for _ in range(n_chunks)]
    a, b = ModelData([C] * n_chunks), ModelData([C] * n_chunks)
    for i, st in enumerate(states):
        upload(a, i, st)
        upload(b, i, st)
    hp = B.hparams(max_grad_norm=0.0)        # no clipping: the streams do not depend on the last bits of the sums
    s = stream_handle()
    pre = [B.Workspace(n_chunks + 2), B.Workspace(n_chunks + 2)]
    grow = [B.Workspace(n_chunks + 2), B.Workspace(n_chunks + 2)]
    for w in pre:
        w.tune(B.AH_TUNE_CARRY_ELEMS, C * n_chunks)
    parts = [(i * C // 2, (i + 1) * C // 2) for i in range(2 * n_chunks)]        # "blocks" of half a chunk
    sums, free = {}, []
    # the growing pair goes first: whatever the runtime itself sets up on the first launch of a
    # kernel (code objects, signal pools) has happened before the pre-sized pair is watched
    for name, md, wss in (("grow", b, grow), ("pre", a, pre)):
        if name == "pre":
            torch.cuda.synchronize()
            free.append(torch.cuda.mem_get_info()[0])
        wss[1].autohete_grad_result_set(0.0, 0, s)
        for it in (1, 2, 3):
            cur, nxt = wss[it % 2], wss[(it + 1) % 2]
            nxt.autohete_grad_result_set(0.0, 0, s)
            for lo, hi in reversed(parts):
                tup = md.range_tuples(lo, hi)
                cur.autohete_adamw_step_carry(nxt, B.chunk_array(tup), len(tup), B.AH_BF16, it, hp, s)
            sums[name, it] = nxt.autohete_grad_result_get(s)[0]
            if name == "pre":
                free.append(torch.cuda.mem_get_info()[0])
    assert len(set(free)) == 1, free
    # a buffer that fills up is folded early: the same sum in another order of fp64 additions
    assert all(abs(sums["pre", it] - sums["grow", it]) <= 1e-13 * sums["grow", it] for it in (1, 2, 3))
    for i in range(n_chunks):
        x, y = download(a, i), download(b, i)
        assert all(x[k].tobytes() == y[k].tobytes() for k in STREAMS)
    with pytest.raises(B.AutoheteError):                 # not while a carried sum is pending
        pre[0].autohete_adamw_step_carry(pre[1], a.chunk_array(), n_chunks, B.AH_BF16, 4, hp, s)
        pre[1].tune(B.AH_TUNE_CARRY_ELEMS, 64 * C * n_chunks)
    for w in pre + grow:
        w.close()


def test_padding_stays_zero_and_checkpoint_resume():
    """Zero padding stays +0 in every stream; 6 steps == 3 steps, state round-trip via host, 3 steps."""
    rng = np.random.default_rng(31)
    n, pad = 50_000, 1234
    st = random_state(n, B.AH_BF16, rng)
    for k in st:
        st[k][-pad:] = 0
    grads = [random_state(n, B.AH_BF16, rng)["grad"] for _ in range(6)]
    for g in grads:
        g[-pad:] = 0
    hp = B.hparams()

    def run(md, ws, lo, hi):
        for t in range(lo, hi):
            upload(md, 0, dict(grad=grads[t - 1]))
            run_gpu(md, ws, B.AH_BF16, t, hp)

    md = ModelData([n])
    upload(md, 0, st)
    ws = B.Workspace(1)
    run(md, ws, 1, 7)
    straight = download(md, 0)
    for s in STREAMS:
        assert not straight[s][-pad:].view(np.uint8).any(), s
    md2 = ModelData([n])
    upload(md2, 0, st)
    ws2 = B.Workspace(1)
    run(md2, ws2, 1, 4)
    saved = download(md2, 0)
    ws2.close()
    md3 = ModelData([n])
    upload(md3, 0, saved)
    ws3 = B.Workspace(1)
    run(md3, ws3, 4, 7)
    resumed = download(md3, 0)
    assert all(straight[s].tobytes() == resumed[s].tobytes() for s in STREAMS)
    ws.close(), ws3.close()


@pytest.mark.parametrize("dtype", [B.AH_BF16, B.AH_FP16])
def test_split_path_master_only_step_then_cast(dtype):
    """autohete_adamw_step_master leaves the 16-bit parameters alone (and accepts NULL for them);
    followed by autohete_cast_params it is bit-identical to the fused step; both match the oracle."""
    rng = np.random.default_rng(77 + dtype)
    numels = [1, 3, 255, 256, 257, 511, 512, 513, 4099, 20_000, 65536 + 5]
    states = [random_state(n, dtype, rng) for n in numels]
    hp = B.hparams(max_grad_norm=0.02)
    fused, split = ModelData(numels), ModelData(numels)
    for i, st in enumerate(states):
        upload(fused, i, st)
        upload(split, i, st)
    ws = B.Workspace(len(numels))
    n = len(numels)
    for step in (1, 2):
        run_gpu(fused, ws, dtype, step, hp)
        arr = split.chunk_array()
        ws.autohete_grad_prep(arr, n, dtype, 1.0, 0.0, stream_handle())
        no_lp = B.chunk_array([(t[0], None) + t[2:] for t in (split.chunk_tuple(i) for i in range(n))])
        before = [download(split, i, ("param_lp",))["param_lp"] for i in range(n)]
        ws.autohete_adamw_step_master(no_lp, n, dtype, step, hp, stream_handle())
        torch.cuda.synchronize()
        for i in range(n):
            assert np.array_equal(download(split, i, ("param_lp",))["param_lp"], before[i])
        ws.autohete_cast_params(arr, n, dtype, stream_handle())
        torch.cuda.synchronize()
        run_oracle(states, dtype, step, hp, ws=ws)
        for i, st in enumerate(states):
            a, b = download(fused, i), download(split, i)
            assert all(a[s].tobytes() == b[s].tobytes() for s in STREAMS), (step, i)
            compare_state(b, st, "split step=%d chunk=%d" % (step, i), st["old"])
        resync(fused, states)
        resync(split, states)
    # cast alone: any fp32 values, incl. ties, overflow to inf (fp16), subnormals, zeros, +-inf; NaN stays NaN
    vals = np.concatenate([rng.normal(0, 1, 5000), [0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e-8, 6e-8, -3e-8, 3.4e38,
                                                    np.inf, -np.inf, np.nan, -np.nan, -65520.0, -3.4e38, 1e-45],
                           np.float32(1.0) + np.arange(0, 64) * np.float32(2.0 ** -12)]).astype(np.float32)
    md = ModelData([vals.size])
    md.view("master", 0).copy_(torch.from_numpy(vals))
    ws.autohete_cast_params(md.chunk_array(), 1, dtype, stream_handle())
    torch.cuda.synchronize()
    got = download(md, 0, ("param_lp",))["param_lp"]
    want = oracle.encode(vals, dtype)
    is_nan = np.isnan(vals)
    assert is_nan.sum() == 2 and np.array_equal(got[~is_nan], want[~is_nan])
    # a NaN stays a NaN (its sign and payload bits are not part of the rule)
    assert np.all(np.isnan(oracle.decode(got[is_nan], dtype))) and np.all(np.isnan(oracle.decode(want[is_nan], dtype)))
    assert np.array_equal(oracle.decode(got[np.isinf(vals)], dtype), vals[np.isinf(vals)])
    lib, s = B.raw(), ctypes.c_void_p(stream_handle())
    t = list(md.chunk_tuple(0))
    t[2] = None
    assert lib.autohete_cast_params(ws._h, B.chunk_array([t]), 1, dtype, s) == B.AH_EINVAL
    t = list(md.chunk_tuple(0))
    t[1] += 2
    assert lib.autohete_cast_params(ws._h, B.chunk_array([t]), 1, dtype, s) == B.AH_EALIGN
    ws.close()


def test_per_block_prep_accumulate_and_backward_order_stepping():
    """One optimizer per transformer block (footnote to Eq. 5): the norm is gathered block by block
    with autohete_grad_prep_accumulate, and each block's slice of the flat model data -- sub-ranges
    of chunks, tensors straddle chunk boundaries -- is stepped on its own, last block first, on a
    second stream.  Must equal the one-shot path bit for bit given the same norm, and the oracle."""
    import synthdata
    d, L, C = 256, 3, 1 << 16
    sizes = [int(x) for x in synthdata.gpt_tensor_numel(d, L, 1000, 64)]
    off, n_chunks, total, pad = B.autohete_chunk_layout(sizes, C)
    # partitions: embedding + positions, then 12 tensors per layer (flat element ranges)
    bounds = [0, off[2]] + [off[2 + 12 * (i + 1)] if 2 + 12 * (i + 1) < len(off) else total for i in range(L)]
    blocks = list(zip(bounds[:-1], bounds[1:]))
    assert blocks[-1][1] == total and all(a % 8 == 0 and b % 8 == 0 for a, b in blocks)
    rng = np.random.default_rng(5)
    states = [random_state(C, B.AH_BF16, rng) for _ in range(n_chunks)]
    for k in states[-1]:
        states[-1][k][C - pad:] = 0
    hp = B.hparams(max_grad_norm=0.05)
    per_block, one_shot = ModelData([C] * n_chunks), ModelData([C] * n_chunks)
    for i, st in enumerate(states):
        upload(per_block, i, st)
        upload(one_shot, i, st)
    ws = B.Workspace(n_chunks + 2)
    side = torch.cuda.Stream()                      # default priority
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        s = side.cuda_stream
        ws.autohete_grad_result_set(0.0, 0, s)
        for a, b in reversed(blocks):               # gradients "land" last block first
            tup = per_block.range_tuples(a, b)
            ws.autohete_grad_prep_accumulate(B.chunk_array(tup), len(tup), B.AH_BF16, 1.0, s)
        sumsq, norm, flag = ws.autohete_grad_result_get(s)
        for a, b in reversed(blocks):
            tup = per_block.range_tuples(a, b)
            ws.autohete_adamw_step(B.chunk_array(tup), len(tup), B.AH_BF16, 2, hp, s)
    side.synchronize()
    assert flag == 0
    ref = sum(float(np.sum(oracle.decode(st["grad"], oracle.BF16).astype(np.float64) ** 2)) for st in states)
    assert abs(sumsq - ref) <= 1e-12 * ref
    ws.autohete_grad_result_set(sumsq, 0, stream_handle())          # same norm -> must be bit-identical
    ws.autohete_adamw_step(one_shot.chunk_array(), n_chunks, B.AH_BF16, 2, hp, stream_handle())
    torch.cuda.synchronize()
    for i in range(n_chunks):
        a, b = download(per_block, i), download(one_shot, i)
        assert all(a[k].tobytes() == b[k].tobytes() for k in STREAMS), i
    run_oracle(states, oracle.BF16, 2, hp)
    for i, st in enumerate(states):
        compare_state(download(per_block, i), st, "per-block chunk=%d" % i, st["old"])
    # a non-finite gradient in ANY block keeps the flag through later accumulations
    bad = states[1]["grad"].copy()
    bad[17] = 0x7F80
    upload(per_block, 1, dict(grad=bad))
    ws.autohete_grad_result_set(0.0, 0, stream_handle())
    for a, b in blocks:
        tup = per_block.range_tuples(a, b)
        ws.autohete_grad_prep_accumulate(B.chunk_array(tup), len(tup), B.AH_BF16, 1.0, stream_handle())
    assert ws.autohete_grad_result_get(stream_handle())[2] == 1
    ws.close()


def test_hybrid_placement_step_matches_oracle():
    """Half of the chunks resident (GPU kernels), half host-owned (gradients D2H -> host AdamW ->
    16-bit parameters H2D through one pinned buffer per chunk): two steps against the oracle."""
    from paper_2503_01890_amd.hybrid import HostChunks, HybridStepper
    C, n_res, n_host = 1 << 16, 3, 3
    rng = np.random.default_rng(41)
    states = [random_state(C, B.AH_BF16, rng) for _ in range(n_res + n_host)]
    md = ModelData([C] * n_res)
    for i in range(n_res):
        upload(md, i, states[i])
    host = HostChunks(n_host, C)
    for c in range(n_host):
        st = states[n_res + c]
        host.master[c][:] = st["master"]
        host.exp_avg[c][:] = st["exp_avg"]
        host.exp_avg_sq[c][:] = st["exp_avg_sq"]
        host.dev_view("param_lp", c).copy_(torch.from_numpy(st["param_lp"].view(np.int16)))
    stepper = HybridStepper(md, host, B.AH_BF16, n_threads=4)
    hp = B.hparams(max_grad_norm=0.05)
    for step in (1, 2):
        for i, st in enumerate(states):
            st["grad"] = random_state(C, B.AH_BF16, rng)["grad"]
            if i < n_res:
                upload(md, i, dict(grad=st["grad"]))
            else:
                host.dev_view("grad", i - n_res).copy_(torch.from_numpy(st["grad"].view(np.int16)))
        torch.cuda.synchronize()
        out = stepper.step(step, hp)
        on, of = run_oracle(states, oracle.BF16, step, hp)
        assert out["found_inf"] == of == 0 and abs(out["norm"] - on) <= 1e-5 * on
        for i, st in enumerate(states):
            if i < n_res:
                got = download(md, i)
            else:
                c = i - n_res
                got = dict(master=host.master[c], exp_avg=host.exp_avg[c], exp_avg_sq=host.exp_avg_sq[c],
                           param_lp=host.dev_view("param_lp", c).cpu().numpy().view(np.uint16))
            compare_state(got, st, "hybrid step=%d chunk=%d" % (step, i), st["old"])
            if i < n_res:                       # oracle -> both halves: the next step starts identical
                upload(md, i, {k: st[k] for k in F32_AND_LP})
            else:
                host.master[c][:], host.exp_avg[c][:], host.exp_avg_sq[c][:] = st["master"], st["exp_avg"], st["exp_avg_sq"]
                host.dev_view("param_lp", c).copy_(torch.from_numpy(st["param_lp"].view(np.int16)))
    # overflow in a HOST-owned gradient: the GPU's norm sees it, both halves skip
    bad = states[n_res + 1]["grad"].copy()
    bad[99] = 0x7F80
    host.dev_view("grad", 1).copy_(torch.from_numpy(bad.view(np.int16)))
    keep_master = [m.copy() for m in host.master]
    keep_lp = host.dev_param_lp.clone()
    keep_res = [download(md, i) for i in range(n_res)]
    out = stepper.step(3, hp)
    assert out["found_inf"] == 1
    assert all(np.array_equal(a, b) for a, b in zip(keep_master, host.master)) and torch.equal(keep_lp, host.dev_param_lp)
    for i in range(n_res):
        now = download(md, i)
        assert all(now[k].tobytes() == keep_res[i][k].tobytes() for k in STREAMS)
    stepper.close()


def test_single_chunk_beyond_2_to_32_elements():
    """64-bit indexing: ONE chunk of 2^32 + 2^20 + 24 elements (68.8 GB of model data).  The norm is
    checked over every element; the update on windows at the start, across element 2^32 and at the
    ragged end, regenerated on the CPU from the same seeds."""
    import synthdata
    from _harness import N_THREADS
    import concurrent.futures as cf
    n = (1 << 32) + (1 << 20) + 24
    free, _ = torch.cuda.mem_get_info()
    if free < n * 16 + (8 << 30):
        pytest.skip("not enough free HBM for a 69 GB chunk")
    w = synthdata.Workload("huge-chunk", [n], n)          # one tensor, one chunk, no padding
    assert w.n_chunks == 1
    md = ModelData([n])
    st = stream_handle()
    synthdata.fill_gpu(md.ptr("param_lp", 0), n, w.spec_param_lp(0), st)
    synthdata.fill_gpu(md.ptr("master", 0), n, w.spec_master(0), st)
    synthdata.fill_gpu(md.ptr("exp_avg", 0), n, w.spec_exp_avg(0), st)
    synthdata.fill_gpu(md.ptr("exp_avg_sq", 0), n, w.spec_exp_avg_sq(0), st)
    synthdata.fill_gpu(md.ptr("grad", 0), n, w.spec_grad(0, 1), st)
    ws = B.Workspace(1)
    hp = B.hparams()
    gn, gf = run_gpu(md, ws, B.AH_BF16, 1, hp)

    def window(spec_fn, lo, cnt, dt, *a):
        spec = spec_fn(0, *a)
        spec.first_index = lo
        return synthdata.fill_cpu(np.empty(cnt, dt), spec)

    piece = 1 << 26
    starts = list(range(0, n, piece))

    def part(lo):
        g = window(w.spec_grad, lo, min(piece, n - lo), np.uint16, 1)
        return oracle.grad_accumulate(g, oracle.BF16, 1.0)

    with cf.ThreadPoolExecutor(N_THREADS) as ex:
        parts = list(ex.map(part, starts))
    on, of = oracle.grad_finish(sum(p[0] for p in parts), max(p[1] for p in parts))
    assert gf == of == 0 and abs(gn - on) <= 1e-5 * on
    cnt = 1 << 16
    for lo in (0, (1 << 32) - cnt // 2, n - cnt + 8, n - 1000):
        k = min(cnt, n - lo)
        ref = dict(grad=window(w.spec_grad, lo, k, np.uint16, 1), param_lp=window(w.spec_param_lp, lo, k, np.uint16),
                   master=window(w.spec_master, lo, k, np.float32), exp_avg=window(w.spec_exp_avg, lo, k, np.float32),
                   exp_avg_sq=window(w.spec_exp_avg_sq, lo, k, np.float32))
        old = dict(master=ref["master"].copy(), exp_avg=ref["exp_avg"].copy(), exp_avg_sq=ref["exp_avg_sq"].copy())
        oracle.adamw_chunk(ref["grad"], ref["param_lp"], ref["master"], ref["exp_avg"], ref["exp_avg_sq"], oracle.BF16,
                           1, oracle_hp(hp), on, 0)
        got = {}
        for s in ("param_lp", "master", "exp_avg", "exp_avg_sq"):
            a = md.view(s, 0)[lo:lo + k].cpu().numpy()
            got[s] = a.view(np.uint16).copy() if a.dtype == np.int16 else a.copy()
        compare_state(got, ref, "huge chunk window at %d" % lo, old, StepCtx(oracle.BF16, hp, 1, on))
    ws.close()


def _random_hparams(rng):
    pick = lambda xs: xs[int(rng.integers(0, len(xs)))]
    return dict(lr=float(pick([1e-5, 1e-4, 3e-3, 0.1, 0.0])), beta1=float(pick([0.0, 0.5, 0.9, 0.99])),
                beta2=float(pick([0.0, 0.9, 0.999, 0.9999])), eps=float(pick([1e-12, 1e-8, 1e-6, 1e-3])),
                weight_decay=float(pick([0.0, 0.01, 0.1, 1.0])), max_grad_norm=float(pick([0.0, -1.0, 1e-3, 0.05, 1.0, 1e6])),
                loss_scale=float(pick([1.0, 3.0, 1000.0, 65536.0, 0.125])))


@pytest.mark.parametrize("seed", range(24))
def test_random_hyperparameters_and_steps(seed):
    """Parity over the hyper-parameter space: zero betas, no decay, no clipping / heavy clipping,
    loss scales that are not powers of two (both sides multiply by the fp64 reciprocal), large t."""
    rng = np.random.default_rng(1000 + seed)
    dtype = B.AH_BF16 if seed % 2 == 0 else B.AH_FP16
    kw = _random_hparams(rng)
    if dtype == B.AH_FP16 and kw["loss_scale"] > 1000.0:
        kw["loss_scale"] = 1000.0                      # keep scaled fp16 gradients finite
    hp, ohp = B.hparams(**kw), oracle.hparams(**kw)
    numels = [int(x) for x in rng.integers(1, 30_000, 5)]
    states = [random_state(n, dtype, rng, scale=kw["loss_scale"]) for n in numels]
    md = ModelData(numels)
    for i, st in enumerate(states):
        upload(md, i, st)
    ws = B.Workspace(len(numels))
    extra = float(rng.choice([0.0, 1e-6, 3.5]))
    for step in (int(rng.integers(1, 5)), int(rng.integers(5, 100_000))):
        arr = md.chunk_array()
        gn, gf = ws.autohete_grad_prep(arr, len(numels), dtype, kw["loss_scale"], extra, stream_handle(), want_result=True)
        ws.autohete_adamw_step(arr, len(numels), dtype, step, hp, stream_handle())
        torch.cuda.synchronize()
        for st in states:
            st["old"] = dict(master=st["master"].copy(), exp_avg=st["exp_avg"].copy(), exp_avg_sq=st["exp_avg_sq"].copy())
        on, of = oracle.full_step(states, dtype, step, ohp, extra)
        check_norm(gn, gf, on, of)
        ctx = StepCtx(dtype, hp, step, on, ws.autohete_grad_result_get(stream_handle())[0])
        for i, st in enumerate(states):
            compare_state(download(md, i), st, "seed=%d %r step=%d chunk=%d" % (seed, kw, step, i), st["old"], ctx)
        resync(md, states)
    ws.close()


def test_seventy_thousand_tiny_chunks_cross_the_grid_row_limit():
    """More chunks than one launch has grid rows (65535): the launcher must split the group."""
    rng = np.random.default_rng(8)
    n_chunks = 70_000
    numels = [int(x) for x in rng.integers(1, 40, n_chunks)]
    total = sum(numels)
    flat = random_state(total, B.AH_BF16, rng)
    md = ModelData(numels, layout="slab")
    # upload through the slabs directly: chunk i sits at md.offset[i]
    idx = np.concatenate([np.arange(o, o + n) for o, n in zip(md.offset, numels)])
    for s in STREAMS:
        a = flat[s]
        slab = md.slab[s]
        slab.zero_()
        slab[torch.from_numpy(idx).to(slab.device)] = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(slab.device)
    ws = B.Workspace(n_chunks)
    hp = B.hparams(max_grad_norm=0.01)
    gn, gf = run_gpu(md, ws, B.AH_BF16, 3, hp)
    old = dict(master=flat["master"].copy(), exp_avg=flat["exp_avg"].copy(), exp_avg_sq=flat["exp_avg_sq"].copy())
    on, of = oracle.full_step([flat], oracle.BF16, 3, oracle_hp(hp))
    check_norm(gn, gf, on, of)
    got = {}
    dev_idx = torch.from_numpy(idx).to(md.slab["master"].device)
    for s in ("param_lp", "master", "exp_avg", "exp_avg_sq"):
        a = md.slab[s][dev_idx].cpu().numpy()
        got[s] = a.view(np.uint16).copy() if a.dtype == np.int16 else a.copy()
    compare_state(got, flat, "70k chunks", old, StepCtx(oracle.BF16, hp, 3, on))
    for s in ("param_lp", "master", "exp_avg", "exp_avg_sq"):      # oracle -> device before the next step
        a = flat[s]
        md.slab[s][dev_idx] = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(dev_idx.device)
    # the norm-carrying update over the same 70k rows: its per-wave slots must stay consecutive across launch groups
    other = B.Workspace(n_chunks)
    other.autohete_grad_result_set(0.0, 0, stream_handle())
    ws.autohete_adamw_step_carry(other, md.chunk_array(), n_chunks, B.AH_BF16, 4, hp, stream_handle())
    torch.cuda.synchronize()
    carried = other.autohete_grad_result_get(stream_handle())[0]
    ref = float(np.sum(oracle.decode(flat["grad"], oracle.BF16).astype(np.float64) ** 2))
    assert abs(carried - ref) <= 1e-12 * ref
    old = dict(master=flat["master"].copy(), exp_avg=flat["exp_avg"].copy(), exp_avg_sq=flat["exp_avg_sq"].copy())
    oracle.adamw_chunk(flat["grad"], flat["param_lp"], flat["master"], flat["exp_avg"], flat["exp_avg_sq"], oracle.BF16, 4,
                       oracle_hp(hp), on, 0)
    for s in ("param_lp", "master", "exp_avg", "exp_avg_sq"):
        a = md.slab[s][dev_idx].cpu().numpy()
        got[s] = a.view(np.uint16).copy() if a.dtype == np.int16 else a.copy()
    compare_state(got, flat, "70k chunks, carry", old, StepCtx(oracle.BF16, hp, 4, on))
    other.close()
    ws.close()


def test_two_workspaces_on_two_streams_do_not_interfere():
    rng = np.random.default_rng(9)
    numels = [300_000, 123_457]
    sets = []
    for k in range(2):
        states = [random_state(n, B.AH_BF16, rng) for n in numels]
        md = ModelData(numels)
        for i, st in enumerate(states):
            upload(md, i, st)
        sets.append((states, md, B.Workspace(2), torch.cuda.Stream(), B.hparams(max_grad_norm=0.03 * (k + 1))))
    torch.cuda.synchronize()
    for rep in range(3):
        for states, md, ws, stream, hp in sets:           # interleave the launches of the two streams
            with torch.cuda.stream(stream):
                arr = md.chunk_array()
                ws.autohete_grad_prep(arr, 2, B.AH_BF16, 1.0, 0.0, stream.cuda_stream)
                ws.autohete_adamw_step(arr, 2, B.AH_BF16, rep + 1, hp, stream.cuda_stream)
        torch.cuda.synchronize()
        for states, md, ws, stream, hp in sets:
            run_oracle(states, oracle.BF16, rep + 1, hp, ws=ws)
            for i, st in enumerate(states):
                compare_state(download(md, i), st, "two streams", st["old"])
            resync(md, states)
    for states, md, ws, stream, hp in sets:
        ws.close()


def _two_copies(states, numels):
    a, b = ModelData(numels), ModelData(numels)
    for i, st in enumerate(states):
        upload(a, i, st)
        upload(b, i, st)
    return a, b


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("dtype", [B.AH_BF16, B.AH_FP16])
def test_norm_carrying_step_equals_accumulate_then_step(variant, dtype):
    """autohete_adamw_step_carry must leave the five streams bit-identical to
    grad_prep_accumulate(next) + adamw_step(current), the next norm equal up to the order of the
    fp64 additions, and both must match the oracle stepping with the norm held by `current`."""
    rng = np.random.default_rng(1000 + variant)
    numels = [int(x) for x in rng.integers(1, 40_000, 19)] + [8192, 256, 1, 8, 65536 + 5, 3 * 16384]
    scale = 1.0 if dtype == B.AH_BF16 else 64.0
    states = [random_state(n, dtype, rng, scale=scale) for n in numels]
    fused, split = _two_copies(states, numels)
    n = len(numels)
    cur, nxt, cur2, nxt2 = (B.Workspace(n) for _ in range(4))
    for w in (cur, cur2):
        w.tune(B.AH_TUNE_STEP_VARIANT, variant)
        w.tune(B.AH_TUNE_STEP_BLOCKS_PER_CU, [0, 3, 64][variant % 3])
    hp = B.hparams(max_grad_norm=0.05, loss_scale=scale)
    s = stream_handle()
    carried_in = 0.37                                    # next-norm accumulations start from a non-zero S
    for w in (cur, cur2):
        w.autohete_grad_result_set(0.09, 0, s)           # "previous iteration": norm 0.3 -> clipping active
    for w in (nxt, nxt2):
        w.autohete_grad_result_set(carried_in, 0, s)
    cur.autohete_adamw_step_carry(nxt, fused.chunk_array(), n, dtype, 3, hp, s)
    nxt2.autohete_grad_prep_accumulate(split.chunk_array(), n, dtype, scale, s)
    cur2.autohete_adamw_step(split.chunk_array(), n, dtype, 3, hp, s)
    torch.cuda.synchronize()
    assert cur.autohete_grad_result_get(s) == cur2.autohete_grad_result_get(s)       # untouched by the call
    sa, na, fa = nxt.autohete_grad_result_get(s)
    sb, nb, fb = nxt2.autohete_grad_result_get(s)
    assert fa == fb == 0 and abs(sa - sb) <= 1e-13 * sb
    ref = carried_in + sum(float(np.sum((oracle.decode(st["grad"], dtype).astype(np.float64) / scale) ** 2))
                           for st in states)
    assert abs(sa - ref) <= 1e-12 * ref
    for i, st in enumerate(states):
        a, b = download(fused, i), download(split, i)
        assert all(a[k].tobytes() == b[k].tobytes() for k in STREAMS), (hex(variant), i)
        old = dict(master=st["master"].copy(), exp_avg=st["exp_avg"].copy(), exp_avg_sq=st["exp_avg_sq"].copy())
        oracle.adamw_chunk(st["grad"], st["param_lp"], st["master"], st["exp_avg"], st["exp_avg_sq"], dtype, 3,
                           oracle_hp(hp), 0.3, 0)
        compare_state(a, st, "carry variant=%x chunk=%d" % (variant, i), old, StepCtx(dtype, hp, 3, 0.3))
    # the same launch again: the carried sum is bit-reproducible
    nxt.autohete_grad_result_set(carried_in, 0, s)
    cur.autohete_grad_result_set(0.0, 1, s)              # flagged: no stream may change, squares still gathered
    before = [download(fused, i) for i in range(n)]
    cur.autohete_adamw_step_carry(nxt, fused.chunk_array(), n, dtype, 4, hp, s)
    torch.cuda.synchronize()
    assert nxt.autohete_grad_result_get(s)[0] == sa
    for i in range(n):
        after = download(fused, i)
        assert all(after[k].tobytes() == before[i][k].tobytes() for k in STREAMS), i
    for w in (cur, nxt, cur2, nxt2):
        w.close()


def test_norm_carrying_step_lagged_pipeline_against_oracle():
    """Three iterations of block-by-block stepping, last block first, each block's update clipped
    with the PREVIOUS iteration's norm while this iteration's is gathered by the same kernels;
    two workspaces alternate.  Oracle: the same schedule written out (norm of iteration t-1 into
    the update of iteration t).  A non-finite gradient in iteration 3 must surface in the carried
    result, and a buffer that has to grow between calls must not disturb anything."""
    import synthdata
    d, L, C = 128, 4, 1 << 15
    sizes = [int(x) for x in synthdata.gpt_tensor_numel(d, L, 500, 32)]
    off, n_chunks, total, pad = B.autohete_chunk_layout(sizes, C)
    bounds = [0, off[2]] + [off[2 + 12 * (i + 1)] if 2 + 12 * (i + 1) < len(off) else total for i in range(L)]
    bounds[-1] = n_chunks * C
    blocks = list(zip(bounds[:-1], bounds[1:]))
    rng = np.random.default_rng(77)
    states = [random_state(C, B.AH_BF16, rng) for _ in range(n_chunks)]
    for k in states[-1]:
        states[-1][k][C - pad:] = 0
    md = ModelData([C] * n_chunks)
    for i, st in enumerate(states):
        upload(md, i, st)
    hp = B.hparams(max_grad_norm=0.02)
    ws = [B.Workspace(n_chunks + 2), B.Workspace(n_chunks + 2)]
    s = stream_handle()
    ws[1].autohete_grad_result_set(0.0, 0, s)            # iteration 1 has no earlier norm: no clipping
    prev_sumsq = 0.0
    for it in (1, 2, 3):
        cur, nxt = ws[it % 2], ws[(it + 1) % 2]
        if it > 1:
            for i, st in enumerate(states):              # fresh gradients
                st["grad"] = random_state(C, B.AH_BF16, rng)["grad"]
                if i == n_chunks - 1:
                    st["grad"][C - pad:] = 0
                if it == 3 and i == 0:
                    st["grad"][4321] = 0x7FC0            # NaN: seen only in the carried result
                upload(md, i, dict(grad=st["grad"]))
        nxt.autohete_grad_result_set(0.0, 0, s)
        for a, b in reversed(blocks):                    # smallest-to-largest calls also exercise buffer growth
            tup = md.range_tuples(a, b)
            cur.autohete_adamw_step_carry(nxt, B.chunk_array(tup), len(tup), B.AH_BF16, it, hp, s)
        sumsq, norm, flag = nxt.autohete_grad_result_get(s)
        o_sumsq, o_flag = 0.0, 0
        for st in states:
            o_sumsq, o_flag = oracle.grad_accumulate(st["grad"], oracle.BF16, 1.0, o_sumsq, o_flag)
        assert flag == o_flag == (1 if it == 3 else 0)
        if not flag:
            assert abs(sumsq - o_sumsq) <= 1e-12 * o_sumsq
        if it < 3:                                       # iteration 3 writes NaN into chunk 0 on both sides
            for i, st in enumerate(states):
                old = dict(master=st["master"].copy(), exp_avg=st["exp_avg"].copy(),
                           exp_avg_sq=st["exp_avg_sq"].copy())
                oracle.adamw_chunk(st["grad"], st["param_lp"], st["master"], st["exp_avg"], st["exp_avg_sq"],
                                   oracle.BF16, it, oracle_hp(hp), float(np.sqrt(prev_sumsq)), 0)
                compare_state(download(md, i), st, "lagged it=%d chunk=%d" % (it, i), old,
                              StepCtx(oracle.BF16, hp, it, float(np.sqrt(prev_sumsq))))
                upload(md, i, st)                        # oracle -> device, so each step starts from equal inputs
        prev_sumsq = o_sumsq
    for w in ws:
        w.close()


def test_norm_carrying_step_rejects_bad_workspaces():
    md = ModelData([1024])
    ws, other = B.Workspace(1), B.Workspace(1)
    hp = B.hparams()
    lib = B.raw()
    args = (md.chunk_array(), 1, B.AH_BF16, 1, ctypes.byref(hp), ctypes.c_void_p(stream_handle()))
    assert lib.autohete_adamw_step_carry(ws._h, None, *args) == B.AH_EINVAL
    assert lib.autohete_adamw_step_carry(ws._h, ws._h, *args) == B.AH_EINVAL
    assert lib.autohete_adamw_step_carry(None, other._h, *args) == B.AH_EINVAL
    assert lib.autohete_adamw_step_carry(ws._h, other._h, md.chunk_array(), 0, B.AH_BF16, 1, ctypes.byref(hp),
                                         ctypes.c_void_p(stream_handle())) == B.AH_OK
    torch.cuda.synchronize()
    ws.close()
    other.close()


def test_carried_norm_joins_the_result_exactly_once():
    """The carried squares are folded lazily; whatever call touches ws_next's result next must see
    them exactly once (reads, accumulations, updates) or drop them (calls that replace the result)."""
    rng = np.random.default_rng(31)
    numels = [50_000, 777, 1 << 16]
    states = [random_state(n, B.AH_BF16, rng) for n in numels]
    md = ModelData(numels)
    for i, st in enumerate(states):
        upload(md, i, st)
    arr, n, s = md.chunk_array(), len(numels), stream_handle()
    cur, nxt = B.Workspace(n), B.Workspace(n)
    hp = B.hparams(lr=0.0, weight_decay=0.0)             # updates leave the master copy alone; gradients are read only
    S = sum(float(np.sum(oracle.decode(st["grad"], oracle.BF16).astype(np.float64) ** 2)) for st in states)

    def carry(times=1):
        for _ in range(times):
            cur.autohete_adamw_step_carry(nxt, arr, n, B.AH_BF16, 1, hp, s)

    cur.autohete_grad_result_set(0.0, 0, s)
    nxt.autohete_grad_result_set(0.0, 0, s)
    carry(3)                                             # three calls appended, one fold
    got = nxt.autohete_grad_result_get(s)[0]
    assert abs(got - 3 * S) <= 1e-12 * S
    assert nxt.autohete_grad_result_get(s)[0] == got     # a second read folds nothing more
    carry()
    nxt.autohete_grad_prep_accumulate(arr, n, B.AH_BF16, 1.0, s)
    assert abs(nxt.autohete_grad_result_get(s)[0] - (got + 2 * S)) <= 1e-12 * S
    carry()
    nxt.autohete_grad_result_set(5.0, 0, s)              # replaced: the carried sum goes with the old result
    assert nxt.autohete_grad_result_get(s) == (5.0, float(np.float32(np.sqrt(5.0))), 0)
    carry()
    nxt.autohete_grad_prep(arr, n, B.AH_BF16, 1.0, 0.0, s)
    assert abs(nxt.autohete_grad_result_get(s)[0] - S) <= 1e-12 * S
    # a different loss scale for later calls: earlier slots keep theirs
    nxt.autohete_grad_result_set(0.0, 0, s)
    carry()
    hp4 = B.hparams(lr=0.0, weight_decay=0.0, loss_scale=4.0)
    cur.autohete_adamw_step_carry(nxt, arr, n, B.AH_BF16, 1, hp4, s)
    assert abs(nxt.autohete_grad_result_get(s)[0] - (S + S / 16.0)) <= 1e-12 * S
    # the workspace that received the sum can clip with it straight away (folded by the update call itself)
    nxt.autohete_grad_result_set(0.0, 0, s)
    carry()
    torch.cuda.synchronize()
    twin = ModelData(numels)
    for i in range(n):
        upload(twin, i, download(md, i))
    clip = B.hparams(max_grad_norm=1e-3)
    nxt.autohete_adamw_step(arr, n, B.AH_BF16, 2, clip, s)
    folded = nxt.autohete_grad_result_get(s)
    assert abs(folded[0] - S) <= 1e-12 * S and folded[2] == 0
    cur.autohete_grad_result_set(folded[0], 0, s)
    cur.autohete_adamw_step(twin.chunk_array(), n, B.AH_BF16, 2, clip, s)
    torch.cuda.synchronize()
    for i in range(n):
        a, b = download(md, i), download(twin, i)
        assert all(a[k].tobytes() == b[k].tobytes() for k in STREAMS), i
    assert any(download(md, i)["master"].tobytes() != states[i]["master"].tobytes() for i in range(n))
    cur.close()
    nxt.close()


@pytest.mark.parametrize("variant", VARIANTS)
def test_nothing_is_written_outside_the_chunks(variant):
    """Every slab is filled with a byte pattern, ragged chunks are placed into it with gaps between
    them (and a guard region after the last), and every entry point runs over them: all bytes that
    belong to no chunk must keep the pattern, for every kernel variant and both 16-bit formats."""
    rng = np.random.default_rng(4242 + variant)
    sizes = [1, 3, 7, 8, 9, 63, 65, 127, 255, 257, 511, 1023, 1025, 2047, 4097, 8191, 65536 + 5, 1000, 128]
    numels = sizes + [256]                                   # the last one is never given to the library
    real = list(range(len(sizes)))
    for dtype in (B.AH_BF16, B.AH_FP16):
        md = ModelData(numels, layout=("group", "slab")[variant % 2], group_chunks=1 + variant % 5)
        for t in md.storages():
            t.fill_(0xA5)
        for i in real:
            upload(md, i, random_state(numels[i], dtype, rng))
        inside = [torch.zeros(t.numel(), dtype=torch.bool, device=md.device) for t in md.storages()]
        for i in real:
            for name in STREAMS:
                k, a, b = md.byte_span(name, i)
                inside[k][a:b] = True
        ws, other = B.Workspace(len(numels)), B.Workspace(len(numels))
        ws.tune(B.AH_TUNE_STEP_VARIANT, variant)
        arr, n, s = md.chunk_array(real), len(real), stream_handle()
        hp = B.hparams()
        ws.autohete_grad_prep(arr, n, dtype, 1.0, 0.0, s)
        ws.autohete_adamw_step(arr, n, dtype, 1, hp, s)
        ws.autohete_adamw_step_master(arr, n, dtype, 2, hp, s)
        ws.autohete_cast_params(arr, n, dtype, s)
        other.autohete_grad_result_set(0.0, 0, s)
        ws.autohete_adamw_step_carry(other, arr, n, dtype, 3, hp, s)
        other.autohete_grad_prep_accumulate(arr, n, dtype, 1.0, s)
        torch.cuda.synchronize()
        assert other.autohete_grad_result_get(s)[2] == 0
        for k, t in enumerate(md.storages()):
            assert bool((t[~inside[k]] == 0xA5).all()), (hex(variant), dtype, k)
        ws.close()
        other.close()


def test_more_chunk_lists_than_cached_tables_and_a_second_stream():
    """Chunk tables are kept on the device by content and replaced least-recently-used.  A hundred
    single-chunk lists (two tables each), cycled three times, overflow that cache of 128; every call
    must still see its own list.  A list first used on one stream and at once on another must be
    complete there too."""
    rng = np.random.default_rng(808)
    numels = [int(x) for x in rng.integers(100, 30_000, 100)]
    states = [random_state(n, B.AH_BF16, rng) for n in numels]
    md = ModelData(numels)
    for i, st in enumerate(states):
        upload(md, i, st)
    ws = B.Workspace(4)
    hp = B.hparams(max_grad_norm=0.01)
    s = stream_handle()
    for step in (1, 2, 3):
        for i in range(100):
            arr = md.chunk_array([i])
            ws.autohete_grad_prep(arr, 1, B.AH_BF16, 1.0, 0.0, s)
            ws.autohete_adamw_step(arr, 1, B.AH_BF16, step, hp, s)
        torch.cuda.synchronize()
        for i, st in enumerate(states):
            run_oracle([st], B.AH_BF16, step, hp)
            compare_state(download(md, i), st, "cycle %d chunk %d" % (step, i), st["old"])
            resync(md, [st], [i])
    side = torch.cuda.Stream()                           # default priority
    torch.cuda.synchronize()
    fresh = md.chunk_array([3, 5, 8])                    # a list this workspace has not seen
    ws.autohete_grad_prep(fresh, 3, B.AH_BF16, 1.0, 0.0, s)            # upload enqueued on the first stream
    with torch.cuda.stream(side):
        ws.autohete_grad_prep(fresh, 3, B.AH_BF16, 1.0, 0.0, side.cuda_stream)   # found in the cache
        got = ws.autohete_grad_result_get(side.cuda_stream)[0]
    torch.cuda.synchronize()
    ref = sum(float(np.sum(oracle.decode(states[i]["grad"], oracle.BF16).astype(np.float64) ** 2)) for i in (3, 5, 8))
    assert abs(got - ref) <= 1e-12 * ref
    ws.close()


@pytest.mark.parametrize("dtype", [B.AH_BF16, B.AH_FP16])
def test_every_finite_16_bit_gradient_pattern(dtype):
    """All 65536 bit patterns as gradients (the non-finite ones replaced by zero so that the step
    is not skipped): subnormals, both zeros, the largest finite values.  The norm of the bf16 set
    is ~1e39, far beyond fp32, so the clip factor is ~1e-39 and only fp64 keeps it from vanishing."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = oracle.decode(bits, dtype)
    grad = np.where(np.isfinite(vals), bits, 0).astype(np.uint16)
    rng = np.random.default_rng(99 + dtype)
    for hp in (B.hparams(max_grad_norm=1.0), B.hparams(max_grad_norm=0.0, loss_scale=2.0 ** 100 if dtype == B.AH_BF16 else 1024.0)):
        st = random_state(65536, dtype, rng)
        st["grad"] = grad.copy()
        md = ModelData([65536])
        upload(md, 0, st)
        ws = B.Workspace(1)
        gn, gf = run_gpu(md, ws, dtype, 1, hp)
        on, of = run_oracle([st], dtype, 1, hp)
        assert gf == of == 0
        s_gpu = ws.autohete_grad_result_get(stream_handle())[0]
        ref = float(np.sum((vals[np.isfinite(vals)].astype(np.float64) / hp.loss_scale) ** 2))
        assert abs(s_gpu - ref) <= 1e-12 * ref                       # fp64 sum of exact squares
        with np.errstate(over="ignore"):
            on32 = np.float32(on)
        if np.isfinite(on32):
            assert abs(gn - on) <= 1e-5 * on
        else:
            assert gn == on32                                        # beyond fp32: both report inf
        compare_state(download(md, 0), st, "all patterns dtype=%d" % dtype, st["old"])
        ws.close()


@pytest.mark.parametrize("variant", [B.step_variant(4, 64, 0), B.step_variant(4, 64, 1), B.step_variant(1, 256, 0)])
def test_degenerate_states_match_the_exact_rule(variant):
    """States a run can reach without any non-finite gradient: a second moment that overflowed
    fp32 (huge finite gradient, clipping off), eps = 0 with no second moment yet, a first moment
    at +-inf.  The fast root / quotient must give what the exact operations give."""
    inf = np.float32(np.inf)
    n = 4096
    rng = np.random.default_rng(3)
    for eps, clip in ((1e-8, 0.0), (0.0, 0.0), (0.0, 1.0)):
        st = random_state(n, B.AH_BF16, rng)
        st["exp_avg_sq"][0::7] = inf                         # overflowed earlier
        st["exp_avg_sq"][1::7] = 0.0
        st["grad"][1::7] = 0                                 # v stays 0: denominator is eps alone
        st["grad"][2::7] = 0x7F7F                            # largest finite bf16: v overflows in this very step
        st["exp_avg"][3::7] = inf
        st["exp_avg"][4::7] = -inf
        st["exp_avg_sq"][4::7] = inf                         # inf / inf
        st["exp_avg"][5::7] = 0.0
        st["grad"][5::7] = 0
        st["exp_avg_sq"][5::7] = 0.0                         # 0 / (0 + eps)
        hp = B.hparams(eps=eps, max_grad_norm=clip)
        md = ModelData([n])
        upload(md, 0, st)
        ws = B.Workspace(1)
        ws.tune(B.AH_TUNE_STEP_VARIANT, variant)
        gn, gf = run_gpu(md, ws, B.AH_BF16, 2, hp)
        with np.errstate(all="ignore"):
            on, of = run_oracle([st], B.AH_BF16, 2, hp)
        assert gf == of == 0
        got = download(md, 0)
        for k in ("master", "exp_avg", "exp_avg_sq"):
            g, o = got[k], st[k]
            assert np.array_equal(np.isnan(g), np.isnan(o)), (eps, clip, k, "NaN pattern")
            assert np.array_equal(np.isinf(g), np.isinf(o)) and np.array_equal(np.sign(g[np.isinf(g)]), np.sign(o[np.isinf(o)])), (eps, clip, k, "inf pattern")
            fin = np.isfinite(o)
            err = np.abs(g[fin].astype(np.float64) - o[fin].astype(np.float64))
            tol = 2.0 * np.spacing(np.abs(o[fin]).astype(np.float32)).astype(np.float64)
            if clip > 0:                                      # the norm (~1e39) is summed in a different order
                tol = np.maximum(tol, 1e-6 * np.abs(o[fin]))
            assert (err <= tol).all(), (eps, clip, k, float(err.max()))
        nan16 = lambda b: (b & 0x7F80) == 0x7F80
        same = got["param_lp"] == st["param_lp"]
        both_nan = nan16(got["param_lp"]) & nan16(st["param_lp"]) & ((got["param_lp"] & 0x7F) != 0) & ((st["param_lp"] & 0x7F) != 0)
        d = np.abs(ordered16_(got["param_lp"]) - ordered16_(st["param_lp"]))
        assert (same | both_nan | (d <= 1)).all(), (eps, clip, "param_lp")
        ws.close()


def ordered16_(bits):
    b = bits.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)


@pytest.mark.parametrize("dtype", [B.AH_BF16, B.AH_FP16])
def test_exact_mode_is_bit_identical_to_the_oracle_given_the_same_norm(dtype):
    """MODE 1 of the update kernel uses correctly rounded fp64 root and divisions in the oracle's
    operation order, so with the same S handed to both sides every stored bit must agree -- four
    million elements, three steps, no tolerance.  The fast mode (Newton iterations) is then held
    against it: it may differ from the exact mode in the last bit of a vanishing fraction only."""
    n = 1 << 22
    rng = np.random.default_rng(2024 + dtype)
    scale = 1.0 if dtype == B.AH_BF16 else 128.0
    st = random_state(n, dtype, rng, scale=scale)
    exact, fast = ModelData([n]), ModelData([n])
    upload(exact, 0, st)
    upload(fast, 0, st)
    ws_e, ws_f = B.Workspace(1), B.Workspace(1)
    ws_e.tune(B.AH_TUNE_STEP_VARIANT, B.step_variant(4, 64, 1))
    hp = B.hparams(max_grad_norm=0.5, loss_scale=scale)
    s = stream_handle()
    for step in (1, 2, 3):
        if step > 1:
            st["grad"] = random_state(n, dtype, rng, scale=scale)["grad"]
            upload(exact, 0, dict(grad=st["grad"]))
            upload(fast, 0, dict(grad=st["grad"]))
        sumsq, flag = oracle.grad_accumulate(st["grad"], dtype, scale)
        assert flag == 0
        norm = float(np.sqrt(sumsq))
        for ws, md in ((ws_e, exact), (ws_f, fast)):
            ws.autohete_grad_result_set(sumsq, 0, s)
            ws.autohete_adamw_step(md.chunk_array(), 1, dtype, step, hp, s)
        torch.cuda.synchronize()
        oracle.adamw_chunk(st["grad"], st["param_lp"], st["master"], st["exp_avg"], st["exp_avg_sq"], dtype, step,
                           oracle_hp(hp), norm, 0)
        got_e, got_f = download(exact, 0), download(fast, 0)
        for k in ("master", "exp_avg", "exp_avg_sq", "param_lp"):
            assert got_e[k].tobytes() == st[k].tobytes(), (step, k, "exact mode differs from the oracle")
        for k in ("master", "exp_avg", "exp_avg_sq"):
            diff = got_f[k].view(np.uint32) != st[k].view(np.uint32)
            assert diff.sum() <= 1e-5 * n, (step, k, int(diff.sum()))
            d = np.abs(got_f[k].view(np.int32).astype(np.int64) - st[k].view(np.int32).astype(np.int64))
            assert d.max() <= 1, (step, k, "fast mode more than one ulp from the exact result")
        assert (got_f["param_lp"] != st["param_lp"]).sum() <= 1e-6 * n
        upload(fast, 0, st)                                  # both continue from the oracle's state
    ws_e.close()
    ws_f.close()


def test_prep_and_step_captured_in_a_hip_graph_replay_like_eager_calls():
    """One optimizer step (autohete_grad_prep + autohete_adamw_step) recorded into a HIP graph.
    After a warm-up call on the capture stream the library finds its chunk tables on the device, so
    the recording holds the two kernels and nothing else (no upload, no memset node).  The graph is
    replayed four times with eager work and synchronisations of the same process in between; after
    every replay the state must equal, bit for bit, that of a second copy stepped eagerly."""
    rng = np.random.default_rng(515)
    numels = [200_000, 65536, 33_333]
    states = [random_state(n, B.AH_BF16, rng) for n in numels]
    graph_md, eager_md = ModelData(numels), ModelData(numels)
    for i, st in enumerate(states):
        upload(graph_md, i, st)
        upload(eager_md, i, st)
    hp = B.hparams(max_grad_norm=0.05)
    ws_g, ws_e = B.Workspace(3), B.Workspace(3)
    side = torch.cuda.Stream()                                     # default priority
    arr_g, arr_e = graph_md.chunk_array(), eager_md.chunk_array()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):                                  # warm-up: the tables are uploaded here
        ws_g.autohete_grad_prep(arr_g, 3, B.AH_BF16, 1.0, 0.0, side.cuda_stream)
        ws_g.autohete_adamw_step(arr_g, 3, B.AH_BF16, 1, hp, side.cuda_stream)
    side.synchronize()
    ws_e.autohete_grad_prep(arr_e, 3, B.AH_BF16, 1.0, 0.0, stream_handle())
    ws_e.autohete_adamw_step(arr_e, 3, B.AH_BF16, 1, hp, stream_handle())
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        ws_g.autohete_grad_prep(arr_g, 3, B.AH_BF16, 1.0, 0.0, side.cuda_stream)
        ws_g.autohete_adamw_step(arr_g, 3, B.AH_BF16, 2, hp, side.cuda_stream)   # the step number is part of the recording
    torch.cuda.synchronize()
    for i in range(3):                                             # recording runs nothing
        a, b = download(graph_md, i), download(eager_md, i)
        assert all(a[k].tobytes() == b[k].tobytes() for k in STREAMS)
    scratch = torch.zeros(1 << 20, device="cuda:0")
    for rep in range(4):
        fresh = [random_state(n, B.AH_BF16, rng)["grad"] for n in numels]
        for i, gr in enumerate(fresh):                             # eager work between the replays
            upload(graph_md, i, dict(grad=gr))
            upload(eager_md, i, dict(grad=gr))
        scratch.add_(1.0)
        torch.cuda.synchronize()
        g.replay()
        ws_e.autohete_grad_prep(arr_e, 3, B.AH_BF16, 1.0, 0.0, stream_handle())
        ws_e.autohete_adamw_step(arr_e, 3, B.AH_BF16, 2, hp, stream_handle())
        torch.cuda.synchronize()
        assert ws_g.autohete_grad_result_get(stream_handle()) == ws_e.autohete_grad_result_get(stream_handle())
        for i in range(3):
            a, b = download(graph_md, i), download(eager_md, i)
            assert all(a[k].tobytes() == b[k].tobytes() for k in STREAMS), (rep, i)
    assert float(scratch[0]) == 4.0
    ws_g.close(), ws_e.close()


def test_bench_prints_one_json_line_with_the_contract_keys():
    """bench.py on the smallest configuration (a process of its own): exactly one JSON line with the
    metric, the timing fields, a roofline object for the dominant kernel and the workload name."""
    import json
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    run = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--workload", "gpt-124m", "--steps", "5",
                          "--warmup", "2", "--no-cpu-baseline"], capture_output=True, text=True, timeout=280)
    assert run.returncode == 0, run.stderr[-2000:]
    lines = [ln for ln in run.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "hbm"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["unit"] == "params/s" and d["data"] == "synthetic"
    assert d["config"]["workload"] == "gpt-124m" and d["vs_baseline"] is None and d["higher_is_better"] is True
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s" and abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12
    assert r["traffic_source"] == "profiles/adamw_step_kernel_gpt-124m_pmc.txt" and r["traffic"] > 0
    assert 0.3 < r["frac"] < 1.0 and 0 < d["ms_per_step"] < 5.0
    assert abs(d["value"] - d["config"]["resident_params"] / (d["ms_per_step"] * 1e-3)) <= 1e-6 * d["value"]
