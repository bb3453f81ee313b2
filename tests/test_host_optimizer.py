"""Host half of the hybrid placement (autohete_host_*): the library's CPU AdamW against the oracle.
Both compute in fp64 in the same operation order, so given the same global sum of squares the
results must be bit-identical -- AVX-512 path and scalar path, any thread count, both formats,
ragged sizes.  Runs without a GPU."""
import ctypes

import numpy as np
import pytest

import oracle
from paper_2503_01890_amd import binding as B

RNG = np.random.default_rng(99)


def lowp(x, dtype):
    return oracle.encode(np.asarray(x, np.float32), dtype)           # inputs only; pinned elsewhere


def make_state(n, dtype, scale=1.0):
    p16 = lowp(RNG.normal(0, 0.02, n), dtype)
    return dict(grad=lowp(RNG.normal(0, 1e-3, n) * scale, dtype), param_lp=p16.copy(), master=oracle.decode(p16, dtype),
                exp_avg=RNG.normal(0, 1e-4, n).astype(np.float32),
                exp_avg_sq=np.abs(RNG.normal(0, 1e-6, n)).astype(np.float32))


def host_chunks(states, with_lp=True):
    return B.chunk_array([(st["grad"].ctypes.data, st["param_lp"].ctypes.data if with_lp else None,
                           st["master"].ctypes.data, st["exp_avg"].ctypes.data, st["exp_avg_sq"].ctypes.data,
                           st["grad"].size) for st in states])


@pytest.fixture(params=[0, 1], ids=["avx512", "scalar"])
def simd(request):
    B.raw().autohete_host_force_scalar(request.param)
    yield request.param
    B.raw().autohete_host_force_scalar(0)


@pytest.mark.parametrize("dtype", [B.AH_BF16, B.AH_FP16])
@pytest.mark.parametrize("threads", [1, 3, 8])
def test_host_step_is_bit_identical_to_the_oracle(simd, dtype, threads):
    scale = 1.0 if dtype == B.AH_BF16 else 512.0
    numels = [1, 7, 8, 9, 15, 16, 17, 1000, 4099, 65536 + 3]
    lib_states = [make_state(n, dtype, scale) for n in numels]
    ora_states = [{k: v.copy() for k, v in st.items()} for st in lib_states]
    hp, ohp = B.hparams(loss_scale=scale, max_grad_norm=0.05), oracle.hparams(loss_scale=scale, max_grad_norm=0.05)
    arr = host_chunks(lib_states)
    for step in (1, 2, 3):
        sumsq, flag = B.autohete_host_grad_sumsq(arr, len(numels), dtype, scale, threads)
        onorm, oflag = oracle.grad_prep([st["grad"] for st in ora_states], dtype, scale)
        assert flag == oflag == 0 and abs(np.sqrt(sumsq) - onorm) <= 1e-13 * onorm
        # same global sum on both sides (the oracle's) -> every stored bit must agree
        B.autohete_host_adamw_step(arr, len(numels), dtype, step, hp, onorm * onorm, 0, threads)
        for st in ora_states:
            oracle.adamw_chunk(st["grad"], st["param_lp"], st["master"], st["exp_avg"], st["exp_avg_sq"], dtype, step,
                               ohp, np.sqrt(onorm * onorm), 0)
        for a, b in zip(lib_states, ora_states):
            for k in a:
                assert a[k].tobytes() == b[k].tobytes(), (step, k, a[k].size)


def test_host_skip_nonfinite_and_no_writeback(simd):
    st = make_state(5000, B.AH_BF16)
    st["grad"][4321] = 0x7F80
    arr = host_chunks([st])
    sumsq, flag = B.autohete_host_grad_sumsq(arr, 1, B.AH_BF16, 1.0, 4)
    assert flag == 1 and not np.isfinite(sumsq)
    before = {k: v.copy() for k, v in st.items()}
    B.autohete_host_adamw_step(arr, 1, B.AH_BF16, 1, B.hparams(), sumsq, flag, 4)
    B.autohete_host_adamw_step(arr, 1, B.AH_BF16, 1, B.hparams(), 1.0, 1, 4)
    assert all(st[k].tobytes() == before[k].tobytes() for k in st)
    # NaN gradient, and no 16-bit write-back when param_lp is NULL
    st["grad"][4321] = 0x7FC0
    assert B.autohete_host_grad_sumsq(arr, 1, B.AH_BF16, 1.0, 2)[1] == 1
    st["grad"][4321] = 0
    stale = st["param_lp"].copy()
    ref = {k: v.copy() for k, v in st.items()}
    B.autohete_host_adamw_step(host_chunks([st], with_lp=False), 1, B.AH_BF16, 2, B.hparams(), 0.25, 0, 5)
    oracle.adamw_chunk(ref["grad"], None, ref["master"], ref["exp_avg"], ref["exp_avg_sq"], oracle.BF16, 2,
                       oracle.hparams(), 0.5, 0)
    assert np.array_equal(st["param_lp"], stale)
    assert all(st[k].tobytes() == ref[k].tobytes() for k in ("master", "exp_avg", "exp_avg_sq"))


def test_host_16bit_conversions_cover_edge_values(simd):
    """Write-back through the host path on values chosen for the format edges (ties, overflow to inf,
    subnormals): lr = 0, wd = 0 keeps master unchanged, so param_lp = RNE(master)."""
    for dtype in (B.AH_BF16, B.AH_FP16):
        vals = np.concatenate([RNG.normal(0, 1, 4000), [0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e-8, 6e-8, -3e-8, 3e38],
                               np.float32(1.0) + np.arange(0, 64) * np.float32(2.0 ** -12),
                               np.arange(0, 40) * np.float32(0.5 * 2.0 ** -24)]).astype(np.float32)
        n = vals.size
        st = dict(grad=np.zeros(n, np.uint16), param_lp=np.zeros(n, np.uint16), master=vals.copy(),
                  exp_avg=np.zeros(n, np.float32), exp_avg_sq=np.zeros(n, np.float32))
        B.autohete_host_adamw_step(host_chunks([st]), 1, dtype, 1, B.hparams(lr=0.0, weight_decay=0.0), 0.0, 0, 3)
        assert np.array_equal(st["master"], vals)
        assert np.array_equal(st["param_lp"], oracle.encode(vals, dtype))
        # and the decode side: the norm of every finite 16-bit pattern
        bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
        x = oracle.decode(bits, dtype).astype(np.float64)
        bits = bits[np.isfinite(x)]
        x = x[np.isfinite(x)]
        g = dict(st, grad=bits.copy())
        arr = B.chunk_array([(g["grad"].ctypes.data, None, None, None, None, bits.size)])
        sumsq, flag = B.autohete_host_grad_sumsq(arr, 1, dtype, 1.0, 2)
        assert flag == 0 and sumsq == pytest.approx(float(np.sum(x * x)), rel=1e-13)


def test_host_errors():
    st = make_state(64, B.AH_BF16)
    arr = host_chunks([st])
    lib = B.raw()
    hp = B.hparams()
    s, f = ctypes.c_double(), ctypes.c_uint32()
    assert lib.autohete_host_grad_sumsq(arr, 1, B.AH_BF16, ctypes.c_float(1.0), 0, ctypes.byref(s), ctypes.byref(f)) == B.AH_EINVAL
    assert lib.autohete_host_grad_sumsq(arr, 1, 5, ctypes.c_float(1.0), 1, ctypes.byref(s), ctypes.byref(f)) == B.AH_EINVAL
    assert lib.autohete_host_grad_sumsq(arr, 1, B.AH_BF16, ctypes.c_float(0.0), 1, ctypes.byref(s), ctypes.byref(f)) == B.AH_EINVAL
    assert lib.autohete_host_grad_sumsq(arr, 1, B.AH_BF16, ctypes.c_float(1.0), 1, None, ctypes.byref(f)) == B.AH_EINVAL
    assert lib.autohete_host_adamw_step(arr, 1, B.AH_BF16, 0, ctypes.byref(hp), 1.0, 0, 1) == B.AH_EINVAL
    bad = B.hparams(beta1=1.0)
    assert lib.autohete_host_adamw_step(arr, 1, B.AH_BF16, 1, ctypes.byref(bad), 1.0, 0, 1) == B.AH_EINVAL
    nul = B.chunk_array([(st["grad"].ctypes.data, None, None, st["exp_avg"].ctypes.data, st["exp_avg_sq"].ctypes.data, 64)])
    assert lib.autohete_host_adamw_step(nul, 1, B.AH_BF16, 1, ctypes.byref(hp), 1.0, 0, 1) == B.AH_EINVAL


@pytest.mark.parametrize("seed", range(12))
def test_host_random_hyperparameters_bit_identical(seed):
    rng = np.random.default_rng(500 + seed)
    pick = lambda xs: xs[int(rng.integers(0, len(xs)))]
    dtype = B.AH_BF16 if seed % 2 == 0 else B.AH_FP16
    kw = dict(lr=float(pick([1e-5, 1e-4, 3e-3, 0.1, 0.0])), beta1=float(pick([0.0, 0.5, 0.9, 0.99])),
              beta2=float(pick([0.0, 0.9, 0.999, 0.9999])), eps=float(pick([1e-12, 1e-8, 1e-6, 1e-3])),
              weight_decay=float(pick([0.0, 0.01, 0.1, 1.0])), max_grad_norm=float(pick([0.0, -1.0, 1e-3, 0.05, 1.0, 1e6])),
              loss_scale=float(pick([1.0, 3.0, 1000.0, 0.125])))
    n = int(rng.integers(1, 50_000))
    a = make_state(n, dtype, kw["loss_scale"])
    b = {k: v.copy() for k, v in a.items()}
    step = int(rng.integers(1, 100_000))
    sumsq = float(rng.choice([0.0, 1e-9, 0.37, 1e4]))
    B.autohete_host_adamw_step(host_chunks([a]), 1, dtype, step, B.hparams(**kw), sumsq, 0, 4)
    oracle.adamw_chunk(b["grad"], b["param_lp"], b["master"], b["exp_avg"], b["exp_avg_sq"], dtype, step,
                       oracle.hparams(**kw), float(np.sqrt(sumsq)), 0)
    for k in a:
        assert a[k].tobytes() == b[k].tobytes(), (kw, step, k)


def test_host_step_degenerate_states(simd):
    """Overflowed second moment, eps = 0 with no second moment, infinite first moments: the host path
    uses the exact root and quotient, so even the NaN / inf patterns must equal the oracle's."""
    n, inf = 4096, np.float32(np.inf)
    for eps in (1e-8, 0.0):
        st = make_state(n, B.AH_BF16)
        st["exp_avg_sq"][0::7] = inf
        st["exp_avg_sq"][1::7] = 0.0
        st["grad"][1::7] = 0
        st["grad"][2::7] = 0x7F7F
        st["exp_avg"][3::7] = inf
        st["exp_avg"][4::7] = -inf
        st["exp_avg_sq"][4::7] = inf
        st["exp_avg"][5::7] = 0.0
        st["grad"][5::7] = 0
        st["exp_avg_sq"][5::7] = 0.0
        ref = {k: v.copy() for k, v in st.items()}
        hp, ohp = B.hparams(eps=eps, max_grad_norm=0.0), oracle.hparams(eps=eps, max_grad_norm=0.0)
        B.autohete_host_adamw_step(host_chunks([st]), 1, B.AH_BF16, 2, hp, 1.0, 0, 3)
        with np.errstate(all="ignore"):
            oracle.adamw_chunk(ref["grad"], ref["param_lp"], ref["master"], ref["exp_avg"], ref["exp_avg_sq"],
                               oracle.BF16, 2, ohp, 1.0, 0)
        for k in ("master", "exp_avg", "exp_avg_sq"):
            a, b = st[k], ref[k]
            assert np.array_equal(np.isnan(a), np.isnan(b)), (eps, k)
            ok = ~np.isnan(b)
            assert a[ok].tobytes() == b[ok].tobytes(), (eps, k)
        nan16 = lambda x: ((x & 0x7F80) == 0x7F80) & ((x & 0x7F) != 0)
        assert np.array_equal(nan16(st["param_lp"]), nan16(ref["param_lp"]))
        ok = ~nan16(ref["param_lp"])
        assert np.array_equal(st["param_lp"][ok], ref["param_lp"][ok])


def test_bias_correction_quotients_without_division_are_the_quotients():
    """The AVX-512 path forms x / (1 - beta^t) from the correctly rounded reciprocal and two fused
    multiply-adds instead of a division.  That is the correctly rounded quotient by theorem; here it
    is held to the oracle's divisions bit for bit over 150 step numbers (each its own pair of
    divisors, including beta = 0 -> divisor 1), states that span forty binades, and gradients that
    include both zeros -- 20 million quotients."""
    B.raw().autohete_host_force_scalar(0)
    rng = np.random.default_rng(2024)
    n = 1 << 16
    steps = [1, 2, 3, 4, 5, 7, 10, 100, 1000, 10_000, 123_457] + [int(x) for x in rng.integers(1, 5000, 139)]
    for k, step in enumerate(steps):
        beta1, beta2 = (0.0, 0.0) if k == 0 else (float(rng.choice([0.9, 0.5, 0.99])), float(rng.choice([0.999, 0.95, 0.9])))
        hp = B.hparams(beta1=beta1, beta2=beta2, max_grad_norm=0.0, lr=1e-3, eps=1e-8)
        ohp = oracle.hparams(beta1=beta1, beta2=beta2, max_grad_norm=0.0, lr=1e-3, eps=1e-8)
        mag = lambda: np.exp2(rng.uniform(-30, 10, n))
        grad = lowp(rng.normal(0, 1, n) * mag(), B.AH_BF16)
        grad[:64] = np.where(np.arange(64) % 2, 0x8000, 0x0000)          # -0 and +0 gradients
        st = dict(grad=grad, param_lp=np.zeros(n, np.uint16), master=(rng.normal(0, 1, n) * mag()).astype(np.float32),
                  exp_avg=(rng.normal(0, 1, n) * mag()).astype(np.float32),
                  exp_avg_sq=(mag() ** 2).astype(np.float32))
        st["exp_avg"][:32] = np.where(np.arange(32) % 4 < 2, -0.0, 0.0)   # zero moments of both signs
        st["exp_avg_sq"][:16] = 0.0
        ref = {k_: v.copy() for k_, v in st.items()}
        B.autohete_host_adamw_step(host_chunks([st]), 1, B.AH_BF16, step, hp, 1.0, 0, 4)
        oracle.adamw_chunk(ref["grad"], ref["param_lp"], ref["master"], ref["exp_avg"], ref["exp_avg_sq"], B.AH_BF16,
                           step, ohp, 1.0, 0)
        for key in st:
            assert st[key].tobytes() == ref[key].tobytes(), (step, beta1, beta2, key)


def test_hand_worked_examples_through_the_host_optimizer(simd):
    """The 16-element examples worked by hand (tests/golden/adamw_hand_worked.txt), through the
    library's host path: every expected value is met exactly."""
    from _golden import load_hand_worked
    for name, c in load_hand_worked().items():
        dtype = B.AH_BF16 if c["dtype"] == "bf16" else B.AH_FP16
        hp = B.hparams(c["lr"], c["beta1"], c["beta2"], c["eps"], c["weight_decay"], c["max_grad_norm"], c["loss_scale"])
        st = dict(grad=lowp(c["grad"], dtype), param_lp=np.zeros(16, np.uint16), master=c["master"].astype(np.float32),
                  exp_avg=c["exp_avg"].astype(np.float32), exp_avg_sq=c["exp_avg_sq"].astype(np.float32))
        arr = host_chunks([st])
        for k in range(1, int(c["steps"]) + 1):
            sumsq, flag = B.autohete_host_grad_sumsq(arr, 1, dtype, c["loss_scale"], 2)
            assert flag == 0 and sumsq == pytest.approx(c["expect_sumsq"], rel=1e-15), name
            B.autohete_host_adamw_step(arr, 1, dtype, int(c["first_step"]) + k - 1, hp, sumsq, flag, 2)
            for key in ("master", "exp_avg", "exp_avg_sq"):
                assert np.array_equal(st[key], c["expect_%s_t%d" % (key, k)].astype(np.float32)), (name, key, k)
            assert np.array_equal(oracle.decode(st["param_lp"], dtype).astype(np.float64), c["expect_param_lp_t%d" % k]), name
