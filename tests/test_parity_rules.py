"""CPU checks of the comparison rules the GPU parity tests use (tests/parity_check.c through
tests/_harness.py): the strict rule for steps taken from identical inputs and the carried bound
for free-running state.  The "GPU" here is a second run of the oracle whose gradient norm differs
in its last bits (as a sum taken in another order does); mistakes are planted into that side and
must be caught."""
import numpy as np
import pytest

import oracle
from _harness import FreeRun, StepCtx, compare_state, random_state

F32 = ("master", "exp_avg", "exp_avg_sq")


def _copy(st):
    return {k: v.copy() for k, v in st.items() if isinstance(v, np.ndarray)}


def _step(st, dtype, step, hp, norm):
    oracle.adamw_chunk(st["grad"], st["param_lp"], st["master"], st["exp_avg"], st["exp_avg_sq"], dtype, step, hp, norm, 0)


def test_one_ulp_is_one_ulp_and_three_fail():
    rng = np.random.default_rng(0)
    ora = random_state(4096, oracle.BF16, rng)
    gpu = _copy(ora)
    gpu["master"] = np.nextafter(ora["master"], np.float32(np.inf))
    gpu["exp_avg_sq"] = np.nextafter(np.nextafter(ora["exp_avg_sq"], np.float32(np.inf)), np.float32(np.inf))
    st = compare_state(gpu, ora, "adjacent")
    assert st["master_mismatch"] == 4096 and st["exp_avg_mismatch"] == 0
    # at a power of two the spacing above is twice the spacing at the value: 1 or 2 "ulp32(ora)" either way
    assert 1.0 <= st["master_max_ulp"] <= 1.0 and 2.0 <= st["exp_avg_sq_max_ulp"] <= 2.0
    assert st["master_beyond"] == st["exp_avg_sq_beyond"] == 0
    bad = _copy(ora)
    x = bad["exp_avg"][17]
    for _ in range(20):                                   # 20 ulp > relative 1e-6 (about 8 to 17 ulp)
        x = np.nextafter(x, np.float32(np.inf))
    bad["exp_avg"][17] = x
    with pytest.raises(AssertionError, match="first at 17"):
        compare_state(bad, ora, "twenty ulp")
    bad = _copy(ora)
    bad["param_lp"][5] += 2
    with pytest.raises(AssertionError, match="param_lp"):
        compare_state(bad, ora, "two ulp16")


def test_third_arm_only_where_the_terms_cancel_and_it_is_counted():
    n = 1024
    hp = oracle.hparams(max_grad_norm=0.0)
    old = dict(master=np.full(n, 0.5, np.float32), exp_avg=np.full(n, 1.0, np.float32), exp_avg_sq=np.ones(n, np.float32))
    # beta1 * m_old = 0.9 and (1 - beta1) * g = -0.9 * (1 - 2^-20): the result is 2^-20 of the terms
    g16 = oracle.encode(np.full(n, -9.0, np.float32), oracle.BF16)
    ora = dict(grad=g16, param_lp=np.zeros(n, np.uint16), master=old["master"].copy(),
               exp_avg=np.full(n, 1e-6, np.float32), exp_avg_sq=np.ones(n, np.float32))
    gpu = _copy(ora)
    gpu["exp_avg"][3] = ora["exp_avg"][3] + np.float32(1e-7)          # 10 % of the tiny result, 0.9 ulp32 of the terms
    ctx = StepCtx(oracle.BF16, hp, 1, 1.0)
    st = compare_state(gpu, ora, "cancelled", old, ctx)
    assert st["exp_avg_beyond"] == 1 and st["exp_avg_max_ulp_T"] < 2.0
    with pytest.raises(AssertionError):                                # without the pre-step state: first two arms only
        compare_state(gpu, ora, "cancelled, no context")
    gpu["exp_avg"][3] = ora["exp_avg"][3] + np.float32(3e-7)          # 2.5 ulp32 of the terms: outside
    with pytest.raises(AssertionError, match="first at 3"):
        compare_state(gpu, ora, "cancelled too far", old, ctx)
    # the count of third-arm elements is held to what the difference between the two norms explains
    many = _copy(ora)
    many["exp_avg"][:200] += np.float32(1e-7)
    with pytest.raises(AssertionError, match="third arm used too often"):
        compare_state(many, ora, "too many", old, StepCtx(oracle.BF16, hp, 1, 1.0, sumsq_gpu=1.0))


@pytest.mark.parametrize("dtype", [oracle.BF16, oracle.FP16])
def test_carried_bound_holds_for_a_second_oracle_with_another_summation_order(dtype):
    """Two oracle trajectories whose norms differ by 1e-10 relative each step, never
    re-synchronised, 60 steps: every element stays inside the carried bound, and a good part of
    the bound is used (it is not vacuous)."""
    rng = np.random.default_rng(5 + dtype)
    n = 1 << 16
    scale = 1.0 if dtype == oracle.BF16 else 1024.0
    hp = oracle.hparams(max_grad_norm=0.1, loss_scale=scale)
    a = random_state(n, dtype, rng, scale=scale)
    b = _copy(a)
    bound = FreeRun(n)
    worst, differed = 0.0, 0
    for step in range(1, 61):
        a["grad"] = random_state(n, dtype, rng, scale=scale)["grad"]
        b["grad"] = a["grad"]
        norm, _ = oracle.grad_prep([a["grad"]], dtype, scale)
        norm_b = norm * (1.0 + (1e-10 if step % 2 else -1e-10))
        old = _copy(a)
        _step(a, dtype, step, hp, norm)
        _step(b, dtype, step, hp, norm_b)
        st = bound.step(b, a, old, StepCtx(dtype, hp, step, norm, sumsq_gpu=norm_b * norm_b), "step %d" % step)
        worst = max(worst, max(st[s + "_max_E_frac"] for s in F32))
        differed += sum(st[s + "_mismatch"] for s in F32)
    assert 0.05 < worst <= 1.0, worst
    assert differed > 100, "the two trajectories should have separated in places"


@pytest.mark.parametrize("mistake", ["beta1", "four_ulp_in_m", "lr", "eps_inside_root", "stale_v"])
def test_carried_bound_catches_planted_mistakes(mistake):
    rng = np.random.default_rng(77)
    n = 1 << 15
    hp = oracle.hparams(max_grad_norm=0.1)
    hp_bad = oracle.hparams(max_grad_norm=0.1)
    a = random_state(n, oracle.BF16, rng)
    b = _copy(a)
    bound = FreeRun(n)
    with pytest.raises(AssertionError, match="free-running"):
        for step in range(1, 13):
            a["grad"] = random_state(n, oracle.BF16, rng)["grad"]
            b["grad"] = a["grad"]
            norm, _ = oracle.grad_prep([a["grad"]], oracle.BF16, 1.0)
            old = _copy(a)
            _step(a, oracle.BF16, step, hp, norm)
            if mistake == "beta1" and step == 6:
                hp_bad.beta1 = np.nextafter(np.float32(0.9), np.float32(1.0))          # one ulp32 off in beta1, once
            if mistake == "lr" and step == 6:
                hp_bad.lr = 1.001e-4
            keep_v = b["exp_avg_sq"].copy()
            _step(b, oracle.BF16, step, hp_bad, norm)
            hp_bad.beta1, hp_bad.lr = hp.beta1, hp.lr
            if mistake == "four_ulp_in_m" and step == 6:
                for _ in range(4):
                    b["exp_avg"][100] = np.nextafter(b["exp_avg"][100], np.float32(np.inf))
            if mistake == "eps_inside_root" and step == 6:                              # sqrt(v^ + eps) for one element
                i = int(np.argmin(a["exp_avg_sq"] + (a["exp_avg_sq"] == 0)))
                bc1, bc2 = 1 - 0.9 ** step, 1 - 0.999 ** step
                m, v, p = float(b["exp_avg"][i]), float(b["exp_avg_sq"][i]), float(old["master"][i])
                b["master"][i] = np.float32(p - 1e-4 * ((m / bc1) / np.sqrt(v / bc2 + 1e-8) + 0.01 * p))
            if mistake == "stale_v" and step == 6:
                b["exp_avg_sq"][7] = keep_v[7]
            bound.step(b, a, old, StepCtx(oracle.BF16, hp, step, norm, sumsq_gpu=norm * norm), "step %d" % step)
