"""Cost model (Eq. 1-5) and strategy search (Eq. 6): the oracle against hand-evaluated points and
properties, then the library against the oracle.  Host only."""
import ctypes

import numpy as np
import pytest

from oracle import strategy_oracle as so
from paper_2503_01890_amd import binding as B

HAND = dict(L=2, Ma=10, Ma1=2, Mp=100, Mgc=50, Mcc=7, Mgpu=1e9, Mcpu=1e9, tfp=1, tbp=2, th2d=4, td2h=0.5, tcpu=3,
            tgpu=0.25)


def to_c(m):
    return B.autohete_cost_model(m["L"], m["Ma"], m["Ma1"], m["Mp"], m["Mgc"], m["Mcc"], m["Mgpu"], m["Mcpu"], m["tfp"],
                                 m["tbp"], m["th2d"], m["td2h"], m["tcpu"], m["tgpu"])


def test_oracle_points_evaluated_by_hand():
    # (c, p, o) = (1, 1, 2):  GPU = 2*2*1 + 2*10*2 + 2*100*2 + 12*100*0 + 50 = 494;  CPU = 14*100*2 + 7 = 2807
    #   T_fwd = max(1*2, 4*2 + 1) = 9;  v = 1: t_sync = 1*max(4-1-2, 0) + 0 = 1
    #   T_bwd = max(2*2 + 1*1 + 0.25*0 + 1, 2 + 0.5 + 3*2) = max(6, 8.5) = 8.5
    s = so.evaluate(HAND, 1, 1, 2)
    assert (s["gpu"], s["cpu"], s["t_fwd"], s["t_sync"], s["t_bwd"], s["feasible"]) == (494, 2807, 9, 1, 8.5, True)
    # (0, 0, 0):  GPU = 0 + 2*10*3 + 2*100*3 + 12*100*2 + 50 = 3110;  CPU = 7
    #   T_fwd = max(2, 0 + 1) = 2;  T_bwd = max(2*2 + 0 + 0.25*2 + 0, 2 + 0.5 + 0) = 4.5
    s = so.evaluate(HAND, 0, 0, 0)
    assert (s["gpu"], s["cpu"], s["t_fwd"], s["t_sync"], s["t_bwd"]) == (3110, 7, 2, 0, 4.5)
    # (0, 2, 2): no checkpointing, both blocks' parameters offloaded: v = 0, t_sync = 2*max(4-2, 0) = 4
    #   GPU = 0 + 60 + 2*100*1 + 0 + 50 = 310;  T_bwd = max(4 + 0 + 0 + 4, 2 + 0.5 + 6) = 8.5
    s = so.evaluate(HAND, 0, 2, 2)
    assert (s["gpu"], s["t_sync"], s["t_bwd"]) == (310, 4, 8.5)
    # (2, 0, 0): both blocks recomputed, everything on the GPU: the GPU arm of Eq. 5 decides
    #   GPU = 2*2*2 + 2*10*1 + 2*100*3 + 12*100*2 + 50 = 3078
    #   T_bwd = max(2*2 + 1*2 + 0.25*2 + 0, 2 + 0.5 + 0) = max(6.5, 2.5) = 6.5
    s = so.evaluate(HAND, 2, 0, 0)
    assert (s["gpu"], s["t_sync"], s["t_bwd"]) == (3078, 0, 6.5)
    # p > o is not a strategy (footnote to the peak-memory model)
    assert not so.evaluate(HAND, 0, 2, 1)["feasible"]
    # the example of the paper's scheduling figure: L = 5, c = 3, p = 1, o = 5 -> one block has both
    fig = dict(HAND, L=5)
    s = so.evaluate(fig, 3, 1, 5)
    assert s["feasible"] and s["t_sync"] == 1 * max(4 - 1 - 2, 0) + 0 and s["t_fwd"] == max(5, 4 * 5 + 1)
    assert s["gpu"] == 2 * 2 * 3 + 2 * 10 * 3 + 2 * 100 * 5 + 0 + 50


def test_oracle_search_properties():
    # memory to spare: nothing is offloaded or recomputed, T = L (t_fp + t_bp + t_optim_gpu)
    best = so.search(HAND)
    assert (best["c"], best["p"], best["o"]) == (0, 0, 0) and best["t_fwd"] + best["t_bwd"] == 2 * (1 + 2 + 0.25)
    # the fp32 states of not even one block fit: every block's optimizer goes to the host
    tight = dict(HAND, Mgpu=700)
    best = so.search(tight)
    assert best["o"] == 2 and best["gpu"] <= 700
    assert so.search(dict(HAND, Mgpu=100)) is None                      # nothing fits
    assert so.search(dict(HAND, Mcpu=6)) is None                        # host constant alone too big
    # more GPU memory never makes the optimum slower; a free GPU optimizer never prefers the host
    rng = np.random.default_rng(0)
    for _ in range(40):
        m = random_model(rng)
        times = []
        for cap in sorted(rng.uniform(0.2, 1.2, 4) * so.evaluate(m, 0, 0, 0)["gpu"]):
            b = so.search(dict(m, Mgpu=cap))
            times.append(np.inf if b is None else b["t_fwd"] + b["t_bwd"])
        assert all(a >= b for a, b in zip(times, times[1:]))
        roomy = so.search(dict(m, Mgpu=1e30, Mcpu=1e30, tgpu=0.0))
        assert roomy["o"] == 0 and roomy["c"] == 0


def random_model(rng):
    L = int(rng.integers(1, 9))
    Ma = float(rng.uniform(1, 100))
    return dict(L=L, Ma=Ma, Ma1=float(rng.uniform(0, Ma)), Mp=float(rng.uniform(1, 100)), Mgc=float(rng.uniform(0, 50)),
                Mcc=float(rng.uniform(0, 50)), Mgpu=float(rng.uniform(500, 20000)), Mcpu=float(rng.uniform(500, 20000)),
                tfp=float(rng.uniform(0.1, 2)), tbp=float(rng.uniform(0.1, 4)), th2d=float(rng.uniform(0.1, 6)),
                td2h=float(rng.uniform(0.1, 6)), tcpu=float(rng.uniform(0.1, 8)), tgpu=float(rng.uniform(0.01, 1)))


def test_library_matches_oracle_pointwise_and_in_search():
    rng = np.random.default_rng(1)
    n_feasible = 0
    for _ in range(300):
        m = random_model(rng)
        cm = to_c(m)
        L = m["L"]
        for _ in range(10):
            c, p, o = (int(x) for x in rng.integers(0, L + 1, 3))
            s, t = B.autohete_strategy_eval(cm, c, p, o), so.evaluate(m, c, p, o)
            assert (s.n_ckpt, s.n_param_offload, s.n_optim_offload, bool(s.feasible)) == (c, p, o, t["feasible"])
            for got, ref in ((s.gpu_bytes, t["gpu"]), (s.cpu_bytes, t["cpu"]), (s.t_fwd, t["t_fwd"]),
                             (s.t_sync, t["t_sync"]), (s.t_bwd, t["t_bwd"])):
                assert got == pytest.approx(ref, rel=1e-13, abs=1e-13)
        ref = so.search(m)
        if ref is None:
            with pytest.raises(B.AutoheteError) as e:
                B.autohete_strategy_search(cm)
            assert e.value.status == B.AH_EINFEASIBLE
        else:
            n_feasible += 1
            got = B.autohete_strategy_search(cm)
            assert got.t_fwd + got.t_bwd == pytest.approx(ref["t_fwd"] + ref["t_bwd"], rel=1e-13)
            assert (got.n_ckpt, got.n_param_offload, got.n_optim_offload) == (ref["c"], ref["p"], ref["o"])
    assert 100 < n_feasible < 300          # the random models exercise both outcomes


def test_library_hand_points_and_errors():
    s = B.autohete_strategy_eval(to_c(HAND), 1, 1, 2)
    assert (s.gpu_bytes, s.cpu_bytes, s.t_fwd, s.t_sync, s.t_bwd, s.feasible) == (494, 2807, 9, 1, 8.5, 1)
    lib = B.raw()
    out = B.autohete_strategy()
    cm = to_c(HAND)
    assert lib.autohete_strategy_eval(ctypes.byref(cm), 3, 0, 0, ctypes.byref(out)) == B.AH_EINVAL   # c > L
    assert lib.autohete_strategy_eval(None, 0, 0, 0, ctypes.byref(out)) == B.AH_EINVAL
    assert lib.autohete_strategy_search(ctypes.byref(cm), None) == B.AH_EINVAL
    for bad in (dict(HAND, L=0), dict(HAND, tfp=-1.0), dict(HAND, Mp=float("nan")), dict(HAND, Ma1=11)):
        bm = to_c(bad)
        assert lib.autohete_strategy_search(ctypes.byref(bm), ctypes.byref(out)) == B.AH_EINVAL


def test_measured_gpu_optimizer_cost_moves_the_plan():
    """With the per-block GPU update time this library measures on MI355X (about 0.9 ms for a 201 M
    parameter block) and a host update ~500x slower per block (0.42 G parameters/s on 16 cores), the
    model offloads only the blocks whose host update hides under the backward pass when memory is
    plentiful, and is pushed to offload more -- at a cost -- when the GPU is small."""
    Mp = 12 * 4096 ** 2 + 13 * 4096
    base = dict(L=32, Ma=8 * 1024 * 4096 * 34.0, Ma1=8 * 1024 * 4096.0, Mp=float(Mp), Mgc=2e9, Mcc=2e9, Mcpu=4e11,
                tfp=0.010, tbp=0.020, th2d=2 * Mp / 50e9, td2h=2 * Mp / 50e9, tcpu=Mp / 0.42e9, tgpu=28 * Mp / 6.5e12)
    plenty = B.autohete_strategy_search(to_c(dict(base, Mgpu=288e9)))
    host_path = base["tbp"] + base["td2h"] + base["tcpu"] * plenty.n_optim_offload
    assert plenty.n_optim_offload <= 2 and host_path <= plenty.t_bwd + 1e-12      # the host work is hidden
    small = B.autohete_strategy_search(to_c(dict(base, Mgpu=80e9)))
    assert plenty.n_optim_offload < small.n_optim_offload <= 32 and small.gpu_bytes <= 80e9
    assert small.t_fwd + small.t_bwd > plenty.t_fwd + plenty.t_bwd
    ref = so.search(dict(base, Mgpu=80e9))
    assert (small.n_ckpt, small.n_param_offload, small.n_optim_offload) == (ref["c"], ref["p"], ref["o"])


def test_ties_go_to_the_least_offloading_by_hand():
    """Eq. 6 does not say which of several equally fast strategies to take; the reading (least
    optimizer offloading, then least parameter offloading, then least checkpointing) is pinned on a
    model whose ties are evaluated by hand.  L = 2, t_fp = 1, t_bp = 2, a free GPU optimizer
    (t_optim_gpu = 0), a host optimizer and copies that hide under the backward pass:
      T_fwd = max(2, 0.5 o + 1) = 2 for every o;  t_sync = 0 (t_h2d < t_bp);
      T_bwd = max(4 + c, 2 + 0.1 + 0.5 o) = 4 + c  ->  T = 6 for every (0, p, o): six-fold tie."""
    m = dict(HAND, tgpu=0.0, th2d=0.5, td2h=0.1, tcpu=0.5)
    for o in range(3):
        for p in range(o + 1):
            s = so.evaluate(m, 0, p, o)
            assert s["feasible"] and s["t_fwd"] + s["t_bwd"] == 6.0
    best = so.search(m)
    assert (best["c"], best["p"], best["o"]) == (0, 0, 0)
    got = B.autohete_strategy_search(to_c(m))
    assert (got.n_ckpt, got.n_param_offload, got.n_optim_offload) == (0, 0, 0)
    # memory that only fits with one block's optimizer states on the host AND one block's parameters
    # offloaded: Eq. 1 at (0, 1, 1) = 2*10*3 + 2*100*2 + 12*100*1 + 50 = 1710, at (0, 0, 1) = 1910
    tight = dict(m, Mgpu=1800)
    assert so.evaluate(tight, 0, 1, 1)["gpu"] == 1710 and so.evaluate(tight, 0, 0, 1)["gpu"] == 1910
    # feasible and tied at T = 6: (0,1,1), (0,1,2), (0,2,2), (0,0,2) [1310 bytes] -> smallest o wins, then p
    best = so.search(tight)
    assert (best["c"], best["p"], best["o"]) == (0, 1, 1)
    got = B.autohete_strategy_search(to_c(tight))
    assert (got.n_ckpt, got.n_param_offload, got.n_optim_offload) == (0, 1, 1)


STRATEGY_MUTATIONS = {
    "v_is_max_not_min": ("v = min(c, p)", "v = max(c, p)"),
    "no_plus_one_activation": ("2 * m[\"Ma\"] * (L - c + 1)", "2 * m[\"Ma\"] * (L - c)"),
    "no_plus_one_parameter": ("2 * m[\"Mp\"] * (L - p + 1)", "2 * m[\"Mp\"] * (L - p)"),
    "states_12_vs_14": ("12 * m[\"Mp\"] * (L - o)", "14 * m[\"Mp\"] * (L - o)"),
    "host_14_vs_12": ("14 * m[\"Mp\"] * o", "12 * m[\"Mp\"] * o"),
    "checkpoint_keeps_all": ("2 * m[\"Ma1\"] * c ", "2 * m[\"Ma\"] * c "),
    "fwd_forgets_last_compute": ("m[\"th2d\"] * o + m[\"tfp\"])", "m[\"th2d\"] * o)"),
    "sync_ignores_recompute": ("max(m[\"th2d\"] - m[\"tfp\"] - m[\"tbp\"], 0)", "max(m[\"th2d\"] - m[\"tbp\"], 0)"),
    "bwd_no_recompute_time": ("+ m[\"tfp\"] * c + m[\"tgpu\"]", "+ m[\"tgpu\"]"),
    "gpu_optim_counts_offloaded": ("m[\"tgpu\"] * (L - o)", "m[\"tgpu\"] * o"),
    "cpu_path_without_d2h": ("m[\"tbp\"] + m[\"td2h\"] + m[\"tcpu\"] * o", "m[\"tbp\"] + m[\"tcpu\"] * o"),
    "bwd_sum_not_max": ("t_bwd = max(on_gpu, on_cpu)", "t_bwd = on_gpu + on_cpu"),
    "p_le_o_dropped": ("and cpu <= m[\"Mcpu\"] and p <= o", "and cpu <= m[\"Mcpu\"]"),
    "cpu_limit_dropped": ("gpu <= m[\"Mgpu\"] and cpu <= m[\"Mcpu\"]", "gpu <= m[\"Mgpu\"]"),
    "gpu_constant_dropped": ("    gpu += m[\"Mgc\"] ", "    gpu += 0 "),
    "tie_prefers_last": ("< best[\"t_fwd\"] + best[\"t_bwd\"]", "<= best[\"t_fwd\"] + best[\"t_bwd\"]"),
    "search_skips_full_offload": ("for o in range(L + 1):", "for o in range(L):"),
}


@pytest.mark.parametrize("name", sorted(STRATEGY_MUTATIONS))
def test_planted_mistake_in_the_strategy_oracle_is_caught(name, monkeypatch):
    """Each case plants one plausible mistake in a copy of the strategy oracle's source and requires
    that one of the hand-evaluated pins above fails against it."""
    import types
    old, new = STRATEGY_MUTATIONS[name]
    text = open(so.__file__).read()
    assert text.count(old) == 1, name
    mutant = types.ModuleType("strategy_mutant")
    exec(compile(text.replace(old, new), "strategy_mutant.py", "exec"), mutant.__dict__)
    monkeypatch.setattr(so, "evaluate", mutant.evaluate)
    monkeypatch.setattr(so, "search", mutant.search)
    caught = False
    for pin in (test_oracle_points_evaluated_by_hand, test_oracle_search_properties,
                test_ties_go_to_the_least_offloading_by_hand):
        try:
            pin()
        except (AssertionError, TypeError, KeyError):
            caught = True
            break
    assert caught, "mutation %r survived every pin" % name
