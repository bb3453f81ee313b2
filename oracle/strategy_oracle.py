"""TEST INFRASTRUCTURE: the paper's cost model and strategy search written out naively.

Eq. 1-6 of section 3.2.2 ("Cost Model and Strategy Search") in plain Python, one line per term, and
an exhaustive triple loop for Eq. 6.  Shares nothing with the library's implementation.
A model is a dict with keys L, Ma, Ma1 (M_a'), Mp, Mgc, Mcc, Mgpu, Mcpu, tfp, tbp, th2d, td2h,
tcpu (t_optim^cpu), tgpu (t_optim^gpu).

READINGS (the paper leaves them implicit): v-hat, the number of blocks with both checkpointing and
parameter offloading, is min(c, p) because both are applied to the earliest blocks (Insight 1);
the footnote's p <= o is a constraint of the search; ties in Eq. 6 go to the smallest o, then p,
then c.

Pins (tests/test_strategy.py): points evaluated by hand, the unlimited-memory optimum, the
optimizer-states-do-not-fit case, monotonicity in the GPU capacity."""


def evaluate(m, c, p, o):
    L = m["L"]
    gpu = 0.0
    gpu += 2 * m["Ma1"] * c                 # checkpointed blocks keep their input activations
    gpu += 2 * m["Ma"] * (L - c + 1)        # the others (and the one being recomputed) keep everything
    gpu += 2 * m["Mp"] * (L - p + 1)        # 16-bit parameters not offloaded (+ the one being prefetched)
    gpu += 12 * m["Mp"] * (L - o)           # fp32 momentum, variance, parameter copy kept on the GPU
    gpu += m["Mgc"]                         # Eq. 1
    cpu = 14 * m["Mp"] * o + m["Mcc"]       # Eq. 2
    t_fwd = max(m["tfp"] * L, m["th2d"] * o + m["tfp"])                                       # Eq. 3
    v = min(c, p)
    t_sync = v * max(m["th2d"] - m["tfp"] - m["tbp"], 0) + (p - v) * max(m["th2d"] - m["tbp"], 0)   # Eq. 4
    on_gpu = m["tbp"] * L + m["tfp"] * c + m["tgpu"] * (L - o) + t_sync
    on_cpu = m["tbp"] + m["td2h"] + m["tcpu"] * o
    t_bwd = max(on_gpu, on_cpu)                                                               # Eq. 5
    feasible = gpu <= m["Mgpu"] and cpu <= m["Mcpu"] and p <= o
    return dict(c=c, p=p, o=o, gpu=gpu, cpu=cpu, t_fwd=t_fwd, t_sync=t_sync, t_bwd=t_bwd, feasible=feasible)


def search(m):
    """Eq. 6 by exhaustion.  Returns the best feasible point or None."""
    best = None
    L = m["L"]
    for o in range(L + 1):
        for p in range(L + 1):
            for c in range(L + 1):
                s = evaluate(m, c, p, o)
                if not s["feasible"]:
                    continue
                if best is None or s["t_fwd"] + s["t_bwd"] < best["t_fwd"] + best["t_bwd"]:
                    best = s
    return best
