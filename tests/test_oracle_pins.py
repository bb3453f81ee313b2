"""Pins of the CPU oracle to things other than itself: closed forms, invariants,
hand-worked examples, brute force, and library routines it does not call
(numpy's float16, torch's bfloat16 conversion, torch.optim.AdamW in fp64).
All CPU; none of this touches the GPU library."""
import numpy as np
import pytest
import torch

import oracle
from _golden import load_hand_worked

BF16, FP16 = oracle.BF16, oracle.FP16
RNG = np.random.default_rng(1234)


def ulp32(x):
    x = np.abs(np.asarray(x, np.float32))
    return np.spacing(np.maximum(x, np.float32(1.1754944e-38))).astype(np.float64)


def lowp(values, dtype):
    """float values that are exactly representable -> 16-bit patterns, via torch/numpy
    (not via the oracle) so inputs do not depend on the code under test."""
    if dtype == FP16:
        return np.asarray(values, np.float32).astype(np.float16).view(np.uint16).copy()
    t = torch.tensor(np.asarray(values, np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def state(n, dtype=BF16, zero_moments=False, rng=RNG):
    p16 = lowp(rng.normal(0, 0.02, n), dtype)
    master = (torch.tensor(p16.view(np.int16)).view(torch.bfloat16 if dtype == BF16 else torch.float16)
              .float().numpy().copy())
    m = np.zeros(n, np.float32) if zero_moments else rng.normal(0, 1e-4, n).astype(np.float32)
    v = np.zeros(n, np.float32) if zero_moments else np.abs(rng.normal(0, 1e-6, n)).astype(np.float32)
    return dict(param_lp=p16, master=master, exp_avg=m, exp_avg_sq=v)


def to_f64(bits, dtype):
    t = torch.tensor(bits.view(np.int16)).view(torch.bfloat16 if dtype == BF16 else torch.float16)
    return t.double().numpy()


# --------------------------------------------------------------------------- 16-bit formats

def test_decode_all_patterns_match_numpy_and_torch():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    for dtype in (BF16, FP16):
        got = oracle.decode(bits, dtype)
        ref = to_f64(bits, dtype).astype(np.float32)
        assert np.array_equal(got.view(np.uint32)[~np.isnan(ref)], ref.view(np.uint32)[~np.isnan(ref)])
        assert np.array_equal(np.isnan(got), np.isnan(ref))


def test_encode_roundtrip_all_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    for dtype in (BF16, FP16):
        x = oracle.decode(bits, dtype)
        back = oracle.encode(x, dtype)
        ok = ~np.isnan(x)
        assert np.array_equal(back[ok], bits[ok])
        assert np.all(np.isnan(oracle.decode(back[~ok], dtype)))


def test_bf16_rne_against_torch_on_ties_and_neighbours():
    hi = np.arange(65536, dtype=np.uint32) << 16
    for tail in (0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF):
        f = (hi | tail).astype(np.uint32).view(np.float32)
        ok = np.isfinite(f)
        ref = torch.tensor(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        got = oracle.encode(f, BF16)
        assert np.array_equal(got[ok], ref[ok]), hex(tail)
    f = RNG.integers(0, 2**32, 2_000_000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    ok = np.isfinite(f)
    ref = torch.tensor(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.encode(f, BF16)[ok], ref[ok])


def test_fp16_rne_against_numpy_incl_subnormals_and_overflow():
    # every fp16 value widened to fp32, nudged by sub-quantum tails incl. exact ties
    base = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16).astype(np.float32)
    base = base[np.isfinite(base)]
    b = base.view(np.uint32)
    for tail in (0x0000, 0x0001, 0x0FFF, 0x1000, 0x1001, 0x1FFF):
        f = (b | tail).view(np.float32)
        with np.errstate(over="ignore"):
            ref = f.astype(np.float16).view(np.uint16)
        assert np.array_equal(oracle.encode(f, FP16), ref), hex(tail)
    # subnormal range: k/2 * 2^-24, i.e. every tie and every grid point, plus neighbours
    k = np.arange(0, 4100, dtype=np.float64)
    for d in (0.0, 1e-12, -1e-12):
        f = (k * 0.5 * 2.0**-24 + d).astype(np.float32)
        ref = f.astype(np.float16).view(np.uint16)
        assert np.array_equal(oracle.encode(f, FP16), ref)
    # random floats over the whole fp16 range and beyond (overflow -> inf at >= 65520)
    e = RNG.uniform(-30, 18, 2_000_000)
    f = (np.exp2(e) * RNG.choice([-1.0, 1.0], e.size)).astype(np.float32)
    with np.errstate(over="ignore"):
        ref = f.astype(np.float16).view(np.uint16)
    assert np.array_equal(oracle.encode(f, FP16), ref)
    edge = np.array([65504.0, 65519.996, 65520.0, 65536.0, -65520.0, np.inf, -np.inf], np.float32)
    assert list(oracle.encode(edge, FP16)) == [0x7BFF, 0x7BFF, 0x7C00, 0x7C00, 0xFC00, 0x7C00, 0xFC00]


# --------------------------------------------------------------------------- chunk layout

def test_chunk_layout_against_cumsum_and_counts():
    sizes = RNG.integers(1, 5000, 300).astype(np.uint64)
    for C in (1, 7, 4096, 2**20):
        off, nc, tot, pad = oracle.chunk_layout(sizes, C)
        assert np.array_equal(off, np.concatenate([[0], np.cumsum(sizes)[:-1]]).astype(np.uint64))
        assert tot == int(sizes.sum())
        assert nc == -(-tot // C) and pad == nc * C - tot and 0 <= pad < C
    off, nc, tot, pad = oracle.chunk_layout(np.array([8, 8], np.uint64), 8)
    assert (list(off), nc, tot, pad) == ([0, 8], 2, 16, 0)
    off, nc, tot, pad = oracle.chunk_layout(np.array([], np.uint64), 8)
    assert (nc, tot, pad) == (0, 0, 0)
    with pytest.raises(ValueError):
        oracle.chunk_layout(np.array([1], np.uint64), 0)


def test_chunk_layout_gpt_byte_accounting():
    # section 2.1: 16 bytes per parameter = 2 (p16) + 2 (g16) + 12 (fp32 states)
    d, L, V, S = 768, 12, 50257, 1024
    per_layer = [d, d, 3 * d * d, 3 * d, d * d, d, d, d, 4 * d * d, 4 * d, 4 * d * d, d]
    sizes = np.array([V * d, S * d] + per_layer * L, np.uint64)
    off, nc, tot, pad = oracle.chunk_layout(sizes, 2**22)
    assert tot == 124_438_272 and nc == 30 and pad == 1_390_848
    assert nc * 2**22 * (2 + 2 + 4 + 4 + 4) == 16 * (tot + pad)


# --------------------------------------------------------------------------- norm / flag

def test_norm_closed_forms():
    for dtype in (BF16, FP16):
        for n, c in ((4**5, 0.25), (4**8, 2.0), (4**3, 2.0**-6)):
            g = lowp(np.full(n, c), dtype)
            norm, flag = oracle.grad_prep([g], dtype, 1.0)
            assert flag == 0 and norm == c * np.sqrt(n)      # exact: dyadic c, n a power of 4
        g = lowp(np.zeros(1000), dtype)
        g[417] = lowp([-3.0], dtype)[0]
        assert oracle.grad_prep([g], dtype, 1.0) == (3.0, 0)
        # loss scale divides the norm; extra_sumsq adds under the root: 3-4-5
        assert oracle.grad_prep([g], dtype, 2.0) == (1.5, 0)
        assert oracle.grad_prep([g], dtype, 1.0, extra_sumsq=16.0) == (5.0, 0)
    # split over several chunks = one chunk
    g = lowp(RNG.normal(0, 1e-3, 10_000), BF16)
    whole = oracle.grad_prep([g], BF16, 1.0)
    parts = oracle.grad_prep([g[:17].copy(), g[17:4096].copy(), g[4096:].copy()], BF16, 1.0)
    assert whole == parts
    # against an independent fp64 numpy sum
    ref = np.sqrt(np.sum(to_f64(g, BF16) ** 2))
    assert abs(whole[0] - ref) <= 1e-12 * ref


@pytest.mark.parametrize("dtype", [BF16, FP16])
@pytest.mark.parametrize("bad", [np.inf, -np.inf, np.nan])
@pytest.mark.parametrize("pos", [0, 511, 999])
def test_nonfinite_sets_flag_and_skips_bit_exactly(dtype, bad, pos):
    n = 1000
    st = state(n, dtype)
    g = lowp(RNG.normal(0, 1e-3, n), dtype)
    g[pos] = {np.inf: 0x7F80, -np.inf: 0xFF80}.get(bad, 0x7FC0) if dtype == BF16 else \
        {np.inf: 0x7C00, -np.inf: 0xFC00}.get(bad, 0x7E00)
    before = {k: a.copy() for k, a in st.items()}
    norm, flag = oracle.full_step([dict(grad=g, **st)], dtype, 1, oracle.hparams())
    assert flag == 1 and np.isnan(norm)
    for k in st:
        assert st[k].tobytes() == before[k].tobytes()


def test_nonfinite_extra_sumsq_sets_flag():
    g = lowp(np.ones(8), BF16)
    for bad in (np.inf, np.nan):
        assert oracle.grad_prep([g], BF16, 1.0, extra_sumsq=bad)[1] == 1


# --------------------------------------------------------------------------- update rule

def test_step1_is_lr_sign_g():
    """m = v = 0, t = 1, wd = 0, no clip, eps -> 0: p1 = p0 - lr*sign(g) (g != 0)."""
    n = 4096
    for dtype in (BF16, FP16):
        st = state(n, dtype, zero_moments=True)
        gv = RNG.normal(0, 1e-3, n)
        gv[gv == 0] = 1e-3
        g = lowp(gv, dtype)
        gd = to_f64(g, dtype)
        assert np.all(gd != 0)
        p0 = st["master"].astype(np.float64)
        hp = oracle.hparams(lr=1e-3, eps=1e-30, weight_decay=0.0, max_grad_norm=0.0)
        oracle.full_step([dict(grad=g, **st)], dtype, 1, hp)
        lr = float(np.float32(1e-3))
        assert np.array_equal(st["master"], (p0 - lr * np.sign(gd)).astype(np.float32))
        b1, b2 = float(np.float32(0.9)), float(np.float32(0.999))
        assert np.array_equal(st["exp_avg"], ((1 - b1) * gd).astype(np.float32))
        assert np.array_equal(st["exp_avg_sq"], ((1 - b2) * (gd * gd)).astype(np.float32))


def test_zero_gradient_is_pure_decay():
    n = 4096
    st = state(n, BF16, zero_moments=True)
    p0 = st["master"].astype(np.float64)
    hp = oracle.hparams(lr=0.125, weight_decay=0.5, max_grad_norm=1.0)   # lr*wd = 1/16 exactly
    g = np.zeros(n, np.uint16)
    norm, flag = oracle.full_step([dict(grad=g, **st)], BF16, 1, hp)
    assert (norm, flag) == (0.0, 0)
    assert np.array_equal(st["master"], (p0 * (1 - 0.0625)).astype(np.float32))  # exact in fp64
    assert not st["exp_avg"].any() and not st["exp_avg_sq"].any()
    ref16 = torch.tensor(st["master"]).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(st["param_lp"], ref16)


def test_constant_gradient_closed_form_every_t():
    """From m = v = 0 with a constant gradient: m_t = (1-b1^t) g, v_t = (1-b2^t) g^2, hence the
    bias-corrected ratio is g/(|g|+eps) at EVERY t and p_t = p_0 - t*lr*g/(|g|+eps) (wd = 0)."""
    n, T = 512, 60
    st = state(n, BF16, zero_moments=True)
    g = lowp(RNG.normal(0, 1e-3, n), BF16)
    gd = to_f64(g, BF16)
    p0 = st["master"].astype(np.float64)
    hp = oracle.hparams(lr=1e-4, eps=1e-8, weight_decay=0.0, max_grad_norm=0.0)
    lr, eps = float(np.float32(1e-4)), float(np.float32(1e-8))
    b1, b2 = float(np.float32(0.9)), float(np.float32(0.999))
    u = gd / (np.abs(gd) + eps)
    for t in range(1, T + 1):
        oracle.full_step([dict(grad=g, **st)], BF16, t, hp)
        # state is re-rounded to fp32 each step: allow t half-ulps of drift
        assert np.all(np.abs(st["exp_avg"] - (1 - b1**t) * gd) <= (t + 1) * ulp32(gd))
        assert np.all(np.abs(st["exp_avg_sq"] - (1 - b2**t) * gd * gd) <= (t + 1) * ulp32(gd * gd))
        # per-step |dp| = lr*|u| to ~1e-6 relative (the fp32 moments carry ~1e-7 relative error)
        assert np.all(np.abs(st["master"] - (p0 - t * lr * u)) <= t * (ulp32(p0) + 2e-6 * lr))
    # a wrong exponent in either bias correction is far outside that band:
    assert lr * abs(1 - (1 - b1**2) / (1 - b1**1)) > 1e-3 * lr


def test_hand_worked_examples():
    for name, c in load_hand_worked().items():
        dtype = BF16 if c["dtype"] == "bf16" else FP16
        hp = oracle.hparams(c["lr"], c["beta1"], c["beta2"], c["eps"], c["weight_decay"],
                            c["max_grad_norm"], c["loss_scale"])
        g = lowp(c["grad"], dtype)
        assert np.array_equal(to_f64(g, dtype), c["grad"]), "fixture gradients must be exact in 16 bits"
        st = dict(param_lp=np.zeros(16, np.uint16), master=c["master"].astype(np.float32),
                  exp_avg=c["exp_avg"].astype(np.float32), exp_avg_sq=c["exp_avg_sq"].astype(np.float32))
        for k in range(1, int(c["steps"]) + 1):
            norm, flag = oracle.full_step([dict(grad=g, **st)], dtype, int(c["first_step"]) + k - 1, hp)
            assert flag == 0 and norm * norm == pytest.approx(c["expect_sumsq"], rel=1e-15), name
            for key in ("master", "exp_avg", "exp_avg_sq"):
                exp = c["expect_%s_t%d" % (key, k)].astype(np.float32)
                assert np.array_equal(st[key], exp), (name, key, k)
            exp16 = c["expect_param_lp_t%d" % k]
            assert np.array_equal(to_f64(st["param_lp"], dtype), exp16), (name, "param_lp", k)


def _torch_adamw_one_step(gd, p, m, v, t, lr, b1, b2, eps, wd):
    P = torch.nn.Parameter(torch.tensor(p, dtype=torch.float64))
    opt = torch.optim.AdamW([P], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd, foreach=False)
    opt.state[P] = dict(step=torch.tensor(float(t - 1)), exp_avg=torch.tensor(m, dtype=torch.float64),
                        exp_avg_sq=torch.tensor(v, dtype=torch.float64))
    P.grad = torch.tensor(gd, dtype=torch.float64)
    opt.step()
    s = opt.state[P]
    return P.detach().numpy(), s["exp_avg"].numpy(), s["exp_avg_sq"].numpy()


@pytest.mark.parametrize("dtype", [BF16, FP16])
def test_against_torch_adamw_fp64(dtype):
    """Library cross-check: one fp64 torch.optim.AdamW step from the same fp32-representable
    state must round to the oracle's fp32 state (<= 1 ulp: double rounding only)."""
    n = 20_000
    st = state(n, dtype)
    scale = 1.0 if dtype == BF16 else 1024.0
    hp = oracle.hparams(lr=1e-4, weight_decay=0.01, max_grad_norm=1.0, loss_scale=scale)
    f = lambda x: float(np.float32(x))
    for t in range(1, 6):
        g = lowp(RNG.normal(0, 1e-3, n) * scale, dtype)
        gd = to_f64(g, dtype) / scale
        norm = float(np.sqrt(np.sum(gd * gd)))
        coef = min(1.0, 1.0 / (norm + 1e-6))
        p, m, v = _torch_adamw_one_step(gd * coef, st["master"], st["exp_avg"], st["exp_avg_sq"], t,
                                        f(1e-4), f(0.9), f(0.999), f(1e-8), f(0.01))
        onorm, flag = oracle.full_step([dict(grad=g, **st)], dtype, t, hp)
        assert flag == 0 and abs(onorm - norm) <= 1e-12 * norm
        for key, ref in (("master", p), ("exp_avg", m), ("exp_avg_sq", v)):
            diff = np.abs(st[key].astype(np.float64) - ref)
            assert np.all(diff <= 0.5000001 * ulp32(ref)), key      # correctly rounded fp64 result
        exp16 = oracle.decode(st["param_lp"], dtype)
        ref16 = torch.tensor(st["master"]).to(torch.bfloat16 if dtype == BF16 else torch.float16).float().numpy()
        assert np.array_equal(exp16, ref16)


def test_clip_invariants():
    n = 2048
    g = lowp(RNG.normal(0, 0.1, n), BF16)          # norm ~ 4.5 > 1
    norm, _ = oracle.grad_prep([g], BF16, 1.0)
    coef = oracle.clip_coef(norm, 1.0)
    assert coef < 1 and coef * norm < 1.0 and abs(coef * norm - 1.0) <= 1.01e-6 / norm
    # clamp: below the threshold (minus the 1e-6 guard) the coefficient is exactly 1 and the
    # clipped step is the unclipped step bit for bit
    assert oracle.clip_coef(0.999998, 1.0) == 1.0 and oracle.clip_coef(5.0, 0.0) == 1.0
    assert oracle.clip_coef(5.0, -1.0) == 1.0
    a, b = state(n, BF16), None
    b = {k: v.copy() for k, v in a.items()}
    oracle.full_step([dict(grad=g, **a)], BF16, 3, oracle.hparams(max_grad_norm=100.0))
    oracle.full_step([dict(grad=g, **b)], BF16, 3, oracle.hparams(max_grad_norm=0.0))
    assert all(a[k].tobytes() == b[k].tobytes() for k in a)
    # clipping by coef == an unclipped step with the loss scale raised by 1/coef
    a, b = state(n, BF16), None
    b = {k: v.copy() for k, v in a.items()}
    oracle.full_step([dict(grad=g, **a)], BF16, 2, oracle.hparams(max_grad_norm=1.0))
    oracle.full_step([dict(grad=g, **b)], BF16, 2, oracle.hparams(max_grad_norm=0.0, loss_scale=1.0 / coef))
    # (the fp32 loss scale carries 6e-8 relative error; bound it by the size of the terms, not of
    # the possibly cancelled result)
    gmag = np.abs(to_f64(g, BF16)) * coef
    term = dict(master=np.abs(a["master"]) + 1e-4, exp_avg=np.abs(a["exp_avg"]) + gmag,
                exp_avg_sq=np.abs(a["exp_avg_sq"]))
    for k in ("master", "exp_avg", "exp_avg_sq"):
        assert np.all(np.abs(a[k].astype(np.float64) - b[k]) <= 1.01 * ulp32(a[k]) + 3e-7 * term[k]), k
    # and it actually clipped: moments differ from the unclipped run
    c = state(n, BF16, zero_moments=True)
    d = {k: v.copy() for k, v in c.items()}
    oracle.full_step([dict(grad=g, **c)], BF16, 1, oracle.hparams(max_grad_norm=1.0))
    oracle.full_step([dict(grad=g, **d)], BF16, 1, oracle.hparams(max_grad_norm=0.0))
    nz = d["exp_avg"] != 0
    ratio = c["exp_avg"][nz].astype(np.float64) / d["exp_avg"][nz]
    assert np.allclose(ratio, coef, rtol=1e-6)


def test_loss_scale_invariance_bit_exact():
    """Scaling every gradient and the loss scale by 2^k changes nothing (power of two: exact)."""
    n = 4096
    gv = RNG.normal(0, 1e-3, n)
    ref = None
    for k in (0, 4, 10):
        st = state(n, FP16, rng=np.random.default_rng(7))
        g = lowp(np.asarray(gv, np.float32).astype(np.float16).astype(np.float64) * 2.0**k, FP16)
        norm, flag = oracle.full_step([dict(grad=g, **st)], FP16, 2, oracle.hparams(loss_scale=2.0**k))
        blob = (norm, flag) + tuple(st[x].tobytes() for x in sorted(st))
        assert np.array_equal(to_f64(g, FP16), to_f64(lowp(gv, FP16), FP16) * 2.0**k)   # exact scaling
        if ref is None:
            ref = blob
        assert blob == ref


def test_partition_invariance():
    """One optimizer per block (footnote to Eq. 5): any grouping of chunks gives the same state."""
    n = 6000
    g = lowp(RNG.normal(0, 1e-3, n), BF16)
    base = state(n, BF16)
    hp = oracle.hparams()
    norm, flag = oracle.grad_prep([g], BF16, 1.0)
    whole = {k: v.copy() for k, v in base.items()}
    oracle.adamw_chunk(g, whole["param_lp"], whole["master"], whole["exp_avg"], whole["exp_avg_sq"],
                       BF16, 4, hp, norm, flag)
    cuts = [0, 1, 8, 9, 2047, 2048, 4099, n]
    parts = {k: v.copy() for k, v in base.items()}
    for a, b in reversed(list(zip(cuts[:-1], cuts[1:]))):     # any order
        sl = {k: parts[k][a:b].copy() for k in parts}
        oracle.adamw_chunk(g[a:b].copy(), sl["param_lp"], sl["master"], sl["exp_avg"], sl["exp_avg_sq"],
                           BF16, 4, hp, norm, flag)
        for k in parts:
            parts[k][a:b] = sl[k]
    assert all(whole[k].tobytes() == parts[k].tobytes() for k in whole)


def test_padding_stays_zero():
    n = 256
    z = dict(grad=np.zeros(n, np.uint16), param_lp=np.zeros(n, np.uint16), master=np.zeros(n, np.float32),
             exp_avg=np.zeros(n, np.float32), exp_avg_sq=np.zeros(n, np.float32))
    live = lowp(RNG.normal(0, 1e-3, n), BF16)
    for t in range(1, 4):
        oracle.full_step([dict(grad=live, **state(n, BF16)), z], BF16, t, oracle.hparams())
        for k in z:
            assert not z[k].view(np.uint8).any(), k          # +0 bit pattern, not -0


def test_split_path_equals_fused_and_cast_is_library_rne():
    """Update without 16-bit write-back + on-demand cast == fused update, bit for bit; the cast is
    the format conversion (checked against torch / numpy, which the oracle does not call)."""
    n = 5000
    for dtype in (BF16, FP16):
        g = lowp(RNG.normal(0, 1e-3, n), dtype)
        fused = state(n, dtype, rng=np.random.default_rng(3))
        split = {k: v.copy() for k, v in fused.items()}
        hp = oracle.hparams()
        norm, flag = oracle.grad_prep([g], dtype, 1.0)
        oracle.adamw_chunk(g, fused["param_lp"], fused["master"], fused["exp_avg"], fused["exp_avg_sq"], dtype, 2, hp,
                           norm, flag)
        stale = split["param_lp"].copy()
        oracle.adamw_chunk(g, None, split["master"], split["exp_avg"], split["exp_avg_sq"], dtype, 2, hp, norm, flag)
        assert np.array_equal(split["param_lp"], stale)                   # untouched without write-back
        oracle.cast_chunk(split["master"], split["param_lp"], dtype)
        assert all(fused[k].tobytes() == split[k].tobytes() for k in fused)
        if dtype == BF16:
            ref = torch.tensor(split["master"]).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        else:
            ref = split["master"].astype(np.float16).view(np.uint16)
        assert np.array_equal(split["param_lp"], ref)


def test_limits_at_infinite_second_moment_and_zero_denominator():
    """Mathematical limits at the corners the update can reach with finite gradients:
    v = +inf (overflowed earlier) makes the Adam term exactly 0, leaving pure decay;
    eps = 0 with v = 0 and m != 0 divides by zero: the parameter runs to -+inf with the sign
    of m; m = v = 0 with eps = 0 is 0/0 (NaN).  The largest finite bf16 gradient overflows v in
    the step itself while the parameter stays finite (its own update still sees a finite v_hat
    only if fp64 holds it: 1e77 does)."""
    n = 64
    st = state(n, BF16)
    p0 = st["master"].astype(np.float64)
    st["exp_avg_sq"][:] = np.inf
    hp = oracle.hparams(lr=0.125, weight_decay=0.5, max_grad_norm=0.0)   # lr*wd = 1/16 exactly
    g = lowp(RNG.normal(0, 1e-3, n), BF16)
    oracle.adamw_chunk(g, st["param_lp"], st["master"], st["exp_avg"], st["exp_avg_sq"], BF16, 3, hp, 0.0, 0)
    assert np.array_equal(st["master"], (p0 * (1 - 0.0625)).astype(np.float32))
    assert np.isinf(st["exp_avg_sq"]).all() and np.isfinite(st["exp_avg"]).all()

    st = state(n, BF16, zero_moments=True)
    st["exp_avg"][: n // 2] = 1e-3
    st["exp_avg"][n // 2:] = -1e-3
    st["exp_avg"][0] = 0.0
    hp0 = oracle.hparams(eps=0.0, weight_decay=0.0, max_grad_norm=0.0)
    with np.errstate(all="ignore"):
        oracle.adamw_chunk(np.zeros(n, np.uint16), st["param_lp"], st["master"], st["exp_avg"], st["exp_avg_sq"],
                           BF16, 2, hp0, 0.0, 0)
    assert np.isnan(st["master"][0])
    assert (st["master"][1: n // 2] == -np.inf).all() and (st["master"][n // 2:] == np.inf).all()

    st = state(n, BF16, zero_moments=True)
    p0 = st["master"].astype(np.float64)
    big = np.full(n, 0x7F7F, np.uint16)                                   # 3.39e38, finite
    hp1 = oracle.hparams(lr=1e-3, weight_decay=0.0, max_grad_norm=0.0)
    with np.errstate(all="ignore"):
        oracle.adamw_chunk(big, st["param_lp"], st["master"], st["exp_avg"], st["exp_avg_sq"], BF16, 1, hp1, 0.0, 0)
    assert np.isinf(st["exp_avg_sq"]).all()                               # 1e-3 * 1.15e77 does not fit fp32
    # step 1: m_hat = g, v_hat = g^2 in fp64 -> update = lr * g / (|g| + eps) = lr to within eps/|g|
    want = p0 - float(np.float32(1e-3))
    assert (np.abs(st["master"].astype(np.float64) - want) <= ulp32(want)).all()
