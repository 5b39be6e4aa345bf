"""Pins of the CPU oracle against things other than itself: closed forms, a hand-worked
example, exhaustive bit-pattern checks against numpy/torch, exact rational brute force, and
an fp64 library optimizer.  No GPU involved."""
import math
import os
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import GRAD_BF16, GRAD_FP16

HP = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.01)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "adam_dyadic_example.txt")


# ---------------------------------------------------------------- helpers (test side only)
def bf16_bits(x):
    """bf16 bit patterns of float values via torch's narrowing (library routine)."""
    t = torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_value(bits):
    return (np.asarray(bits, dtype=np.uint32) << 16).view(np.float32)


def f32(x):
    return np.float32(x)


def round_f32(x: Fraction) -> np.float32:
    """Exact round-to-nearest-even of a rational to fp32 (overflow -> inf)."""
    if x == 0:
        return np.float32(0.0)
    fmax = Fraction(float(np.finfo(np.float32).max))
    half_ulp_max = Fraction(2) ** 103
    if abs(x) >= fmax + half_ulp_max:
        return np.float32(math.copysign(math.inf, x))
    with np.errstate(over="ignore"):
        c = np.float32(float(x))
    if not np.isfinite(c):
        c = np.float32(math.copysign(float(np.finfo(np.float32).max), x))
    cands = [c, np.nextafter(c, np.float32(np.inf)), np.nextafter(c, np.float32(-np.inf))]
    cands = [k for k in cands if np.isfinite(k)]
    best = None
    for k in cands:
        d = abs(Fraction(float(k)) - x)
        even = (int(np.float32(k).view(np.uint32)) & 1) == 0
        key = (d, 0 if even else 1)
        if best is None or key < best[0]:
            best = (key, k)
    return np.float32(best[1])


def exact_adamw(g: Fraction, p, m, v, hp, t, s: Fraction, adamw=1, bias_correction=1):
    """One element of AdamW in exact rational arithmetic (square root to 60 digits)."""
    getcontext().prec = 80
    lr, b1, b2, eps, wd = (Fraction(float(f32(hp[k]))) for k in
                           ("lr", "beta1", "beta2", "eps", "wd"))
    p, m, v = Fraction(float(p)), Fraction(float(m)), Fraction(float(v))
    g = g * s
    if not adamw:
        g = g + wd * p
    mn = b1 * m + (1 - b1) * g
    vn = b2 * v + (1 - b2) * g * g
    bc1 = 1 - b1 ** t if bias_correction else Fraction(1)
    bc2 = 1 - b2 ** t if bias_correction else Fraction(1)
    vhat = vn / bc2
    root = Decimal(vhat.numerator) / Decimal(vhat.denominator)
    root = Fraction(root.sqrt())
    pn = p - (lr * wd * p if adamw else 0) - lr * (mn / bc1) / (root + eps)
    return pn, mn, vn


def run_oracle(gbits, dtype, p, m, v, t, s=1.0, hp=HP, **kw):
    g = np.ascontiguousarray(gbits, dtype=np.uint16)
    p = np.array(p, dtype=np.float32)
    m = np.array(m, dtype=np.float32)
    v = np.array(v, dtype=np.float32)
    q = np.zeros(g.size, dtype=np.uint16)
    oracle.adamw_step(g, dtype, p, m, v, q, t=t, s=s, **hp, **kw)
    return p, m, v, q


def ulp_diff(a, b):
    a = np.asarray(a, dtype=np.float32).view(np.int32).astype(np.int64)
    b = np.asarray(b, dtype=np.float32).view(np.int32).astype(np.int64)
    a = np.where(a < 0, -(a & 0x7FFFFFFF), a)
    b = np.where(b < 0, -(b & 0x7FFFFFFF), b)
    return np.abs(a - b)


# ---------------------------------------------------------------- 16-bit formats
def test_decode_fp16_exhaustive_vs_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.decode16(int(b), GRAD_FP16) for b in bits])
    assert np.array_equal(np.isnan(want), np.isnan(got))
    ok = ~np.isnan(want)
    assert np.array_equal(want[ok], got[ok])
    assert np.array_equal(np.signbit(want[ok]), np.signbit(got[ok]))


def test_decode_bf16_exhaustive_vs_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    want = bf16_value(bits).astype(np.float64)
    got = np.array([oracle.decode16(int(b), GRAD_BF16) for b in bits])
    assert np.array_equal(np.isnan(want), np.isnan(got))
    ok = ~np.isnan(want)
    assert np.array_equal(want[ok], got[ok])
    assert np.array_equal(np.signbit(want[ok]), np.signbit(got[ok]))


@pytest.mark.parametrize("dtype", [GRAD_BF16, GRAD_FP16])
def test_nonfinite_scan_exhaustive(dtype):
    bits = np.arange(65536, dtype=np.uint16)
    vals = bits.view(np.float16).astype(np.float64) if dtype == GRAD_FP16 else \
        bf16_value(bits).astype(np.float64)
    want = ~np.isfinite(vals)
    got = np.array([oracle.is_nonfinite16(int(b), dtype) for b in bits])
    assert np.array_equal(want, got)
    # and the bucket-level count over all patterns at once
    _, cnt = oracle.grad_stats(bits.copy(), dtype, 1.0)
    assert cnt == int(want.sum())


def test_bf16_rounding_exhaustive_vs_torch_and_definition():
    lowers = [0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF]
    upper = np.arange(65536, dtype=np.uint32)
    for lo in lowers:
        u = (upper << 16) | lo
        x = u.view(np.float32)
        want = bf16_bits(x)
        got = np.array([oracle.f32_to_bf16(float(v)) if not np.isnan(v) else 0 for v in x],
                       dtype=np.uint16)
        ok = ~np.isnan(x)
        assert np.array_equal(want[ok], got[ok]), hex(lo)
    # definition: nearest representable, ties to even fraction, on a few named values
    assert oracle.f32_to_bf16(1.0) == 0x3F80
    assert oracle.f32_to_bf16(-0.0) == 0x8000
    assert oracle.f32_to_bf16(float(np.float32(3.3895314e38))) == 0x7F7F      # largest finite
    assert oracle.f32_to_bf16(float(np.finfo(np.float32).max)) == 0x7F80      # rounds to inf
    assert oracle.f32_to_bf16(float(np.uint32(0x3F808000).view(np.float32))) == 0x3F80  # tie
    assert oracle.f32_to_bf16(float(np.uint32(0x3F818000).view(np.float32))) == 0x3F82  # tie
    assert oracle.f32_to_bf16(float(np.uint32(0x00010000).view(np.float32))) == 0x0001
    nan_bits = oracle.f32_to_bf16(float("nan"))
    assert (nan_bits & 0x7F80) == 0x7F80 and (nan_bits & 0x7F) != 0


def test_cast_lp_is_the_pinned_rounding_element_by_element():
    """The array cast against torch's / numpy's own conversions on every finite and infinite
    fp32 whose low half is one of the tie patterns, and NaN stays NaN."""
    import torch
    upper = np.arange(65536, dtype=np.uint32)
    for lo in (0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0x1000, 0x0FFF, 0x1001, 0xFFFF):
        x = ((upper << 16) | lo).view(np.float32)
        ok = ~np.isnan(x)
        got_b, got_h = oracle.cast_lp(x, 0), oracle.cast_lp(x, 1)
        want_b = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        with np.errstate(over="ignore"):
            want_h = x.astype(np.float16).view(np.uint16)
        assert np.array_equal(got_b[ok], want_b[ok]) and np.array_equal(got_h[ok], want_h[ok]), hex(lo)
        assert np.all((got_b[~ok] & 0x7F80) == 0x7F80) and np.all((got_b[~ok] & 0x7F) != 0)
        assert np.all((got_h[~ok] & 0x7C00) == 0x7C00) and np.all((got_h[~ok] & 0x3FF) != 0)
    assert oracle.cast_lp(np.zeros(0, np.float32)).size == 0
    # the same bits as the step's own store
    gb = bf16_bits([1e-3, -2e-3, 0.5])
    p, m, v, q = run_oracle(gb, GRAD_BF16, [0.1, 70000.0, -3e-6], np.zeros(3), np.zeros(3), 1)
    assert np.array_equal(q, oracle.cast_lp(p))


def test_fp16_rounding_exhaustive_vs_numpy():
    lowers = [0x0000, 0x0001, 0x0FFF, 0x1000, 0x1001, 0x1FFF, 0x2000, 0x3000, 0xFFFF]
    upper = np.arange(65536, dtype=np.uint32)
    for lo in lowers:
        x = ((upper << 16) | lo).view(np.float32)
        ok = ~np.isnan(x)
        with np.errstate(over="ignore"):
            want = x.astype(np.float16).view(np.uint16)
        got = np.array([oracle.f32_to_fp16(float(v)) if not np.isnan(v) else 0 for v in x], dtype=np.uint16)
        assert np.array_equal(want[ok], got[ok]), hex(lo)
    assert oracle.f32_to_fp16(65504.0) == 0x7BFF and oracle.f32_to_fp16(65520.0) == 0x7C00
    assert oracle.f32_to_fp16(65519.99) == 0x7BFF and oracle.f32_to_fp16(-0.0) == 0x8000
    assert oracle.f32_to_fp16(2.0 ** -24) == 0x0001 and oracle.f32_to_fp16(2.0 ** -25) == 0x0000   # tie to even
    assert oracle.f32_to_fp16(1.5 * 2.0 ** -24) == 0x0002
    nanb = oracle.f32_to_fp16(float("nan"))
    assert (nanb & 0x7C00) == 0x7C00 and (nanb & 0x3FF) != 0
    # and through the step: the fp16 working copy is the rounding of the stored parameter
    gb = bf16_bits([1e-3, -2e-3, 0.5])
    p, m, v, q = run_oracle(gb, GRAD_BF16, [0.1, 70000.0, -3e-6], np.zeros(3), np.zeros(3), 1, lp_fp16=1)
    assert np.array_equal(q, p.astype(np.float16).view(np.uint16))


# ---------------------------------------------------------------- golden hand-worked example
def _golden():
    out = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, val = [s.strip() for s in line.split("=")]
        out[k] = int(val, 16) if val.startswith("0x") else Fraction(val)
    return out


def test_golden_dyadic_example():
    G = _golden()
    hp = dict(lr=0.5, beta1=0.5, beta2=0.75, eps=1.0, wd=0.0)
    one, neg = bf16_bits([1.0])[0], bf16_bits([-1.0])[0]
    p, m, v = [1.0], [0.0], [0.0]
    for t, gb in enumerate([one, neg, one], start=1):
        p, m, v, q = run_oracle([gb], GRAD_BF16, p, m, v, t, hp=hp)
        if t < 3:   # exact while the inputs are still exactly the rationals
            assert m[0] == round_f32(G[f"A.t{t}.m"])
            assert v[0] == round_f32(G[f"A.t{t}.v"])
            assert p[0] == round_f32(G[f"A.t{t}.p"])
        else:
            assert ulp_diff(p[0], round_f32(G["A.t3.p"])) <= 1
            assert m[0] == round_f32(G["A.t3.m"]) and v[0] == round_f32(G["A.t3.v"])
        if t == 1:
            assert q[0] == G["A.t1.q_bits"]
    # fp16 container gives the same result as bf16 for the value 1.0
    p16, m16, v16, _ = run_oracle([0x3C00], GRAD_FP16, [1.0], [0.0], [0.0], 1, hp=hp)
    assert p16[0] == round_f32(G["A.t1.p"]) and m16[0] == 0.5 and v16[0] == 0.25
    # decoupled decay
    hpB = dict(hp, wd=0.25)
    p, m, v, q = run_oracle([one], GRAD_BF16, [1.0], [0.0], [0.0], 1, hp=hpB)
    assert p[0] == round_f32(G["B.t1.p"]) and q[0] == G["B.t1.q_bits"]
    # gradient multiplier s
    p, m, v, q = run_oracle([one], GRAD_BF16, [1.0], [0.0], [0.0], 1, s=0.5, hp=hp)
    assert (m[0], v[0], p[0]) == (round_f32(G["C.t1.m"]), round_f32(G["C.t1.v"]),
                                  round_f32(G["C.t1.p"]))
    # classic Adam: decay enters through the gradient
    hpD = dict(hp, wd=1.0)
    p, m, v, q = run_oracle([0], GRAD_BF16, [1.0], [0.0], [0.0], 1, hp=hpD, adamw=0)
    assert p[0] == round_f32(G["D.t1.p"])


# ---------------------------------------------------------------- closed forms
def test_step1_closed_form():
    """From m=v=0 at t=1: p1 = p0 (1 - lr wd) - lr g / (|g| + eps)."""
    rng = np.random.default_rng(1)
    gv = np.concatenate([rng.normal(0, 1e-3, 200), [1e-9, -1e-9, 1e-12, 3.0, -2.5e4, 1e-30]])
    gb = bf16_bits(gv)
    p0 = rng.normal(0, 0.02, gb.size).astype(np.float32)
    p, m, v, q = run_oracle(gb, GRAD_BF16, p0, np.zeros_like(p0), np.zeros_like(p0), 1)
    lr, eps, wd = (Fraction(float(f32(HP[k]))) for k in ("lr", "eps", "wd"))
    b1, b2 = Fraction(float(f32(HP["beta1"]))), Fraction(float(f32(HP["beta2"])))
    for i in range(gb.size):
        g = Fraction(float(bf16_value(gb[i:i + 1])[0]))
        pe = Fraction(float(p0[i])) * (1 - lr * wd) - lr * g / (abs(g) + eps)
        assert p[i] == round_f32(pe), i
        assert m[i] == round_f32((1 - b1) * g) and v[i] == round_f32((1 - b2) * g * g)
        assert q[i] == bf16_bits([p[i]])[0]
    # |g| >> eps: the step has magnitude lr whatever g is (up to eps/|g|)
    big = np.abs(bf16_value(gb).astype(np.float64)) > 1e-4
    hp0 = dict(HP, wd=0.0)
    p, *_ = run_oracle(gb, GRAD_BF16, p0, np.zeros_like(p0), np.zeros_like(p0), 1, hp=hp0)
    step = (p0.astype(np.float64) - p.astype(np.float64))[big]
    assert np.allclose(np.abs(step), 1e-4, rtol=2e-3)
    assert np.array_equal(np.sign(step), np.sign(bf16_value(gb).astype(np.float64)[big]))


def test_constant_gradient_trajectory():
    """g = c for all t: mhat = c, vhat = c^2 exactly; with wd = 0 the parameter moves on a
    line p_t = p0 - t lr c/(|c|+eps); m_t = c(1-b1^t), v_t = c^2(1-b2^t)."""
    hp = dict(HP, wd=0.0)
    cs = bf16_value(bf16_bits([1e-3, -2e-3, 0.5, -7.0]))
    gb = bf16_bits(cs)
    p0 = np.array([0.3, -0.2, 1.0, 2.0], dtype=np.float32)
    p, m, v = p0.copy(), np.zeros(4, np.float32), np.zeros(4, np.float32)
    b1, b2 = float(f32(hp["beta1"])), float(f32(hp["beta2"]))
    lr, eps = float(f32(hp["lr"])), float(f32(hp["eps"]))
    for t in range(1, 31):
        p, m, v, _ = run_oracle(gb, GRAD_BF16, p, m, v, t, hp=hp)
        c = cs.astype(np.float64)
        assert np.allclose(m, c * (1 - b1 ** t), rtol=3e-7, atol=0)
        assert np.allclose(v, c * c * (1 - b2 ** t), rtol=3e-7 * t, atol=0)
        line = p0.astype(np.float64) - t * lr * c / (np.abs(c) + eps)
        # each step rounds p once: at most half an ulp of drift per step
        half_ulp = 0.5 * np.spacing(np.maximum(np.abs(p0), np.abs(p)).astype(np.float32))
        assert np.all(np.abs(p - line) <= t * half_ulp.astype(np.float64) * 1.001)


def test_zero_gradient_is_pure_decay():
    p0 = np.array([1.0, -0.5, 0.02, 123.0], dtype=np.float32)
    p, m, v = p0.copy(), np.zeros(4, np.float32), np.zeros(4, np.float32)
    g = np.zeros(4, dtype=np.uint16)
    lr, wd = float(f32(HP["lr"])), float(f32(HP["wd"]))
    T = 50
    for t in range(1, T + 1):
        p, m, v, _ = run_oracle(g, GRAD_BF16, p, m, v, t)
        assert not m.any() and not v.any()
    want = p0.astype(np.float64) * (1 - lr * wd) ** T
    assert np.all(ulp_diff(p, want.astype(np.float32)) <= T // 2 + 1)
    assert np.allclose(p, want, rtol=1e-6)
    assert np.all(np.abs(p) < np.abs(p0))


def test_lr_zero_moves_moments_only():
    hp = dict(HP, lr=0.0)
    gb = bf16_bits([1e-3, -4e-3, 2.0])
    p0 = np.array([0.1, 0.2, -0.3], dtype=np.float32)
    p, m, v, q = run_oracle(gb, GRAD_BF16, p0, np.zeros(3), np.zeros(3), 1, hp=hp)
    assert np.array_equal(p, p0)
    assert np.all(m != 0) and np.all(v > 0)
    assert np.array_equal(q, bf16_bits(p0))


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("dtype", [GRAD_BF16, GRAD_FP16])
@pytest.mark.parametrize("n", [1, 3, 8, 13, 64])
def test_bruteforce_exact_rational(dtype, n):
    rng = np.random.default_rng(100 + n + dtype)
    if dtype == GRAD_BF16:
        gb = bf16_bits(rng.normal(0, 1e-3, n))
        special = [0x0001, 0x7F7F, 0xFF7F, 0x8000, 0x0080]     # subnormal, +-max, -0, min normal
        dec = lambda b: Fraction(float(bf16_value(np.array([b]))[0]))
    else:
        gb = rng.normal(0, 60.0, n).astype(np.float16).view(np.uint16)
        special = [0x0001, 0x7BFF, 0xFBFF, 0x8000, 0x0400]
        dec = lambda b: Fraction(float(np.array([b], dtype=np.uint16).view(np.float16)[0]))
    gb = gb.copy()
    for k, sbits in enumerate(special[:n]):
        gb[k] = sbits
    p = rng.normal(0, 0.02, n).astype(np.float32)
    m = rng.normal(0, 1e-4, n).astype(np.float32)
    v = (rng.normal(0, 1e-4, n) ** 2).astype(np.float32)
    s = f32(0.0896 if dtype == GRAD_BF16 else 1.0 / 65536.0)
    for t in (1, 7):
        po, mo, vo, qo = run_oracle(gb, dtype, p, m, v, t, s=s)
        for i in range(n):
            pe, me, ve = exact_adamw(dec(int(gb[i])), p[i], m[i], v[i], HP, t,
                                     Fraction(float(s)))
            assert mo[i] == round_f32(me), (t, i)
            assert vo[i] == round_f32(ve), (t, i)
            assert po[i] == round_f32(pe), (t, i)
            assert qo[i] == bf16_bits([po[i]])[0]
        # variants: classic Adam and no bias correction
        for kw in (dict(adamw=0), dict(bias_correction=0)):
            po2, mo2, vo2, _ = run_oracle(gb, dtype, p, m, v, t, s=s, **kw)
            for i in range(n):
                if dtype == GRAD_BF16 and i < 3 and not kw.get("adamw", 1):
                    continue     # max-finite g overflows fp32 v either way; covered above
                pe, me, ve = exact_adamw(dec(int(gb[i])), p[i], m[i], v[i], HP, t,
                                         Fraction(float(s)), **kw)
                assert (mo2[i], vo2[i], po2[i]) == (round_f32(me), round_f32(ve),
                                                    round_f32(pe)), (kw, t, i)


# ---------------------------------------------------------------- library cross-checks
@pytest.mark.parametrize("adamw", [1, 0])
def test_against_torch_fp64_optimizer(adamw):
    n, T = 4096, 12
    rng = np.random.default_rng(7)
    p0 = rng.normal(0, 0.02, n).astype(np.float32)
    hp32 = {k: float(f32(val)) for k, val in HP.items()}
    w = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    cls = torch.optim.AdamW if adamw else torch.optim.Adam
    opt = cls([w], lr=hp32["lr"], betas=(hp32["beta1"], hp32["beta2"]), eps=hp32["eps"],
              weight_decay=hp32["wd"])
    p, m, v = p0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    for t in range(1, T + 1):
        gb = bf16_bits(rng.normal(0, 1e-3, n))
        w.grad = torch.tensor(bf16_value(gb), dtype=torch.float64)
        opt.step()
        p, m, v, _ = run_oracle(gb, GRAD_BF16, p, m, v, t, adamw=adamw)
    st = opt.state[w]
    assert np.allclose(p, w.detach().numpy(), rtol=1e-6, atol=1e-9)
    assert np.allclose(m, st["exp_avg"].numpy(), rtol=1e-6, atol=1e-10)
    assert np.allclose(v, st["exp_avg_sq"].numpy(), rtol=3e-6, atol=1e-16)


# ---------------------------------------------------------------- norm / clip / scale
def test_norm_exactly_representable():
    for e in (-10, 0, 3):
        for j in (0, 1, 5, 8):
            k = 4 ** j
            g = np.full(k, bf16_bits([2.0 ** e])[0], dtype=np.uint16)
            s, c = oracle.grad_stats(g, GRAD_BF16, 1.0)
            assert c == 0 and s == k * 4.0 ** e and math.sqrt(s) == 2.0 ** (e + j)
    g = np.full(16, 0x4400, dtype=np.uint16)            # fp16 4.0, unscaled by 1/4 -> 1.0
    s, c = oracle.grad_stats(g, GRAD_FP16, 0.25)
    assert (s, c) == (16.0, 0)
    # 3-4-5 and sign independence
    s, _ = oracle.grad_stats(bf16_bits([3.0, -4.0]), GRAD_BF16, 1.0)
    assert s == 25.0


def test_norm_statistical():
    import synth
    n = 1 << 20
    g = synth.normal_16bit(11, synth.STREAM_GRAD, 1, 0, n, 1e-3)
    s, c = oracle.grad_stats(g.view(torch.int16).numpy().view(np.uint16), GRAD_BF16, 1.0)
    assert c == 0
    assert abs(math.sqrt(s) / (1e-3 * math.sqrt(n)) - 1) < 5e-3
    assert math.isclose(s, float((g.double() ** 2).sum()), rel_tol=1e-12)


@pytest.mark.parametrize("dt,code", [(torch.bfloat16, GRAD_BF16), (torch.float16, GRAD_FP16)])
def test_library_primitive_norm_equals_scalar_loop(dt, code):
    """The torch-ops statement of the norm used at multi-billion scale against the C loop."""
    import synth
    n = 300_007
    g = synth.normal_16bit(4, synth.STREAM_GRAD, 2, 0, n, 1e-3 if code == GRAD_BF16 else 50.0, dt)
    raw = g.view(torch.int16)
    raw[17], raw[4000], raw[n - 1] = (0x7F80, 0x7FC1, -128) if code == GRAD_BF16 else (0x7C00, 0x7E01, -1024)
    bits = raw.numpy().view(np.uint16).copy()
    for inv in (1.0, 1.0 / 65536.0, 0.37):
        s0, c0 = oracle.grad_stats(bits, code, inv)
        s1, c1 = oracle.grad_stats_blas(g, inv, chunk=65536)
        assert c0 == c1 == 3 == oracle.count_nonfinite_blas(g, chunk=4096)
        assert math.isclose(s0, s1, rel_tol=1e-12)
    allbits = torch.arange(65536, dtype=torch.int32).to(torch.int16).view(dt)
    s0, c0 = oracle.grad_stats(np.arange(65536, dtype=np.uint16), code, 1.0)
    s1, c1 = oracle.grad_stats_blas(allbits, 1.0)
    assert c0 == c1 == oracle.count_nonfinite_blas(allbits) and math.isclose(s0, s1, rel_tol=1e-12)


def test_nonfinite_elements_are_counted_and_left_out_of_the_sum():
    g = bf16_bits([1.0, 2.0, 0.0, 0.0, 0.0])
    g[2], g[3], g[4] = 0x7F80, 0xFF80, 0x7FC1
    s, c = oracle.grad_stats(g, GRAD_BF16, 1.0)
    assert (s, c) == (5.0, 3)


def test_clip_coefficient():
    assert oracle.clip_coef(0.5, 1.0) == 1.0
    assert oracle.clip_coef(1.0 - 1e-6, 1.0) == 1.0         # norm + 1e-6 <= max_norm
    assert oracle.clip_coef(123.0, 0.0) == 1.0              # clipping off
    c = oracle.clip_coef(11.155, 1.0)
    assert math.isclose(c, 1.0 / (11.155 + 1e-6), rel_tol=1e-15) and abs(c - 0.08964) < 1e-4
    assert oracle.clip_coef(1.0, 1.0) < 1.0


def test_power_of_two_loss_scale_is_exact():
    """Scaling gradients by 2^k and unscaling by 2^-k changes nothing, bit for bit."""
    rng = np.random.default_rng(3)
    n = 257
    gv = bf16_value(bf16_bits(rng.normal(0, 1e-3, n)))
    p0 = rng.normal(0, 0.02, n).astype(np.float32)
    a = run_oracle(bf16_bits(gv), GRAD_BF16, p0, np.zeros(n), np.zeros(n), 1, s=1.0)
    b = run_oracle(bf16_bits(gv * 65536.0), GRAD_BF16, p0, np.zeros(n), np.zeros(n), 1,
                   s=1.0 / 65536.0)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


# ---------------------------------------------------------------- iteration protocol
def _mk_trainer(n=300, nb=3, **kw):
    rng = np.random.default_rng(5)
    buckets = [oracle.Bucket(rng.normal(0, 0.02, n)) for _ in range(nb)]
    return oracle.Trainer(buckets, **HP, **kw), rng


def test_overflow_iteration_is_skipped_and_scale_halved():
    tr, rng = _mk_trainer(grad_dtype=GRAD_FP16, loss_scale=65536.0)
    g = [(rng.normal(0, 1e-3, 300) * 65536).astype(np.float16).view(np.uint16).copy()
         for _ in range(3)]
    assert tr.iteration(g) and tr.t == 2
    snaps = [b.snapshot() for b in tr.buckets]
    g2 = [x.copy() for x in g]
    g2[1][17] = 0x7C00                                  # +inf
    g2[2][5] = 0x7E00                                   # NaN
    assert not tr.iteration(g2)
    assert tr.t == 2 and tr.loss_scale == 32768.0
    assert tr.log[-1]["nonfinite"] == 2
    for b, s in zip(tr.buckets, snaps):
        for x, y in zip((b.p, b.m, b.v, b.q), s):
            assert x.tobytes() == y.tobytes()


def test_clipped_iteration_matches_manual_scaling():
    tr, rng = _mk_trainer(max_norm=1.0)
    g = [bf16_bits(rng.normal(0, 0.2, 300)) for _ in range(3)]
    ref = [oracle.Bucket(b.p) for b in tr.buckets]
    tr.iteration(g)
    allg = np.concatenate([bf16_value(x) for x in g]).astype(np.float64)
    norm = math.sqrt(float((allg ** 2).sum()))
    assert math.isclose(tr.log[-1]["norm"], norm, rel_tol=1e-12)
    clip = 1.0 / (norm + 1e-6)
    assert clip < 1 and math.isclose(tr.log[-1]["clip"], clip, rel_tol=1e-12)
    for b, r, gi in zip(tr.buckets, ref, g):
        oracle.adamw_step(gi, GRAD_BF16, r.p, r.m, r.v, r.q, t=1, s=np.float32(clip), **HP)
        assert np.array_equal(b.p, r.p) and np.array_equal(b.q, r.q)
    # unclipped when the norm is under the threshold: identical to max_norm = 0
    tr1, rng1 = _mk_trainer(max_norm=1e9)
    tr0, rng0 = _mk_trainer(max_norm=0.0)
    tr1.iteration(g)
    tr0.iteration(g)
    for a, b in zip(tr1.buckets, tr0.buckets):
        assert a.p.tobytes() == b.p.tobytes() and a.v.tobytes() == b.v.tobytes()


def test_speculate_then_rollback_equals_synchronous():
    """Speculative step + rollback + clipped redo leaves exactly the synchronous state."""
    tr, rng = _mk_trainer(max_norm=1.0)
    g = [bf16_bits(rng.normal(0, 0.2, 300)) for _ in range(3)]
    spec = [oracle.Bucket(b.p) for b in tr.buckets]
    snaps = [b.snapshot() for b in spec]
    for b, gi in zip(spec, g):                                     # speculate with s = 1
        oracle.adamw_step(gi, GRAD_BF16, b.p, b.m, b.v, b.q, t=1, s=1.0, **HP)
    _, bad, norm = tr.stats(g)
    s, clip = tr.scale_for(norm)
    assert bad == 0 and clip < 1
    for b, sn, gi in zip(spec, snaps, g):                          # roll back, redo clipped
        b.restore(sn)
        oracle.adamw_step(gi, GRAD_BF16, b.p, b.m, b.v, b.q, t=1, s=s, **HP)
    tr.iteration(g)
    for a, b in zip(tr.buckets, spec):
        for x, y in zip((a.p, a.m, a.v, a.q), (b.p, b.m, b.v, b.q)):
            assert x.tobytes() == y.tobytes()


def test_loss_scale_growth_follows_the_hand_worked_walk():
    """The growth rule of the loss scale (the paper gives none; the usual one is taken): the
    same hand-worked walk the host-logic test holds the library to."""
    from test_host_logic import LOSS_SCALE_WALK
    b = oracle.Bucket(np.ones(4, dtype=np.float32))
    tr = oracle.Trainer([b], loss_scale=8.0, min_loss_scale=1.0, growth_interval=2,
                        max_loss_scale=16.0, **HP)
    clean_g = bf16_bits([1.0, -2.0, 0.5, 0.25])
    bad_g = clean_g.copy()
    bad_g[2] = 0x7F80                       # +inf
    t = 1
    for overflow, want in LOSS_SCALE_WALK:
        applied = tr.iteration([bad_g if overflow else clean_g])
        assert applied == (not overflow) and tr.loss_scale == want
        t += 0 if overflow else 1
        assert tr.t == t


def test_threaded_norm_is_the_scalar_loop_chunk_by_chunk():
    """grad_stats_threaded: exactly representable sums equal the single loop for any chunking
    and thread count; on random data it matches the single loop to rounding, never depends on
    the thread count, and counts NaN/Inf exactly."""
    g = np.full(4 ** 6, bf16_bits([2.0 ** -3])[0], dtype=np.uint16)
    for chunk, threads in ((1 << 20, 1), (1000, 3), (77, 2)):
        s, c = oracle.grad_stats_threaded(g, GRAD_BF16, 1.0, threads=threads, chunk=chunk)
        assert (s, c) == (4 ** 6 * 2.0 ** -6, 0)
    import synth
    n = 250_003
    gt = synth.normal_16bit(5, synth.STREAM_GRAD, 3, 0, n, 1e-3)
    raw = gt.view(torch.int16)
    raw[5], raw[n - 2] = 0x7F80, 0x7FC5
    bits = raw.numpy().view(np.uint16).copy()
    s0, c0 = oracle.grad_stats(bits, GRAD_BF16, 0.5)
    got = [oracle.grad_stats_threaded(bits, GRAD_BF16, 0.5, threads=t, chunk=4096) for t in (1, 2, 5)]
    assert got[0] == got[1] == got[2]
    assert got[0][1] == c0 == 2 and math.isclose(got[0][0], s0, rel_tol=1e-13)


def test_layout_definition_matches_the_hand_worked_example():
    path = os.path.join(os.path.dirname(__file__), "golden", "layout_example.txt")
    rows, meta = [], {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if "=" in line:
            k, v = line.split("=")
            meta[k.strip()] = [int(x) for x in v.split()]
        else:
            rows.append(tuple(int(x) for x in line.split()))
    slices, nb = oracle.layout_plan(meta["numel"], meta["bucket"][0])
    assert slices == rows and nb == meta["buckets"][0]
    # invariants on other inputs: every element covered once, in order; no slice crosses a
    # bucket or tensor boundary; empty tensors produce nothing
    for numel, bucket in (([3, 0, 9, 1], 4), ([16], 16), ([5, 5], 100), ([1] * 9, 2)):
        slices, nb = oracle.layout_plan(numel, bucket)
        assert nb == -(-sum(numel) // bucket)
        flat = 0
        for t, to, bk, bo, ln in slices:
            assert ln > 0 and to + ln <= numel[t] and bo + ln <= bucket
            assert bk * bucket + bo == flat == sum(numel[:t]) + to
            flat += ln
        assert flat == sum(numel)
