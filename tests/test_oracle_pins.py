"""Pins for the CPU oracle: it is checked against what the paper and the
mathematics fix (closed forms, invariants, exact dyadic hand-worked cases,
library routines, brute force on tiny inputs), never against itself.

Citations: Eq. 2 (GlobalGC), Eq. 3 (AdaGC coefficient and EMA), Alg. 1 (warm-up
branch, AdaGC branch, AdamW statements), Sec. 4.3 (one fp32 of state per tensor).
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import Hyper

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_defaults.txt")


def golden():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            parts = line.split()
            out[parts[0]] = float(parts[1])
    return out


def f32(x):
    return float(np.float32(x))


# ------------------------------------------------------------------ norm (Sec. 4.1, Eq. 3)

def test_norm_hand_values():
    assert oracle.l2_norm(np.array([3, 4], dtype=np.float32)) == 5.0
    assert oracle.l2_norm(np.array([-5, 12], dtype=np.float32)) == 13.0
    assert oracle.l2_norm(np.array([1, 2, 2], dtype=np.float32)) == 3.0
    assert oracle.l2_norm(np.array([0], dtype=np.float32)) == 0.0
    assert oracle.l2_norm(np.array([-7], dtype=np.float32)) == 7.0


@pytest.mark.parametrize("n", [1, 4, 9, 16, 1024, 65536, 1000000])
def test_norm_all_ones_perfect_square(n):
    assert oracle.l2_norm(np.ones(n, dtype=np.float32)) == math.sqrt(n)


def test_norm_exact_rational_bruteforce():
    rng = np.random.default_rng(1)
    for n in range(1, 17):
        g = (rng.standard_normal(n) * 10 ** rng.uniform(-4, 2)).astype(np.float32)
        exact = sum(Fraction(float(x)) ** 2 for x in g)
        got = oracle.sum_squares(g)
        assert abs(Fraction(got) - exact) <= exact * Fraction(n, 2 ** 52)


def test_norm_vs_library_nrm2():
    rng = np.random.default_rng(2)
    for n in (17, 1000, 123457):
        g = rng.standard_normal(n).astype(np.float32) * 3e-3
        ref = np.linalg.norm(g.astype(np.float64))
        assert oracle.l2_norm(g) == pytest.approx(ref, rel=1e-13)


def test_norm_sign_and_order_independent():
    rng = np.random.default_rng(3)
    g = rng.standard_normal(1000).astype(np.float32)
    a = oracle.l2_norm(g)
    assert oracle.l2_norm(-g) == a
    assert oracle.l2_norm(np.ascontiguousarray(g[::-1])) == pytest.approx(a, rel=1e-14)
    # homogeneity with an exact scale
    assert oracle.l2_norm(g * np.float32(4.0)) == 4.0 * a


def test_norm_bf16_input_is_widened_exactly():
    vals = torch.tensor([3.0, -4.0, 0.5, 1.0078125, -2.5e-3], dtype=torch.float32).to(torch.bfloat16)
    bits = vals.view(torch.int16).numpy().view(np.uint16).copy()
    ref = math.sqrt(sum(float(x) ** 2 for x in vals.to(torch.float64)))
    assert oracle.l2_norm(bits) == pytest.approx(ref, rel=1e-15)
    assert oracle.l2_norm(np.array([0x4040, 0xC080], dtype=np.uint16)) == 5.0   # bf16(3), bf16(-4)


# ------------------------------------------------------------------ bf16 conversion (format definition)

def test_bf16_rne_vs_library_cast():
    rng = np.random.default_rng(4)
    x = np.concatenate([
        rng.standard_normal(5000).astype(np.float32) * 10.0 ** rng.integers(-30, 30, 5000),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 1.0039063, 1.0039062,
                  np.inf, -np.inf, 3.3895314e38, 3.4028235e38, 1e-40, -1e-45], dtype=np.float32),
    ]).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.float_to_bf16_rne(x)
    assert np.array_equal(got, ref)
    # ties go to the even neighbour: 1 + 2^-8 is halfway between 1.0 (even) and 1 + 2^-7
    assert oracle.float_to_bf16_rne(np.array([1.00390625], np.float32))[0] == 0x3F80
    # 1 + 3*2^-8 is halfway between 1+2^-7 (odd) and 1+2^-6 (even)
    assert oracle.float_to_bf16_rne(np.array([1.01171875], np.float32))[0] == 0x3F82
    nan_bits = oracle.float_to_bf16_rne(np.array([np.nan], np.float32))[0]
    assert (nan_bits & 0x7F80) == 0x7F80 and (nan_bits & 0x007F) != 0


def test_bf16_widen_vs_library():
    bits = np.arange(0, 65536, 7, dtype=np.uint16)
    ref = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32).numpy()
    got = oracle.bf16_to_float(bits)
    # NaN payloads do not survive a float -> Python float -> float round trip; compare them as NaN
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


# ------------------------------------------------------------------ Eq. 3: coefficient, EMA

def test_rule_hand_values_dyadic():
    # gamma=1, lambda=2, beta=0.5: threshold 2.  norm 8 -> h = 1/4, EMA takes the clipped norm 2.
    h, g, c = oracle.adagc_rule(8.0, 1.0, 2.0, 0.5)
    assert (h, g, c) == (0.25, 1.5, True)
    # norm 1.5 < 2: no clip, EMA takes the raw norm
    h, g, c = oracle.adagc_rule(1.5, 1.0, 2.0, 0.5)
    assert (h, g, c) == (1.0, 1.25, False)
    # tie: strict inequality, not active, h = 1
    h, g, c = oracle.adagc_rule(2.0, 1.0, 2.0, 0.5)
    assert (h, g, c) == (1.0, 1.5, False)


def test_rule_paper_defaults_growth_factor():
    gold = golden()
    lam, beta = gold["lambda_rel"], gold["ema_beta"]
    h, g, c = oracle.adagc_rule(100.0, 1.0, lam, beta)
    assert c and h == pytest.approx(lam / 100.0, rel=1e-15)
    assert g == pytest.approx(gold["always_clip_growth"], rel=1e-12)


def test_rule_clipped_norm_invariant():
    """After scaling, the tensor's norm is at most lambda_rel*gamma, and equal to it when the
    clip is active (sentence after Eq. 3)."""
    rng = np.random.default_rng(5)
    for _ in range(200):
        n = int(rng.integers(1, 64))
        g = (rng.standard_normal(n) * 10 ** rng.uniform(-3, 1)).astype(np.float32)
        gamma = f32(10 ** rng.uniform(-3, 1))
        lam = f32(1.04)
        norm = oracle.l2_norm(g)
        h, gnew, clipped = oracle.adagc_rule(norm, gamma, lam, f32(0.99))
        scaled = np.linalg.norm(g.astype(np.float64) * h)
        thr = lam * gamma
        assert 0.0 < h <= 1.0
        assert scaled <= thr * (1 + 1e-12)
        if clipped:
            assert norm > thr
            assert scaled == pytest.approx(thr, rel=1e-12)
        else:
            assert h == 1.0 and norm <= thr


def test_rule_scale_invariance():
    for c in (0.125, 2.0, 1024.0):
        a = oracle.adagc_rule(3.0, 1.0, 1.5, 0.75)
        b = oracle.adagc_rule(3.0 * c, 1.0 * c, 1.5, 0.75)
        assert a[0] == b[0] and a[2] == b[2] and b[1] == a[1] * c


def test_rule_degenerate_cases():
    # zero gradient: no division, h = 1, EMA decays toward 0
    assert oracle.adagc_rule(0.0, 2.0, 1.04, 0.5) == (1.0, 1.0, False)
    # zero EMA with a non-zero gradient: literal reading of Eq. 3 gives h = 0 and gamma stays 0
    assert oracle.adagc_rule(3.0, 0.0, 1.04, 0.99) == (0.0, 0.0, True)
    # both zero
    assert oracle.adagc_rule(0.0, 0.0, 1.04, 0.99) == (1.0, 0.0, False)
    # infinite lambda_rel: never active, also with gamma = 0 (threshold is NaN there)
    h, g, c = oracle.adagc_rule(3.0, 2.0, math.inf, 0.5)
    assert (h, g, c) == (1.0, 2.5, False)
    h, g, c = oracle.adagc_rule(3.0, 0.0, math.inf, 0.5)
    assert (h, g, c) == (1.0, 1.5, False)
    # NaN norm: compare is false, no clip, NaN flows into the EMA as it would into AdamW
    h, g, c = oracle.adagc_rule(math.nan, 1.0, 1.04, 0.99)
    assert h == 1.0 and not c and math.isnan(g)


def test_ema_closed_forms():
    gold = golden()
    lam, beta = gold["lambda_rel"], gold["ema_beta"]
    k = 50
    # (a) every step clipped: gamma_k = gamma_0 * rho^k, rho = beta + (1-beta)*lambda_rel
    g0 = 0.7
    gamma = g0
    for _ in range(k):
        h, gamma, c = oracle.adagc_rule(1e6, gamma, lam, beta)
        assert c
    assert gamma == pytest.approx(g0 * gold["always_clip_growth"] ** k, rel=1e-12)
    # (b) constant norm below threshold: gamma_k = n + beta^k (gamma_0 - n)
    n, g0 = 2.0, 2.5
    gamma = g0
    for _ in range(k):
        h, gamma, c = oracle.adagc_rule(n, gamma, lam, beta)
        assert not c and h == 1.0
    assert gamma == pytest.approx(n + beta ** k * (g0 - n), rel=1e-12)
    # (c) never clipped, varying norms: gamma_k = beta^k gamma_0 + (1-beta) sum beta^(k-j) n_j
    rng = np.random.default_rng(6)
    ns = 1.0 + 0.01 * rng.random(k)           # within 1% of 1 => below 1.04*gamma throughout
    g0 = 1.0
    gamma = g0
    for j in range(k):
        h, gamma, c = oracle.adagc_rule(float(ns[j]), gamma, lam, beta)
        assert not c
    closed = beta ** k * g0 + (1 - beta) * sum(beta ** (k - 1 - j) * ns[j] for j in range(k))
    assert gamma == pytest.approx(closed, rel=1e-12)


def test_ema_step_bounds():
    """beta*gamma <= gamma_new <= (beta + (1-beta)*lambda_rel)*gamma, whatever the norm."""
    rng = np.random.default_rng(7)
    for _ in range(500):
        gamma = 10 ** rng.uniform(-4, 2)
        norm = gamma * 10 ** rng.uniform(-3, 3)
        h, gnew, c = oracle.adagc_rule(norm, gamma, 1.04, 0.99)
        assert 0.99 * gamma * (1 - 1e-15) <= gnew <= 1.0004 * gamma * (1 + 1e-15)


# ------------------------------------------------------------------ Eq. 2 / warm-up branch of Alg. 1

def test_globalgc_coef():
    assert oracle.globalgc_coef(13.0, 6.5) == 0.5
    assert oracle.globalgc_coef(0.5, 1.0) == 1.0
    assert oracle.globalgc_coef(1.0, 1.0) == 1.0
    assert oracle.globalgc_coef(0.0, 1.0) == 1.0
    assert oracle.globalgc_coef(7.0, math.inf) == 1.0


def test_warmup_gamma_running_min():
    assert oracle.warmup_gamma(123.0, 5.0, True) == 5.0      # gamma_0 = ||ghat_1||
    assert oracle.warmup_gamma(0.0, 5.0, True) == 5.0
    assert oracle.warmup_gamma(5.0, 3.0, False) == 3.0
    assert oracle.warmup_gamma(5.0, 8.0, False) == 5.0


def _lists(arrs, dtype=np.float32):
    return [np.array(a, dtype=dtype) for a in arrs]


def test_step_warmup_branch_hand_worked():
    """Two tensors [3,4] and [12]: global norm 13, lambda_abs 6.5 -> h = 1/2 for both.
    Step 1 sets gamma to the clipped norms (2.5, 6); step 2 keeps the running minimum."""
    theta = _lists([[0, 0], [0]])
    m = _lists([[0, 0], [0]])
    v = _lists([[0, 0], [0]])
    gamma = np.zeros(2, dtype=np.float32)
    hp = Hyper(lr=0.0, beta1=0.5, beta2=0.75, eps=0.0, weight_decay=0.0, lambda_abs=6.5, t_start=2)
    norms, coefs, clipped = oracle.adagc_step(theta, _lists([[3, 4], [12]]), m, v, gamma, hp, 1)
    assert list(norms) == [5.0, 12.0] and list(coefs) == [0.5, 0.5] and list(clipped) == [1, 1]
    assert list(gamma) == [2.5, 6.0]
    # m takes the globally clipped gradient: (1-beta1)*h*g
    assert list(m[0]) == [0.75, 1.0] and list(m[1]) == [3.0]
    # v takes its square: (1-beta2)*(h*g)^2
    assert list(v[0]) == [0.5625, 1.0] and list(v[1]) == [9.0]
    # step 2 (still warm-up): small gradients, no global clip; min() keeps 2.5 and lowers 6 -> 4
    norms, coefs, clipped = oracle.adagc_step(theta, _lists([[0, 3], [4]]), m, v, gamma, hp, 2)
    assert list(coefs) == [1.0, 1.0] and list(clipped) == [0, 0]
    assert list(gamma) == [2.5, 4.0]
    # step 3: warm-up over (t_start = 2) -> AdaGC branch with Eq. 3
    hp.lambda_rel, hp.ema_beta = 2.0, 0.5
    norms, coefs, clipped = oracle.adagc_step(theta, _lists([[6, 8], [4]]), m, v, gamma, hp, 3)
    assert list(norms) == [10.0, 4.0]
    assert list(coefs) == [0.5, 1.0] and list(clipped) == [1, 0]      # 10 > 2*2.5 ; 4 <= 2*4
    assert list(gamma) == [0.5 * 2.5 + 0.5 * 5.0, 0.5 * 4.0 + 0.5 * 4.0]


def test_step_init_step_without_global_clip():
    """t_start = 1 with infinite lambda_abs: step 1 passes gradients through and sets gamma to
    their norms; AdaGC is live from step 2."""
    theta, m, v = _lists([[1, 1]]), _lists([[0, 0]]), _lists([[0, 0]])
    gamma = np.array([77.0], dtype=np.float32)
    hp = Hyper(lr=0.0, lambda_rel=2.0, ema_beta=0.5)
    norms, coefs, clipped = oracle.adagc_step(theta, _lists([[3, 4]]), m, v, gamma, hp, 1)
    assert coefs[0] == 1.0 and clipped[0] == 0 and gamma[0] == 5.0
    norms, coefs, clipped = oracle.adagc_step(theta, _lists([[30, 40]]), m, v, gamma, hp, 2)
    assert norms[0] == 50.0 and clipped[0] == 1 and coefs[0] == 0.2 and gamma[0] == 7.5


def test_step_t_start_zero_uses_caller_gamma():
    theta, m, v = _lists([[1, 1]]), _lists([[0, 0]]), _lists([[0, 0]])
    gamma = np.array([1.0], dtype=np.float32)
    hp = Hyper(lr=0.0, lambda_rel=2.0, ema_beta=0.5, t_start=0)
    norms, coefs, clipped = oracle.adagc_step(theta, _lists([[3, 4]]), m, v, gamma, hp, 1)
    assert clipped[0] == 1 and coefs[0] == 0.4 and gamma[0] == 1.5


# ------------------------------------------------------------------ AdamW statements of Alg. 1

def test_adamw_dyadic_hand_worked_two_steps():
    """beta1=1/2, beta2=3/4, lr=1/2, eps=0, wd=1/4, theta0=4, g=4 scaled by h=1/2 (ghat=2).
    t=1: m=1, v=1, mhat=2, vhat=4, theta = 4 - 1/2*1/4*4 - 1/2*2/2 = 3.
    t=2: m=3/2, v=7/4, mhat=2, vhat=4, theta = 3 - 3/8 - 1/2 = 17/8."""
    hp = Hyper(lr=0.5, beta1=0.5, beta2=0.75, eps=0.0, weight_decay=0.25)
    theta, m, v = (np.array([4.0], np.float32), np.zeros(1, np.float32), np.zeros(1, np.float32))
    g = np.array([4.0], np.float32)
    copy = np.zeros(1, np.uint16)
    oracle.adamw_update(theta, m, v, g, 0.5, hp, 1, copy)
    assert (theta[0], m[0], v[0]) == (3.0, 1.0, 1.0)
    assert copy[0] == 0x4040                                   # bf16(3.0)
    oracle.adamw_update(theta, m, v, g, 0.5, hp, 2, copy)
    assert (theta[0], m[0], v[0]) == (2.125, 1.5, 1.75)
    assert copy[0] == 0x4008                                   # bf16(2.125) = 2 + 2^-3


def test_updates_read_bf16_gradients_as_their_values():
    """The two hand-worked dyadic cases again, with the gradient given as bf16 bits
    (4.0 = 0x4080, -8.0 = 0xC100): the results are the same numbers."""
    hp = Hyper(lr=0.5, beta1=0.5, beta2=0.75, eps=0.0, weight_decay=0.25, grad_dtype=oracle.GRAD_BF16)
    theta, m, v = (np.array([4.0], np.float32), np.zeros(1, np.float32), np.zeros(1, np.float32))
    oracle.adamw_update(theta, m, v, np.array([0x4080], np.uint16), 0.5, hp, 1)
    assert (theta[0], m[0], v[0]) == (3.0, 1.0, 1.0)
    hp = Hyper(lr=0.25, beta1=0.5, beta2=0.75, weight_decay=0.5, optimizer=oracle.LION, grad_dtype=oracle.GRAD_BF16)
    theta, m = np.array([1.0], np.float32), np.array([2.0], np.float32)
    oracle.lion_update(theta, m, np.array([0xC100], np.uint16), 0.5, hp)
    assert (theta[0], m[0]) == (1.125, 0.5)


@pytest.mark.parametrize("optimizer", [oracle.ADAMW, oracle.LION])
def test_step_on_bf16_gradients_equals_step_on_the_widened_values(optimizer):
    """Every bf16 value is an fp32 value (same sign, exponent, top 7 mantissa bits), so a step fed bf16 bits
    must leave exactly the state of a step fed those values as fp32; the widening here is a plain shift."""
    rng = np.random.default_rng(21)
    numels = [1, 5, 300, 77]
    bits = [(rng.standard_normal(n) * 0.05).astype(np.float32).view(np.uint32) >> 16 for n in numels]
    bits = [b.astype(np.uint16) for b in bits]
    wide = [(b.astype(np.uint32) << 16).view(np.float32) for b in bits]
    states = []
    for grads, gd in ((bits, oracle.GRAD_BF16), (wide, oracle.GRAD_F32)):
        hp = Hyper(optimizer=optimizer, grad_dtype=gd, lambda_abs=0.5, t_start=2)
        theta = [np.full(n, 0.25, np.float32) for n in numels]
        m = [np.zeros(n, np.float32) for n in numels]
        v = [np.zeros(n, np.float32) for n in numels] if optimizer == oracle.ADAMW else None
        gamma = np.zeros(len(numels), np.float32)
        outs = [oracle.adagc_step(theta, grads, m, v, gamma, hp, t) for t in (1, 2, 3)]
        states.append((theta, m, v, gamma, outs))
    a, b = states
    for x, y in zip(a[0] + a[1] + (a[2] or []) + [a[3]], b[0] + b[1] + (b[2] or []) + [b[3]]):
        assert np.array_equal(x, y)
    for (n1, c1, f1), (n2, c2, f2) in zip(a[4], b[4]):
        assert np.array_equal(n1, n2) and np.array_equal(c1, c2) and np.array_equal(f1, f2)
    assert not np.array_equal(a[0][2], np.full(300, 0.25, np.float32))


def test_adamw_step1_closed_form():
    """m0=v0=0, t=1: m=(1-b1)g, v=(1-b2)g^2, theta1 = theta0(1-lr*wd) - lr*g/(|g|+eps)."""
    rng = np.random.default_rng(8)
    n = 257
    hp = Hyper()
    theta0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    g = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    theta, m, v = theta0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    oracle.adamw_update(theta, m, v, g, 1.0, hp, 1)
    b1, b2, lr, wd, eps = map(f32, (hp.beta1, hp.beta2, hp.lr, hp.weight_decay, hp.eps))
    gd, td = g.astype(np.float64), theta0.astype(np.float64)
    np.testing.assert_allclose(m, (1 - b1) * gd, rtol=1e-7)
    np.testing.assert_allclose(v, (1 - b2) * gd * gd, rtol=1e-7)
    np.testing.assert_allclose(theta, td * (1 - lr * wd) - lr * gd / (np.abs(gd) + eps),
                               rtol=2e-7, atol=1e-12)


@pytest.mark.parametrize("eps", [1e-8, 1e-3])
def test_adamw_matches_library_adamw_when_never_clipped(eps):
    """lambda_rel = +inf: the whole step is plain AdamW.  The library routine runs in float64;
    the oracle stores float32 after each step, so agreement is to a few float32 roundings."""
    rng = np.random.default_rng(9)
    sizes = [1, 5, 64, 1000]
    hp = Hyper(lr=1e-2, beta1=0.9, beta2=0.95, eps=eps, weight_decay=0.1, lambda_rel=math.inf)
    theta = [(rng.standard_normal(n) * 0.5).astype(np.float32) for n in sizes]
    m = [np.zeros(n, np.float32) for n in sizes]
    v = [np.zeros(n, np.float32) for n in sizes]
    gamma = np.zeros(len(sizes), np.float32)
    tp = [torch.tensor(t.astype(np.float64), requires_grad=True) for t in theta]
    opt = torch.optim.AdamW(tp, lr=f32(hp.lr), betas=(f32(hp.beta1), f32(hp.beta2)), eps=f32(eps),
                            weight_decay=f32(hp.weight_decay), foreach=False)
    for step in range(1, 8):
        grads = [(rng.standard_normal(n) * 10 ** rng.uniform(-4, 0)).astype(np.float32) for n in sizes]
        norms, coefs, clipped = oracle.adagc_step(theta, grads, m, v, gamma, hp, step)
        assert not clipped.any() and (coefs == 1.0).all()
        for p, g in zip(tp, grads):
            p.grad = torch.tensor(g.astype(np.float64))
        opt.step()
        for i, p in enumerate(tp):
            st = opt.state[p]
            # theta crosses zero under lr-sized steps: absolute slack of a few float32 roundings
            np.testing.assert_allclose(theta[i], p.detach().numpy(), rtol=2e-6, atol=1e-6 * f32(hp.lr))
            # m can cancel: absolute slack of a few float32 roundings of its largest entry
            m_ref = st["exp_avg"].numpy()
            np.testing.assert_allclose(m[i], m_ref, rtol=2e-6, atol=1e-6 * np.abs(m_ref).max())
            np.testing.assert_allclose(v[i], st["exp_avg_sq"].numpy(), rtol=2e-6, atol=1e-20)


def test_adamw_clip_enters_before_the_moments():
    """The coefficient multiplies g before m and v (Alg. 1): updating with (g, h) equals updating
    with (h*g, 1) when h*g is exact."""
    rng = np.random.default_rng(10)
    n = 100
    g = rng.standard_normal(n).astype(np.float32)
    hp = Hyper()
    a = [np.full(n, 0.3, np.float32), np.full(n, 0.01, np.float32), np.full(n, 1e-4, np.float32)]
    b = [x.copy() for x in a]
    oracle.adamw_update(a[0], a[1], a[2], g, 0.25, hp, 3)
    oracle.adamw_update(b[0], b[1], b[2], g * np.float32(0.25), 1.0, hp, 3)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


# ------------------------------------------------------------------ Lion (imported rule)

def test_lion_dyadic_hand_worked():
    """beta1=1/2, beta2=3/4, lr=1/4, wd=1/2; m=2, ghat=-4, theta=1:
    c = 1 - 2 = -1 -> sign -1; theta = 1 - 1/4(-1 + 1/2) = 9/8; m = 3/2 - 1 = 1/2."""
    hp = Hyper(lr=0.25, beta1=0.5, beta2=0.75, weight_decay=0.5, optimizer=oracle.LION)
    theta, m = np.array([1.0], np.float32), np.array([2.0], np.float32)
    copy = np.zeros(1, np.uint16)
    oracle.lion_update(theta, m, np.array([-8.0], np.float32), 0.5, hp, copy)
    assert (theta[0], m[0]) == (1.125, 0.5)
    assert copy[0] == 0x3F90


def test_lion_interpolation_uses_beta1_and_momentum_uses_beta2():
    """m=1, g=-3: with beta1=0.9 c=+0.6 (sign +), with beta2=0.5 the new m is -1.
    Swapping the two betas would flip the sign of the update."""
    hp = Hyper(lr=0.125, beta1=0.9, beta2=0.5, weight_decay=0.0, optimizer=oracle.LION)
    theta, m = np.array([0.0], np.float32), np.array([1.0], np.float32)
    oracle.lion_update(theta, m, np.array([-3.0], np.float32), 1.0, hp)
    assert theta[0] == -0.125 and m[0] == -1.0


def test_lion_update_magnitude_and_sign_zero():
    rng = np.random.default_rng(11)
    n = 500
    hp = Hyper(lr=1e-4, beta1=0.9, beta2=0.99, weight_decay=0.1, optimizer=oracle.LION)
    theta0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    g = rng.standard_normal(n).astype(np.float32)
    g[:10] = 0.0
    theta, m = theta0.copy(), np.zeros(n, np.float32)
    oracle.lion_update(theta, m, g, 1.0, hp)
    lr, wd = f32(hp.lr), f32(hp.weight_decay)
    decayed = theta0.astype(np.float64) * (1 - lr * wd)
    delta = theta.astype(np.float64) - decayed
    # first step, m = 0: sign(c) = sign(g); zero gradient gives sign 0 (only the decay acts)
    np.testing.assert_allclose(delta, -lr * np.sign(g), atol=4e-9)
    np.testing.assert_allclose(m, (1 - f32(hp.beta2)) * g.astype(np.float64), rtol=1e-7)


# ------------------------------------------------------------------ whole step: indexing

def test_step_tensors_are_independent_and_permutable():
    rng = np.random.default_rng(12)
    sizes = [3, 1, 16, 7, 40]
    hp = Hyper(t_start=0)

    def fresh():
        r = np.random.default_rng(13)
        theta = [r.standard_normal(n).astype(np.float32) for n in sizes]
        m = [r.standard_normal(n).astype(np.float32) * 0.1 for n in sizes]
        v = [(r.standard_normal(n).astype(np.float32) * 0.1) ** 2 for n in sizes]
        g = [r.standard_normal(n).astype(np.float32) * (10.0 ** (i - 2)) for i, n in enumerate(sizes)]
        gamma = np.array([0.5, 0.05, 50.0, 1.0, 1e4], np.float32)
        return theta, g, m, v, gamma

    theta, g, m, v, gamma = fresh()
    n0, c0, f0 = oracle.adagc_step(theta, g, m, v, gamma, hp, 5)
    assert f0.any() and not f0.all()
    perm = [3, 0, 4, 2, 1]
    t2, g2, m2, v2, gm2 = fresh()
    tp, gp, mp, vp = ([x[i] for i in perm] for x in (t2, g2, m2, v2))
    gmp = gm2[perm].copy()
    n1, c1, f1 = oracle.adagc_step(tp, gp, mp, vp, gmp, hp, 5)
    for k, i in enumerate(perm):
        assert n1[k] == n0[i] and c1[k] == c0[i] and f1[k] == f0[i] and gmp[k] == gamma[i]
        assert np.array_equal(tp[k], theta[i]) and np.array_equal(mp[k], m[i]) and np.array_equal(vp[k], v[i])
    # each tensor alone gives the same result as inside the list (per-tensor rule)
    t3, g3, m3, v3, gm3 = fresh()
    for i in range(len(sizes)):
        gi = gm3[i:i + 1].copy()
        ni, ci, fi = oracle.adagc_step([t3[i]], [g3[i]], [m3[i]], [v3[i]], gi, hp, 5)
        assert ni[0] == n0[i] and ci[0] == c0[i] and gi[0] == gamma[i]
        assert np.array_equal(t3[i], theta[i])


def test_step_equals_pieces():
    """The list step is the composition norm -> rule -> update, tensor by tensor."""
    rng = np.random.default_rng(14)
    n = 33
    hp = Hyper(t_start=0)
    theta = rng.standard_normal(n).astype(np.float32)
    g = rng.standard_normal(n).astype(np.float32)
    m, v = np.zeros(n, np.float32), np.zeros(n, np.float32)
    gamma = np.array([1.0], np.float32)
    t_ref, m_ref, v_ref = theta.copy(), m.copy(), v.copy()
    norm = oracle.l2_norm(g)
    h, gnew, c = oracle.adagc_rule(norm, 1.0, f32(hp.lambda_rel), f32(hp.ema_beta))
    oracle.adamw_update(t_ref, m_ref, v_ref, g, h, hp, 4)
    norms, coefs, clipped = oracle.adagc_step([theta], [g], [m], [v], gamma, hp, 4)
    assert norms[0] == norm and coefs[0] == h and bool(clipped[0]) == c and c
    assert gamma[0] == np.float32(gnew)
    assert np.array_equal(theta, t_ref) and np.array_equal(m, m_ref) and np.array_equal(v, v_ref)


def test_step_rejects_bad_arguments():
    theta, m, v = _lists([[1]]), _lists([[0]]), _lists([[0]])
    gamma = np.zeros(1, np.float32)
    with pytest.raises(ValueError):
        oracle.adagc_step(theta, _lists([[1]]), m, v, gamma, Hyper(), 0)       # step is 1-based
    with pytest.raises(ValueError):
        oracle.adagc_step(theta, _lists([[1]]), m, None, gamma, Hyper(), 1)    # AdamW needs v


def test_gamma_state_is_one_float32_per_tensor():
    """Sec. 4.3: the extra state is a single 32-bit float per tensor."""
    theta, m, v = _lists([[1, 2, 3]]), _lists([[0, 0, 0]]), _lists([[0, 0, 0]])
    gamma = np.zeros(1, np.float32)
    g = _lists([[0.1, 0.2, 0.3]])
    oracle.adagc_step(theta, g, m, v, gamma, Hyper(), 1)
    assert gamma.dtype == np.float32 and gamma.nbytes == 4
    assert gamma[0] == np.float32(oracle.l2_norm(g[0]))


# ------------------------------------------------------------------ chunk enumeration

def test_enumerate_chunks_covers_every_element_once():
    rng = np.random.default_rng(15)
    numels = [int(x) for x in rng.integers(1, 200, 40)] + [1, 16, 17, 32, 64]
    for chunk in (1, 16, 17):
        chunks, begin = oracle.enumerate_chunks(numels, chunk)
        seen = [np.zeros(n, np.int32) for n in numels]
        for (i, first, length) in chunks:
            assert 1 <= length <= chunk and first % chunk == 0
            seen[i][first:first + length] += 1
        assert all((s == 1).all() for s in seen)
        assert sum(c[2] for c in chunks) == sum(numels)
        assert begin[0] == 0 and begin[-1] == len(chunks)
        for i in range(len(numels)):
            own = chunks[begin[i]:begin[i + 1]]
            assert all(c[0] == i for c in own) and len(own) == -(-numels[i] // chunk)


# ------------------------------------------------------------------ global-statistic modes (Eq. 2; ablation study, Sec. 5.6)

def test_globalgc_mode_hand_worked_and_equals_endless_warmup():
    """Mode GlobalGC applies Eq. 2 on every step and keeps no per-tensor state.  Tensors [3,4] and
    [12]: global norm 13, lambda_abs 6.5 -> h = 1/2.  The same numbers come out of Alg. 1's warm-up
    branch when T_start never ends."""
    def fresh():
        return (_lists([[1, 1], [1]]), _lists([[0, 0], [0]]), _lists([[0, 0], [0]]))
    g = _lists([[3, 4], [12]])
    th_a, m_a, v_a = fresh()
    gam_a = np.array([7.0, 9.0], np.float32)
    hp_a = Hyper(lr=0.25, beta1=0.5, beta2=0.75, eps=0.0, weight_decay=0.0, lambda_abs=6.5, t_start=0,
                 clip_mode=oracle.MODE_GLOBALGC)
    norms, coefs, clipped = oracle.adagc_step(th_a, g, m_a, v_a, gam_a, hp_a, 5)
    assert list(norms) == [5.0, 12.0] and list(coefs) == [0.5, 0.5] and list(clipped) == [1, 1]
    assert list(gam_a) == [7.0, 9.0]                      # untouched
    th_b, m_b, v_b = fresh()
    gam_b = np.array([7.0, 9.0], np.float32)
    hp_b = Hyper(lr=0.25, beta1=0.5, beta2=0.75, eps=0.0, weight_decay=0.0, lambda_abs=6.5, t_start=1000)
    oracle.adagc_step(th_b, g, m_b, v_b, gam_b, hp_b, 5)
    for x, y in zip(th_a + m_a + v_a, th_b + m_b + v_b):
        assert np.array_equal(x, y)
    assert list(m_a[0]) == [0.75, 1.0] and list(m_a[1]) == [3.0]
    # below the threshold nothing is clipped
    hp_a.lambda_abs = 13.0
    norms, coefs, clipped = oracle.adagc_step(th_a, g, m_a, v_a, gam_a, hp_a, 6)
    assert list(coefs) == [1.0, 1.0] and list(clipped) == [0, 0]


def test_global_adagc_on_one_tensor_is_adagc():
    """With a single tensor the model's norm is the tensor's norm: both modes must agree bit for bit,
    through the warm-up and after it."""
    rng = np.random.default_rng(20)
    n = 50
    def run(mode):
        r = np.random.default_rng(21)
        theta = [r.standard_normal(n).astype(np.float32)]
        m, v = [np.zeros(n, np.float32)], [np.zeros(n, np.float32)]
        gamma = np.zeros(1, np.float32)
        hp = Hyper(lambda_abs=0.9, t_start=3, clip_mode=mode)
        out = []
        for step in range(1, 12):
            scale = 10.0 if step in (2, 7) else (0.3 if step == 9 else 1.0)
            g = [(r.standard_normal(n) * 0.1 * scale).astype(np.float32)]
            out.append(oracle.adagc_step(theta, g, m, v, gamma, hp, step) + (gamma.copy(),))
        return theta, m, v, out
    a, b = run(oracle.MODE_ADAGC), run(oracle.MODE_GLOBAL_ADAGC)
    for x, y in zip(a[0] + a[1] + a[2], b[0] + b[1] + b[2]):
        assert np.array_equal(x, y)
    flags = []
    for (na, ca, fa, ga), (nb, cb, fb, gb) in zip(a[3], b[3]):
        assert na[0] == nb[0] and ca[0] == cb[0] and fa[0] == fb[0] and ga[0] == gb[0]
        flags.append(int(fa[0]))
    assert 0 < sum(flags) < len(flags)


def test_global_adagc_on_a_list_is_adagc_on_the_concatenation():
    rng = np.random.default_rng(22)
    sizes = [3, 17, 1, 40]
    hp_g = Hyper(t_start=0, clip_mode=oracle.MODE_GLOBAL_ADAGC)
    hp_t = Hyper(t_start=0)
    theta = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    m = [rng.standard_normal(n).astype(np.float32) * 0.01 for n in sizes]
    v = [(rng.standard_normal(n).astype(np.float32) * 0.01) ** 2 for n in sizes]
    g = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    cat = lambda xs: [np.concatenate(xs)]
    th_c, m_c, v_c, g_c = cat(theta), cat(m), cat(v), cat(g)
    gamma_g = np.array([0.5, 123.0, 456.0, 789.0], np.float32)      # only element 0 is the model's gamma
    gamma_c = np.array([0.5], np.float32)
    n_g, c_g, f_g = oracle.adagc_step(theta, g, m, v, gamma_g, hp_g, 4)
    n_c, c_c, f_c = oracle.adagc_step(th_c, g_c, m_c, v_c, gamma_c, hp_t, 4)
    assert f_c[0] == 1 and f_g.all()
    assert len(set(c_g.tolist())) == 1 and c_g[0] == pytest.approx(c_c[0], rel=1e-14)
    assert gamma_g[0] == gamma_c[0] and list(gamma_g[1:]) == [123.0, 456.0, 789.0]
    np.testing.assert_allclose(np.concatenate(theta), th_c[0], rtol=1e-6, atol=1e-9)
    np.testing.assert_allclose(np.concatenate(m), m_c[0], rtol=1e-6, atol=1e-9)
    # the model's clipped norm equals lambda_rel * gamma
    total = math.sqrt(sum(oracle.sum_squares(x) for x in g))
    assert c_g[0] * total == pytest.approx(f32(1.04) * 0.5, rel=1e-12)


def test_global_adagc_warmup_sets_then_minimises_the_single_gamma():
    theta, m, v = _lists([[0, 0], [0]]), _lists([[0, 0], [0]]), _lists([[0, 0], [0]])
    gamma = np.array([99.0, 55.0], np.float32)
    hp = Hyper(lr=0.0, lambda_abs=6.5, t_start=2, lambda_rel=2.0, ema_beta=0.5, clip_mode=oracle.MODE_GLOBAL_ADAGC)
    n, c, f = oracle.adagc_step(theta, _lists([[3, 4], [12]]), m, v, gamma, hp, 1)      # ||g|| = 13 -> h = 1/2
    assert list(c) == [0.5, 0.5] and list(gamma) == [6.5, 55.0]
    n, c, f = oracle.adagc_step(theta, _lists([[0, 3], [4]]), m, v, gamma, hp, 2)       # ||g|| = 5, no clip
    assert list(c) == [1.0, 1.0] and list(gamma) == [5.0, 55.0]
    n, c, f = oracle.adagc_step(theta, _lists([[6, 8], [0]]), m, v, gamma, hp, 3)       # Eq. 3: 10 = 2*5, tie
    assert list(c) == [1.0, 1.0] and list(f) == [0, 0] and gamma[0] == 7.5
    n, c, f = oracle.adagc_step(theta, _lists([[18, 24], [0]]), m, v, gamma, hp, 4)     # 30 > 15 -> h = 1/2
    assert list(c) == [0.5, 0.5] and list(f) == [1, 1] and gamma[0] == 0.5 * 7.5 + 0.5 * 15.0


def test_step_rejects_unknown_mode():
    theta, m, v = _lists([[1]]), _lists([[0]]), _lists([[0]])
    with pytest.raises(ValueError):
        oracle.adagc_step(theta, _lists([[1]]), m, v, np.zeros(1, np.float32), Hyper(clip_mode=99), 1)


# ------------------------------------------------------------------ state norms (Fig. 2 quantities)

def test_state_norms_hand_values_and_library():
    before = np.array([1.0, 1.0, 1.0], np.float32)
    after = np.array([4.0, 5.0, 1.0], np.float32)            # update (3, 4, 0)
    m = np.array([1.0, 2.0, 2.0], np.float32)
    v = np.array([0.0, 5.0, 12.0], np.float32)
    assert oracle.state_norms(before, after, m, v) == (3.0, 13.0, 5.0)
    assert oracle.state_norms(before, after, m) == (3.0, 0.0, 5.0)       # Lion keeps no second moment
    rng = np.random.default_rng(30)
    a, b, mm, vv = (rng.standard_normal(1000).astype(np.float32) for _ in range(4))
    got = oracle.state_norms(a, b, mm, vv)
    ref = (np.linalg.norm(mm.astype(np.float64)), np.linalg.norm(vv.astype(np.float64)),
           np.linalg.norm(b.astype(np.float64) - a.astype(np.float64)))
    assert got == pytest.approx(ref, rel=1e-13)
    assert oracle.state_norms(a, a, mm, vv)[2] == 0.0


def test_state_norms_after_first_adamw_step_closed_form():
    """m0 = v0 = 0, t = 1: ||m|| = (1-b1)||h g||, ||v|| = (1-b2)||(h g)^2||, and without weight decay
    every coordinate moves by about lr, so ||update|| ~ lr*sqrt(n)."""
    rng = np.random.default_rng(31)
    n = 400
    hp = Hyper(weight_decay=0.0, eps=0.0)
    g = (rng.standard_normal(n) * 0.3).astype(np.float32)
    theta = (rng.standard_normal(n) * 0.02).astype(np.float32)
    before = theta.copy()
    m, v = np.zeros(n, np.float32), np.zeros(n, np.float32)
    oracle.adamw_update(theta, m, v, g, 0.5, hp, 1)
    mn, vn, un = oracle.state_norms(before, theta, m, v)
    gd = 0.5 * g.astype(np.float64)
    assert mn == pytest.approx((1 - f32(0.9)) * np.linalg.norm(gd), rel=1e-6)
    assert vn == pytest.approx((1 - f32(0.95)) * np.linalg.norm(gd * gd), rel=1e-6)
    assert un == pytest.approx(f32(3e-4) * math.sqrt(n), rel=1e-4)


# ------------------------------------------------------------------ ZClip (Table 2; appendix "Clipping Hyper-Parameters")
# The paper prints the coefficient, tau and z; the adjustment function xi and the statistics' update are a
# reading (see oracle_zclip_rule): "parity unpinned by the paper" for those, pinned here by hand values,
# invariants and closed forms.

def test_zclip_paper_hyper_parameters():
    paper = golden()
    assert paper["zclip_alpha"] == 0.97 and paper["zclip_z_thres"] == 2.0
    assert oracle.Hyper().z_thres == paper["zclip_z_thres"]


def test_zclip_rule_hand_values_dyadic():
    # mu 4, sigma 1, norm 8: z = 4 > 2, xi = 2^2/4 = 1, tau = 5, h = 5/8; alpha 1/2: mu' = 4.5, var' = .5 + .5*(.5)^2
    assert oracle.zclip_rule(8.0, 4.0, 1.0, 0.5, 2.0) == (0.625, 4.5, 0.625, True)
    # norm 6: z = 2 is not above the threshold: no clip, the statistics take the raw norm
    assert oracle.zclip_rule(6.0, 4.0, 1.0, 0.5, 2.0) == (1.0, 5.0, 1.0, False)
    # sigma = 2 (var 4), mu 1, norm 17: z = 8, xi = 9/8 with z_thres 3, tau = 1 + 9/4 = 3.25, h = 3.25/17
    h, mu, var, c = oracle.zclip_rule(17.0, 1.0, 4.0, 0.75, 3.0)
    assert c and h == 3.25 / 17.0 and mu == 0.75 + 0.25 * 3.25 and var == 0.75 * 4.0 + 0.25 * (3.25 - mu) ** 2
    # a norm below the mean is never clipped
    assert oracle.zclip_rule(1.0, 4.0, 1.0, 0.5, 2.0)[::3] == (1.0, False)


def test_zclip_threshold_as_table_2_prints_it():
    """tau = mu + xi(z) sigma with z = (norm - mu)/sigma and h = min{1, tau/norm}; with the reciprocal xi,
    tau lies strictly between the mean and the activation boundary mu + z_thres sigma, falls as the norm
    grows, and meets the norm at the boundary (h continuous)."""
    rng = np.random.default_rng(21)
    for _ in range(300):
        mu, sigma, zt = rng.uniform(0.1, 10), rng.uniform(0.01, 3), rng.uniform(0.5, 4)
        norm = mu + sigma * zt * rng.uniform(1.0001, 30)
        h, mu_new, var_new, c = oracle.zclip_rule(norm, mu, sigma * sigma, 0.97, zt)
        assert c and 0.0 < h < 1.0
        tau = h * norm
        z = (norm - mu) / sigma
        assert abs(tau - (mu + zt * zt / z * sigma)) <= 1e-12 * tau
        assert mu < tau < mu + zt * sigma < norm
        h2 = oracle.zclip_rule(norm * 1.5, mu, sigma * sigma, 0.97, zt)[0]
        assert h2 * norm * 1.5 < tau                       # further out, lower threshold
        assert abs(mu_new - (0.97 * mu + 0.03 * tau)) <= 1e-12 * mu_new          # statistics take the clipped norm
    # continuity at the boundary, from above
    h = oracle.zclip_rule(4.0 + 2.0 * (1 + 1e-9), 4.0, 1.0, 0.97, 2.0)[0]
    assert 1.0 - 1e-8 < h < 1.0


def test_zclip_scale_invariance():
    for c in (0.125, 8.0, 1024.0):
        a = oracle.zclip_rule(9.0, 3.0, 2.25, 0.75, 2.0)
        b = oracle.zclip_rule(9.0 * c, 3.0 * c, 2.25 * c * c, 0.75, 2.0)
        assert a[0] == b[0] and a[3] == b[3] and b[1] == a[1] * c and b[2] == a[2] * c * c


def test_zclip_zero_variance_needs_no_special_case():
    assert oracle.zclip_rule(6.0, 4.0, 0.0, 0.5, 2.0) == (4.0 / 6.0, 4.0, 0.0, True)      # tau = mu
    assert oracle.zclip_rule(4.0, 4.0, 0.0, 0.5, 2.0) == (1.0, 4.0, 0.0, False)            # z = 0/0
    assert oracle.zclip_rule(3.0, 4.0, 0.0, 0.5, 2.0) == (1.0, 3.5, 0.125, False)
    h, mu, var, c = oracle.zclip_rule(float("nan"), 4.0, 1.0, 0.5, 2.0)
    assert h == 1.0 and not c and math.isnan(mu)


def test_zclip_statistics_are_exponential_moving_mean_and_variance():
    """Never clipped (z_thres = inf): mu_k = a^k mu_0 + (1-a) sum a^(k-j) n_j, and the variance follows
    var_k = a var_{k-1} + (1-a)(n_k - mu_k)^2, in exact rationals on dyadic inputs."""
    from fractions import Fraction as F
    a = F(3, 4)
    norms = [F(5), F(3, 2), F(9, 4), F(7), F(1, 8), F(33, 16)]
    mu, var = F(2), F(1, 4)
    fmu, fvar = float(mu), float(var)
    for k, n in enumerate(norms):
        mu = a * mu + (1 - a) * n
        var = a * var + (1 - a) * (n - mu) ** 2
        h, fmu, fvar, c = oracle.zclip_rule(float(n), fmu, fvar, float(a), float("inf"))
        assert h == 1.0 and not c
        assert fmu == float(mu) and fvar == float(var)
    closed = a ** len(norms) * F(2) + (1 - a) * sum(a ** (len(norms) - 1 - j) * n for j, n in enumerate(norms))
    assert mu == closed
    # the mean is the library's exponentially weighted mean (adjust=False) of the same sequence
    import pandas as pd
    ew = pd.Series([2.0] + [float(n) for n in norms]).ewm(alpha=float(1 - a), adjust=False).mean().iloc[-1]
    assert abs(ew - fmu) <= 1e-15 * fmu
    # a constant norm: the mean converges to it geometrically and the variance decays
    mu_c, var_c = 1.0, 1.0
    for k in range(1, 60):
        _, mu_c, var_c, _ = oracle.zclip_rule(3.0, mu_c, var_c, 0.5, float("inf"))
        assert abs(mu_c - (3.0 - 2.0 * 0.5 ** k)) <= 1e-15
    assert var_c < 1e-15


def test_zclip_gather():
    assert oracle.zclip_gather(5.0, 123.0, 456.0, 0.5, True) == (5.0, 0.0)             # first step: set
    assert oracle.zclip_gather(7.0, 5.0, 0.0, 0.5, False) == (6.0, 0.5)                # then the same EMA
    assert oracle.zclip_gather(7.0, 5.0, 0.0, 0.5, False) == oracle.zclip_rule(7.0, 5.0, 0.0, 0.5, float("inf"))[1:3]


def test_zclip_step_hand_worked():
    """[3,4] and [12]: global norm 13.  mu 5, var 4 (sigma 2), z_thres 2: z = 4, xi = 1, tau = 7, h = 7/13 for
    every tensor; alpha 1/2: mu' = 6, var' = 2 + .5*1 = 2.5.  The update is plain AdamW on h*g."""
    theta = [np.array([1.0, -1.0], np.float32), np.array([0.5], np.float32)]
    g = [np.array([3.0, 4.0], np.float32), np.array([12.0], np.float32)]
    hp = oracle.Hyper(clip_mode=oracle.MODE_ZCLIP, ema_beta=0.5, z_thres=2.0, t_start=0)
    m, v = _lists([np.zeros(2), np.zeros(1)]), _lists([np.zeros(2), np.zeros(1)])
    state = np.array([5.0, 4.0], np.float32)
    th = [x.copy() for x in theta]
    norms, coefs, clipped = oracle.adagc_step(th, g, m, v, state, hp, 3)
    assert norms.tolist() == [5.0, 12.0] and clipped.tolist() == [1, 1]
    assert coefs.tolist() == [7.0 / 13.0, 7.0 / 13.0]
    assert state.tolist() == [6.0, 2.5]
    for i in range(2):
        t2, m2, v2 = theta[i].copy(), np.zeros_like(theta[i]), np.zeros_like(theta[i])
        oracle.adamw_update(t2, m2, v2, g[i], 7.0 / 13.0, hp, 3)
        assert np.array_equal(t2, th[i]) and np.array_equal(m2, m[i]) and np.array_equal(v2, v[i])
    # an ordinary step (z = 0.5): nothing clipped, statistics move
    state = np.array([12.0, 4.0], np.float32)
    norms, coefs, clipped = oracle.adagc_step(th, g, m, v, state, hp, 4)
    assert coefs.tolist() == [1.0, 1.0] and clipped.tolist() == [0, 0]
    assert state.tolist() == [12.5, 2.0 + 0.5 * 0.25]


def test_zclip_step_gathers_statistics_under_globalgc_first():
    """Steps 1..t_start: Eq. 2's coefficient, and the statistics gathered from the globally clipped norm
    (set on step 1, moving averages afterwards); the z-score rule starts on step t_start + 1."""
    g = [np.array([3.0, 4.0], np.float32), np.array([12.0], np.float32)]
    hp = oracle.Hyper(clip_mode=oracle.MODE_ZCLIP, ema_beta=0.5, z_thres=2.0, t_start=2, lambda_abs=6.5)
    th, m, v = _lists([np.ones(2), np.ones(1)]), _lists([np.zeros(2), np.zeros(1)]), _lists([np.zeros(2), np.zeros(1)])
    state = np.array([99.0, 99.0], np.float32)
    _, coefs, clipped = oracle.adagc_step(th, g, m, v, state, hp, 1)
    assert coefs.tolist() == [0.5, 0.5] and clipped.tolist() == [1, 1] and state.tolist() == [6.5, 0.0]
    g2 = [x * np.float32(0.5) for x in g]                 # norm 6.5: not clipped by lambda_abs = 6.5
    _, coefs, clipped = oracle.adagc_step(th, g2, m, v, state, hp, 2)
    assert coefs.tolist() == [1.0, 1.0] and state.tolist() == [6.5, 0.0]
    _, coefs, clipped = oracle.adagc_step(th, g, m, v, state, hp, 3)   # z = +inf: tau = mu
    assert coefs.tolist() == [0.5, 0.5] and clipped.tolist() == [1, 1] and state.tolist() == [6.5, 0.0]


def test_zclip_on_a_list_sees_only_the_global_norm():
    rng = np.random.default_rng(8)
    parts = [rng.standard_normal(n).astype(np.float32) for n in (5, 1, 9)]
    whole = [np.concatenate(parts)]
    hp = oracle.Hyper(clip_mode=oracle.MODE_ZCLIP, t_start=0, ema_beta=0.97)
    s1, s2 = np.array([1.0, 0.04], np.float32), np.array([1.0, 0.04], np.float32)
    a = oracle.adagc_step(_lists([np.zeros(5), np.zeros(1), np.zeros(9)]), parts, _lists([np.zeros(5), np.zeros(1), np.zeros(9)]),
                          _lists([np.zeros(5), np.zeros(1), np.zeros(9)]), np.concatenate([s1, [0]]).astype(np.float32), hp, 2)
    b = oracle.adagc_step(_lists([np.zeros(15)]), whole, _lists([np.zeros(15)]), _lists([np.zeros(15)]), s2, hp, 2)
    assert a[1][0] == a[1][1] == a[1][2] == b[1][0] and b[2][0] == 1


# ------------------------------------------------------------------ AGC and Clippy (Table 2; update clipping)
# Table 2 prints both coefficients; what Delta is, which theta enters and what a unit is are readings
# (see oracle_agc_coef): pinned here by hand values, invariants and a cross-check of the direction's norms
# against the update routine.

def test_update_clipping_paper_hyper_parameters():
    paper = golden()
    assert paper["agc_lambda_rel"] == 1e-3 and paper["clippy_lambda_abs"] == 0.5 and paper["clippy_lambda_rel"] == 1e-2


def test_agc_coef_hand_values_and_invariant():
    assert oracle.agc_coef(10.0, 5.0, 0.25) == (0.5, True)        # 0.25*10/5
    assert oracle.agc_coef(10.0, 2.0, 0.25) == (1.0, False)       # ratio 1.25
    assert oracle.agc_coef(8.0, 2.0, 0.25) == (1.0, False)        # ratio exactly 1: not clipped
    assert oracle.agc_coef(10.0, 0.0, 0.25) == (1.0, False)       # no update to clip
    assert oracle.agc_coef(0.0, 0.0, 0.25) == (1.0, False)        # 0/0
    assert oracle.agc_coef(0.0, 3.0, 0.25) == (0.0, True)         # no floor on ||theta||: literal
    rng = np.random.default_rng(4)
    for _ in range(200):
        th, d, lam = rng.uniform(0.01, 50), rng.uniform(0.01, 50), rng.uniform(1e-4, 2)
        c, clipped = oracle.agc_coef(th, d, lam)
        assert 0.0 < c <= 1.0 and clipped == (lam * th < d)
        assert c * d <= lam * th * (1 + 1e-15) or not clipped     # ||c Delta|| <= lambda ||theta||
        if clipped:
            assert abs(c * d - lam * th) <= 1e-15 * lam * th
        assert oracle.agc_coef(th * 8, d * 8, lam) == (c, clipped)    # scale invariant


def test_clippy_coef_hand_values_and_invariant():
    assert oracle.clippy_coef(2.0, 8.0, 0.5, 1.0, 0.5) == (0.5, True)        # (0.5*2+1)/(0.5*8)
    assert oracle.clippy_coef(2.0, 4.0, 0.5, 1.0, 0.5) == (1.0, False)       # ratio exactly 1
    assert oracle.clippy_coef(2.0, 1.0, 0.5, 1.0, 0.5) == (1.0, False)
    assert oracle.clippy_coef(0.0, 8.0, 0.5, 1.0, 0.5) == (0.25, True)       # the absolute term keeps zeros moving
    assert oracle.clippy_coef(2.0, 0.0, 0.5, 1.0, 0.5) == (1.0, False)
    rng = np.random.default_rng(5)
    for _ in range(200):
        th, d = rng.uniform(0, 5), rng.uniform(0.01, 50)
        lr, lam, ab = rng.uniform(1e-4, 1), rng.uniform(1e-4, 1), rng.uniform(0.01, 1)
        c, clipped = oracle.clippy_coef(th, d, lam, ab, lr)
        assert 0.0 < c <= 1.0
        assert lr * c * d <= (lam * th + ab) * (1 + 1e-15)          # the largest step stays within the budget
        if clipped:
            assert abs(lr * c * d - (lam * th + ab)) <= 1e-15 * (lam * th + ab)


def test_direction_norms_hand_worked_and_against_the_update_routine():
    # step 1 from zero moments with eps = 0: Delta = g/|g| = sign(g)
    hp = Hyper(lr=0.25, beta1=0.5, beta2=0.75, eps=0.0, weight_decay=0.0)
    theta = np.array([3.0, -4.0, 0.0, 0.0], np.float32)
    g = np.array([1.0, -2.0, 0.5, 8.0], np.float32)
    z = np.zeros(4, np.float32)
    assert oracle.direction_norms(theta, z, z, g, hp, 1) == (5.0, 2.0, 4.0, 1.0)
    # general case: the direction is what the update routine applies; recover it with lr = 1, wd = 0, theta = 0
    rng = np.random.default_rng(17)
    n = 4000
    m = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    v = ((rng.standard_normal(n) * 1e-2) ** 2).astype(np.float32)
    g = (rng.standard_normal(n) * 3e-2).astype(np.float32)
    theta = (rng.standard_normal(n) * 0.02).astype(np.float32)
    hp = Hyper(lr=1.0, weight_decay=0.0, eps=1e-8)
    t0, m2, v2 = np.zeros(n, np.float32), m.copy(), v.copy()
    oracle.adamw_update(t0, m2, v2, g, 1.0, hp, 7)
    delta = -t0.astype(np.float64)                                  # fp32-rounded direction
    th2, d2, thinf, dinf = oracle.direction_norms(theta, m, v, g, hp, 7)
    assert abs(d2 - np.linalg.norm(delta)) <= 1e-6 * d2 and abs(dinf - np.abs(delta).max()) <= 1e-6 * dinf
    assert abs(th2 - np.linalg.norm(theta.astype(np.float64))) <= 1e-14 * th2
    assert thinf == float(np.abs(theta).max())
    # Lion: the direction is the sign of the interpolation
    hpl = Hyper(beta1=0.5, beta2=0.75, optimizer=oracle.LION)
    m = np.array([1.0, -1.0, 2.0, 0.0, 0.0], np.float32)
    g = np.array([1.0, 1.0, -1.0, 0.0, -3.0], np.float32)          # c = 1, 0, .5, 0, -1.5
    th = np.array([0.5, 0.5, 0.5, 0.5, -2.0], np.float32)
    assert oracle.direction_norms(th, m, None, g, hpl, 3) == (math.sqrt(5.0), math.sqrt(3.0), 2.0, 1.0)


def test_update_clipped_scales_the_direction_only():
    """lr 1/4, beta1 1/2, beta2 3/4, eps 0, step 1: Delta = sign(g).  With coefficient 1/2 the parameter
    moves by lr/2; the moments are those of the unclipped gradient; weight decay is applied in full."""
    hp = Hyper(lr=0.25, beta1=0.5, beta2=0.75, eps=0.0, weight_decay=0.0)
    theta = np.array([3.0, -4.0, 1.0], np.float32)
    g = np.array([2.0, -6.0, 0.5], np.float32)
    th, m, v = theta.copy(), np.zeros(3, np.float32), np.zeros(3, np.float32)
    oracle.adamw_update_clipped(th, m, v, g, 0.5, hp, 1)
    assert th.tolist() == [3.0 - 0.125, -4.0 + 0.125, 1.0 - 0.125]
    assert m.tolist() == [1.0, -3.0, 0.25] and v.tolist() == [1.0, 9.0, 0.0625]
    hpw = Hyper(lr=0.25, beta1=0.5, beta2=0.75, eps=0.0, weight_decay=0.5)
    th = theta.copy()
    oracle.adamw_update_clipped(th, np.zeros(3, np.float32), np.zeros(3, np.float32), g, 0.5, hpw, 1)
    assert th.tolist() == [3.0 - 0.375 - 0.125, -4.0 + 0.5 + 0.125, 1.0 - 0.125 - 0.125]
    # coefficient 1 is the plain step, bit for bit
    rng = np.random.default_rng(2)
    a = [(rng.standard_normal(500) * s).astype(np.float32) for s in (0.02, 1e-3, 1e-3, 1e-2)]
    a[2] = a[2] ** 2
    p1, m1, v1 = a[0].copy(), a[1].copy(), a[2].copy()
    p2, m2, v2 = a[0].copy(), a[1].copy(), a[2].copy()
    oracle.adamw_update(p1, m1, v1, a[3], 1.0, Hyper(), 9)
    oracle.adamw_update_clipped(p2, m2, v2, a[3], 1.0, Hyper(), 9)
    assert np.array_equal(p1, p2) and np.array_equal(m1, m2) and np.array_equal(v1, v2)
    # Lion: theta -= lr (coef*sign(c) + wd*theta); momentum from the unclipped gradient
    hpl = Hyper(lr=0.25, beta1=0.5, beta2=0.75, weight_decay=0.5, optimizer=oracle.LION)
    th, m = np.array([8.0, -2.0], np.float32), np.array([1.0, 1.0], np.float32)
    oracle.lion_update_clipped(th, m, np.array([1.0, -3.0], np.float32), 0.5, hpl)
    assert th.tolist() == [8.0 - 0.25 * (0.5 + 4.0), -2.0 - 0.25 * (-0.5 - 1.0)]
    assert m.tolist() == [0.75 + 0.25, 0.75 - 0.75]


def test_agc_and_clippy_steps_hand_worked():
    """theta [3,4,0,0] (l2 5, l-inf 4) and [0,0]; first step, eps 0: Delta is the sign of g.
    AGC, lambda_rel 0.2: ratios 0.2*5/2 = 0.5 and 0 -> the first tensor moves by lr/2, the second not at all.
    Clippy, lambda_rel 1/16, lambda_abs 1/4, lr 1: ratios (0.25+0.25)/1 = 0.5 and 0.25."""
    def fresh():
        return (_lists([[3, 4, 0, 0], [0, 0]]), _lists([[0] * 4, [0] * 2]), _lists([[0] * 4, [0] * 2]))
    g = _lists([[1, -2, 0.5, 8], [4, -4]])
    gamma = np.array([7.0, 9.0], np.float32)
    th, m, v = fresh()
    hp = Hyper(lr=0.25, beta1=0.5, beta2=0.75, eps=0.0, weight_decay=0.0, lambda_rel=0.2, clip_mode=oracle.MODE_AGC)
    norms, coefs, clipped = oracle.adagc_step(th, g, m, v, gamma, hp, 1)
    assert norms.tolist() == [2.0, math.sqrt(2.0)]                  # reported: the direction's l2 norm
    assert coefs.tolist() == [f32(0.2) * 5.0 / 2.0, 0.0] and clipped.tolist() == [1, 1]
    c = f32(0.2) * 5.0 / 2.0
    np.testing.assert_array_equal(th[0], np.array([3 - 0.25 * c, 4 + 0.25 * c, -0.25 * c, -0.25 * c], np.float32))
    assert th[1].tolist() == [0.0, 0.0]
    assert m[0].tolist() == [0.5, -1.0, 0.25, 4.0] and m[1].tolist() == [2.0, -2.0]      # unclipped gradient
    assert gamma.tolist() == [7.0, 9.0]                              # no state
    th, m, v = fresh()
    hp = Hyper(lr=1.0, beta1=0.5, beta2=0.75, eps=0.0, weight_decay=0.0, lambda_rel=0.0625, lambda_abs=0.25,
               clip_mode=oracle.MODE_CLIPPY)
    norms, coefs, clipped = oracle.adagc_step(th, g, m, v, gamma, hp, 1)
    assert norms.tolist() == [1.0, 1.0] and coefs.tolist() == [0.5, 0.25] and clipped.tolist() == [1, 1]
    assert th[0].tolist() == [2.5, 4.5, -0.5, -0.5] and th[1].tolist() == [-0.25, 0.25]
    # generous thresholds: nothing is clipped and the step is plain AdamW
    th, m, v = fresh()
    th2, m2, v2 = fresh()
    hp = Hyper(lambda_rel=1e6, clip_mode=oracle.MODE_AGC, t_start=0)
    th[1][:] = 1.0
    th2[1][:] = 1.0
    _, coefs, clipped = oracle.adagc_step(th, g, m, v, gamma, hp, 4)
    oracle.adagc_step(th2, g, m2, v2, gamma.copy(), Hyper(lambda_rel=float("inf"), t_start=0), 4)
    assert coefs.tolist() == [1.0, 1.0] and clipped.tolist() == [0, 0]
    for x, y in zip(th + m + v, th2 + m2 + v2):
        assert np.array_equal(x, y)
