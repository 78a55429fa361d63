"""The all-cores build of the oracle (the same C source compiled with -fopenmp) against the one-thread
build, which stays the definition.  Only after this holds may the all-cores build stand in for it where
billions of parameters have to be replayed.

What must hold: theta, m, v and the bf16 copies are computed element by element with the same
statements, so they are bit-identical; a sum of squares is the same sum in another rounding order
(one contiguous block per thread, block sums added in block order), so norms, coefficients and gamma
agree to the rounding error of a double sum over N terms (~sqrt(N) * 1.1e-16; 1e-12 is asserted),
and clip decisions are identical away from the threshold.
"""
import numpy as np
import pytest

import oracle

SUM_RTOL = 1e-12


def _case(seed, numels, bf16=False, lion=False):
    rng = np.random.default_rng(seed)
    theta = [(rng.standard_normal(n) * 0.02).astype(np.float32) for n in numels]
    m = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for n in numels]
    v = None if lion else [(rng.standard_normal(n) * 1e-3).astype(np.float32) ** 2 for n in numels]
    sig = np.exp(rng.uniform(np.log(1e-4), np.log(1e-1), len(numels)))
    g = [(rng.standard_normal(n) * s).astype(np.float32) for n, s in zip(numels, sig)]
    if bf16:
        g = [(x.view(np.uint32) >> 16).astype(np.uint16) for x in g]
    copies = [np.zeros(n, np.uint16) for n in numels]
    gamma = np.array([oracle.l2_norm(x) for x in g], np.float32)
    gamma[::2] *= np.float32(0.5)            # every other tensor clips
    return theta, g, m, v, gamma, copies


def _clone(case):
    return tuple(None if part is None else ([a.copy() for a in part] if isinstance(part, list) else part.copy())
                 for part in case)


NUMELS = [1, 2, 3, 7, 17, 1000, 4097, 65536, 300001, 1 << 20]


def test_all_cores_build_really_uses_several_threads():
    assert oracle.num_threads() == 1
    with oracle.all_cores():
        assert oracle.num_threads() >= 1      # a one-core host is allowed; the box that needs it has many
    assert oracle.num_threads() == 1


@pytest.mark.parametrize("bf16", [False, True])
def test_sum_of_squares_same_sum_in_another_order(bf16):
    rng = np.random.default_rng(5)
    for n in [1, 2, 5, 8, 9, 63, 1000, 1 << 20, 3_000_017]:
        g = (rng.standard_normal(n) * 3e-3).astype(np.float32)
        if bf16:
            g = (g.view(np.uint32) >> 16).astype(np.uint16)
        one = oracle.sum_squares(g)
        with oracle.all_cores():
            many = oracle.sum_squares(g)
        assert abs(many - one) <= SUM_RTOL * one, (n, one, many)
    ones = np.ones(1 << 22, np.float32)      # exact in any order
    with oracle.all_cores():
        assert oracle.sum_squares(ones) == float(1 << 22)


@pytest.mark.parametrize("lion,bf16,mode,t_start,step", [
    (False, False, oracle.MODE_ADAGC, 1, 5),
    (False, True, oracle.MODE_ADAGC, 1, 2),
    (True, True, oracle.MODE_ADAGC, 1, 3),
    (True, False, oracle.MODE_ADAGC, 1, 3),
    (False, False, oracle.MODE_ADAGC, 100, 7),         # warm-up branch
    (False, False, oracle.MODE_GLOBALGC, 0, 4),
    (False, False, oracle.MODE_GLOBAL_ADAGC, 2, 9),
])
def test_step_is_bit_identical_in_state_and_close_in_norms(lion, bf16, mode, t_start, step):
    case = _case(11, NUMELS, bf16=bf16, lion=lion)
    hp = oracle.Hyper(optimizer=oracle.LION if lion else oracle.ADAMW,
                      grad_dtype=oracle.GRAD_BF16 if bf16 else oracle.GRAD_F32, clip_mode=mode, t_start=t_start,
                      lambda_abs=0.05 if (mode or t_start > 1) else float("inf"))
    a = _clone(case)
    b = _clone(case)
    na, ca, fa = oracle.adagc_step(a[0], a[1], a[2], a[3], a[4], hp, step, a[5])
    with oracle.all_cores():
        nb, cb, fb = oracle.adagc_step(b[0], b[1], b[2], b[3], b[4], hp, step, b[5])
    np.testing.assert_allclose(nb, na, rtol=SUM_RTOL, atol=0)
    np.testing.assert_array_equal(fb, fa)
    np.testing.assert_allclose(cb, ca, rtol=4 * SUM_RTOL, atol=0)
    np.testing.assert_allclose(b[4].astype(np.float64), a[4].astype(np.float64), rtol=1.2e-7, atol=0)   # <= 1 fp32 ulp
    # with the coefficient held equal the elementwise statements are the same: replay with the one-thread h
    for i, n in enumerate(NUMELS):
        th1, m1 = case[0][i].copy(), case[2][i].copy()
        th2, m2 = case[0][i].copy(), case[2][i].copy()
        c1, c2 = np.zeros(n, np.uint16), np.zeros(n, np.uint16)
        if lion:
            oracle.lion_update(th1, m1, case[1][i], ca[i], hp, c1)
            with oracle.all_cores():
                oracle.lion_update(th2, m2, case[1][i], ca[i], hp, c2)
        else:
            v1, v2 = case[3][i].copy(), case[3][i].copy()
            oracle.adamw_update(th1, m1, v1, case[1][i], ca[i], hp, step, c1)
            with oracle.all_cores():
                oracle.adamw_update(th2, m2, v2, case[1][i], ca[i], hp, step, c2)
            assert np.array_equal(v1.view(np.uint32), v2.view(np.uint32))
        assert np.array_equal(th1.view(np.uint32), th2.view(np.uint32))
        assert np.array_equal(m1.view(np.uint32), m2.view(np.uint32))
        assert np.array_equal(c1, c2)


def test_unclipped_step_is_bit_identical_end_to_end():
    """h = 1 exactly on both builds when nothing clips, so the whole step must agree bit for bit."""
    case = _case(3, NUMELS)
    case[4][:] = np.float32(1e6)             # thresholds far above every norm
    hp = oracle.Hyper(t_start=0)
    a, b = _clone(case), _clone(case)
    oracle.adagc_step(a[0], a[1], a[2], a[3], a[4], hp, 6, a[5])
    with oracle.all_cores():
        oracle.adagc_step(b[0], b[1], b[2], b[3], b[4], hp, 6, b[5])
    for k in (0, 2, 3, 5):
        for x, y in zip(a[k], b[k]):
            assert np.array_equal(x.view(np.uint8), y.view(np.uint8))
