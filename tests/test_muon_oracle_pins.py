"""Pins of the Muon oracle (oracle/muon.py).  The paper prints no Muon rule ("parity unpinned by the paper");
the published algorithm written out there is pinned to the mathematics: the exact Newton-Schulz iteration is an
odd polynomial acting on the singular values (checked through the library's SVD), its fixed-point region, the
invariances of the iteration, the bf16 rounding against the library cast, hand-worked momentum steps."""
import importlib.util
import math
import os

import numpy as np
import torch

import oracle
from oracle import muon as M

if os.environ.get("ADAGC_MUON_ORACLE_SRC"):
    # tests/test_muon_pins_catch_planted_mistakes.py runs this file against altered copies of the oracle's source
    _spec = importlib.util.spec_from_file_location("muon_under_test", os.environ["ADAGC_MUON_ORACLE_SRC"])
    M = importlib.util.module_from_spec(_spec)
    _spec.loader.exec_module(M)


def test_bf16_rounding_matches_the_library_cast():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-30, 30, 20000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.001953125, 1.005859375, np.inf, -np.inf, 3.3895314e38])])
    ref = torch.from_numpy(x).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(M.to_bf16(x), ref)
    assert np.isnan(M.to_bf16(np.array([np.nan]))[0])
    bits = M.bf16_bits(M.to_bf16(x[:1000]))
    back = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.array_equal(back, M.to_bf16(x[:1000]))


def test_exact_iteration_is_the_polynomial_on_the_singular_values():
    rng = np.random.default_rng(1)
    for shape in [(6, 6), (5, 9), (9, 5), (1, 7), (16, 40)]:
        u = rng.standard_normal(shape)
        uu, s, vt = np.linalg.svd(u, full_matrices=False)
        s0 = s / (np.linalg.norm(u) + M.NS_EPS)
        closed = (uu * M.ns_scalar_map(s0)) @ vt
        got = M.newton_schulz(u, storage="exact")
        assert np.abs(got - closed).max() <= 1e-12 * max(1.0, np.abs(closed).max()), shape
        # one step, by hand: a X + b (X X^T) X + c (X X^T)^2 X
        x = u / (np.linalg.norm(u) + M.NS_EPS)
        if shape[0] > shape[1]:
            x = x.T
        g = x @ x.T
        a, b, c = M.NS_COEFFS
        one = a * x + b * g @ x + c * g @ g @ x
        got1 = M.newton_schulz(u, steps=1, storage="exact")
        got1 = got1.T if shape[0] > shape[1] else got1
        assert np.abs(got1 - one).max() <= 1e-14


def test_singular_values_end_near_one():
    """Five steps take every singular value above ~1e-2 of the Frobenius norm into [0.68, 1.14]: the published
    coefficients trade exactness for speed.  Checked on the scalar map and on matrices, bf16 storage included."""
    s = M.ns_scalar_map(np.linspace(0.02, 1.0, 2000))
    assert s.min() > 0.66 and s.max() < 1.14
    assert abs(M.ns_scalar_map(1e-6) / 1e-6 - M.NS_COEFFS[0] ** 5) < 1e-3 * M.NS_COEFFS[0] ** 5     # tiny values grow by a^5
    rng = np.random.default_rng(2)
    for shape, storage in [((32, 32), "bf16"), ((24, 80), "bf16"), ((80, 24), "bf16"), ((24, 80), "exact")]:
        o = M.newton_schulz(rng.standard_normal(shape), storage=storage)
        sv = np.linalg.svd(o, compute_uv=False)
        assert sv.max() < 1.2 and sv.min() > 0.3, (shape, storage, sv.min(), sv.max())


def test_iteration_invariances():
    rng = np.random.default_rng(3)
    u = rng.standard_normal((12, 20))
    for storage in ("exact", "bf16"):
        o = M.newton_schulz(u, storage=storage)
        assert np.array_equal(M.newton_schulz(u.T, storage=storage), o.T)            # tall matrices run transposed
        assert np.array_equal(M.newton_schulz(-u, storage=storage), -o)              # odd map
    o = M.newton_schulz(u, storage="exact")
    assert np.abs(M.newton_schulz(64.0 * u, storage="exact") - o).max() < 1e-7       # scale goes away (up to the 1e-7 guard)
    q, _ = np.linalg.qr(rng.standard_normal((12, 12)))
    assert np.abs(M.newton_schulz(q @ u, storage="exact") - q @ o).max() < 1e-12     # rotations pass through
    # bf16 storage stays close to the exact iteration (its perturbations are ~2^-9 per stored value)
    ob = M.newton_schulz(u, storage="bf16")
    assert np.abs(ob - o).max() < 0.05 and np.sqrt(np.mean((ob - o) ** 2)) < 0.02


def test_stored_intermediates_are_bf16_values_in_the_stated_order():
    rng = np.random.default_rng(4)
    trace = []
    M.newton_schulz(rng.standard_normal((8, 8)), steps=2, trace=trace)
    assert [n for n, _ in trace] == ["X0", "A1", "B1", "X1", "A2", "B2", "X2"]
    for name, mat in trace:
        assert np.array_equal(M.to_bf16(mat), mat), name
    x0, a1, b1, x1 = (trace[i][1] for i in range(4))
    a, b, c = M.NS_COEFFS
    assert np.array_equal(a1, M.to_bf16(x0 @ x0.T))
    assert np.array_equal(b1, M.to_bf16(b * a1 + c * (a1 @ a1)))
    assert np.array_equal(x1, M.to_bf16(a * x0 + b1 @ x0))


def test_update_scale():
    assert M.update_scale(4, 16) == 1.0 and M.update_scale(16, 16) == 1.0 and M.update_scale(64, 16) == 2.0


def test_muon_update_hand_worked():
    """mu 1/2, coefficient 1/2, g = [[4, 0], [0, 8]], M = [[2, 0], [0, -4]]:
    ghat = [[2,0],[0,4]], M' = [[3,0],[0,2]], Nesterov U = ghat + M'/2 = [[3.5,0],[0,5]] (diagonal: the iteration
    acts on each entry as the scalar map); plain momentum U = M'."""
    g = np.array([[4.0, 0.0], [0.0, 8.0]], np.float32)
    for nesterov, diag in ((True, [3.5, 5.0]), (False, [3.0, 2.0])):
        theta = np.array([[1.0, 2.0], [3.0, 4.0]], np.float32)
        mom = np.array([[2.0, 0.0], [0.0, -4.0]], np.float32)
        o = M.muon_update(theta, g, mom, 0.5, lr=0.25, weight_decay=0.5, mu=0.5, nesterov=nesterov, storage="exact")
        assert mom.tolist() == [[3.0, 0.0], [0.0, 2.0]]
        nrm = math.hypot(*diag) + M.NS_EPS
        want = np.diag(M.ns_scalar_map(np.array(diag) / nrm))
        assert np.abs(o - want).max() < 1e-14
        th0 = np.array([[1.0, 2.0], [3.0, 4.0]])
        np.testing.assert_array_equal(theta, (th0 - 0.25 * (0.5 * th0 + want)).astype(np.float32))
    # the clip coefficient enters before the momentum: h = 0 leaves only the decayed momentum
    theta = np.ones((2, 2), np.float32)
    mom = np.array([[2.0, 0.0], [0.0, -4.0]], np.float32)
    M.muon_update(theta, g, mom, 0.0, lr=0.25, weight_decay=0.0, mu=0.5, storage="exact")
    assert mom.tolist() == [[1.0, 0.0], [0.0, -2.0]]
    # tall matrices are scaled by sqrt(rows/cols)
    rng = np.random.default_rng(5)
    gt = rng.standard_normal((8, 2)).astype(np.float32)
    th, mo = np.zeros((8, 2), np.float32), np.zeros((8, 2), np.float32)
    o = M.muon_update(th, gt, mo, 1.0, lr=1.0, weight_decay=0.0, mu=0.0, storage="exact")
    np.testing.assert_allclose(th, (-2.0 * o).astype(np.float32), rtol=0, atol=0)


def test_coefficients_are_the_published_ones():
    """(a, b, c) and the guard are constants of the published algorithm (the paper prints none of them): kept as a
    text fixture with its citation, and checked for what the publication says of them: slope a at zero, and a band
    around one that five steps reach from 0.02 upwards."""
    vals = {}
    for line in open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "muon_published.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            vals[k.strip()] = float(v)
    assert M.NS_COEFFS == (vals["ns_a"], vals["ns_b"], vals["ns_c"]) and M.NS_EPS == vals["ns_eps"]
    a, b, c = M.NS_COEFFS
    one_step = lambda s: a * s + b * s ** 3 + c * s ** 5
    assert abs(one_step(1e-9) / 1e-9 - a) < 1e-6
    assert abs(one_step(1.0) - (a + b + c)) < 1e-15 and 0.69 < a + b + c < 0.71
