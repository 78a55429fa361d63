"""GPU parity of the Muon path against the numpy oracle (oracle/muon.py), through the C ABI."""
import math

import numpy as np
import pytest
import torch

from oracle import muon as OM
from paper_2502_11034_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


def bf16_dev(x64, ld=None):
    """float64 host matrix of bf16-representable values -> bf16 device matrix, optionally inside wider rows."""
    t = torch.from_numpy(np.ascontiguousarray(x64, dtype=np.float32)).to(torch.bfloat16)
    if ld is None:
        return t.to(DEV)
    buf = torch.full((x64.shape[0], ld), float("nan"), dtype=torch.bfloat16, device=DEV)   # the padding is never read
    buf[:, :x64.shape[1]] = t.to(DEV)
    return buf[:, :x64.shape[1]]


def host64(t):
    return t.to(torch.float32).cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("M,N,K,ld_extra", [(128, 128, 128, 0), (256, 384, 384, 8), (128, 512, 1024, 64), (1024, 1024, 4096, 0),
                                              (4096, 4096, 256, 0)])       # the last one runs on 256 x 256 tiles
def test_matrix_core_product_matches_the_oracle(M, N, K, ld_extra):
    rng = np.random.default_rng(M + N + K)
    P = OM.to_bf16(rng.standard_normal((M, K)) * 0.05)
    Q = OM.to_bf16(rng.standard_normal((N, K)) * 0.05)
    D = OM.to_bf16(rng.standard_normal((M, N)) * 0.3)
    alpha, beta = 2.0315, -4.775
    dP, dQ, dDt = bf16_dev(P, K + ld_extra), bf16_dev(Q, K + ld_extra), bf16_dev(D.T.copy(), M + ld_extra)
    C = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    Ct = torch.zeros((N, M), dtype=torch.bfloat16, device=DEV)
    B.adagc_muon_gemm_nt(dP, dQ, alpha, beta, dDt, C, Ct)
    torch.cuda.synchronize()
    f = lambda v: float(np.float32(v))
    exact = f(alpha) * (P @ Q.T) + f(beta) * D
    ref = OM.to_bf16(exact)
    got = host64(C)
    assert np.array_equal(host64(Ct), got.T), "row-major and transposed results differ"
    # fp32 accumulation against the exact sum: within 1e-5 of the sum of magnitudes before rounding, so the bf16
    # results are equal or neighbouring values
    slack = 1e-5 * (np.abs(f(alpha)) * (np.abs(P) @ np.abs(Q).T) + np.abs(f(beta) * D))
    err = np.abs(got - ref)
    assert (err <= 2.0 ** -7 * np.abs(ref) + slack).all(), "max error %g" % err.max()
    differ = float((got != ref).mean())
    say("gemm %dx%dx%d: %.3f %% of the results are not the oracle's bf16 value (neighbouring value instead)" % (M, N, K, 100 * differ))
    assert differ < 0.03
    # without D, and with only one of the two outputs
    C2 = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    B.adagc_muon_gemm_nt(dP, dQ, 1.0, 0.0, None, C2, None)
    Ct2 = torch.zeros((N, M), dtype=torch.bfloat16, device=DEV)
    B.adagc_muon_gemm_nt(dP, dQ, 1.0, 0.0, None, None, Ct2)
    torch.cuda.synchronize()
    ref2 = OM.to_bf16(P @ Q.T)
    g2 = host64(C2)
    assert np.array_equal(host64(Ct2), g2.T)
    assert (np.abs(g2 - ref2) <= 2.0 ** -7 * np.abs(ref2) + 1e-5 * (np.abs(P) @ np.abs(Q).T)).all()


@pytest.mark.parametrize("M,K", [(128, 128), (384, 256), (1024, 512), (4096, 128), (6144, 128)])   # 4096: 256 x 256 tiles
def test_symmetric_matrix_core_product(M, K):
    """P = Q: only the tiles on and below the diagonal are computed and each is stored twice.  The result must be
    exactly symmetric and equal to the full product's (the same sums in the same order)."""
    rng = np.random.default_rng(M + K)
    P = OM.to_bf16(rng.standard_normal((M, K)) * 0.05)
    D = rng.standard_normal((M, M)) * 0.3
    D = OM.to_bf16(D + D.T)
    dP, dD = bf16_dev(P), bf16_dev(D)
    S = torch.full((M, M), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.adagc_muon_gemm_nt(dP, dP, 2.0315, -4.775, dD, None, S, symmetric=True)
    F = torch.zeros((M, M), dtype=torch.bfloat16, device=DEV)
    B.adagc_muon_gemm_nt(dP, dP, 2.0315, -4.775, dD, F, None)
    torch.cuda.synchronize()
    got = host64(S)
    assert not np.isnan(got).any(), "a tile was not written"
    assert np.array_equal(got, got.T)
    assert np.array_equal(got, host64(F))
    f = lambda v: float(np.float32(v))
    ref = OM.to_bf16(f(2.0315) * (P @ P.T) + f(-4.775) * D)
    slack = 1e-5 * (np.abs(f(2.0315)) * (np.abs(P) @ np.abs(P).T) + np.abs(f(-4.775) * D))
    assert (np.abs(got - ref) <= 2.0 ** -7 * np.abs(ref) + slack).all()
    with pytest.raises(B.AdagcError):
        B.adagc_muon_gemm_nt(dP, bf16_dev(P), 1.0, 0.0, None, None, S, symmetric=True)      # P and Q must be the same array


@pytest.mark.parametrize("batch,M,N,K,symmetric", [(3, 128, 256, 128, False), (5, 384, 384, 256, True), (2, 4096, 4096, 128, True),
                                                     (8, 1024, 2048, 128, False), (32, 512, 512, 128, True)])
def test_batched_matrix_core_product_equals_the_single_ones(batch, M, N, K, symmetric):
    """One launch over a batch of products of one shape: every matrix's result is, bit for bit, what the single
    launch gives for it (whatever tile size either launch picks: a result element is the same sum in the same
    order on both tiles), and nothing outside the batch's outputs is written."""
    rng = np.random.default_rng(batch * 1000 + M + N + K)
    gen = torch.Generator(device="cpu").manual_seed(int(rng.integers(1 << 30)))
    P = (torch.randn((batch, M, K), generator=gen) * 0.05).to(torch.bfloat16).to(DEV)
    Q = P if symmetric else (torch.randn((batch, N, K), generator=gen) * 0.05).to(torch.bfloat16).to(DEV)
    D = torch.randn((batch, N, M), generator=gen) * 0.3
    if symmetric:
        D = D + D.transpose(1, 2)
    Dt = D.to(torch.bfloat16).to(DEV)
    guard = 7.0
    Ct = torch.full((batch + 1, N, M), guard, dtype=torch.bfloat16, device=DEV)
    C = None if symmetric else torch.full((batch + 1, M, N), guard, dtype=torch.bfloat16, device=DEV)
    B.adagc_muon_gemm_nt_batched(P, Q, 2.0315, -4.775, Dt, None if symmetric else C[:batch], Ct[:batch], symmetric=symmetric)
    torch.cuda.synchronize()
    assert (Ct[batch] == guard).all() and (symmetric or (C[batch] == guard).all())
    for z in range(batch):
        one_t = torch.zeros((N, M), dtype=torch.bfloat16, device=DEV)
        one = None if symmetric else torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
        B.adagc_muon_gemm_nt(P[z], Q[z], 2.0315, -4.775, Dt[z], one, one_t, symmetric=symmetric)
        torch.cuda.synchronize()
        assert torch.equal(Ct[z].view(torch.int16), one_t.view(torch.int16)), "matrix %d of the batch" % z
        if not symmetric:
            assert torch.equal(C[z].view(torch.int16), one.view(torch.int16)), "matrix %d of the batch (row-major)" % z
    # and one matrix of the batch against the oracle's product
    z = batch - 1
    f = lambda v: float(np.float32(v))
    p64, q64, d64 = host64(P[z]), host64(Q[z]), host64(Dt[z]).T
    ref = OM.to_bf16(f(2.0315) * (p64 @ q64.T) + f(-4.775) * d64)
    slack = 1e-5 * (f(2.0315) * (np.abs(p64) @ np.abs(q64).T) + np.abs(f(-4.775) * d64))
    assert (np.abs(host64(Ct[z]).T - ref) <= 2.0 ** -7 * np.abs(ref) + slack).all()
    if batch == 3:
        buf = torch.zeros(batch * (N * M + 4), dtype=torch.bfloat16, device=DEV)
        with pytest.raises(B.AdagcError):            # a stride that is not a multiple of 8 elements
            B.adagc_muon_gemm_nt_batched(P, Q, 1.0, 0.0, None, None, buf.as_strided((batch, N, M), (N * M + 4, M, 1)))


def test_matrix_core_product_places_every_element():
    """Index check with exactly representable data: P row i holds i+1 at column i (others 0), Q row j holds small
    integers, so C[i][j] = (i+1) * Q[j][i] exactly, and a misplaced lane or register shows as a wrong integer."""
    M, N, K = 256, 128, 256
    P = np.zeros((M, K))
    P[np.arange(M), np.arange(M) % K] = (np.arange(M) % 7) + 1.0
    rng = np.random.default_rng(1)
    Q = rng.integers(-8, 9, (N, K)).astype(np.float64)
    C = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    B.adagc_muon_gemm_nt(bf16_dev(P), bf16_dev(Q), 1.0, 0.0, None, C, None)
    torch.cuda.synchronize()
    assert np.array_equal(host64(C), P @ Q.T)


def test_matrix_core_product_rejects_shapes_it_does_not_tile():
    z = torch.zeros((128, 128), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros((128, 128), dtype=torch.bfloat16, device=DEV)
    for P, Q in [(z[:100], z), (z[:, :64], z[:, :64])]:
        with pytest.raises(B.AdagcError) as e:
            B.adagc_muon_gemm_nt(P, Q, 1.0, 0.0, None, out[:P.shape[0]], None)
        assert e.value.code == B.ADAGC_ERR_INVALID_ARG
    with pytest.raises(B.AdagcError):
        B.adagc_muon_gemm_nt(z, z, 1.0, 0.0, None, None, None)
    assert B.lib().adagc_muon_workspace_bytes(None) == 0
    # every access is a 16-byte vector: an operand that starts 8 bytes into an allocation is refused
    shifted = torch.zeros(128 * 128 + 8, dtype=torch.bfloat16, device=DEV)[4:4 + 128 * 128].view(128, 128)
    for args in [(shifted, z, None, out), (z, z, shifted, out), (z, z, None, shifted)]:
        with pytest.raises(B.AdagcError) as e:
            B.adagc_muon_gemm_nt(args[0], args[1], 1.0, 0.0, args[2], args[3], None)
        assert e.value.code == B.ADAGC_ERR_INVALID_ARG


# --------------------------------------------------------------------------- the Muon step

import oracle
from paper_2502_11034_amd.workloads import to_numpy

SHAPES = [(64, 200), (300, 100), (128, 128), (256, 640), (1, 50), (40, 40), (512, 128)]


def _inputs(seed, shapes=SHAPES, spike=None):
    rng = np.random.default_rng(seed)
    sig = np.exp(rng.uniform(np.log(1e-3), np.log(1e-1), len(shapes)))
    g = [(rng.standard_normal(s) * sig[i] * (spike if spike and i % 2 == 0 else 1.0)).astype(np.float32) for i, s in enumerate(shapes)]
    m = [(rng.standard_normal(s) * sig[i] * 0.5).astype(np.float32) for i, s in enumerate(shapes)]
    th = [(rng.standard_normal(s) * 0.02).astype(np.float32) for s in shapes]
    return g, m, th


def _dev(arrs):
    return [torch.from_numpy(a.reshape(-1).copy()).to(DEV) for a in arrs]


def _gpu_muon(shapes, g, m, th, gamma, hp, mh, step, copies=False):
    """One adagc_muon_step from the given host state.  Returns (theta, momentum, gamma, norms, coefs, flags[, copies])."""
    ctx = B.AdaGC([r * c for r, c in shapes], B.ADAGC_OPT_MUON, B.ADAGC_GRAD_F32, copies)
    ctx.muon_attach(shapes)
    dg, dm, dth = _dev(g), _dev(m), _dev(th)
    dgam = torch.from_numpy(gamma.copy()).to(DEV)
    dcp = None
    if copies:
        dcp = [torch.zeros(r * c, dtype=torch.bfloat16, device=DEV) for r, c in shapes]
        ctx.set_param_copies(dcp)
    ctx.muon_step(dth, dg, dm, dgam, hp, mh, step)
    norms, coefs, flags = ctx.get_norms()
    out = ([to_numpy(t).reshape(s) for t, s in zip(dth, shapes)], [to_numpy(t).reshape(s) for t, s in zip(dm, shapes)],
           to_numpy(dgam), norms, coefs, flags)
    if copies:
        out += ([to_numpy(t).reshape(s) for t, s in zip(dcp, shapes)],)
    ctx.close()
    return out


def _direction(shapes, g, m, gamma, hp_kw, mh, step):
    """O of every tensor as the GPU computes it: theta = 0, lr = 1, no decay gives theta' = fp32(-scale * O); dividing by
    the scale and rounding to the nearest bf16 value gives O back exactly (fp32's rounding error is far below bf16's
    spacing)."""
    hp = B.make_hyper(lr=1.0, weight_decay=0.0, **hp_kw)
    th0 = [np.zeros(s, np.float32) for s in shapes]
    res = _gpu_muon(shapes, g, m, th0, gamma, hp, mh, step)
    return [OM.to_bf16(-(t.astype(np.float64)) / OM.update_scale(*s)) for t, s in zip(res[0], shapes)], res


def _bf16_ulps(a, b):
    """Distance in bf16 steps between two arrays of bf16-representable values."""
    def key(x):
        bits = OM.bf16_bits(x).astype(np.int32)
        return np.where(bits & 0x8000, -(bits & 0x7FFF), bits & 0x7FFF)
    return np.abs(key(a) - key(b))


def test_muon_momentum_normalisation_and_update_without_iteration():
    """ns_steps = 0: O is X0 = bf16(U / ||U||_F), so this checks the clip coefficient entering the momentum, the
    Nesterov form, the norm, the transposed orientation of tall matrices, the padding and the parameter update."""
    g, m, th = _inputs(1)
    lam, beta = float(np.float32(1.04)), float(np.float32(0.99))
    gamma = np.array([oracle.l2_norm(x.reshape(-1)) for x in g], np.float32)
    gamma[::2] *= np.float32(0.5)                              # every other tensor is clipped
    for nesterov in (True, False):
        mh = B.make_muon_hyper(momentum=0.95, nesterov=nesterov, ns_steps=0)
        O, res = _direction(SHAPES, g, m, gamma, dict(t_start=0), mh, 7)
        _, m_gpu, gam_gpu, norms, coefs, flags = res
        clipped = 0
        for i, s in enumerate(SHAPES):
            n = oracle.l2_norm(g[i].reshape(-1))
            h, g_new, c = oracle.adagc_rule(n, float(gamma[i]), lam, beta)
            np.testing.assert_allclose(norms[i], n, rtol=1e-5)
            np.testing.assert_allclose(coefs[i], h, rtol=1e-5)
            np.testing.assert_allclose(gam_gpu[i], np.float32(g_new), rtol=1e-5)
            assert flags[i] == c
            clipped += c
            th_ref, m_ref = np.zeros(s, np.float32), m[i].copy()
            o_ref = OM.muon_update(th_ref, g[i], m_ref, h, lr=1.0, weight_decay=0.0, mu=0.95, nesterov=nesterov, steps=0)
            assert (np.abs(m_gpu[i].astype(np.float64) - m_ref) <= 1e-5 * np.abs(m_ref)).all(), "momentum of tensor %d" % i
            assert (m_gpu[i].view(np.uint32) != m_ref.view(np.uint32)).mean() < 1e-3
            d = _bf16_ulps(O[i], o_ref)
            assert d.max() <= 1 and (d > 0).mean() < 0.01, "X0 of tensor %d: max %d steps, %.3f %% differ" % (i, d.max(), 100 * (d > 0).mean())
        assert 3 <= clipped <= 4
    # the update itself: theta' = theta - lr (wd theta + scale O) with the O the GPU produced, and the bf16 copies
    mh = B.make_muon_hyper(ns_steps=0)
    O, _ = _direction(SHAPES, g, m, gamma, dict(t_start=0), mh, 7)
    hp = B.make_hyper(lr=0.02, weight_decay=0.1, t_start=0)
    res = _gpu_muon(SHAPES, g, m, th, gamma, hp, mh, 7, copies=True)
    for i, s in enumerate(SHAPES):
        t64 = th[i].astype(np.float64)
        ref = (t64 - float(np.float32(0.02)) * (float(np.float32(0.1)) * t64 + OM.update_scale(*s) * O[i])).astype(np.float32)
        assert (np.abs(res[0][i].astype(np.float64) - ref) <= 1e-5 * np.abs(ref)).all(), "theta of tensor %d" % i
        exact = torch.from_numpy(res[0][i]).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(res[6][i], exact)


def test_muon_newton_schulz_step_by_step():
    """Lockstep through the iteration: the GPU's X_k (read back through a step with theta = 0) is handed to the oracle,
    whose one step is compared with the GPU's X_(k+1).  Within one step the GPU accumulates its products in fp32 where
    the oracle is exact, so a stored bf16 value can be the oracle's neighbour, and a neighbour in A or B moves X by a
    few more steps at most: every value within 4 bf16 steps or 2^-9 of the row's largest value, 98 % identical."""
    g, m, _ = _inputs(2)
    gamma = np.full(len(SHAPES), 1e9, np.float32)               # nothing clipped here
    prev = None
    for k in range(0, 6):
        O, _ = _direction(SHAPES, g, m, gamma, dict(t_start=0), B.make_muon_hyper(ns_steps=k), 3)
        X = [o.T if s[0] > s[1] else o for o, s in zip(O, SHAPES)]            # the wide orientation the iteration runs on
        if prev is not None:
            worst, frac = 0.0, 0.0
            for i, s in enumerate(SHAPES):
                ref = OM.ns_iterate(prev[i], 1)
                d = _bf16_ulps(X[i], ref)
                rel = np.abs(X[i] - ref) / np.abs(ref).max(axis=1, keepdims=True)
                assert ((d <= 4) | (rel <= 2.0 ** -9)).all(), "step %d tensor %d: %d bf16 steps apart" % (k, i, d.max())
                worst, frac = max(worst, float(rel.max())), max(frac, float((d > 0).mean()))
                assert (d > 0).mean() < 0.02
            say("Newton-Schulz step %d: at most %.1e of the row's largest value from the oracle's step, %.3f %% of values not identical"
                % (k, worst, 100 * frac))
        prev = X


def test_muon_five_steps_end_to_end():
    """The whole iteration against the oracle's, started from the same U: rounding differences of single values are
    carried through five steps, so the comparison is in the large: root-mean-square difference below 1 % of the
    result's own, and the same singular values to 0.01 (the iteration leaves them in about [0.68, 1.2], except those that
    started too close to zero for five steps)."""
    g, m, _ = _inputs(3)
    gamma = np.full(len(SHAPES), 1e9, np.float32)
    O, _ = _direction(SHAPES, g, m, gamma, dict(t_start=0), B.make_muon_hyper(), 3)
    for i, s in enumerate(SHAPES):
        th_ref, m_ref = np.zeros(s, np.float32), m[i].copy()
        o_ref = OM.muon_update(th_ref, g[i], m_ref, 1.0, lr=1.0, weight_decay=0.0, mu=0.95)
        rms = np.sqrt(np.mean(o_ref ** 2))
        diff = np.sqrt(np.mean((O[i] - o_ref) ** 2))
        sv = np.linalg.svd(O[i], compute_uv=False)
        say("tensor %d %s: rms difference %.2e of rms %.2e; singular values %.3f .. %.3f" % (i, s, diff, rms, sv.min(), sv.max()))
        assert diff <= 0.01 * rms
        sv_ref = np.linalg.svd(o_ref, compute_uv=False)
        assert np.abs(sv - sv_ref).max() <= 0.01 and sv.max() < 1.25


def test_muon_matrices_iterated_in_batches_give_the_results_of_single_ones():
    """Matrices whose padded extents agree share batched launches (here: 64 x 200, 200 x 64 and 100 x 250 all pad to
    128 x 256, wide and tall ones mixed; 40 of one shape make two batches of 20).  Every tensor's parameters and momentum
    must be, bit for bit, what a context holding that tensor alone produces."""
    shapes = [(64, 200), (300, 100), (200, 64), (64, 200), (100, 250), (100, 300), (128, 128)] + [(130, 300)] * 40
    g, m, th = _inputs(8, shapes)
    gamma = np.array([oracle.l2_norm(x.reshape(-1)) for x in g], np.float32)
    gamma[::3] *= np.float32(0.4)
    hp = B.make_hyper(lr=0.02, weight_decay=0.1, t_start=0)
    mh = B.make_muon_hyper()
    ctx = B.AdaGC([r * c for r, c in shapes], B.ADAGC_OPT_MUON, B.ADAGC_GRAD_F32)
    ctx.muon_attach(shapes)
    # the largest batch: 20 matrices padded to 256 x 384, each 4 x 256 x 384 + 2 x 256 x 256 bf16 values
    assert ctx.muon_workspace_bytes() == 20 * (4 * 256 * 384 + 2 * 256 * 256) * 2
    ctx.close()
    together = _gpu_muon(shapes, g, m, th, gamma, hp, mh, 4)
    for i in list(range(8)) + [26, 27, 46]:
        alone = _gpu_muon([shapes[i]], [g[i]], [m[i]], [th[i]], gamma[i:i + 1], hp, mh, 4)
        assert np.array_equal(together[0][i].view(np.uint32), alone[0][0].view(np.uint32)), "parameters of tensor %d" % i
        assert np.array_equal(together[1][i].view(np.uint32), alone[1][0].view(np.uint32)), "momentum of tensor %d" % i
        assert together[4][i] == alone[4][0]
    # and against the oracle, as for the single ones
    for i in (0, 2, 4, 30):
        th_ref, m_ref = th[i].copy(), m[i].copy()
        OM.muon_update(th_ref, g[i], m_ref, float(together[4][i]), lr=0.02, weight_decay=0.1, mu=0.95)
        diff = np.sqrt(np.mean((together[0][i].astype(np.float64) - th_ref) ** 2))
        assert diff <= 0.02 * OM.update_scale(*shapes[i]) * 0.01 * 0.2


def test_muon_trajectory_with_adagc_clipping():
    """Three steps with the paper's schedule in small (one warm-up step, then Eq. 3), a spike on the third step:
    norms, coefficients, flags and gamma against the C oracle's rule, the momentum against the oracle to 1e-5."""
    shapes = SHAPES
    hp = B.make_hyper(lr=0.02, weight_decay=0.1, t_start=1)
    mh = B.make_muon_hyper()
    ctx = B.AdaGC([r * c for r, c in shapes], B.ADAGC_OPT_MUON, B.ADAGC_GRAD_F32)
    ctx.muon_attach(shapes)
    _, m0, th0 = _inputs(5)
    dm, dth = _dev([np.zeros_like(x) for x in m0]), _dev(th0)
    dgam = torch.zeros(len(shapes), dtype=torch.float32, device=DEV)
    h_m = [np.zeros(s, np.float32) for s in shapes]
    h_th = [t.copy() for t in th0]
    h_gam = np.zeros(len(shapes), np.float32)
    lam, beta = float(np.float32(1.04)), float(np.float32(0.99))
    total_clipped = 0
    for step in (1, 2, 3):
        g, _, _ = _inputs(10 + step, spike=30.0 if step == 3 else None)
        ctx.muon_step(dth, _dev(g), dm, dgam, hp, mh, step)
        norms, coefs, flags = ctx.get_norms()
        for i, s in enumerate(shapes):
            n = oracle.l2_norm(g[i].reshape(-1))
            if step == 1:
                h, g_new, c = 1.0, n, False
            else:
                h, g_new, c = oracle.adagc_rule(n, float(h_gam[i]), lam, beta)
            h_gam[i] = np.float32(g_new)
            np.testing.assert_allclose(norms[i], n, rtol=1e-5)
            np.testing.assert_allclose(coefs[i], h, rtol=1e-5)
            assert flags[i] == c
            total_clipped += int(c)
            OM.muon_update(h_th[i], g[i], h_m[i], h, lr=0.02, weight_decay=0.1, mu=0.95)
            gm = to_numpy(dm[i]).reshape(s)
            assert (np.abs(gm.astype(np.float64) - h_m[i]) <= 1e-5 * np.abs(h_m[i])).all()
            gt = to_numpy(dth[i]).reshape(s).astype(np.float64)
            # theta differs only through O: |lr * scale * (O_gpu - O_ref)|, O's values are below 0.5 in magnitude here
            assert np.sqrt(np.mean((gt - h_th[i]) ** 2)) <= 0.02 * OM.update_scale(*s) * 0.01 * 0.2 * step
        np.testing.assert_allclose(to_numpy(dgam), h_gam, rtol=1e-5)
    assert total_clipped >= 4
    ctx.close()


def test_muon_argument_checks():
    ctx = B.AdaGC([128 * 64, 10], B.ADAGC_OPT_MUON)
    z = [torch.zeros(128 * 64, device=DEV), torch.zeros(10, device=DEV)]
    gam = torch.zeros(2, device=DEV)
    with pytest.raises(B.AdagcError) as e:
        ctx.muon_step(z, z, z, gam, B.make_hyper(), B.make_muon_hyper(), 1)       # not attached
    assert e.value.code == B.ADAGC_ERR_STATE
    with pytest.raises(B.AdagcError) as e:
        ctx.muon_attach([(128, 64), (3, 4)])                                          # 3*4 != 10
    assert e.value.code == B.ADAGC_ERR_INVALID_ARG
    ctx.muon_attach([(128, 64), (2, 5)])
    with pytest.raises(B.AdagcError) as e:
        ctx.muon_attach([(128, 64), (2, 5)])                                          # once
    assert e.value.code == B.ADAGC_ERR_STATE
    with pytest.raises(B.AdagcError) as e:
        ctx.step(z, z, z, z, gam, B.make_hyper(), 1)                                  # the wrong entry point
    assert e.value.code == B.ADAGC_ERR_STATE
    for bad in (B.make_muon_hyper(momentum=1.0), B.make_muon_hyper(ns_steps=17), B.make_muon_hyper(ns_steps=-1)):
        with pytest.raises(B.AdagcError) as e:
            ctx.muon_step(z, z, z, gam, B.make_hyper(), bad, 1)
        assert e.value.code == B.ADAGC_ERR_INVALID_ARG
    with pytest.raises(B.AdagcError) as e:
        ctx.muon_step(z, z, z, gam, B.make_hyper(clip_mode=B.ADAGC_MODE_AGC), B.make_muon_hyper(), 1)
    assert e.value.code == B.ADAGC_ERR_INVALID_ARG
    ctx.muon_step(z, z, z, gam, B.make_hyper(), B.make_muon_hyper(), 1)               # zeros in, zeros out
    torch.cuda.synchronize()
    assert not z[0].any() and not z[1].any()
    ctx.close()
    adam = B.AdaGC([16])
    with pytest.raises(B.AdagcError) as e:
        adam.muon_attach([(4, 4)])
    assert e.value.code == B.ADAGC_ERR_STATE
    adam.close()


# --------------------------------------------------------------------------- Llama-3-8B shapes

def _sampled_rows_check(name, P, Q, alpha, beta, D, got, rows):
    """Rows of bf16(alpha P Q^T + beta D) computed one by one by the oracle's arithmetic."""
    f = lambda v: float(np.float32(v))
    for i in rows:
        exact = f(alpha) * (P[i] @ Q.T)
        slack = 1e-5 * np.abs(f(alpha)) * (np.abs(P[i]) @ np.abs(Q).T)
        if D is not None:
            exact = exact + f(beta) * D[i]
            slack = slack + 1e-5 * np.abs(f(beta) * D[i])
        ref = OM.to_bf16(exact)
        assert (np.abs(got[i] - ref) <= 2.0 ** -7 * np.abs(ref) + slack).all(), "%s row %d" % (name, i)


def test_newton_schulz_products_at_llama3_8b_ffn_shape():
    """One step's three products at the size of a 4096 x 14336 weight, on the 256 x 256 tiles the step uses there (the
    step runs them batched over equal-shaped matrices; a batched product equals the single one bit for bit, which
    test_batched_matrix_core_product_equals_the_single_ones checks): each checked on sampled rows that the oracle
    computes one by one from the GPU's own operands, and the symmetric ones for exact symmetry."""
    m, n = 4096, 14336
    gen = torch.Generator(device=DEV).manual_seed(9)
    x = (torch.randn(m, n, device=DEV, generator=gen) * (1.0 / np.sqrt(m * n)) * 3.0).to(torch.bfloat16)      # like a normalised U
    y = x.t().contiguous()
    a_, b_, c_ = 3.4445, -4.7750, 2.0315
    A = torch.empty((m, m), dtype=torch.bfloat16, device=DEV)
    Bm = torch.empty((m, m), dtype=torch.bfloat16, device=DEV)
    X2 = torch.empty((m, n), dtype=torch.bfloat16, device=DEV)
    Y2 = torch.empty((n, m), dtype=torch.bfloat16, device=DEV)
    B.adagc_muon_gemm_nt(x, x, 1.0, 0.0, None, None, A, symmetric=True)
    B.adagc_muon_gemm_nt(A, A, c_, b_, A, None, Bm, symmetric=True)
    B.adagc_muon_gemm_nt(Bm, y, 1.0, a_, y, X2, Y2)
    torch.cuda.synchronize()
    hx, hA, hB, hX2 = host64(x), host64(A), host64(Bm), host64(X2)
    assert np.array_equal(hA, hA.T) and np.array_equal(hB, hB.T)
    assert torch.equal(Y2, X2.t().contiguous())
    rows = [0, 1, 127, 128, 2047, 2048, 3000, 4095]
    _sampled_rows_check("A = X X^T", hx, hx, 1.0, 0.0, None, hA, rows)
    _sampled_rows_check("B = b A + c A A", hA, hA, c_, b_, hA, hB, rows)
    _sampled_rows_check("X' = a X + B X", hB, hx.T.copy(), 1.0, a_, hx, hX2, rows)
    say("Newton-Schulz products at 4096 x 14336: %d sampled rows of each product agree with the oracle" % len(rows))


def test_muon_step_at_llama3_8b_attention_shapes():
    """The whole step on a k-projection (1024 x 4096) and a q-projection (4096 x 4096) at real size, five steps of the
    iteration, against the oracle's (numpy, float64 products): root-mean-square difference and singular values."""
    shapes = [(1024, 4096), (4096, 4096)]
    g, m, _ = _inputs(21, shapes)
    gamma = np.full(len(shapes), 1e9, np.float32)
    O, _ = _direction(shapes, g, m, gamma, dict(t_start=0), B.make_muon_hyper(), 3)
    for i, s in enumerate(shapes):
        th_ref, m_ref = np.zeros(s, np.float32), m[i].copy()
        o_ref = OM.muon_update(th_ref, g[i], m_ref, 1.0, lr=1.0, weight_decay=0.0, mu=0.95)
        rms = np.sqrt(np.mean(o_ref ** 2))
        diff = np.sqrt(np.mean((O[i] - o_ref) ** 2))
        same = float((O[i] == o_ref).mean())
        say("%s: rms difference %.2e of rms %.2e, %.1f %% of the values identical" % (s, diff, rms, 100 * same))
        assert diff <= 0.01 * rms
        if s[0] < s[1]:
            sv, sv_ref = np.linalg.svd(O[i], compute_uv=False), np.linalg.svd(o_ref, compute_uv=False)
            assert np.abs(sv - sv_ref).max() <= 0.01 and 0.6 < sv.min() and sv.max() < 1.25


@pytest.mark.parametrize("shape,with_oracle", [((4096, 4096), True), ((14336, 4096), False)])
def test_muon_batch_of_32_at_llama3_8b_shapes(shape, with_oracle):
    """The launch configuration the benchmark times: 32 equal matrices iterated in one batch (symmetric products
    32 x 136 tiles of 256 x 256), for a q-projection and for a gate-projection (tall: iterated transposed, 17 GB of
    workspace).  The first and the last matrix of the batch must be, bit for bit, what a context holding one matrix
    produces; for the square shape the last one is also compared with the oracle's five steps (the oracle's check at
    4096 x 14336 is test_newton_schulz_products_at_llama3_8b_ffn_shape)."""
    count = 32
    gen = torch.Generator(device=DEV).manual_seed(33)
    sig = torch.exp(torch.empty(count, device=DEV).uniform_(-6.0, -2.0, generator=gen))
    g = [torch.randn(shape[0] * shape[1], device=DEV, generator=gen) * sig[i] for i in range(count)]
    m = [torch.randn(shape[0] * shape[1], device=DEV, generator=gen) * sig[i] * 0.5 for i in range(count)]
    th = [torch.zeros(shape[0] * shape[1], device=DEV) for _ in range(count)]
    hp = B.make_hyper(lr=1.0, weight_decay=0.0, t_start=0)
    mh = B.make_muon_hyper()
    m_before = {i: to_numpy(m[i]).reshape(shape) for i in (0, count - 1)}
    g_host = {i: to_numpy(g[i]).reshape(shape) for i in (0, count - 1)}
    ctx = B.AdaGC([shape[0] * shape[1]] * count, B.ADAGC_OPT_MUON, B.ADAGC_GRAD_F32)
    ctx.muon_attach([shape] * count)
    assert ctx.muon_workspace_bytes() == count * (4 * shape[0] * shape[1] + 2 * 4096 * 4096) * 2
    gamma = torch.full((count,), 1e9, dtype=torch.float32, device=DEV)
    ctx.muon_step(th, g, m, gamma, hp, mh, 3)
    torch.cuda.synchronize()
    ctx.close()
    for i in (0, count - 1):
        alone = _gpu_muon([shape], [g_host[i]], [m_before[i]], [np.zeros(shape, np.float32)], np.full(1, 1e9, np.float32), hp, mh, 3)
        assert np.array_equal(to_numpy(th[i]).reshape(shape).view(np.uint32), alone[0][0].view(np.uint32)), "matrix %d of the batch" % i
        assert np.array_equal(to_numpy(m[i]).reshape(shape).view(np.uint32), alone[1][0].view(np.uint32))
    if not with_oracle:
        return
    i = count - 1
    O = OM.to_bf16(-(to_numpy(th[i]).reshape(shape).astype(np.float64)))
    th_ref, m_ref = np.zeros(shape, np.float32), m_before[i].copy()
    o_ref = OM.muon_update(th_ref, g_host[i], m_ref, 1.0, lr=1.0, weight_decay=0.0, mu=0.95)
    rms = np.sqrt(np.mean(o_ref ** 2))
    diff = np.sqrt(np.mean((O - o_ref) ** 2))
    say("matrix %d of a batch of %d at %s: rms difference %.2e of rms %.2e, %.1f %% of the values identical"
        % (i, count, shape, diff, rms, 100 * float((O == o_ref).mean())))
    assert diff <= 0.01 * rms


# --------------------------------------------------------------------------- the comparisons have teeth

def _oracle_with_mistake(k):
    """oracle/muon.py with mistake k of tests/test_muon_pins_catch_planted_mistakes.py planted (None: unmodified), as a module."""
    import types
    import test_muon_pins_catch_planted_mistakes as planted_muon
    mod = types.ModuleType("muon_with_mistake")
    exec(compile(planted_muon._mutated(k), "muon_with_mistake.py", "exec"), mod.__dict__)
    return mod


def _compare_one_newton_schulz_step(om, x0, x1):
    """The bar of test_muon_newton_schulz_step_by_step for the first step."""
    for i in range(len(x0)):
        ref = om.ns_iterate(x0[i], 1)
        d = _bf16_ulps(x1[i], ref)
        rel = np.abs(x1[i] - ref) / np.abs(ref).max(axis=1, keepdims=True)
        assert ((d <= 4) | (rel <= 2.0 ** -9)).all() and (d > 0).mean() < 0.02, "tensor %d" % i


def _compare_step_without_iteration(om, shapes, g, m, th, coefs, gpu_theta, gpu_m):
    """The bars of test_muon_momentum_normalisation_and_update_without_iteration: momentum to 1e-5, parameters through
    X0 = bf16(U / ||U||) to one bf16 step of X0."""
    lr, wd = float(np.float32(0.02)), float(np.float32(0.1))
    for i, s in enumerate(shapes):
        th_ref, m_ref = th[i].copy(), m[i].copy()
        o_ref = om.muon_update(th_ref, g[i], m_ref, float(coefs[i]), lr=0.02, weight_decay=0.1, mu=0.95, steps=0)
        assert (np.abs(gpu_m[i].astype(np.float64) - m_ref) <= 1e-5 * np.abs(m_ref)).all(), "momentum of tensor %d" % i
        bound = 1e-5 * np.abs(th_ref) + lr * om.update_scale(*s) * 2.0 ** -7 * np.abs(o_ref) + 1e-12
        assert (np.abs(gpu_theta[i].astype(np.float64) - th_ref) <= bound).all(), "parameters of tensor %d" % i


def test_muon_comparisons_notice_a_wrong_oracle():
    """Mistakes planted in a copy of the Muon oracle (on the CPU; the GPU library is the one under test, unaltered):
    the comparisons used above must fail against every one of them, and pass against the unmodified copy."""
    import test_muon_pins_catch_planted_mistakes as planted_muon
    names = [n for n, _, _ in planted_muon.MISTAKES]
    g, m, th = _inputs(6)
    gamma = np.array([oracle.l2_norm(x.reshape(-1)) for x in g], np.float32)
    gamma[::2] *= np.float32(0.5)
    # one Newton-Schulz step: X0 and X1 from the GPU
    big = np.full(len(SHAPES), 1e9, np.float32)
    X = []
    for k in (0, 1):
        O, _ = _direction(SHAPES, g, m, big, dict(t_start=0), B.make_muon_hyper(ns_steps=k), 3)
        X.append([o.T if s[0] > s[1] else o for o, s in zip(O, SHAPES)])
    # a step without iteration, every other tensor clipped
    hp = B.make_hyper(lr=0.02, weight_decay=0.1, t_start=0)
    res = _gpu_muon(SHAPES, g, m, th, gamma, hp, B.make_muon_hyper(ns_steps=0), 7)
    lam, beta = float(np.float32(1.04)), float(np.float32(0.99))
    coefs = [oracle.adagc_rule(oracle.l2_norm(g[i].reshape(-1)), float(gamma[i]), lam, beta)[0] for i in range(len(SHAPES))]
    assert sum(c < 1.0 for c in coefs) >= 3
    clean = _oracle_with_mistake(None)
    _compare_one_newton_schulz_step(clean, X[0], X[1])
    _compare_step_without_iteration(clean, SHAPES, g, m, th, coefs, res[0], res[1])
    # (where a stored value is rounded -- "A not rounded when stored", "A A from the unrounded A" -- moves results by less
    # than the fp32-against-exact accumulation slack of these comparisons; the oracle's own pins fix those points)
    in_step = ["b and c exchanged", "a dropped from the update of X", "polynomial applied from the right", "one step short"]
    in_update = ["spectral norm instead of Frobenius", "Nesterov term without the momentum factor", "Nesterov and plain momentum exchanged",
                 "clip coefficient dropped", "momentum as an average", "update scale without the root", "update scale upside down",
                 "decay outside the learning rate", "tall matrices not transposed", "result of a tall matrix not transposed back"]
    unnoticed = []
    for name in in_step + in_update:
        om = _oracle_with_mistake(names.index(name))
        try:
            if name in in_step:
                _compare_one_newton_schulz_step(om, X[0], X[1])
            else:
                _compare_step_without_iteration(om, SHAPES, g, m, th, coefs, res[0], res[1])
            unnoticed.append(name)
        except (AssertionError, ValueError):          # ValueError: a shape mismatch the mistake causes
            pass
    say("Muon comparisons: %d of %d planted oracle mistakes noticed" % (len(in_step) + len(in_update) - len(unnoticed), len(in_step) + len(in_update)))
    assert not unnoticed, unnoticed


def test_muon_with_bf16_gradients():
    """Gradients handed over as bf16 (widened exactly in the kernels): the oracle gets the same values as float32.
    Without iteration the momentum and X0 are held to the strict bars; with five steps the result to 1 % rms."""
    shapes = SHAPES + [(96, 130)]
    g, m, th = _inputs(9, shapes)
    g = [OM.to_bf16(x).astype(np.float32) for x in g]                    # bf16-representable values
    gamma = np.array([oracle.l2_norm(x.reshape(-1)) for x in g], np.float32)
    gamma[::2] *= np.float32(0.5)
    lam, beta = float(np.float32(1.04)), float(np.float32(0.99))
    for ns_steps in (0, 5):
        ctx = B.AdaGC([r * c for r, c in shapes], B.ADAGC_OPT_MUON, B.ADAGC_GRAD_BF16)
        ctx.muon_attach(shapes)
        dg = [torch.from_numpy(x.reshape(-1).copy()).to(torch.bfloat16).to(DEV) for x in g]
        dm = _dev(m)
        dth = _dev([np.zeros(s, np.float32) for s in shapes])
        dgam = torch.from_numpy(gamma.copy()).to(DEV)
        ctx.muon_step(dth, dg, dm, dgam, B.make_hyper(lr=1.0, weight_decay=0.0, t_start=0), B.make_muon_hyper(ns_steps=ns_steps), 5)
        norms, coefs, flags = ctx.get_norms()
        ctx.close()
        clipped = 0
        for i, s in enumerate(shapes):
            n = oracle.l2_norm(g[i].reshape(-1))
            h, _, c = oracle.adagc_rule(n, float(gamma[i]), lam, beta)
            np.testing.assert_allclose(norms[i], n, rtol=1e-5)
            np.testing.assert_allclose(coefs[i], h, rtol=1e-5)
            assert flags[i] == c
            clipped += c
            th_ref, m_ref = np.zeros(s, np.float32), m[i].copy()
            o_ref = OM.muon_update(th_ref, g[i], m_ref, h, lr=1.0, weight_decay=0.0, mu=0.95, steps=ns_steps)
            gm = to_numpy(dm[i]).reshape(s)
            assert (np.abs(gm.astype(np.float64) - m_ref) <= 1e-5 * np.abs(m_ref)).all(), "momentum of tensor %d" % i
            O = OM.to_bf16(-(to_numpy(dth[i]).reshape(s).astype(np.float64)) / OM.update_scale(*s))
            if ns_steps == 0:
                d = _bf16_ulps(O, o_ref)
                assert d.max() <= 1 and (d > 0).mean() < 0.01, "X0 of tensor %d" % i
            else:
                assert np.sqrt(np.mean((O - o_ref) ** 2)) <= 0.01 * np.sqrt(np.mean(o_ref ** 2)), "tensor %d" % i
        assert clipped >= 3


@pytest.mark.parametrize("mode", [B.ADAGC_MODE_GLOBALGC, B.ADAGC_MODE_GLOBAL_ADAGC, B.ADAGC_MODE_ZCLIP])
def test_muon_with_the_global_clipping_rules(mode):
    """Muon takes its clip coefficient from the same rule kernels as AdamW and Lion: the model-wide rules (GlobalGC on
    every step, Global AdaGC, ZClip) over four steps with a spike on the last; norms, coefficients, flags and the rule's
    state against the C oracle's list step (run with Lion on scratch arrays: the rule does not depend on the optimizer),
    the momentum against the Muon oracle with that coefficient."""
    shapes = SHAPES
    n = len(shapes)
    grads = [[x * (np.float32(6.0) if step == 4 else np.float32(1.0)) for x in _inputs(40 + step, shapes)[0]] for step in (1, 2, 3, 4)]
    global_norm = math.sqrt(sum(oracle.l2_norm(x.reshape(-1)) ** 2 for x in grads[0]))
    kw = dict(lr=0.02, weight_decay=0.1, lambda_abs=0.8 * global_norm, t_start=2, clip_mode=mode,
              ema_beta=0.97 if mode == B.ADAGC_MODE_ZCLIP else 0.99)
    hp = B.make_hyper(**kw)
    oh = oracle.Hyper(optimizer=oracle.LION, **kw)
    mh = B.make_muon_hyper()
    ctx = B.AdaGC([r * c for r, c in shapes], B.ADAGC_OPT_MUON, B.ADAGC_GRAD_F32)
    ctx.muon_attach(shapes)
    _, _, th0 = _inputs(5, shapes)
    dm, dth = _dev([np.zeros(s, np.float32) for s in shapes]), _dev(th0)
    dgam = torch.zeros(max(n, 2), dtype=torch.float32, device=DEV)
    h_gam = np.zeros(max(n, 2), np.float32)
    h_m = [np.zeros(s, np.float32) for s in shapes]
    h_th = [t.copy() for t in th0]
    scratch_th = [np.zeros(r * c, np.float32) for r, c in shapes]
    scratch_m = [np.zeros(r * c, np.float32) for r, c in shapes]
    clipped_steps = 0
    for step, g in zip((1, 2, 3, 4), grads):
        ctx.muon_step(dth, _dev(g), dm, dgam, hp, mh, step)
        norms, coefs, flags = ctx.get_norms()
        o_norms, o_coefs, o_flags = oracle.adagc_step(scratch_th, [x.reshape(-1) for x in g], scratch_m, None, h_gam, oh, step)
        np.testing.assert_allclose(norms, o_norms, rtol=1e-5)
        np.testing.assert_allclose(coefs, o_coefs, rtol=1e-5)
        assert np.array_equal(flags, o_flags)
        np.testing.assert_allclose(to_numpy(dgam), h_gam, rtol=1e-5)
        clipped_steps += int(o_flags.any())
        for i, s in enumerate(shapes):
            OM.muon_update(h_th[i], g[i], h_m[i], float(o_coefs[i]), lr=0.02, weight_decay=0.1, mu=0.95)
            gm = to_numpy(dm[i]).reshape(s)
            assert (np.abs(gm.astype(np.float64) - h_m[i]) <= 1e-5 * np.abs(h_m[i])).all(), "step %d tensor %d" % (step, i)
    assert clipped_steps >= 1 and o_flags.all()          # the spike step clips the whole model
    ctx.close()


def test_muon_step_on_a_side_stream_equals_the_default_stream():
    """Every launch of the step goes to the caller's stream: a step enqueued on a side stream (after an event that orders
    it behind the inputs' uploads) gives, bit for bit, the default stream's result."""
    shapes = [(64, 200), (300, 100), (128, 128), (128, 128)]
    g, m, th = _inputs(12, shapes)
    gamma = np.array([oracle.l2_norm(x.reshape(-1)) for x in g], np.float32) * np.float32(0.7)
    hp = B.make_hyper(lr=0.02, weight_decay=0.1, t_start=0)
    mh = B.make_muon_hyper()
    ref = _gpu_muon(shapes, g, m, th, gamma, hp, mh, 4)
    ctx = B.AdaGC([r * c for r, c in shapes], B.ADAGC_OPT_MUON, B.ADAGC_GRAD_F32)
    ctx.muon_attach(shapes)
    dg, dm, dth = _dev(g), _dev(m), _dev(th)
    dgam = torch.from_numpy(gamma.copy()).to(DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    ctx.muon_step(dth, dg, dm, dgam, hp, mh, 4, stream=side.cuda_stream)
    side.synchronize()
    for i, s in enumerate(shapes):
        assert np.array_equal(to_numpy(dth[i]).reshape(s).view(np.uint32), ref[0][i].view(np.uint32))
        assert np.array_equal(to_numpy(dm[i]).reshape(s).view(np.uint32), ref[1][i].view(np.uint32))
    assert np.array_equal(to_numpy(dgam), ref[2])
    ctx.close()


def test_muon_attach_takes_smaller_batches_when_memory_is_short():
    """32 matrices of 14336 x 4096 want 17.2 GB of workspace; with about 12 GB free the attach settles for batches of 16
    (8.6 GB) instead of failing.  Only the context is created: attach needs no tensor."""
    shape, count = (14336, 4096), 32
    per_matrix = (4 * 4096 * 14336 + 2 * 4096 * 4096) * 2
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    leave = 12 << 30
    if free < leave + (1 << 30):
        pytest.skip("not enough free device memory to stage the shortage")
    hog = torch.empty(free - leave, dtype=torch.uint8, device=DEV)
    try:
        ctx = B.AdaGC([shape[0] * shape[1]] * count, B.ADAGC_OPT_MUON, B.ADAGC_GRAD_F32)
        ctx.muon_attach([shape] * count)
        assert ctx.muon_workspace_bytes() == 16 * per_matrix
        ctx.close()
    finally:
        del hog
        torch.cuda.empty_cache()
    ctx = B.AdaGC([shape[0] * shape[1]] * count, B.ADAGC_OPT_MUON, B.ADAGC_GRAD_F32)
    ctx.muon_attach([shape] * count)
    assert ctx.muon_workspace_bytes() == 32 * per_matrix
    ctx.close()
