"""GPU parity of the Muon path against the numpy oracle (oracle/muon.py), through the C ABI."""
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


@pytest.mark.parametrize("M,N,K,ld_extra", [(128, 128, 64, 0), (256, 384, 192, 8), (128, 512, 1024, 64), (1024, 1024, 4096, 0)])
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
    z = torch.zeros((128, 64), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros((128, 128), dtype=torch.bfloat16, device=DEV)
    for P, Q in [(z[:100], z), (z[:, :32], z[:, :32])]:
        with pytest.raises(B.AdagcError) as e:
            B.adagc_muon_gemm_nt(P, Q, 1.0, 0.0, None, out[:P.shape[0]], None)
        assert e.value.code == B.ADAGC_ERR_INVALID_ARG
    with pytest.raises(B.AdagcError):
        B.adagc_muon_gemm_nt(z, z, 1.0, 0.0, None, None, None)
