"""Two measurements of the bf16 matrix-core product of the Muon path, through the library's own entry point
(adagc_muon_gemm_nt_batched).  A measurement tool like memory_probe.py, not part of the library.

  1. the rate of one shape on operands of different values (zeros, ones, sparse, normal random): on a part that runs
     against its power limit, the same instruction stream is faster on data that toggles fewer bits;
  2. time per round of 256 output tiles against the depth K, for the three output combinations the Newton-Schulz
     products use: the slope is the main loop's time per 64-deep operand tile, the intercept the fixed cost per
     output tile (first operand load, epilogue).

    python3 -m paper_2502_11034_amd.gemm_probe
"""
import torch

from . import binding as B

DEV = "cuda:0"


def timed(fn, reps):
    for _ in range(2):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def operand_values():
    batch, M, N, K = 2, 4096, 4096, 32768
    C = torch.zeros(batch, M, N, dtype=torch.bfloat16, device=DEV)
    Ct = torch.zeros(batch, N, M, dtype=torch.bfloat16, device=DEV)
    gens = [("zeros", lambda s: torch.zeros(s, device=DEV)),
            ("ones", lambda s: torch.ones(s, device=DEV)),
            ("normal random, one value in eight non-zero", lambda s: torch.randn(s, device=DEV) * (torch.rand(s, device=DEV) < 0.125)),
            ("normal random", lambda s: torch.randn(s, device=DEV) * 0.05),
            ("zeros again", lambda s: torch.zeros(s, device=DEV))]
    print("1. %d products of %d x %d x %d (C and Ct written, no D), by operand values" % (batch, M, N, K))
    for name, gen in gens:
        P = gen((batch, M, K)).to(torch.bfloat16)
        Q = gen((batch, N, K)).to(torch.bfloat16)
        ms = timed(lambda: B.adagc_muon_gemm_nt_batched(P, Q, 1.0, 0.0, None, C, Ct), 10)
        print("   %-46s %8.3f ms %8.0f TFLOP/s" % (name, ms, batch * 2.0 * M * N * K / ms / 1e9), flush=True)


def fixed_cost():
    batch, M, N = 16, 4096, 4096
    rounds = batch * (M // 256) * (N // 256) / 256.0
    Dt = (torch.randn(batch, N, M, device=DEV) * 0.05).to(torch.bfloat16)
    C = torch.zeros(batch, M, N, dtype=torch.bfloat16, device=DEV)
    Ct = torch.zeros(batch, N, M, dtype=torch.bfloat16, device=DEV)
    print("2. %d products of %d x %d x K on 256 x 256 tiles (%d rounds of 256 tiles): microseconds per round" % (batch, M, N, rounds))
    for mode, kw in (("Ct", dict(Dt=None, C=None, Ct=Ct)), ("C + Ct", dict(Dt=None, C=C, Ct=Ct)), ("D + C + Ct", dict(Dt=Dt, C=C, Ct=Ct))):
        pts = []
        for K in (128, 256, 512, 1024, 2048, 4096, 8192):
            P = (torch.randn(batch, M, K, device=DEV) * 0.05).to(torch.bfloat16)
            Q = (torch.randn(batch, N, K, device=DEV) * 0.05).to(torch.bfloat16)
            ms = timed(lambda: B.adagc_muon_gemm_nt_batched(P, Q, 1.0, 0.5, kw["Dt"], kw["C"], kw["Ct"]), 5)
            pts.append((K // 64, ms * 1000.0 / rounds))
        xs, ys = [p[0] for p in pts[2:]], [p[1] for p in pts[2:]]             # least squares over K >= 512
        n = len(xs)
        mx, my = sum(xs) / n, sum(ys) / n
        slope = sum((x - mx) * (y - my) for x, y in zip(xs, ys)) / sum((x - mx) ** 2 for x in xs)
        print("   %-11s %s  ->  %.2f us per 64-deep operand tile + %.1f us per output tile"
              % (mode, " ".join("K=%d: %.1f" % (k * 64, t) for k, t in pts), slope, my - slope * mx), flush=True)


if __name__ == "__main__":
    operand_values()
    fixed_cost()
