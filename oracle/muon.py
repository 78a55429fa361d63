"""CPU oracle for Muon with AdaGC on 2-D parameter tensors (numpy, float64).

TEST INFRASTRUCTURE ONLY: nothing in the GPU library or its binding imports this, and this imports
nothing of theirs.

The paper states that AdaGC "integrates" with Muon (Sec. 4.2; "Optimizer Compatibility: Muon and Lion",
Sec. 5.4) and prints neither Muon's rule nor its precision: "parity unpinned by the paper" for all of it.
What is written out here is the published algorithm (Jordan et al., "Muon: an optimizer for hidden layers
in neural networks"), with AdaGC's clipped gradient h*g in the place of the gradient, as Alg. 1 does for
AdamW:

    n = ||g||, h and gamma from Eq. 3 (or the warm-up branch)               -- the C oracle's functions
    M  <- mu M + h g                                                        (momentum, stored as float32)
    U   = h g + mu M            (Nesterov form)   or   U = M
    O   = NewtonSchulz(U)                                                   (approximately U's polar factor)
    theta <- theta - eta (lambda_w theta + sqrt(max(1, rows/cols)) O)       (stored as float32)

Newton-Schulz, 5 steps with (a, b, c) = (3.4445, -4.7750, 2.0315):
    X = U / (||U||_F + 1e-7), transposed if rows > cols
    A = X X^T;  B = b A + c A A;  X <- a X + B X
Storage of the iteration: the published reference runs it in bf16, and so does the GPU (bf16 matrix-core
operands, wider accumulation): X, A and B are rounded to bf16 (via float32, round to nearest even) once each
time they are produced.  storage="exact" keeps float64 throughout: that form has a closed form through the
SVD (the odd polynomial acts on the singular values), which is what pins it.
"""
import math

import numpy as np

NS_COEFFS = (3.4445, -4.7750, 2.0315)
NS_EPS = 1e-7


def to_bf16(x):
    """float64 array -> the same values rounded to float32 and then to bf16 (nearest even), as float64."""
    f = np.ascontiguousarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32)
    kept = u >> 16
    dropped = u & 0xFFFF
    up = (dropped > 0x8000) | ((dropped == 0x8000) & ((kept & 1) == 1))
    out = ((kept + up.astype(np.uint32)) << 16).astype(np.uint32)
    nan = np.isnan(f)
    res = out.view(np.float32).astype(np.float64)
    res[nan] = np.nan
    return res


def bf16_bits(x):
    """The bf16 bit patterns (uint16) of values that are already bf16-representable."""
    return (np.ascontiguousarray(x, dtype=np.float64).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)


def ns_iterate(x, steps, coeffs=NS_COEFFS, storage="bf16", trace=None):
    """`steps` passes of A = X X^T; B = b A + c A A; X <- a X + B X on an already normalised wide matrix."""
    a, b, c = coeffs
    rnd = to_bf16 if storage == "bf16" else (lambda z: z)
    x = np.asarray(x, dtype=np.float64)
    for k in range(steps):
        gram = rnd(x @ x.T)
        poly = rnd(b * gram + c * (gram @ gram))
        x = rnd(a * x + poly @ x)
        if trace is not None:
            trace += [("A%d" % (k + 1), gram), ("B%d" % (k + 1), poly), ("X%d" % (k + 1), x)]
    return x


def normalise(u, storage="bf16"):
    """X0: U over its Frobenius norm (plus the 1e-7 guard), transposed if it is tall, as stored."""
    rnd = to_bf16 if storage == "bf16" else (lambda z: z)
    u = np.asarray(u, dtype=np.float64)
    x = u.T if u.shape[0] > u.shape[1] else u
    return rnd(x / (math.sqrt(float(np.sum(u * u))) + NS_EPS))


def newton_schulz(u, steps=5, coeffs=NS_COEFFS, storage="bf16", trace=None):
    """The iteration above on one matrix (float64 in, float64 out, same shape).  trace: a list that
    receives (name, matrix) for every stored intermediate, in the order they are produced."""
    u = np.asarray(u, dtype=np.float64)
    x = normalise(u, storage)
    if trace is not None:
        trace.append(("X0", x))
    x = ns_iterate(x, steps, coeffs, storage, trace)
    return x.T if u.shape[0] > u.shape[1] else x


def ns_scalar_map(sigma, steps=5, coeffs=NS_COEFFS):
    """What the exact iteration does to one singular value: the odd polynomial, `steps` times."""
    a, b, c = coeffs
    s = np.asarray(sigma, dtype=np.float64)
    for _ in range(steps):
        s = a * s + b * s ** 3 + c * s ** 5
    return s


def update_scale(rows, cols):
    return math.sqrt(max(1.0, rows / cols))


def muon_update(theta, g, momentum, h, lr, weight_decay, mu, nesterov=True, steps=5, storage="bf16"):
    """One tensor: theta, momentum float32 2-D arrays updated in place; g float32; h the gradient's clip
    coefficient.  Hyper-parameters are taken as the float32 values a caller hands over.  Returns O."""
    f = lambda v: float(np.float32(v))
    lr, weight_decay, mu = f(lr), f(weight_decay), f(mu)
    ghat = h * g.astype(np.float64)
    m_new = (mu * momentum.astype(np.float64) + ghat).astype(np.float32)
    momentum[...] = m_new
    u = ghat + mu * m_new.astype(np.float64) if nesterov else m_new.astype(np.float64)
    o = newton_schulz(u, steps=steps, storage=storage)
    th = theta.astype(np.float64)
    theta[...] = (th - lr * (weight_decay * th + update_scale(*theta.shape) * o)).astype(np.float32)
    return o
