"""Strength of the Muon oracle's pins: each plausible mistake below is planted in a COPY of oracle/muon.py (a textual
replacement, in a temporary directory) and tests/test_muon_oracle_pins.py is run against the copy; every one must be
noticed, and the unmodified copy must pass."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "muon.py")

MISTAKES = [
    ("b and c exchanged", "poly = rnd(b * gram + c * (gram @ gram))", "poly = rnd(c * gram + b * (gram @ gram))"),
    ("a dropped from the update of X", "x = rnd(a * x + poly @ x)", "x = rnd(x + poly @ x)"),
    ("polynomial applied from the right", "x = rnd(a * x + poly @ x)", "x = rnd(a * x + (x @ poly if x.shape[0] == x.shape[1] else poly @ x))"),
    ("tall matrices not transposed", "x = u.T if u.shape[0] > u.shape[1] else u\n    return rnd(", "x = u\n    return rnd("),
    ("spectral norm instead of Frobenius", "math.sqrt(float(np.sum(u * u)))", "float(np.linalg.norm(u, 2))"),
    ("guard dropped from the norm", "math.sqrt(float(np.sum(u * u))) + NS_EPS", "math.sqrt(float(np.sum(u * u)))"),
    ("Nesterov term without the momentum factor", "u = ghat + mu * m_new.astype(np.float64) if nesterov", "u = ghat + m_new.astype(np.float64) if nesterov"),
    ("Nesterov and plain momentum exchanged", "u = ghat + mu * m_new.astype(np.float64) if nesterov else m_new.astype(np.float64)",
     "u = m_new.astype(np.float64) if nesterov else ghat + mu * m_new.astype(np.float64)"),
    ("clip coefficient dropped", "ghat = h * g.astype(np.float64)", "ghat = g.astype(np.float64)"),
    ("momentum as an average", "m_new = (mu * momentum.astype(np.float64) + ghat)", "m_new = (mu * momentum.astype(np.float64) + (1.0 - mu) * ghat)"),
    ("update scale without the root", "return math.sqrt(max(1.0, rows / cols))", "return max(1.0, rows / cols)"),
    ("update scale upside down", "return math.sqrt(max(1.0, rows / cols))", "return math.sqrt(max(1.0, cols / rows))"),
    ("decay outside the learning rate", "(th - lr * (weight_decay * th + update_scale(*theta.shape) * o))", "(th - weight_decay * th - lr * update_scale(*theta.shape) * o)"),
    ("bf16 ties always round up", "(dropped > 0x8000) | ((dropped == 0x8000) & ((kept & 1) == 1))", "(dropped >= 0x8000)"),
    ("A not rounded when stored", "gram = rnd(x @ x.T)", "gram = x @ x.T"),
    ("B not rounded when stored", "poly = rnd(b * gram + c * (gram @ gram))", "poly = b * gram + c * (gram @ gram)"),
    ("one step short", "for k in range(steps):", "for k in range(steps - 1):"),
    ("first coefficient mistyped", "NS_COEFFS = (3.4445,", "NS_COEFFS = (3.4455,"),
    ("A A from the unrounded A", "poly = rnd(b * gram + c * (gram @ gram))", "poly = rnd(b * gram + c * ((x @ x.T) @ (x @ x.T)))"),
    ("result of a tall matrix not transposed back", "return x.T if u.shape[0] > u.shape[1] else x", "return x"),
]


def _mutated(k):
    text = open(SRC).read()
    if k is None:
        return text
    _, old, new = MISTAKES[k]
    assert text.count(old) == 1, "mistake %d: its anchor occurs %d times in the oracle's source" % (k, text.count(old))
    return text.replace(old, new)


def _pins_pass(path):
    env = dict(os.environ, ADAGC_MUON_ORACLE_SRC=path)
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_muon_oracle_pins.py"), "-x", "-q",
                          "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    return res.returncode == 0, res.stdout[-2000:]


def test_every_planted_mistake_is_caught(tmp_path):
    paths = []
    for k in [None] + list(range(len(MISTAKES))):
        path = os.path.join(str(tmp_path), "muon_%s.py" % ("clean" if k is None else "m%02d" % k))
        with open(path, "w") as f:
            f.write(_mutated(k))
        paths.append(path)
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(_pins_pass, paths))
    assert results[0][0], "the unmodified oracle fails its own pins:\n" + results[0][1]
    survivors = [MISTAKES[k][0] for k, (ok, _) in enumerate(results[1:]) if ok]
    assert not survivors, "mistakes the pins do not notice: %s" % survivors
