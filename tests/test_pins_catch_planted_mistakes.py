"""Strength of the oracle's pins: each plausible mistake below is planted in a COPY of the oracle's source
(on the CPU, in a temporary directory), built, and the pin suite is run against it; every one must be
noticed.  The unmodified copy must pass."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "adagc_oracle.c")

MISTAKES = [
    ("epsilon inside the square root", "(sqrt(vhat) + hp->eps)", "sqrt(vhat + hp->eps)"),
    ("weight decay dropped from AdamW", "th - hp->lr * hp->weight_decay * th - ", "th - "),
    ("EMA fed the unclipped norm", "double clipped_norm = active ? threshold : norm;", "double clipped_norm = norm;"),
    ("clip on >= instead of >", "int active = (norm > threshold);", "int active = (norm >= threshold);"),
    ("second bias correction uses beta1", "double bias2 = 1.0 - pow(hp->beta2", "double bias2 = 1.0 - pow(hp->beta1"),
    ("Lion interpolation uses beta2", "double c = hp->beta1 * mprev + (1.0 - hp->beta1)",
     "double c = hp->beta2 * mprev + (1.0 - hp->beta2)"),
    ("Lion momentum built from the interpolation", "double mj = hp->beta2 * mprev + (1.0 - hp->beta2) * ghat;",
     "double mj = hp->beta2 * mprev + (1.0 - hp->beta2) * c;"),
    ("second moment without the square", "(1.0 - hp->beta2) * ghat * ghat", "(1.0 - hp->beta2) * ghat"),
    ("warm-up one step short", "int warmup = (step - 1) < hp->t_start;", "int warmup = step < hp->t_start;"),
    ("running maximum instead of minimum", "return clipped_norm < gamma_prev ? clipped_norm : gamma_prev;",
     "return clipped_norm > gamma_prev ? clipped_norm : gamma_prev;"),
    ("bf16 ties always round up", "(dropped == 0x8000u && (kept & 1u))", "(dropped == 0x8000u)"),
    ("coefficient applied after the moments", "double mj = hp->beta1 * (double)m[j] + (1.0 - hp->beta1) * ghat;",
     "double mj = hp->beta1 * (double)m[j] + (1.0 - hp->beta1) * grad_at(g, j, grad_dtype);"),
    ("global norm without the root", "double global_norm = sqrt(s);", "double global_norm = s;"),
    ("EMA weights swapped", "*gamma_new = beta * gamma_prev + (1.0 - beta) * clipped_norm;",
     "*gamma_new = (1.0 - beta) * gamma_prev + beta * clipped_norm;"),
    ("first bias correction dropped", "double mhat = mj / bias1;", "double mhat = mj;"),
    ("second bias correction dropped", "double vhat = vj / bias2;", "double vhat = vj;"),
    ("bias corrections one step late", "double bias1 = 1.0 - pow(hp->beta1, (double)t);",
     "double bias1 = 1.0 - pow(hp->beta1, (double)(t + 1));"),
    ("coefficient inverted", "double coef = active ? threshold / norm : 1.0;", "double coef = active ? norm / threshold : 1.0;"),
    ("warm-up minimum fed the unclipped norm", "gamma_new = oracle_warmup_gamma(gamma_prev, h * norm, step == 1);",
     "gamma_new = oracle_warmup_gamma(gamma_prev, norm, step == 1);"),
    ("first step keeps the initial gamma", "    if (first_step)\n        return clipped_norm;\n", ""),
    ("warm-up applies no global coefficient", "                h = h_global;\n                clipped = clipped_global;\n                gamma_new",
     "                h = 1.0;\n                clipped = 0;\n                gamma_new"),
    ("Lion: sign(0) taken as +1", "double sgn = (c > 0.0) ? 1.0 : ((c < 0.0) ? -1.0 : 0.0);",
     "double sgn = (c >= 0.0) ? 1.0 : -1.0;"),
    ("Lion: update from the new momentum", "double sgn = (c > 0.0) ? 1.0 : ((c < 0.0) ? -1.0 : 0.0);",
     "double cm = hp->beta2 * mprev + (1.0 - hp->beta2) * ghat; double sgn = (cm > 0.0) ? 1.0 : ((cm < 0.0) ? -1.0 : 0.0);"),
    ("GlobalGC coefficient not capped at 1", "return active ? lambda_abs / global_norm : 1.0;",
     "return lambda_abs / global_norm;"),
    ("updates read bf16 bits as integers", "return (double)oracle_bf16_to_float(((const uint16_t *)g)[j]);",
     "return (double)(((const uint16_t *)g)[j]);"),
    ("weight decay dropped from Lion", "th = th - hp->lr * (sgn + hp->weight_decay * th);", "th = th - hp->lr * sgn;"),
]


def _pins_pass(tmp_path, tag, source):
    c = os.path.join(str(tmp_path), "oracle_%s.c" % tag)
    so = os.path.join(str(tmp_path), "liboracle_%s.so" % tag)
    with open(c, "w") as f:
        f.write(source)
    subprocess.run(["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-w",
                    "-o", so, c, "-lm"], check=True)
    env = dict(os.environ, ADAGC_ORACLE_LIB=so)
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                          "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    return res.returncode == 0, res.stdout[-2000:]


def test_every_planted_mistake_is_caught(tmp_path):
    with open(SRC) as f:
        original = f.read()
    jobs = [("clean", original)]
    for k, (what, old, new) in enumerate(MISTAKES):
        assert original.count(old) >= 1, "pattern of '%s' no longer occurs in the oracle" % what
        jobs.append(("m%02d" % k, original.replace(old, new)))
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda j: _pins_pass(tmp_path, *j), jobs))
    assert results[0][0], "the unmodified oracle fails its own pins:\n" + results[0][1]
    survivors = [MISTAKES[k][0] for k, (ok, _) in enumerate(results[1:]) if ok]
    assert not survivors, "mistakes the pins do not notice: %s" % survivors
