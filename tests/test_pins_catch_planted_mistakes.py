"""Strength of the oracle's pins: each plausible mistake of tests/planted.py is planted in a COPY of the
oracle's source (on the CPU, in a temporary directory), built, and the pin suite is run against it; every
one must be noticed.  The unmodified copy must pass."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import planted


def _pins_pass(so):
    env = dict(os.environ, ADAGC_ORACLE_LIB=so)
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(planted.ROOT, "tests", "test_oracle_pins.py"),
                          "-x", "-q", "-p", "no:cacheprovider"], cwd=planted.ROOT, env=env, capture_output=True,
                         text=True, timeout=600)
    return res.returncode == 0, res.stdout[-2000:]


def test_every_planted_mistake_is_caught(tmp_path):
    libs = [planted.build(tmp_path, "clean", planted.source())]
    libs += [planted.build(tmp_path, "m%02d" % k, planted.mutated_source(k)) for k in range(len(planted.MISTAKES))]
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(_pins_pass, libs))
    assert results[0][0], "the unmodified oracle fails its own pins:\n" + results[0][1]
    survivors = [planted.MISTAKES[k][0] for k, (ok, _) in enumerate(results[1:]) if ok]
    assert not survivors, "mistakes the pins do not notice: %s" % survivors
