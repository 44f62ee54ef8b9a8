"""Are the checker's pins tight?  Every entry of tests/oracle_mutants.py is one plausible slip
(a dropped term, a wrong sign or index, a transposed operand, a missing square, an off-by-one)
planted in a COPY of oracle/tabx_ref.cpp; the pin tests, run against that copy, must fail.
CPU only; nothing here touches the GPU library or the committed checker.
"""
import concurrent.futures as cf
import os
import subprocess
import sys

from tests.oracle_mutants import MUTANTS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "tabx_ref.cpp")
# the pin tests, quickest killers first
PINS = ["tests/test_oracle_pins.py", "tests/test_oracle_pins_edges.py",
        "tests/test_oracle_policy.py", "tests/test_oracle_policy_roles.py", "tests/test_oracle_levels.py",
        "tests/test_oracle_hurtbox_variants.py", "tests/test_oracle_dynamics.py",
        "tests/test_oracle_rollouts.py"]


def test_every_planted_mistake_occurs_exactly_once_in_the_checker():
    src = open(SRC).read()
    names = [n for n, _, _ in MUTANTS]
    assert len(set(names)) == len(names)
    for name, old, new in MUTANTS:
        assert src.count(old) == 1, name
        assert old != new, name


def _pins_fail_on(args):
    name, old, new, src, tmp = args
    d = os.path.join(tmp, name)
    os.makedirs(d)
    cpp, lib = os.path.join(d, "tabx_ref.cpp"), os.path.join(d, "libtabx_ref_mutant.so")
    with open(cpp, "w") as f:
        f.write(src.replace(old, new))
    c = subprocess.run(["g++", "-O1", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-shared",
                        "-fPIC", "-I", os.path.join(ROOT, "oracle"), cpp, "-o", lib],
                       capture_output=True, text=True)
    if c.returncode != 0:
        return name, "does not compile: " + c.stderr[-300:]
    t = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + PINS,
                       capture_output=True, text=True, cwd=ROOT, timeout=600,
                       env=dict(os.environ, TABX_REF_LIB=lib))
    if t.returncode == 1:          # pytest: tests were collected and run, some failed
        return name, None
    return name, f"pins gave exit status {t.returncode}: " + t.stdout[-300:]


def test_pins_fail_on_every_planted_mistake(tmp_path):
    src = open(SRC).read()
    jobs = [(n, o, r, src, str(tmp_path)) for n, o, r in MUTANTS]
    workers = max(1, min(8, os.cpu_count() or 1))
    with cf.ThreadPoolExecutor(workers) as ex:
        verdicts = list(ex.map(_pins_fail_on, jobs))
    survivors = [(n, why) for n, why in verdicts if why is not None]
    assert not survivors, survivors
