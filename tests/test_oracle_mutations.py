"""How strong are the oracle's pins?  Plant one plausible mistake at a time in a COPY of the oracle's C
source (a dropped scale, a wrong head map, a reversed tie-break, a transposed index ...), rebuild the
copy and run tests/test_oracle_pins.py against it: every mutant must fail at least one pin.  The
repository's own oracle is never touched; nothing here uses the GPU."""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)

# (name, text in oracle/mage_oracle.c, replacement)
MUTANTS = [
    ("logit scale dropped", "return acc / sqrt((double)d);", "return acc;"),
    ("query head -> KV head interleaved", "const int h = g / G;", "const int h = g % Hkv;"),
    ("attention rows: KV head interleaved", "g = r % Hq, h = g / G;", "g = r % Hq, h = g % Hkv;"),
    ("tie-break to the larger index", "return (x->j > y->j) - (x->j < y->j);", "return (x->j < y->j) - (x->j > y->j);"),
    ("block average not divided by B", "row[j] /= (double)B;", "row[j] /= 1.0;"),
    ("group average not divided by G", "= acc / (double)G;", "= acc;"),
    ("in-block keys ignored", "const int nb = k_blk ? nb_in : 0;", "const int nb = 0;"),
    ("value row taken by position in the set, not by index", "vrow = vc + ((size_t)j * Hkv + h) * d;", "vrow = vc + ((size_t)t * Hkv + h) * d;"),
    ("query layout [Hq,B,d] instead of [B,Hq,d]", "const float *qrow = q1 + ((size_t)q * Hq + g) * d;", "const float *qrow = q1 + ((size_t)g * B + q) * d;"),
    ("log-sum-exp without its maximum", "(float)(m + log(Z))", "(float)(log(Z))"),
    ("group sum over interleaved heads", "for (int g = h * G; g < (h + 1) * G; ++g)\n                    acc", "for (int g = h; g < Hq; g += Hkv)\n                    acc"),
    ("page estimate: group sum over interleaved heads", "for (int g = h * G; g < (h + 1) * G; ++g)\n            for (int qi", "for (int g = h; g < Hq; g += Hkv)\n            for (int qi"),
    # second workload (page estimator, overlap)
    ("page bound from the maxima alone", "acc += a > b ? a : b;", "acc += a;"),
    ("page bound takes the smaller product", "acc += a > b ? a : b;", "acc += a < b ? a : b;"),
    ("page bound not scaled by 1/sqrt(d)", "kmin + ((size_t)P * Hkv + h) * d, d) /\n                                     sqrt((double)d);", "kmin + ((size_t)P * Hkv + h) * d, d);"),
    ("page minimum is the maximum", "if (v < mn) mn = v;", "if (v > mn || mn == INFINITY) mn = v;"),
    ("estimate not averaged over the block", "row[j] /= (double)G * (double)B;", "row[j] /= (double)G;"),
    ("overlap compares position by position", "for (int j = 0; j < k; ++j)\n            if (a[i] == b[j]) {", "for (int j = i; j <= i; ++j)\n            if (a[i] == b[j]) {"),
    ("overlap divided by the wrong size", "return (double)common / (double)k;", "return (double)common / (double)(k + 1);"),
]


def _run_mutant(args):
    i, (name, old, new), base = args
    d = os.path.join(base, f"m{i}")
    os.makedirs(os.path.join(d, "tests"))
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(d, "oracle"),
                    ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    for f in ("conftest.py", "test_oracle_pins.py"):
        shutil.copy(os.path.join(HERE, f), os.path.join(d, "tests", f))
    src = os.path.join(d, "oracle", "mage_oracle.c")
    text = open(src).read()
    if text.count(old) < 1:
        return name, "pattern not found in the oracle source"
    open(src, "w").write(text.replace(old, new))
    env = dict(os.environ, PYTHONDONTWRITEBYTECODE="1", OMP_NUM_THREADS="2")
    env.pop("PYTHONPATH", None)
    # the stored-output fixture would notice any change of arithmetic: it is left out, so that only
    # the independent pins (closed forms, library routines, invariants) count
    r = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-p", "no:cacheprovider",
                        "-k", "not worked_example"],
                       cwd=d, env=env, capture_output=True, text=True, timeout=600)
    if r.returncode == 0:
        return name, "SURVIVED: no pin noticed"
    if " failed" not in r.stdout:
        return name, "did not run: " + (r.stdout + r.stderr)[-500:]
    return name, None


def test_every_planted_mistake_fails_a_pin(tmp_path):
    jobs = [(i, m, str(tmp_path)) for i, m in enumerate(MUTANTS)]
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(_run_mutant, jobs))
    bad = [(n, why) for n, why in results if why]
    assert not bad, bad
