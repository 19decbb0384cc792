"""Do the pins bite?  Each case plants ONE plausible mistake in a private copy of the oracle's C
source (a wrong band edge, modulus, prime, slot stride, a dropped clamp or term, a transposed
operand, a wrong rounding ...), rebuilds that copy and runs the oracle's pin tests against it in a
child process: a pin must fail (or the mutant must crash under the pins).  The unmodified copy must
pass, so a failure is the mistake's.
CPU only; nothing here touches the GPU path or the real oracle files."""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["test_oracle_sampling.py", "test_oracle_spmm.py", "test_oracle_quant.py"]

# (name, text in oracle/aes_oracle.c, replacement); every text occurs exactly once
MUTATIONS = [
    ("Table 1: band edge 36 -> 35", "row_nnz <= 36 * sh_width", "row_nnz <= 35 * sh_width"),
    ("Table 1: band edge 54 -> 56", "row_nnz <= 54 * sh_width", "row_nnz <= 56 * sh_width"),
    ("Table 1: R <= 2 read as R < 2", "row_nnz <= 2 * sh_width", "row_nnz < 2 * sh_width"),
    ("Table 1: sample counts 8 and 16 swapped", "c = 8;", "c = 16; /* swapped */"),
    ("rows that fit are no longer kept whole", "if (row_nnz <= sh_width) {", "if (row_nnz < sh_width) {"),
    ("clamp sample_cnt <= W dropped", "if (c > sh_width) c = sh_width;", ""),
    ("clamp N >= 1 dropped", "if (n < 1) n = 1;", ""),
    ("Eq. 3: prime 1429 -> 1427", "prime_num = 1429u", "prime_num = 1427u"),
    ("Eq. 3: modulus row_nnz - N + 1 -> row_nnz - N + 2", "(uint64_t)(row_nnz - N + 1)", "(uint64_t)(row_nnz - N + 2)"),
    ("Eq. 3: modulus forgets N", "(uint64_t)(row_nnz - N + 1)", "(uint64_t)(row_nnz + 1 - 1)"),
    ("slot layout: runs stored one after another", "const int64_t slot = pos * sample_cnt + run;", "const int64_t slot = run * N + pos;"),
    ("a run repeats its first element", "slot_col[slot] = col_ind[first + pos];", "slot_col[slot] = col_ind[first];"),
    ("value taken from the neighbouring element", "slot_val[slot] = val[first + pos];",
     "slot_val[slot] = val[first + (pos + 1 < N ? pos + 1 : pos)];"),
    ("seed offset: odd multiplier lost", "(2u * (uint64_t)rid + 1u)", "(2u * (uint64_t)rid)"),
    ("AFS and SFS exchanged", "} else if (mode == 1) {", "} else if (mode == 2) {"),
    ("multiply stage: last slot of a row dropped", "k < s_rowptr[r + 1]; ++k", "k < s_rowptr[r + 1] - 1; ++k"),
    ("multiply stage: X indexed transposed", "const float *x = X + (int64_t)s_col[k] * ldx;",
     "const float *x = X + (int64_t)s_col[k];"),
    ("one-pass form: X indexed transposed", "X[(int64_t)sh_col[k] * ldx + c]", "X[(int64_t)sh_col[k] + c * ldx]"),
    ("one-pass form: value not applied", "(double)sh_val[k] * (double)X[", "(double)X["),
    ("sum of |terms| accumulates signed terms", "if (ya) ya[c] += fabs(p);", "if (ya) ya[c] += p;"),
    ("combination: Theta transposed", "Theta[c * ldt + o]", "Theta[o * ldt + c]"),
    ("Eq. 1: floor -> round to nearest", "q = (int)floorf(t);", "q = (int)rintf(t);"),
    ("Eq. 1: 255 levels -> 256", "t = t * 255.0f;", "t = t * 256.0f;"),
    ("Eq. 1: x_min not subtracted", "float t = (x - lo[g]) / d;", "float t = x / d;"),
    ("symmetric: round half even -> truncate", "int q = (int)rintf(t);", "int q = (int)(t);"),
    ("symmetric: 127 -> 128", "a / 127.0f", "a / 128.0f"),
    ("symmetric: absolute value forgotten", "x = fabsf(x);", "x = x;"),
    ("Eq. 2: zero point dropped", "Xhat[i * ldx + c] = t + zero[g];", "Xhat[i * ldx + c] = t;"),
    ("Eq. 2: unsigned codes read as signed", "(float)((const uint8_t *)Xq)[i * ldq + c]", "(float)Xq[i * ldq + c]"),
    ("groups: per column and per row exchanged", "granularity == ORC_Q_PER_COLUMN ? c : i",
     "granularity == ORC_Q_PER_COLUMN ? i : c"),
]


def _run_pins(copy_root):
    env = dict(os.environ, PYTHONPATH="", OMP_NUM_THREADS="1")
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"]
    cmd += [os.path.join(copy_root, "tests", f) for f in PIN_FILES]
    return subprocess.run(cmd, cwd=copy_root, env=env, capture_output=True, text=True)


def _sandbox(root, source_text):
    """A private tree with the oracle (its C source = source_text) and its pin tests; conftest
    resolves `oracle` next to `tests`, so the child process never sees the real oracle."""
    os.makedirs(os.path.join(root, "oracle"))
    shutil.copy(os.path.join(ROOT, "oracle", "__init__.py"), os.path.join(root, "oracle", "__init__.py"))
    with open(os.path.join(root, "oracle", "aes_oracle.c"), "w") as f:
        f.write(source_text)
    os.makedirs(os.path.join(root, "tests"))
    for f in PIN_FILES + ["conftest.py", "helpers.py"]:
        shutil.copy(os.path.join(ROOT, "tests", f), os.path.join(root, "tests", f))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(root, "tests", "golden"))
    os.symlink(os.path.join(ROOT, "workloads"), os.path.join(root, "workloads"))
    return root


def test_every_planted_mistake_is_caught(tmp_path):
    original = open(os.path.join(ROOT, "oracle", "aes_oracle.c")).read()
    for name, old, _ in MUTATIONS:
        assert original.count(old) == 1, f"mutation site of '{name}' not found exactly once: {old!r}"

    def attempt(job):
        k, (name, old, new) = job
        text = original if old is None else original.replace(old, new)
        done = _run_pins(_sandbox(str(tmp_path / f"m{k}"), text))
        last = (done.stdout.strip().splitlines() or [""])[-1]
        return name, done.returncode, last, done.stderr[-300:]

    jobs = list(enumerate([("unmodified", None, None)] + MUTATIONS))
    with ThreadPoolExecutor(max_workers=6) as pool:
        results = list(pool.map(attempt, jobs))
    name, rc, last, err = results[0]
    assert rc == 0, f"the pins must pass on the unmodified copy: {last} {err}"
    survivors, broken = [], []
    for name, rc, last, err in results[1:]:
        if rc == 0:
            survivors.append(name)
        elif rc > 0 and " failed" not in last:          # neither a failed pin nor a crash of the mutant: a build problem
            broken.append((name, last, err))
    assert not survivors, f"no pin noticed: {survivors}"
    assert not broken, broken
