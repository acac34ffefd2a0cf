"""Mutation sweep over the CPU oracle (not collected by pytest; run by hand: python tests/oracle_mutation_sweep.py).

Every arithmetic or comparison operator of oracle/gp_dense.py is swapped for its counterpart and every numeric
literal is changed, one at a time; each mutant is copied to a scratch directory together with the oracle's pin tests
(tests/test_oracle_*.py, tests/golden/) and the suite is run against it. A mutant that the pins do not reject is
printed. The survivors that remain are listed, with the reason each is harmless, in the design notes.

CPU only; about five minutes on eight cores. Optional arguments: line numbers of gp_dense.py to restrict the sweep to.
"""
import io
import os
import re
import shutil
import subprocess
import sys
import tempfile
import tokenize
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SWAP = {"+": "-", "-": "+", "*": "/", "/": "*", "<": ">=", ">": "<=", "<=": ">", ">=": "<", "+=": "-=", "-=": "+=",
        "**": "*"}


def mutants(src):
    out = []
    for t in tokenize.generate_tokens(io.StringIO(src).readline):
        if t.start[0] != t.end[0]:
            continue
        if t.type == tokenize.OP and t.string in SWAP:
            out.append((t.start, t.end, SWAP[t.string]))
        elif t.type == tokenize.NUMBER:
            try:
                v = float(t.string)
            except ValueError:
                continue
            out.append((t.start, t.end, str(int(v) + 1) if re.fullmatch(r"\d+", t.string) else repr(v * 1.5 + 0.25)))
    return out


def run_one(lines, mut):
    (row, c0), (_, c1), new = mut
    changed = list(lines)
    old = changed[row - 1]
    changed[row - 1] = old[:c0] + new + old[c1:]
    work = tempfile.mkdtemp(prefix="oracle_mutant_")
    try:
        for sub in ("oracle", "workloads"):
            shutil.copytree(os.path.join(ROOT, sub), os.path.join(work, sub), ignore=shutil.ignore_patterns("__pycache__"))
        os.makedirs(os.path.join(work, "tests"))
        shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(work, "tests", "golden"))
        for f in os.listdir(os.path.join(ROOT, "tests")):
            if f.startswith("test_oracle") or f == "conftest.py":
                shutil.copy(os.path.join(ROOT, "tests", f), os.path.join(work, "tests", f))
        with open(os.path.join(work, "oracle", "gp_dense.py"), "w") as fh:
            fh.write("\n".join(changed))
        env = dict(os.environ, OMP_NUM_THREADS="1", OPENBLAS_NUM_THREADS="1", MKL_NUM_THREADS="1",
                   PYTHONDONTWRITEBYTECODE="1")
        try:
            res = subprocess.run([sys.executable, "-m", "pytest", "tests", "-x", "-q", "-m", "not gpu", "-p",
                                  "no:cacheprovider"], cwd=work, env=env, capture_output=True, text=True, timeout=900)
            survived = res.returncode == 0
        except subprocess.TimeoutExpired:
            survived = False
        return survived, f"line {row}, column {c0}: '{old[c0:c1]}' -> '{new}'   | {old.strip()}"
    finally:
        shutil.rmtree(work, ignore_errors=True)


def main():
    src = open(os.path.join(ROOT, "oracle", "gp_dense.py")).read()
    lines = src.split("\n")
    muts = mutants(src)
    keep = {int(a) for a in sys.argv[1:]}
    if keep:
        muts = [m for m in muts if m[0][0] in keep]
    print(len(muts), "mutants", flush=True)
    survivors = 0
    with ThreadPoolExecutor(max(1, min(7, (os.cpu_count() or 2) - 1))) as pool:
        for survived, what in pool.map(lambda m: run_one(lines, m), muts):
            if survived:
                survivors += 1
                print("SURVIVED", what, flush=True)
    print("survivors:", survivors, "of", len(muts), flush=True)


if __name__ == "__main__":
    main()
