"""Mutation check of the CPU oracle (no GPU, not collected by pytest): plant one small mistake at a time --
an operator, a comparison, a constant, an index, a cast -- in a private copy of oracle/lioncub_oracle.c
(or, with MUT_FILE=__init__.py, of the Python side), rebuild, run the oracle's pin tests on the copy, and
list the mistakes that no pin catches.  What survives should be equivalent code (a cast of a value that
already has the type, a bound that no caller reaches); anything else is a missing pin.

    python tests/oracle_mutation_check.py            # about ten minutes on 8 cores
"""
import os
import re
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FILE = os.environ.get("MUT_FILE", "lioncub_oracle.c")
IS_PYTHON = FILE.endswith(".py")
SOURCE = open(os.path.join(ROOT, "oracle", FILE)).read().split("\n")
TESTS = ["test_oracle_pins.py", "test_oracle_l1.py"] + sys.argv[1:]
WORKERS = 8

# (pattern, replacement): every match on a code line is one planted mistake
RULES = [
    (r"(?<![+\-eE(,=*/<>&|!?:] )(?<![+\-eE(,=])\s\+\s", " - "), (r"\s-\s", " + "), (r"\s\*\s", " + "), (r"\s/\s", " * "),
    (r"\s<\s", " <= "), (r"\s<=\s", " < "), (r"\s>\s", " >= "), (r"\s>=\s", " > "), (r"\s<\s", " > "), (r"\s>\s", " < "),
    (r"==", "!="), (r"!=", "=="), (r"&&", "||"), (r"\|\|", "&&"), (r"\+=", "-="), (r"-=", "+="),
    (r"\b0\b", "1"), (r"\b1\b", "0"), (r"\b1\b", "2"), (r"\b2\b", "1"), (r"\b2\b", "3"), (r"<<", ">>"), (r">>", "<<"),
    (r"\s&\s", " | "), (r"\s\|\s", " & "), (r"\b63\b", "62"), (r"\b64\b", "63"), (r"\b8\b", "7"),
    (r"\b0\.0f?\b", "1.0f"), (r"\b1\.0f?\b", "0.5f"), (r"\b0\.5\b", "0.25"),
    (r"\bi\]", "i + 1]"), (r"\bw\]", "w + 1]"), (r"\+\+", "--"), (r"\? (\S+) : (\S+?)([;)])", r"? \2 : \1\3"),
    (r"-1\b", "1"), (r"\bfloor\b", "ceil"), (r"\bfabs\b", ""), (r"\bfabsf\b", ""), (r"\(float\)", ""), (r"\(double\)", "(float)"),
]


def code_lines():
    """(line number, code, trailing comment) of every line that holds code: block comments, docstrings,
    preprocessor lines and, on the Python side, the ctypes signature table at the top are skipped."""
    in_block = False
    mark = '"""' if IS_PYTHON else "/*"
    for ln, line in enumerate(SOURCE):
        st = line.strip()
        if in_block:
            in_block = ('"""' not in st) if IS_PYTHON else ("*/" not in st)
            continue
        if st.startswith(mark):
            closed = st.count('"""') >= 2 if IS_PYTHON else "*/" in st
            in_block = not closed
            continue
        if not st or st.startswith("#") or st.startswith("//") or st.startswith("*") or (IS_PYTHON and ln < 28):
            continue
        at = line.find("#" if IS_PYTHON else "//")
        yield (ln, line, "") if at < 0 else (ln, line[:at], line[at:])


def mutants():
    out = []
    for ln, body, tail in code_lines():
        for pattern, replacement in RULES:
            for found in re.finditer(pattern, body):
                new = body[:found.start()] + found.expand(replacement) + body[found.end():]
                if new != body:
                    out.append((ln, new + tail))
    return out


def worker(slot, jobs, work, results):
    """A private tree (oracle/ and the pin tests) per worker; one mutant at a time goes through it."""
    tree = os.path.join(work, "w%d" % slot)
    os.makedirs(os.path.join(tree, "oracle"))
    os.makedirs(os.path.join(tree, "tests"))
    for f in ("__init__.py", "build.py", "lioncub_oracle.c"):
        shutil.copy(os.path.join(ROOT, "oracle", f), os.path.join(tree, "oracle", f))
    for f in TESTS + ["conftest.py"]:
        shutil.copy(os.path.join(ROOT, "tests", f), os.path.join(tree, "tests", f))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(tree, "tests", "golden"))
    for ln, new in jobs:
        lines = list(SOURCE)
        lines[ln] = new
        with open(os.path.join(tree, "oracle", FILE), "w") as f:
            f.write("\n".join(lines))
        built = subprocess.run([sys.executable, os.path.join(tree, "oracle", "build.py")], cwd=tree, capture_output=True)
        if built.returncode != 0:
            results.append((ln, new, "does not compile"))
            continue
        try:
            run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + ["tests/" + t for t in TESTS],
                                 cwd=tree, capture_output=True, timeout=120)
            results.append((ln, new, "caught" if run.returncode != 0 else "SURVIVED"))
        except subprocess.TimeoutExpired:
            results.append((ln, new, "caught (time limit)"))
        if len(results) % 50 == 0:
            print(len(results), "done", flush=True)


def main():
    planted = mutants()
    print(len(planted), "mistakes to plant in oracle/%s" % FILE, flush=True)
    work = tempfile.mkdtemp(prefix="oracle_mutants_")
    results = []
    try:
        with ThreadPoolExecutor(WORKERS) as pool:
            for slot in range(WORKERS):
                pool.submit(worker, slot, planted[slot::WORKERS], work, results)
    finally:
        shutil.rmtree(work, ignore_errors=True)
    results.sort()
    tally = {}
    for _, _, verdict in results:
        tally[verdict] = tally.get(verdict, 0) + 1
    print(tally)
    for ln, new, verdict in results:
        if verdict == "SURVIVED":
            print("%4d | %s\n     > %s" % (ln + 1, SOURCE[ln].strip(), new.strip()))


if __name__ == "__main__":
    main()
