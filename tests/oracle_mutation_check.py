"""Mutation check of the CPU oracle (no GPU, not collected by pytest): plant one small mistake at a time --
an operator, a comparison, a constant, an index, a cast -- in a private copy of oracle/lioncub_oracle.c
(or, with MUT_FILE=__init__.py, of the Python side), rebuild, run the oracle's pin tests on the copy, and
list the mistakes that no pin catches.  What survives should be equivalent code (a cast of a value that
already has the type, a bound that no caller reaches); anything else is a missing pin.

    python tests/oracle_mutation_check.py            # about ten minutes on 8 cores
"""
import os, re, shutil, subprocess, sys, tempfile
from concurrent.futures import ThreadPoolExecutor
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FILE = os.environ.get("MUT_FILE", "lioncub_oracle.c")
PY = FILE.endswith(".py")
SRC = open(os.path.join(ROOT, "oracle", FILE)).read().split("\n")
WORK = tempfile.mkdtemp(prefix="oracle_mutants_")
TESTS = ["test_oracle_pins.py", "test_oracle_l1.py"] + sys.argv[1:]

RULES = [(r"(?<![+\-eE(,=*/<>&|!?:] )(?<![+\-eE(,=])\s\+\s", " - "), (r"\s-\s", " + "), (r"\s\*\s", " + "), (r"\s/\s", " * "),
         (r"\s<\s", " <= "), (r"\s<=\s", " < "), (r"\s>\s", " >= "), (r"\s>=\s", " > "), (r"\s<\s", " > "), (r"\s>\s", " < "),
         (r"==", "!="), (r"!=", "=="), (r"&&", "||"), (r"\|\|", "&&"), (r"\+=", "-="), (r"-=", "+="),
         (r"\b0\b", "1"), (r"\b1\b", "0"), (r"\b1\b", "2"), (r"\b2\b", "1"), (r"\b2\b", "3"), (r"<<", ">>"), (r">>", "<<"),
         (r"\s&\s", " | "), (r"\s\|\s", " & "), (r"\b63\b", "62"), (r"\b64\b", "63"), (r"\b8\b", "7"), (r"\b0\.0f?\b", "1.0f"), (r"\b1\.0f?\b", "0.5f"),
         (r"\b0\.5\b", "0.25"), (r"\bi\]", "i + 1]"), (r"\bw\]", "w + 1]"), (r"\+\+", "--"), (r"\? (\S+) : (\S+?)([;)])", r"? \2 : \1\3"),
         (r"-1\b", "1"), (r"\bfloor\b", "ceil"), (r"\bfabs\b", ""), (r"\bfabsf\b", ""), (r"\(float\)", ""), (r"\(double\)", "(float)")]

def mutants():
    out = []
    in_comment = False
    for ln, line in enumerate(SRC):
        code = line
        st = code.strip()
        if in_comment:
            if "*/" in code: in_comment = False
            continue
        if st.startswith("/*"):
            if "*/" not in code: in_comment = True
            continue
        if PY:
            if st.count('"""') == 1: in_doc = not globals().get("in_doc", False); globals()["in_doc"] = in_doc; continue
            if globals().get("in_doc", False) or st.startswith('"""') or st.startswith("#") or not st or ln < 28: continue
        elif st.startswith("//") or st.startswith("#") or not st or st.startswith("*"):
            continue
        cpos = code.find("#" if PY else "//")
        body = code if cpos < 0 else code[:cpos]
        tail = "" if cpos < 0 else code[cpos:]
        for pat, rep in RULES:
            for mt in re.finditer(pat, body):
                new = body[:mt.start()] + mt.expand(rep) + body[mt.end():]
                if new != body:
                    out.append((ln, new + tail))
    return out

def worker(slot, jobs, results):
    d = os.path.join(WORK, "w%d" % slot)
    shutil.rmtree(d, ignore_errors=True)
    os.makedirs(os.path.join(d, "oracle")); os.makedirs(os.path.join(d, "tests"))
    for f in ("__init__.py", "build.py", "lioncub_oracle.c"): shutil.copy(os.path.join(ROOT, "oracle", f), os.path.join(d, "oracle", f))
    for f in TESTS + ["conftest.py"]: shutil.copy(os.path.join(ROOT, "tests", f), os.path.join(d, "tests", f))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(d, "tests", "golden"))
    for ln, new in jobs:
        lines = list(SRC); lines[ln] = new
        open(os.path.join(d, "oracle", FILE), "w").write("\n".join(lines))
        b = subprocess.run([sys.executable, os.path.join(d, "oracle", "build.py")], cwd=d, capture_output=True, text=True)
        if b.returncode != 0:
            results.append((ln, new, "nocompile")); continue
        try:
            r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + ["tests/" + t for t in TESTS], cwd=d, capture_output=True, text=True, timeout=120)
            results.append((ln, new, "caught" if r.returncode != 0 else "SURVIVED"))
        except subprocess.TimeoutExpired:
            results.append((ln, new, "caught(timeout)"))
        print(len(results), flush=True) if len(results) % 50 == 0 else None

if __name__ == "__main__":
    ms = mutants()
    print(len(ms), "mutants", flush=True)
    results = []
    with ThreadPoolExecutor(8) as ex:
        for s in range(8): ex.submit(worker, s, ms[s::8], results)
    results.sort()
    n = {}
    for ln, new, res in results: n[res] = n.get(res, 0) + 1
    print(n)
    for ln, new, res in results:
        if res == "SURVIVED": print("%4d | %s\n     > %s" % (ln + 1, SRC[ln].strip(), new.strip()))
    shutil.rmtree(WORK, ignore_errors=True)
