"""Planted mistakes for the oracle's pins (not collected by pytest; run by hand, CPU only):

    python tests/oracle_mutation_run.py <mutants> <seed> <workers>

Takes `mutants` random single-token changes of oracle/tangram_oracle.cpp (a comparison made strict or
lax, a sign, `&&` for `||`, `min` for `max`, `++` for `--`, ...), each in a scratch copy of oracle/, tests/,
gen/ and include/ under the system's temporary directory, and runs the CPU tests of the oracle on it.  Prints
one JSON line per change; "SURVIVED" marks a change that no pin caught - either it has no effect on any result
or a pin is missing.  Nothing here touches the GPU or the product library."""
import json
import os
import random
import re
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SWAPS = [(" < ", " <= "), (" <= ", " < "), (" > ", " >= "), (" >= ", " > "), (" + ", " - "), (" - ", " + "), (" && ", " || "),
         (" == ", " != "), (" != ", " == "), ("std::min(", "std::max("), ("std::max(", "std::min("), (" += ", " -= "),
         (" -= ", " += "), ("++", "--"), (" * ", " + "), (" / ", " * ")]


def candidates(src):
    first = next(i for i, l in enumerate(src) if l.startswith("int64_t duration("))
    out = []
    for i in range(first, len(src)):
        code = src[i].split("//")[0]
        if not code.strip() or code.strip().startswith(("#", "*", "/*")):
            continue
        for a, b in SWAPS:
            for m in re.finditer(re.escape(a), code):
                if "for (" in code and a in ("++", " < ", " <= "):
                    continue                                   # loop headers: a hang, not arithmetic
                out.append((i, m.start(), a, b))
    return out


def run_one(src, cand, scratch):
    i, pos, a, b = cand
    shutil.rmtree(scratch, ignore_errors=True)
    os.makedirs(os.path.join(scratch, "paper_2603_13019_amd"))
    for sub in ("oracle", "tests", "gen", "include"):
        shutil.copytree(os.path.join(ROOT, sub), os.path.join(scratch, sub), ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    lines = list(src)
    lines[i] = lines[i][:pos] + b + lines[i][pos + len(a):]
    with open(os.path.join(scratch, "oracle", "tangram_oracle.cpp"), "w") as f:
        f.write("\n".join(lines))
    try:
        p = subprocess.run([sys.executable, "-m", "pytest", "tests", "-x", "-q", "-m", "not gpu", "-k", "oracle", "-p", "no:cacheprovider"],
                           cwd=scratch, capture_output=True, text=True, timeout=600)
        out = p.stdout.strip().split("\n")
        status = "caught" if p.returncode != 0 else "SURVIVED"
        first = next((l for l in out if l.startswith(("FAILED", "ERROR"))), out[-1] if out else "")
    except subprocess.TimeoutExpired:
        status, first = "caught", "timeout"
    shutil.rmtree(scratch, ignore_errors=True)
    rec = dict(line=i + 1, swap=f"{a.strip()} -> {b.strip()}", text=src[i].strip()[:110], status=status, first=first[:120])
    print(json.dumps(rec), flush=True)
    return rec


def main():
    n, seed, workers = int(sys.argv[1]), int(sys.argv[2]), int(sys.argv[3])
    with open(os.path.join(ROOT, "oracle", "tangram_oracle.cpp")) as f:
        src = f.read().split("\n")
    cands = candidates(src)
    random.Random(seed).shuffle(cands)
    cands = cands[:n]
    base = tempfile.mkdtemp(prefix="oracle_mutants_")
    with ThreadPoolExecutor(workers) as ex:
        res = list(ex.map(lambda k: run_one(src, cands[k], os.path.join(base, f"m{k}")), range(len(cands))))
    shutil.rmtree(base, ignore_errors=True)
    print("survivors:", sum(r["status"] == "SURVIVED" for r in res), "of", len(res), flush=True)


if __name__ == "__main__":
    main()
