"""Mutation check of the oracle's pins (CPU only; not collected by pytest: run it by hand).

Every code line of oracle/*.py is changed in up to four ways, one change at a time (a sign, a comparison, an index, a
constant, source and destination swapped, sine for cosine, a sum over the other axis ...), in a scratch copy of the
tree under /tmp, and the CPU test suite (`-m "not gpu"`) is run on the copy: a change that no test notices is printed
as SURVIVED.  What should remain are changes that compute the same thing (len(src) for len(dst), the parity of
l1 - l2 + l3 for that of l1 + l2 + l3, `>` for `>=` where both sides agree at equality, a loop bound whose extra terms
are skipped by the next line).  Six worker processes, about a quarter of an hour.

usage: python tests/mutation_check.py [oracle file ...]"""
import os, re, shutil, subprocess, sys, tokenize, io
from concurrent.futures import ThreadPoolExecutor
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FILES = sys.argv[1:] or ["oracle/egnn_oracle.py", "oracle/so2_oracle.py", "oracle/hamiltonian_oracle.py", "oracle/partition_oracle.py"]
NW = 6
OPS = [(" + ", " - "), (" - ", " + "), (" += ", " -= "), (" -= ", " += "), (" * ", " * 1.01 * "), ("np.cos(", "np.sin("), ("np.sin(", "np.cos("),
       ("src", "dst"), ("dst", "src"), ("[0]", "[1]"), ("[:, 0", "[:, 1"), ("** 2", "** 3"), (" / ", " * "), ("1.0", "2.0"), (".sum(", ".max("), ("j + 1", "j + 2"), ("lmax + 1", "lmax + 2"), ("m1", "m2"), ("l1", "l2"), (" < ", " <= "), (" <= ", " < "), (" > ", " >= "), ("2.0", "3.0"), ("0.5", "0.25"), (".T", ""), ("axis=0", "axis=1"), ("axis=1", "axis=0")]
def code_lines(path):
    src = open(path).read()
    skip = set()
    for tok in tokenize.generate_tokens(io.StringIO(src).readline):
        if tok.type == tokenize.STRING and tok.string.startswith(('"""', "'''", 'r"""')):
            for l in range(tok.start[0], tok.end[0] + 1): skip.add(l)
    out = []
    for i, line in enumerate(src.split("\n"), 1):
        s = line.strip()
        if i in skip or not s or s.startswith(("#", "def ", "import ", "from ", "assert ", "raise ", "return None", "class ", "@", '"""')): continue
        code = line.split("  #")[0]
        out.append((i, code))
    return src.split("\n"), out
def mutants(path):
    lines, cl = code_lines(path)
    res = []
    for i, code in cl:
        done = 0
        for a, b in OPS:
            if a in code and done < 4:
                res.append((path, i, a, b)); done += 1
    return res
def prepare(w):
    d = f"/tmp/mut{w}"
    if os.path.exists(d): shutil.rmtree(d)
    os.makedirs(d)
    for sub in ["oracle", "tests", "paper_2507_03840_amd", "include"]:
        shutil.copytree(os.path.join(ROOT, sub), os.path.join(d, sub), ignore=shutil.ignore_patterns("__pycache__", "_build", "*.npz", "*.o"))
    for f in ["__graft_entry__.py", "bench.py"]:
        shutil.copy(os.path.join(ROOT, f), d)
    return d
def run(args):
    w, (path, i, a, b) = args
    d = f"/tmp/mut{w}"
    orig = open(os.path.join(ROOT, path)).read().split("\n")
    m = list(orig); m[i - 1] = m[i - 1].replace(a, b, 1)
    open(os.path.join(d, path), "w").write("\n".join(m))
    try:
        # (the tests of the input generators are left out: slow, and not pins of the oracle)
        r = subprocess.run([sys.executable, "-m", "pytest", "tests", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                            "--ignore", "tests/test_synth_recipes.py"], cwd=d, capture_output=True, text=True, timeout=300,
                           env=dict(os.environ, OMP_NUM_THREADS="1", PYTHONDONTWRITEBYTECODE="1"))
        caught = r.returncode != 0
        first = next((l for l in r.stdout.splitlines() if l.startswith("FAILED") or l.startswith("ERROR")), "")
    except subprocess.TimeoutExpired:
        caught, first = True, "timeout"
    finally:
        open(os.path.join(d, path), "w").write("\n".join(orig))
    return (path, i, a, b, caught, first, orig[i - 1].strip())
allm = []
for f in FILES: allm += mutants(f)
print(len(allm), "mutants", flush=True)
import queue, threading
q = queue.Queue()
for mu in allm: q.put(mu)
results = []
def worker(w):
    prepare(w)
    while True:
        try: mu = q.get_nowait()
        except queue.Empty: return
        r = run((w, mu)); results.append(r)
        if not r[4]: print("SURVIVED", r[0], r[1], repr(r[2]), "->", repr(r[3]), "|", r[6], flush=True)
ths = [threading.Thread(target=worker, args=(w,)) for w in range(NW)]
[t.start() for t in ths]; [t.join() for t in ths]
print("caught", sum(r[4] for r in results), "of", len(results))
