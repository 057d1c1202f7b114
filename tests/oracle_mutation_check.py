"""Mutation check of the CPU oracle against its pins (CPU only).

    python tests/oracle_mutation_check.py [every_kth] [--write]

Plants one small mistake at a time in a copy of oracle/sinkhorn_oracle.c (a flipped sign, a
swapped index, a transposed subscript, a changed constant or comparison, exp for exp2, ...),
builds the copy into a library of its own and runs tests/test_oracle_pins.py against it.  A
mutant that passes every pin is built once more with gcc's address and undefined-behaviour
sanitizers and runs the pins again (a loop bound one past the end passes on the allocator's slack
and dies there).  What passes both is printed: either it changes nothing a caller can see (a
comparison at a tolerance, a dead initial value, the thread-count setter) or a pin is missing.
The oracle in the tree is never touched.  `--write` stores the survivors of a FULL run in
tests/golden/oracle_mutation_survivors.txt (the mutated source lines, which are what the
collected test tests/test_oracle_mutation_sample.py allows a sampled mutant to survive as)."""
import concurrent.futures as cf
import os
import re
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "sinkhorn_oracle.c")
GCC = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC"]
GCC_SAN = ["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-shared", "-fPIC"]


def sanitizer_env(threads_each):
    """Environment of a child that loads a sanitized library into the uninstrumented interpreter."""
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True,
                          text=True).stdout.strip()
    env = dict(os.environ, OMP_NUM_THREADS=str(threads_each))
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1"
    return env

RUNNER = """
import sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {tests!r})
import oracle
oracle._LIB = sys.argv[1]
oracle.build = lambda force=False: sys.argv[1]
import pytest
sys.exit(pytest.main(["-x", "-q", "-p", "no:cacheprovider", {pins!r}]))
"""

OPERATORS = [
    (r"\+=", "-="), (r"-=", "+="), (r"\*=", "/="),
    (r" \+ ", " - "), (r" - ", " + "), (r" \* ", " + "), (r" / ", " * "),
    (r"\[i\]", "[j]"), (r"\[j\]", "[i]"), (r"\[k\]", "[0]"),
    (r"i \* ld \+ j", "j * ld + i"), (r"i \* m \+ k", "k * m + i"),
    (r" < ", " <= "), (r" > ", " < "), (r" >= ", " > "),
    (r"\b1\.0\b", "0.5"), (r"\b0\.0\b", "1.0"), (r"\b2\.0\b", "1.0"),
    (r"\bexp\(", "exp2("), (r"\blog\(", "log2("), (r"\bfabs\(", "("), (r"\bsqrt\(", "("),
    (r"eta", "(1.0 - eta)"), (r"\+ 1\b", "+ 0"), (r"- 1\b", "- 0"),
]


def mutants(lines):
    out, in_comment = [], False
    for ln, text in enumerate(lines):
        s = text.strip()
        if in_comment:
            in_comment = "*/" not in s
            continue
        if s.startswith("/*"):
            in_comment = "*/" not in s
            continue
        if not s or s[0] in "#*" or s.startswith("//"):
            continue
        code = text.split("//")[0]
        for pat, rep in OPERATORS:
            for hit in re.finditer(pat, code):
                new = text[:hit.start()] + rep + text[hit.end():]
                if new != text:
                    out.append((ln, new))
    return out


def run_mutants(todo, workers=4, threads_each=2, progress=None):
    """Builds and tests every (line number, mutated line) of `todo`; returns (line, text, verdict)
    triples with verdict in {"killed", "killed under the sanitizers", "survived",
    "does not compile"}."""
    lines = open(SRC).read().split("\n")
    work = tempfile.mkdtemp(prefix="oracle_mut_")
    runner = os.path.join(work, "run_pins.py")
    with open(runner, "w") as fh:
        fh.write(RUNNER.format(root=ROOT, tests=os.path.join(ROOT, "tests"),
                               pins=os.path.join(ROOT, "tests", "test_oracle_pins.py")))

    def run(job):
        idx, (ln, new) = job
        src, lib = os.path.join(work, f"m{idx}.c"), os.path.join(work, f"m{idx}.so")
        body = list(lines)
        body[ln] = new
        with open(src, "w") as fh:
            fh.write("\n".join(body))
        verdict = "does not compile"
        if subprocess.run(GCC + [src, "-o", lib, "-lm"], capture_output=True).returncode == 0:
            try:
                rc = subprocess.run([sys.executable, runner, lib], capture_output=True, timeout=600,
                                    env=dict(os.environ, OMP_NUM_THREADS=str(threads_each))).returncode
                verdict = "survived" if rc == 0 else "killed"
            except subprocess.TimeoutExpired:
                verdict = "killed"
            os.remove(lib)
            if verdict == "survived" and \
                    subprocess.run(GCC_SAN + [src, "-o", lib, "-lm"], capture_output=True).returncode == 0:
                try:
                    rc = subprocess.run([sys.executable, runner, lib], capture_output=True, timeout=1800,
                                        env=sanitizer_env(threads_each)).returncode
                except subprocess.TimeoutExpired:
                    rc = 1
                if rc != 0:
                    verdict = "killed under the sanitizers"
                os.remove(lib)
        os.remove(src)
        return ln, new, verdict

    out = []
    with cf.ThreadPoolExecutor(workers) as pool:
        for done, res in enumerate(pool.map(run, list(enumerate(todo)))):
            out.append(res)
            if progress:
                progress(done, res)
    return out


def all_mutants():
    return mutants(open(SRC).read().split("\n"))


SURVIVORS = os.path.join(ROOT, "tests", "golden", "oracle_mutation_survivors.txt")


def main():
    args = [a for a in sys.argv[1:] if not a.startswith("--")]
    todo = all_mutants()
    if args:
        todo = todo[::int(args[0])]
    print(len(todo), "mutants", flush=True)

    def progress(done, res):
        ln, new, verdict = res
        if verdict == "survived":
            print(f"SURVIVED line {ln + 1}: {new.strip()}", flush=True)
        if done % 100 == 0:
            print("done", done, flush=True)

    res = run_mutants(todo, progress=progress)
    alive = [new.strip() for _, new, verdict in res if verdict == "survived"]
    print("survivors:", len(alive), "of", len(todo), "(killed only under the sanitizers:",
          sum(verdict == "killed under the sanitizers" for _, _, verdict in res), ")")
    if "--write" in sys.argv:
        if args:
            raise SystemExit("--write needs the full run")
        with open(SURVIVORS, "w") as fh:
            fh.write("# Mutated lines of oracle/sinkhorn_oracle.c that pass every pin in a full run of\n"
                     "# tests/oracle_mutation_check.py (" + str(len(todo)) + " mutants), also when built with the address and\n"
                     "# undefined-behaviour sanitizers.  Each changes nothing a caller can see: a comparison at a\n"
                     "# tolerance turned into <=, a loop bound whose extra trip stays inside its buffer, the\n"
                     "# thread-count setter, a dead initial value.\n")
            for line in sorted(set(alive)):
                fh.write(line + "\n")


if __name__ == "__main__":
    main()
