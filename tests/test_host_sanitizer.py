"""The host side of the library (planner, prefix tree, device-table builder, argument validation)
built with g++ -fsanitize=address,undefined and driven over random cases whose expected plan words
come from the CPU oracle.  No device code and no GPU involved."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import planner as opl
from oracle import trie as otrie

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2602_06072_amd", "csrc")


def vec(v):
    v = [] if v is None else [int(x) for x in v]
    return " ".join([str(len(v))] + [str(x) for x in v])


def plan_line(rng, bad=False):
    n = int(rng.integers(0, 40))
    C = int(rng.choice([1, 4, 37, 300, 5000]))
    hr = int(rng.integers(0, 4))
    decode = rng.random() < 0.5
    if rng.random() < 0.5:
        kv = rng.integers(1, 400, size=n)
        pid = plen = None
    else:
        nf = int(rng.integers(1, 5))
        fl = rng.integers(0, 90, size=nf)
        pid = rng.integers(-1, nf, size=n)
        plen = np.where(pid >= 0, fl[np.maximum(pid, 0)], 0)
        kv = plen + rng.integers(1, 70, size=n)
    q = np.ones(n, dtype=np.int64) if decode else np.minimum(kv, rng.integers(1, 200, size=n))
    rc = 0
    if bad and n > 0:
        kv = kv.copy()
        kv[int(rng.integers(0, n))] = 0                  # a request without tokens
        rc = -1
    words = [] if rc else opl.make_plan([int(x) for x in kv], [int(x) for x in q],
                                        None if pid is None else [int(x) for x in pid],
                                        None if plen is None else [int(x) for x in plen], C, hr).words()
    return f"plan {C} {hr} 1 {0 if pid is None else 1} {vec(kv)} {vec(q)} {vec(pid)} {vec(plen)} {rc} {vec(words)}"


def tree_line(rng):
    n = int(rng.integers(2, 12))
    seqs = [[int(t) for t in rng.integers(0, 3, size=int(rng.integers(1, 9)))] for _ in range(n)]
    mp = int(rng.integers(1, 4))
    C = int(rng.choice([8, 40, 1000]))
    hr = int(rng.integers(0, 3))
    par, nl, rn, saved = otrie.trie_tree(seqs, mp)
    lens = [len(s) for s in seqs]
    words = opl.make_plan_tree(lens, [1] * n, par, nl, rn, C, hr).words()
    toks = [t for s in seqs for t in s]
    return f"tree {mp} {C} {hr} {vec(lens)} {vec(toks)} {vec(par)} {vec(nl)} {vec(rn)} {saved} {vec(words)}"


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_code_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "host_sanitizer_driver")
    srcs = [os.path.join(CSRC, f) for f in ("planner.cpp", "schedule.cpp", "trie.cpp", "api.cpp")]
    srcs.append(os.path.join(ROOT, "tests", "native", "host_sanitizer_driver.cpp"))
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-static-libasan", "-static-libubsan",
           "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", *srcs, "-L/opt/rocm/lib", "-lamdhip64",
           "-Wl,-rpath,/opt/rocm/lib", "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    rng = np.random.default_rng(2024)
    lines = [plan_line(rng, bad=(k % 9 == 8)) for k in range(260)] + [tree_line(rng) for _ in range(120)]
    cases = tmp_path / "cases.txt"
    cases.write_text("\n".join(lines) + "\n")
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe, str(cases)], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert "380 cases, 0 failures" in run.stdout
