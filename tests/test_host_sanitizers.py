"""The library's host functions (csrc/draft_host.cpp) built with AddressSanitizer and
UndefinedBehaviorSanitizer and replayed on random cycles; results are compared with the oracle."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import goose_draft as dr
from test_draft_host import _plan_ref

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path_factory.mktemp("san") / "host_sanitizer_driver")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"),
           os.path.join(ROOT, "paper_2604_02047_amd", "csrc", "draft_host.cpp"), "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        pytest.skip("sanitizer build not available here: " + res.stderr[-300:])
    return exe


def test_host_functions_are_clean_under_the_sanitizers(driver):
    rng = np.random.default_rng(5)
    lines, expect = [], []
    for trial in range(250):
        V, K = int(rng.choice([12, 40, 200])), int(rng.choice([1, 4, 10]))
        ids = rng.integers(-1, V, size=(V, K)).astype(np.int32)
        if trial % 2 == 0:
            ids[rng.random(size=V) < 0.6] = -1
        sc = (rng.random(size=(V, K)) * (rng.random(size=(V, K)) < 0.7)).astype(np.float32)
        n = int(rng.integers(1, 60))
        seq = rng.integers(0, min(V, int(rng.choice([3, 6, V]))), size=n).tolist()
        anchor, lens = int(seq[-1]), (3, 4, 5)
        max_spine = int(rng.choice([4, 20]))
        B = int(rng.integers(1 + max_spine, 129))
        p_hat, thr, bypass = float(rng.random()), float(rng.choice([0.01, 0.0, 0.3])), int(rng.choice([3, 8]))
        lines.append("plan %d %s %d %s %d %d %d %d %s %s %d %r 0.5 6 %r %d" % (
            n, " ".join(map(str, seq)), len(lens), " ".join(map(str, lens)), max_spine, anchor, V, K,
            " ".join(map(str, ids.ravel().tolist())), " ".join(repr(float(x)) for x in sc.ravel()), B, p_hat, thr, bypass))
        t, p, s, mode = _plan_ref(seq, lens, max_spine, anchor, ids, sc, B, p_hat, 0.5, 6, thr, bypass)
        expect.append([0, mode, len(t)] + list(map(int, t)) + list(map(int, p)) + list(map(int, s)))
        par = list(map(int, p))
        if trial % 5 == 0 and len(par) > 2:
            par[2] = 2                                        # not a tree in topological order
        lines.append("chk %d %s" % (len(par), " ".join(map(str, par))))
        expect.append([0 if all(q < i for i, q in enumerate(par)) and par[0] == -1 else -4])
    res = subprocess.run([driver], input="\n".join(lines) + "\n", capture_output=True, text=True,
                         env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0"))
    assert res.returncode == 0, res.stderr[-2000:]
    got = [list(map(int, ln.split())) for ln in res.stdout.strip().split("\n")]
    assert got == expect
