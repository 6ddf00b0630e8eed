"""The CPU oracle under the host sanitizers: gmp_oracle.c is built with AddressSanitizer and
UndefinedBehaviorSanitizer into a small C program (oracle/sanitize_driver.c) that replays the hand-derived
trajectories of tests/golden/ and calls every entry point with awkward sizes.  Any report ends the program
with a non-zero status."""
import json
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLD = os.path.join(ROOT, "tests", "golden")


def _ints(v):
    return " ".join(str(int(x)) for x in v)


def _lines():
    out = []
    for kind, name in (("F", "ring_trajectories.json"), ("K", "walker_trajectories.json")):
        for c in json.load(open(os.path.join(GOLD, name)))["cases"]:
            vis = c["expected_visited_in_order"]
            vis = list(range(*vis["range"])) if "range" in vis else vis["list"]
            head = [c["N"], c["R"], 1 if c["monotone"] == "increasing" else -1]
            head += [c["W"], c["L"], c["k"], c["max_iters"]] if kind == "F" else [c["T"], c["k"]]
            out.append(f"{kind} {_ints(head)} {len(c['seed'])} {_ints(c['seed'])} {len(c['expected_ids'])} "
                       f"{_ints(c['expected_ids'])} {len(vis)} {_ints(vis)} {c['n_expanded']} {c['n_scored']} {c['n_iters']}")
    return out


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", os.path.join(ROOT, "oracle", "gmp_oracle.c"),
           os.path.join(ROOT, "oracle", "sanitize_driver.c"), "-o", exe, "-lm"]
    subprocess.run(cmd, check=True)
    lines = _lines()
    assert len(lines) >= 9
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="2")
    res = subprocess.run([exe], input="\n".join(lines) + "\n", capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert f"ok, {len(lines)} hand cases" in res.stdout
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr
