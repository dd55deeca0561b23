"""The sampling kernel resolves Floyd's "already chosen" test for all slots of a vertex at once
(paper_2605_29346_amd/csrc/zg_floyd.h); the CPU checker keeps the sequential algorithm.  This CPU-only test
compiles the kernel's rule for the host, runs it in a lockstep harness (tests/floyd_lockstep.cpp) and compares it
with the checker over EVERY candidate sequence of small (deg, F), up to fanout 8 - chains of collisions included,
which the randomised GPU parity runs only meet by chance."""
import math
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PAIRS = [(5, 3), (6, 2), (4, 3), (7, 4), (3, 1), (6, 5), (2, 1), (7, 6), (8, 7), (9, 6), (10, 5), (12, 4), (9, 8)]


@pytest.fixture(scope="module")
def harness(tmp_path_factory):
    d = tmp_path_factory.mktemp("floyd")
    obj = d / "zg_oracle.o"
    exe = d / "floyd_lockstep"
    subprocess.run(["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-c", os.path.join(ROOT, "oracle", "zg_oracle.c"),
                    "-I", os.path.join(ROOT, "oracle"), "-o", str(obj)], check=True)
    subprocess.run(["g++", "-std=c++17", "-O2", "-Wall", "-Werror", os.path.join(ROOT, "tests", "floyd_lockstep.cpp"), str(obj),
                    "-I", os.path.join(ROOT, "paper_2605_29346_amd", "csrc"), "-I", os.path.join(ROOT, "oracle"),
                    "-o", str(exe)], check=True)
    return str(exe)


def test_parallel_rule_equals_sequential_floyd_on_every_candidate_sequence(harness):
    args = [str(x) for pair in PAIRS for x in pair]
    r = subprocess.run([harness] + args, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    cases, bad = (int(x) for x in r.stdout.split())
    expect = sum(math.prod(deg - F + j + 1 for j in range(F)) for deg, F in PAIRS)
    assert cases == expect and bad == 0


def test_harness_notices_a_wrong_rule(harness, tmp_path):
    # the same harness over a deliberately broken copy of the rule (the chase clause dropped) must report mismatches:
    # otherwise agreement above would prove nothing
    src = open(os.path.join(ROOT, "paper_2605_29346_amd", "csrc", "zg_floyd.h")).read()
    assert "const bool nc = dup || (chase && ca);" in src
    inc = tmp_path / "inc"
    inc.mkdir()
    (inc / "zg_floyd.h").write_text(src.replace("const bool nc = dup || (chase && ca);", "const bool nc = dup;"))
    obj = tmp_path / "o.o"
    exe = tmp_path / "broken"
    subprocess.run(["gcc", "-std=c11", "-O2", "-c", os.path.join(ROOT, "oracle", "zg_oracle.c"), "-I", os.path.join(ROOT, "oracle"),
                    "-o", str(obj)], check=True)
    subprocess.run(["g++", "-std=c++17", "-O2", os.path.join(ROOT, "tests", "floyd_lockstep.cpp"), str(obj), "-I", str(inc),
                    "-I", os.path.join(ROOT, "oracle"), "-o", str(exe)], check=True)
    r = subprocess.run([str(exe), "5", "3", "7", "4"], capture_output=True, text=True)
    assert r.returncode == 1 and int(r.stdout.split()[1]) > 0
