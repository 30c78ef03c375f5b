"""The library's host side (validation, both step tables, the table accessor) under AddressSanitizer and
UndefinedBehaviorSanitizer, on valid plans and on plans damaged on purpose: wild indices, lying counts, absurd
sizes, options out of range.  The driver (tests/sanitize/plan_fuzz_driver.cpp) is built from the library's own
plan.cpp with g++; arrays are allocated exactly as long as the case's descriptors claim at most, so reading
past them is a report.  No GPU code is involved (sanitizers run on host code only)."""
import os
import random
import shutil
import subprocess

import numpy as np
import pytest

from oracle import collective as col

from random_cases import random_case

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2008_08708_amd", "csrc")
WILD = [-1, 0, 1, 2, 63, 64, 65, 255, 256, 1 << 16, 1 << 30, (1 << 31) - 1, -(1 << 31), -2]
NUM_CASES = int(os.environ.get("SCCL_SANITIZE_CASES", "1500"))


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    if shutil.which("g++") is None:
        pytest.skip("no g++")
    exe = str(tmp_path_factory.mktemp("sanitize") / "plan_fuzz_driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-static-libasan", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
           os.path.join(ROOT, "tests", "sanitize", "plan_fuzz_driver.cpp"), os.path.join(CSRC, "plan.cpp"), "-o", exe]
    done = subprocess.run(cmd, capture_output=True, text=True)
    if done.returncode != 0 and "asan" in done.stderr.lower() and "cannot find" in done.stderr.lower():
        pytest.skip("the sanitizer runtime is not installed")
    assert done.returncode == 0, done.stderr[-2000:]
    return exe


def case_text(rng, seed):
    """One plan description; with probability 3/4 damaged in one to three places."""
    _, topo, coll, sched, dtype, _, epc = random_case(seed)
    P, G = topo.num_nodes, coll.num_chunks
    bw = [[sorted(L), b, len(L)] for (L, b) in topo.bw]                  # edges, chunks per round, stated edge count
    pre, post = coll.pre.astype(np.int64).copy(), coll.post.astype(np.int64).copy()
    sends = np.asarray(sched.sends, dtype=np.int64).reshape(-1, 5).copy()
    rounds = list(sched.rounds)
    S, N = len(rounds), sends.shape[0]
    slot, positions = None, 0
    if rng.random() < 0.3:
        slot, positions = col.compact_slots(coll, sched.sends)
        slot = slot.astype(np.int64)
    dt = {"i32": 0, "f32": 1, "f16": 2}[dtype]
    opts = [1, 0, 0, 0, 0, 0, 0, 0]                                        # flags = host only; the rest default
    for _ in range(rng.randrange(0, 4)):
        kind, w = rng.randrange(14), rng.choice(WILD)
        if kind == 0 and len(sends):
            sends[rng.randrange(len(sends)), rng.randrange(5)] = w
        elif kind == 1 and len(sends):
            sends[rng.randrange(len(sends)), rng.randrange(5)] += rng.choice([-1, 1])
        elif kind == 2:
            rounds[rng.randrange(len(rounds))] = w
        elif kind == 3:
            bw[rng.randrange(len(bw))][1] = w
        elif kind == 4:
            e = bw[rng.randrange(len(bw))][0]
            if e:
                e[rng.randrange(len(e))] = (rng.choice(WILD), rng.choice(WILD))
        elif kind == 5:
            epc = rng.choice([0, 1, 3, -1, 1 << 40, 1 << 61, (1 << 62) + 5, (1 << 63) - 1])
        elif kind == 6 and slot is not None:
            slot[rng.randrange(G), rng.randrange(P)] = w
        elif kind == 7 and slot is not None:
            positions = w
        elif kind == 8:
            opts[1 + rng.randrange(7)] = w
        elif kind == 9:
            pre[rng.randrange(G), rng.randrange(P)] ^= 1
        elif kind == 10:
            post[rng.randrange(G), rng.randrange(P)] ^= 1
        elif kind == 11:
            N = rng.choice([0, -1, max(0, N - 1)])
        elif kind == 12:
            S = rng.choice([0, -1, max(1, S - 1)])
        elif kind == 13:
            dt = w
    lines = [f"{P} {len(bw)}"]
    for edges, b, stated in bw:
        lines.append(f"{b} {stated} {len(edges)} " + " ".join(f"{s} {d}" for s, d in edges))
    lines.append(f"{G} {G} {P} {int(coll.combining)} {dt} {epc}")
    lines.append(" ".join(map(str, pre.ravel().tolist())))
    lines.append(" ".join(map(str, post.ravel().tolist())))
    lines.append(f"{0 if slot is None else 1} {positions}")
    if slot is not None:
        lines.append(" ".join(map(str, slot.ravel().tolist())))
    lines.append(f"{S} {len(rounds)} " + " ".join(map(str, rounds)))
    lines.append(f"{N} {sends.shape[0]}")
    lines.extend(" ".join(map(str, row)) for row in sends.tolist())
    lines.append(" ".join(map(str, opts)))
    return "\n".join(lines)


def test_host_compiler_is_clean_under_the_sanitizers(driver):
    rng = random.Random(20080)
    cases = [case_text(rng, 1000 + rng.randrange(3000)) for _ in range(NUM_CASES)]
    text = f"{len(cases)}\n" + "\n".join(cases) + "\n"
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    done = subprocess.run([driver], input=text, capture_output=True, text=True, env=env, timeout=600)
    assert done.returncode == 0, (done.stderr[-3000:], done.stdout[-300:])
    assert "runtime error" not in done.stderr and "AddressSanitizer" not in done.stderr, done.stderr[-3000:]
    rows = [line.split() for line in done.stdout.splitlines()]
    assert len(rows) == NUM_CASES
    status = [int(r[1]) for r in rows]
    assert status.count(0) >= NUM_CASES // 5                             # undamaged and harmlessly damaged plans compile
    assert len(set(status)) >= 6                                         # and the damage reaches many different checks
    for r in rows:
        if int(r[1]) == 0:
            assert int(r[2]) > 0 or int(r[3]) != 0                       # a compiled plan has a table to read back
