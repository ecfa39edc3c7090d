"""The library's host C++ (partitioner and its variants, pass orders, pipeline timeline) built with gcc under
AddressSanitizer + UndefinedBehaviorSanitizer and driven over seeded random arguments with exactly-sized heap
arrays: any out-of-bounds access, signed overflow or misuse of a caller-sized array aborts the driver, and every
value it prints is compared with the oracle."""
import os
import random
import shutil
import subprocess

import pytest

from oracle import partition as P
from oracle import pipeline as PL
from oracle import schedule as SCH

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2406_03488_amd", "csrc")
SOURCES = [os.path.join(CSRC, f) for f in ("s1f_partition.cpp", "s1f_schedule.cpp", "s1f_pipeline.cpp")]


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path_factory.mktemp("san") / "host_sanitizer_driver")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-Werror", f"-I{os.path.join(ROOT, 'include')}",
           os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"), *SOURCES, "-o", exe]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    assert proc.returncode == 0, proc.stderr
    return exe


def _run(exe, commands):
    text = "\n".join(" ".join(str(x) for x in c) for c in commands) + "\n"
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    proc = subprocess.run([exe], input=text, capture_output=True, text=True, env=env, timeout=300)
    assert proc.returncode == 0, f"driver exited with {proc.returncode}:\n{proc.stderr[-4000:]}"
    lines = proc.stdout.strip().split("\n")
    assert len(lines) == len(commands)
    return [ln.split() for ln in lines]


def test_partitioners_under_sanitizers(driver):
    rng = random.Random(31)
    cmds, want = [], []
    for _ in range(300):
        n = rng.choice((rng.randint(1, 60), rng.randint(1, 5000), 131072))
        k = rng.randint(1, min(n, 33))
        hidden = rng.choice((1, 3, 64, 4096, 8192))
        align = rng.choice((1, 1, 2, 8, 128))
        if (n - 1) // align < k - 1:
            align = 1
        which = rng.randrange(3)
        if which == 0:
            cmds.append(("part", n, k, hidden, 1)); want.append(P.partition(n, k, hidden, 1))
        elif which == 1:
            cmds.append(("partex", n, k, hidden, 1, 0, align)); want.append(P.partition(n, k, hidden, 1, align))
        elif n <= 400:   # the oracle's dynamic programme is quadratic
            cmds.append(("partex", n, k, hidden, 1, 1, align)); want.append(P.partition_literal(n, k, hidden, 1, align))
    for _ in range(200):
        k = rng.randint(1, 8)
        align = rng.choice((1, 1, 2, 4))
        b = [0]
        for _ in range(k):
            b.append(b[-1] + rng.randint(1, 50))
        cost = [rng.choice((0, rng.randint(1, 1000), rng.randint(1, 10**12))) for _ in range(k)]
        if sum(cost) == 0 or (b[-1] - 1) // align < k - 1:
            continue
        cmds.append(("rebal", k, align, *b, *cost)); want.append(P.rebalance(b, cost, align))
    # rejected arguments must not touch the arrays either
    bad = [("part", 3, 4, 4, 1), ("part", 8, 0, 4, 1), ("partex", 8, 3, 1, 1, 0, 4), ("partex", 8, 2, 1, 1, 2, 1),
           ("rebal", 3, 1, 0, 4, 4, 8, 1, 1, 1), ("rebal", 2, 0, 0, 4, 8, 1, 1)]
    got = _run(driver, cmds + bad)
    for c, g, w in zip(cmds, got, want):
        assert g[0] == "0" and [int(x) for x in g[1:]] == list(w), c
    for c, g in zip(bad, got[len(cmds):]):
        assert g == ["1"], c


def test_orders_and_timeline_under_sanitizers(driver):
    rng = random.Random(32)
    cmds, want = [], []
    for _ in range(200):
        Pp, M, k = rng.choice((1, 2, 3, 4, 8)), rng.randint(1, 20), rng.randint(1, 8)
        i = rng.randint(1, Pp)
        cmds.append(("warm", Pp, i, M, k)); want.append([SCH.warmup_count(Pp, i, M, k)])
        cmds.append(("order", Pp, i, M, k))
        want.append([x for kind, m, j in SCH.stage_order(Pp, i, M, k) for x in (int(kind == "B"), m, j)])
        ws = [SCH.warmup_count(Pp, j, M, k) for j in range(1, Pp + 1)]
        if sum(ws) > 0:
            cmds.append(("share", Pp, i, M, k)); want.append([ws[i - 1], sum(ws)])
    for Pp, M, k, n in ((2, 4, 2, 2), (4, 8, 4, 2), (4, 6, 2, 3), (8, 16, 4, 2), (4, 4, 1, 4), (1, 3, 1, 2)):
        for i in range(1, Pp + 1):
            cmds.append(("iwarm", Pp, i, M, k, n)); want.append([PL.interleaved_warmup(Pp, i, M, k, n)])
            cmds.append(("iorder", Pp, i, M, k, n))
            want.append([x for kind, m, j, c in PL.interleaved_order(Pp, i, M, k, n)
                         for x in (int(kind == "B"), m, j, c)])
    sims = []
    while len(sims) < 60:
        Pp, k, n = rng.choice((1, 2, 4, 8)), rng.choice((1, 2, 4)), rng.choice((1, 1, 2))
        M = rng.randint(1, 10)
        if n > 1 and not ((M * k) % Pp == 0 and Pp % k == 0):
            continue
        split, has_tok = rng.randrange(2), rng.randrange(2)
        cap, comm = rng.randint(0, 6), rng.choice((0, 0, 3, 17))
        tf = [rng.randint(1, 50) for _ in range(k)]; tb = [rng.randint(1, 90) for _ in range(k)]
        tw = [rng.randint(1, 40) for _ in range(k)] if split else None
        tok = [rng.randint(1, 9) for _ in range(k)] if has_tok else None
        cmd = ["sim", Pp, M, k, n, split, cap, comm, has_tok, *tf, *tb, *(tw or []), *(tok or [])]
        r = PL.simulate(Pp, n, PL.device_orders(Pp, M, k, n), tf, tb, tw, comm, cap, tok)
        assert r is not None
        sims.append((cmd, [r["makespan"], *r["busy"], *r["peak_live"], *r["peak_pending"]], PL.bubble_ratio(r, Pp)))
    bad = [("warm", 4, 5, 4, 2), ("order", 0, 1, 4, 2), ("iorder", 4, 1, 4, 3, 2), ("share", 1, 1, 3, 1)]
    got = _run(driver, cmds + [s[0] for s in sims] + bad)
    for c, g, w in zip(cmds, got, want):
        assert g[0] == "0" and [int(x) for x in g[1:]] == w, c
    for (c, w, bubble), g in zip(sims, got[len(cmds):]):
        assert g[0] == "0" and [int(x) for x in g[1:-1]] == w and abs(float(g[-1]) - bubble) < 1e-12, c
    for c, g in zip(bad, got[len(cmds) + len(sims):]):
        assert g[0] in ("1", "2") and len(g) == 1, c
