"""The library's host-only code (the NPFP** scheduling decisions, Sec. IV) built for the CPU
with AddressSanitizer and UndefinedBehaviorSanitizer and replayed on seeded random cases,
its output compared with the scheduling oracle.  Output buffers in the driver are heap
arrays of exactly the promised size.  (The argument checks of the GPU entry points live in a
file that needs the HIP runtime; tests/test_abi.py exercises them without a sanitizer.)"""
import math
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import npfp_oracle as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
POLICIES = ["C", "CF", "[C]F", "C[F]", "[C][F]"]
ACTIONS = {"idle": 0, "coarse": 1, "fine": 2}


def _table(rng, levels, nmax):
    base = np.sort(rng.uniform(0.3, 2.0, levels))
    return [[0.0] + [float(base[l] * (1 + rng.uniform(0.3, 0.9) * (n - 1))) for n in range(1, nmax + 1)]
            for l in range(levels)]


def _flat(tab):
    return f"{len(tab)} {len(tab[0]) - 1} " + " ".join(repr(float(x)) for row in tab for x in row)


def _nums(v):
    return " ".join(repr(x) if isinstance(x, float) else str(int(x)) for x in v)


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no host compiler")
    out = str(tmp_path_factory.mktemp("san") / "sched_san")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
           "-DCFDETR_API=", "-x", "c++",
           os.path.join(ROOT, "paper_2505_23317_amd", "csrc", "sched.hip"),
           os.path.join(ROOT, "tests", "san", "sched_driver.cc"), "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    return out


def test_scheduling_code_is_clean_under_the_host_sanitizers(driver, tmp_path):
    rng = np.random.default_rng(11)
    lines, want = [], []
    for _ in range(200):                                   # Lemma 1
        n = int(rng.integers(1, 9))
        period = np.sort(rng.uniform(2.0, 30.0, n)).tolist()
        c = rng.uniform(0.1, 3.0, n).tolist()
        lines.append(f"R {n} {_nums(period)} {_nums(c)}")
        ok, R = S.response_times(period, c)
        want.append(("R", 0, int(ok), R))
    for n, t, nxt in [(4, 10.0, 13.0), (4, 10.0, 12.9), (4, 10.0, 11.4), (1, 0.0, 9.0),
                      (0, 0.0, 9.0), (3, 10.0, 10.5)]:     # Algo. 2
        c = [0.0, 1.0, 1.5, 2.5, 3.0]
        lines.append(f"B {n} {t!r} {nxt!r} {len(c)} {_nums(c)}")
        want.append(("B", S.coarse_batch_size(n, t, nxt, c)))
    for _ in range(300):                                   # Algo. 3
        n = int(rng.integers(0, 13))
        levels = int(rng.integers(1, 4))
        C = _table(rng, levels, 12)
        w = rng.integers(0, levels, n).tolist()
        t = float(rng.uniform(0, 10))
        dl = (t + rng.uniform(0.5, 12.0, n)).tolist()
        nxt = t + float(rng.uniform(0.5, 12.0))
        lines.append(f"F {n} {_nums(w)} {_nums(dl)} {t!r} {nxt!r} {_flat(C)}")
        want.append(("F",) + tuple(S.fine_batches(w, dl, t, nxt, C)))
    for _ in range(300):                                   # Algo. 1
        n = int(rng.integers(1, 9))
        Cc = [0.0] + np.cumsum(rng.uniform(0.2, 1.0, n)).tolist()
        C = _table(rng, 3, n)
        ac = sorted(rng.choice(n, int(rng.integers(0, n + 1)), replace=False).tolist())
        rest = [i for i in range(n) if i not in ac]
        af = sorted(rng.choice(rest, int(rng.integers(0, len(rest) + 1)), replace=False).tolist()) \
            if rest else []
        w = rng.integers(0, 3, len(af)).tolist()
        t = float(rng.uniform(0, 10))
        dl = (t + rng.uniform(0.3, 6.0, len(af))).tolist()
        nxt = t + float(rng.uniform(0.1, 6.0))
        for p, pol in enumerate(POLICIES):
            lines.append(f"D {p} {t!r} {len(ac)} {_nums(ac)} {len(af)} {_nums(af)} {_nums(w)} "
                         f"{_nums(dl)} {nxt!r} {len(Cc)} {_nums(Cc)} {_flat(C)}")
            want.append(("D",) + tuple(S.decide(pol, t, ac, af, w, dl, nxt, Cc, C)))
    # argument errors must be refused, not run into
    lines.append("F 2 0 5 9.0 9.0 0.0 9.0 3 4 " + " ".join(["1.0"] * 15))     # level 5 of 3
    want.append(("E",))
    lines.append("R 2 1.0 -2.0 0.1 0.1")                                        # negative period
    want.append(("E",))
    path = tmp_path / "cases.txt"
    path.write_text("\n".join(lines) + "\n")
    r = subprocess.run([driver, str(path)], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, (r.returncode, r.stderr[-3000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
    got = r.stdout.strip().split("\n")
    assert len(got) == len(want)
    for g, w_ in zip(got, want):
        f = g.split()
        if w_[0] == "E":
            assert int(f[1]) != 0
        elif w_[0] == "R":
            assert int(f[1]) == 0 and int(f[2]) == w_[2]
            assert [float(x) for x in f[3:]] == [float(x) for x in w_[3]]
        elif w_[0] == "B":
            assert int(f[1]) == w_[1]
        elif w_[0] == "F":
            order, cuts, dba = w_[1], w_[2], w_[3]
            parts = g.split("|")
            head = parts[0].split()
            assert int(head[1]) == 0 and int(head[2]) == len(cuts)
            assert [int(x) for x in parts[1].split()] == list(order)
            assert [int(x) for x in parts[2].split()] == [b for (_, b) in cuts]
            assert [float(x) for x in parts[3].split()] == [float(x) for x in dba]
        else:
            kind, tasks = w_[1], w_[2]
            parts = g.split("|")
            head = parts[0].split()
            assert int(head[1]) == 0 and int(head[2]) == ACTIONS[kind]
            batches = [[int(x) for x in b.split()] for b in parts[1].split("/") if b.strip()]
            if kind == "coarse":
                assert batches == [list(tasks)]
            elif kind == "fine":
                assert batches == [list(b) for b in tasks]
            else:
                assert batches == []
