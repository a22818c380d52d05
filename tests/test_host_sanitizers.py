"""The host half of the library (allocator, bookkeeping, background recalibrator) under sanitizers.

``odma_host.cpp`` builds with g++ alone (no hipcc: the device half installs its copy routine when it is present), so
it can be compiled together with a small driver (``tests/native/host_trace_driver.cpp``) under AddressSanitizer +
UndefinedBehaviorSanitizer and under ThreadSanitizer.  The driver replays traces of calls whose expected results this
test wrote from the allocator oracle -- random traces with invalid ids, failures and recalibrations -- and runs the
background recalibrator with two reporting threads beside the pool's driver thread.  A sanitizer report or a
difference from the oracle fails the test.
"""
import os
import shutil
import subprocess

import numpy as np
import pytest

import workloads as wl
from oracle import allocator as al

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CXX = shutil.which("g++")
pytestmark = pytest.mark.skipif(CXX is None, reason="needs g++")

SAN = {"asan": ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan", "-static-libubsan"],
       "tsan": ["-fsanitize=thread", "-static-libtsan"]}


@pytest.fixture(scope="module")
def drivers(tmp_path_factory):
    out = {}
    d = tmp_path_factory.mktemp("san")
    for name, flags in SAN.items():
        exe = str(d / f"driver_{name}")
        cmd = [CXX, "-O1", "-g", "-std=c++17", "-pthread", "-ffp-contract=off", "-I", os.path.join(ROOT, "include"),
               "-I", os.path.join(ROOT, "paper_2512_09427_amd", "csrc"), *flags,
               os.path.join(ROOT, "tests", "native", "host_trace_driver.cpp"),
               os.path.join(ROOT, "paper_2512_09427_amd", "csrc", "odma_host.cpp"), "-o", exe]
        subprocess.run(cmd, check=True, capture_output=True, text=True, timeout=300)
        out[name] = exe
    return out


def run(exe, *args):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               TSAN_OPTIONS="exitcode=66:halt_on_error=0")
    r = subprocess.run([exe, *args], capture_output=True, text=True, timeout=300, env=env)
    report = r.stdout + r.stderr
    assert "Sanitizer" not in report and "runtime error" not in report, report[-3000:]
    assert r.returncode == 0, report[-3000:]
    return r.stdout


def fmt(v):
    return "-" if v is None else " ".join(str(int(x)) for x in v)


def write_trace(path, seed, steps=400):
    """Random calls, including invalid and duplicate ids, failures and per-call boundaries; expectations from the oracle."""
    rng = np.random.default_rng(seed)
    bounds = (32, 64, 128, 256)
    sim = al.PoolSim(2048, 1024, 512, max_requests=48, window=64, boundaries=bounds)
    lines = [f"C 2048 1024 512 16 48 64 4 {fmt(bounds)}"]

    def snapshot():
        rows = sim.snapshot()
        flat = [len(rows)] + [x for r in rows for x in r]
        ext = []
        for arena in (0, 1):
            e = sim.free_extents(arena)
            ext += [len(e)] + [x for pair in e for x in pair]
        lines.append(f"S # {fmt(flat)} | {fmt(ext)}")

    for step in range(steps):
        op = rng.choice(["assign", "assign", "release", "advance", "migrate", "recal"])
        if op == "assign":
            k = int(rng.integers(1, 6))
            ids, pred = rng.integers(-1, 50, k), rng.integers(-2, 600, k)
            u = rng.random(k).astype(np.float32) if rng.random() < 0.7 else None
            prompt = rng.integers(0, 40, k) if rng.random() < 0.5 else None
            b = tuple(sorted(rng.choice(np.arange(16, 513, 16), 3, replace=False).tolist())) if rng.random() < 0.2 else None
            bk, off, cap, st = sim.assign(ids.tolist(), pred.tolist(), u, None if prompt is None else prompt.tolist(), b)
            ubits = None if u is None else u.view(np.uint32)
            lines.append(f"A {k} | {fmt(ids)} | {fmt(pred)} | {fmt(ubits)} | {fmt(prompt)} | {fmt(b)} # {fmt(bk)} | {fmt(off)} | {fmt(cap)} | {fmt(st)}")
        elif op == "release":
            ids = rng.integers(0, 48, int(rng.integers(1, 4)))
            lines.append(f"R {len(ids)} | {fmt(ids)} # {fmt(sim.release(ids.tolist()))}")
        elif op == "advance":
            ids = rng.integers(0, 48, int(rng.integers(1, 8)))
            nn = rng.integers(0, 70, len(ids)) if rng.random() < 0.7 else None
            ov, st = sim.advance(ids.tolist(), None if nn is None else nn.tolist())
            lines.append(f"V {len(ids)} | {fmt(ids)} | {fmt(nn)} # {fmt(ov)} | {fmt(st)}")
        elif op == "migrate":
            rid = int(rng.integers(0, 48))
            st, noff, ncap, _, _ = sim.migrate(rid)
            lines.append(f"M {rid} # {st} {noff} {ncap}")
        else:
            lens = wl.pareto(rng, int(rng.integers(0, 40)), 1.2, 4, 2000).tolist()
            lines.append(f"K {len(lens)} | {fmt(lens)} # {fmt(sim.recalibrate(lens))}")
        if step % 10 == 9:
            snapshot()
    snapshot()
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")
    return len(lines)


@pytest.mark.parametrize("san", ["asan", "tsan"])
def test_random_traces_under_sanitizers(drivers, tmp_path, san):
    for seed in range(4):
        trace = str(tmp_path / f"trace_{seed}.txt")
        n = write_trace(trace, seed)
        out = run(drivers[san], "replay", trace)
        assert f"replayed {n} calls: all equal" in out


def test_a_planted_mistake_in_the_trace_is_caught(drivers, tmp_path):
    trace = str(tmp_path / "trace.txt")
    write_trace(trace, 9, steps=60)
    lines = open(trace).read().splitlines()
    i = next(k for k, l in enumerate(lines) if l.startswith("A ") and " 0" in l.split("#")[1])
    head, want = lines[i].split("#")
    parts = want.split("|")
    parts[1] = " " + " ".join(str(int(x) + 16) for x in parts[1].split()) + " "     # every expected offset off by one block
    lines[i] = head + "#" + "|".join(parts)
    open(trace, "w").write("\n".join(lines) + "\n")
    r = subprocess.run([drivers["asan"], "replay", trace], capture_output=True, text=True, timeout=120)
    assert r.returncode == 1 and "assign: offset differs from the oracle" in r.stdout


@pytest.mark.parametrize("san", ["tsan", "asan"])
def test_background_recalibrator_under_threads(drivers, san):
    out = run(drivers[san], "threads", "60")
    fields = out.split()
    epoch, got, bad = int(fields[1]), tuple(int(x) for x in fields[3:7]), int(fields[8])
    assert bad == 0
    assert epoch == (2 * 60 * 25 + 300) // 50
    # what the window holds in the end: the last 256 of the 300 values the driver thread reported last
    sim = al.PoolSim(16, 16, 65536, window=256, boundaries=(512, 1024, 2048, 4096))
    assert got == tuple(sim.recalibrate([64 + (j * 37) % 5000 for j in range(300)]))
