"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer, without a GPU: the scheduler
and cache-manager sources (csrc/serving.cpp, csrc/kvm.cpp) replay the oracle's random drives and
loop traces and must take the oracle's decisions; the C oracle runs its pins; the plain C client
runs its host part.  The sanitizer runtimes are linked statically into small programs of their
own, so nothing is preloaded into the Python process."""
import os
import subprocess

import numpy as np
import pytest

from oracle.kv_manager import IterationLoop, ProactiveCacheManager
from oracle.scheduler import SkipJoinMLFQ
from tests.test_kv_manager_oracle import OracleWorld, random_drive

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
PKG = os.path.join(ROOT, "paper_2305_05920_amd")
FLAGS = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
         "-static-libasan"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def run(cmd, **kw):
    return subprocess.run(cmd, capture_output=True, text=True, timeout=300, **kw)


@pytest.fixture(scope="module")
def library():
    lib = os.path.join(PKG, "libfastserve.so")
    if not os.path.exists(lib):
        from paper_2305_05920_amd import build
        build.build_library()
    return lib


@pytest.fixture(scope="module")
def replay_exe(library):
    exe = os.path.join(SAN, "replay_san")
    out = run(["g++", "-std=c++17", *FLAGS, "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"),
               "-I", "/opt/rocm/include", os.path.join(PKG, "csrc", "serving.cpp"), os.path.join(PKG, "csrc", "kvm.cpp"),
               os.path.join(SAN, "replay.cpp"), "-o", exe, "-L", PKG, "-lfastserve", "-L", "/opt/rocm/lib", "-lamdhip64",
               f"-Wl,-rpath,{PKG}", "-Wl,-rpath,/opt/rocm/lib"])
    assert out.returncode == 0, out.stderr
    return exe


class Recorder(OracleWorld):
    """The oracle's world; every event is also written down as a script line, every decision as the
    line the replay program has to print."""

    def __init__(self, s, k):
        super().__init__(s, k)
        self.script, self.expect = [], []

    def state(self):
        k = self.k
        live = sorted(j for j, c in k.jobs.items() if not c.released)
        self.script.append(f"state {len(live)} " + " ".join(map(str, live)))
        jobs = "".join(f" {j}:{k.jobs[j].where}:{k.jobs[j].length}:" +
                       ",".join(map(str, k.jobs[j].blocks if k.jobs[j].where in (0, 3) else k.jobs[j].slots))
                       for j in live)
        self.expect.append(f"state {len(k.free_blocks)} {len(k.free_slots)} {k.reserve} {k.blocks_out} {k.blocks_in} "
                           f"{len(k.moves)}{jobs}")
        self.script.append("batch")
        self.expect.append("batch" + "".join(f" {j}" for j in self.s.schedule()))

    def admit(self, j, tokens, init_time):
        ok = self.k.admit(j, tokens)
        self.script.append(f"admit {j} {tokens}")
        self.expect.append(f"admit {int(ok)}")
        if ok:
            q = self.s.add_job(j, init_time, 1.0)
            self.script.append(f"add {j} {init_time!r} 1.0")
            self.expect.append(f"add {q}")
        self.state()
        return ok

    def grow(self, j, n):
        ok = super().grow(j, n)
        self.script.append(f"grow {j} {n}")
        self.expect.append(f"grow {int(ok)}")
        self.state()
        return ok

    def iteration(self, elapsed):
        batch = super().iteration(elapsed)
        self.script.append(f"done {elapsed!r} {len(batch)} " + " ".join(map(str, batch)) + " 0")
        self.state()
        return batch

    def start_swaps(self, want):
        running, moves = super().start_swaps(want)
        self.script.append(f"swaps {want} {len(running)} " + " ".join(map(str, running)))
        self.state()
        return running, moves

    def retire(self, n):
        got = super().retire(n)
        self.script.append(f"retire {n}")
        self.expect.append(f"retire {got}")
        self.state()
        return got

    def observe(self, d):
        super().observe(d)
        self.script.append(f"observe {d}")
        self.state()

    def release(self, j):
        super().release(j)
        self.script += [f"release {j}", f"ready {j} 1", f"done 0.0 1 {j} 1 {j}"]
        self.state()


@pytest.mark.parametrize("seed", [0, 1])
def test_scheduler_and_manager_replay_the_oracles_drive_under_sanitizers(replay_exe, seed):
    s = SkipJoinMLFQ(4, 1.0, 1, 6.0, 3)
    k = ProactiveCacheManager(s, 24, 30, 16, 6, reserve_idle_blocks=2, reserve_window=8, reserve_quantile=0.75)
    rec = Recorder(s, k)
    random_drive(rec, np.random.default_rng(900 + seed), 500)
    assert k.blocks_out > 0 and k.blocks_in > 0
    script = "sched 4 1.0 1 6.0 3\nkvm 24 30 16 6 2 8 0.75\n" + "\n".join(rec.script) + "\n"
    out = run([replay_exe], input=script, env=ENV)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-4000:]
    got = out.stdout.splitlines()
    assert got[-1] == "replay ok" and "runtime error" not in out.stderr and "AddressSanitizer" not in out.stderr
    assert got[:-1] == rec.expect


def test_iteration_loop_replays_an_oracle_trace_under_sanitizers(replay_exe):
    rng = np.random.default_rng(77)
    n = 40
    prompts = np.clip(np.round(rng.exponential(60.0, n)), 1, 200).astype(int)
    outputs = np.clip(np.floor(rng.pareto(1.2, n) * 6 + 1), 1, 60).astype(int)
    arrival = np.sort(rng.integers(0, 30, size=n))
    ora = IterationLoop(5, 1.0, 1, 12.0, 4, 256, num_blocks=60, num_host_blocks=400, block_size=16, table_width=20,
                        reserve_idle_blocks=4, reserve_window=16, reserve_quantile=0.8)
    script = ["loop 5 1.0 1 12.0 4 256 60 400 16 20 4 16 0.8"]
    for j in range(n):
        init = float(prompts[j]) / 16.0
        ora.submit(j, int(arrival[j]), int(prompts[j]), int(outputs[j]), init, 1.0)
        script.append(f"submit {j} {arrival[j]} {prompts[j]} {outputs[j]} {init!r} 1.0")
    expect = []
    while ora.jobs:
        left = len(ora.jobs)
        p = ora.plan()
        expect.append("plan first" + "".join(f" {j}" for j in p["first"]) + " decode" +
                      "".join(f" {j}@{L}" for j, L in zip(p["decode"], p["lens_before"])) +
                      f" waiting {len(ora.waiting)} left {left}")
        script.append("plan")
        live = sorted(j for j, c in ora.kvm.jobs.items() if not c.released)
        script.append(f"state {len(live)} " + " ".join(map(str, live)))
        k = ora.kvm
        expect.append(f"state {len(k.free_blocks)} {len(k.free_slots)} {k.reserve} {k.blocks_out} {k.blocks_in} "
                      f"{len(k.moves)}" + "".join(
                          f" {j}:{k.jobs[j].where}:{k.jobs[j].length + (int(prompts[j]) if j in p['first'] else 1 if j in p['decode'] else 0)}:" +
                          ",".join(map(str, k.jobs[j].blocks if k.jobs[j].where in (0, 3) else k.jobs[j].slots))
                          for j in live))
        ora.complete()
    expect.append(f"stats {ora.iteration} {ora.job_tokens} {ora.prompt_tokens} {ora.finished}")
    out = run([replay_exe], input="\n".join(script) + "\n", env=ENV)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-4000:]
    got = out.stdout.splitlines()
    assert got[-1] == "replay ok" and "runtime error" not in out.stderr and "AddressSanitizer" not in out.stderr
    assert ora.kvm.blocks_out > 0
    # the replay program completes an iteration right after planning it, so the state it prints shows
    # finished jobs gone: compare those lines job by job for the jobs still there
    for g, e in zip(got[:-1], expect):
        if e.startswith("state"):
            ge, ee = g.split(), e.split()
            assert ge[0] == "state"
            gone = {x.split(":")[0] for x in ge[7:] if x.endswith(":gone")}
            assert [x for x in ge[7:] if not x.endswith(":gone")] == [x for x in ee[7:] if x.split(":")[0] not in gone]
        else:
            assert g == e
    assert len(got) - 1 == len(expect)


def test_c_oracle_runs_its_pins_under_sanitizers():
    exe = os.path.join(SAN, "oracle_pins_san")
    out = run(["gcc", "-std=c11", *FLAGS, "-Wall", os.path.join(SAN, "oracle_pins.c"),
               os.path.join(ROOT, "oracle", "fs_oracle.c"), "-o", exe, "-lm"])
    assert out.returncode == 0, out.stderr
    out = run([exe], env=ENV)
    assert out.returncode == 0 and "oracle pins ok" in out.stdout, out.stdout + out.stderr
    assert "runtime error" not in out.stderr and "AddressSanitizer" not in out.stderr


def test_c_client_host_part_under_sanitizers(library):
    exe = os.path.join(SAN, "client_san")
    out = run(["gcc", "-std=c11", *FLAGS, "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"),
               "-I", "/opt/rocm/include", os.path.join(ROOT, "tests", "c_client", "client.c"), "-o", exe, "-L", PKG,
               "-lfastserve", "-L", "/opt/rocm/lib", "-lamdhip64", "-lm", f"-Wl,-rpath,{PKG}", "-Wl,-rpath,/opt/rocm/lib"])
    assert out.returncode == 0, out.stderr
    out = run([exe, "host"], env=dict(ENV, ASAN_OPTIONS="detect_leaks=0"))     # the HIP runtime keeps its own globals
    assert out.returncode == 0 and "host checks ok" in out.stdout, out.stdout + out.stderr
    assert "runtime error" not in out.stderr and "AddressSanitizer" not in out.stderr
