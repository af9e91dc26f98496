"""The boundary is a C ABI: a caller written in plain C (tests/c_client/client.c, compiled with
gcc against the two public headers) uses it without Python or a tensor library.  Its host part
(argument checks, error strings, the scheduler) runs anywhere; its GPU part runs a tiny decode
step in both forms and checks closed forms."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "c_client", "client.c")
EXE = os.path.join(ROOT, "tests", "c_client", "client")


def build_client(force: bool = False) -> str:
    lib = os.path.join(ROOT, "paper_2305_05920_amd", "libfastserve.so")
    if not os.path.exists(lib):
        pytest.skip("library not built")
    stale = not os.path.exists(EXE) or os.path.getmtime(EXE) < max(os.path.getmtime(SRC), os.path.getmtime(lib))
    if force or stale:
        tmp = EXE + f".tmp{os.getpid()}"
        subprocess.check_call([
            "gcc", "-std=c11", "-O1", "-Wall", "-Werror", "-D__HIP_PLATFORM_AMD__",
            "-I", os.path.join(ROOT, "include"), "-I", "/opt/rocm/include", SRC, "-o", tmp,
            "-L", os.path.join(ROOT, "paper_2305_05920_amd"), "-lfastserve", "-L", "/opt/rocm/lib", "-lamdhip64", "-lm",
            "-Wl,-rpath,$ORIGIN/../../paper_2305_05920_amd", "-Wl,-rpath,/opt/rocm/lib"])
        os.replace(tmp, EXE)
    return EXE


def test_c_client_builds_with_gcc_and_its_host_part_passes():
    exe = build_client(force=True)
    out = subprocess.run([exe, "host"], capture_output=True, text=True, timeout=60)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "host checks ok" in out.stdout


@pytest.mark.gpu
def test_c_client_runs_the_decode_step_on_the_gpu():
    exe = EXE if os.path.exists(EXE) else build_client()
    out = subprocess.run([exe, "gpu"], capture_output=True, text=True, timeout=120)
    print(out.stdout, out.stderr, flush=True)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "gpu checks ok" in out.stdout
