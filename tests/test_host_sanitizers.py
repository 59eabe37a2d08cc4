"""The planner behind the C ABI under AddressSanitizer + UndefinedBehaviorSanitizer.

tests/host_fuzz.cpp is compiled together with the library's host sources (the kernel launcher is a stub,
nothing touches a device) and run on a range of seeds: random well-formed layer graphs of every operator must
compile, the same graphs with fields overwritten by arbitrary values must come back with a status, and the
sanitizers must stay silent (any finding aborts the driver).
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2410_21120_amd", "csrc")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    gxx = shutil.which("g++")
    if gxx is None or not os.path.exists(os.path.join(ROCM, "include", "hip", "hip_runtime.h")):
        pytest.skip("needs g++ and the HIP headers")
    exe = str(tmp_path_factory.mktemp("host_fuzz") / "host_fuzz")
    cmd = [gxx, "-std=c++17", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-static-libasan", "-static-libubsan", "-D__HIP_PLATFORM_AMD__", "-w",
           "-I" + os.path.join(ROCM, "include"), "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
           os.path.join(CSRC, "fi_plan.cpp"), os.path.join(CSRC, "fi_api.cpp"), os.path.join(CSRC, "fi_sched.cpp"),
           os.path.join(ROOT, "tests", "host_fuzz.cpp"),
           "-L" + os.path.join(ROCM, "lib"), "-lamdhip64", "-lpthread", "-Wl,-rpath," + os.path.join(ROCM, "lib"), "-o", exe]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0 and "asan" in r.stdout.lower() and "cannot find" in r.stdout.lower():
        pytest.skip("static sanitizer runtimes are not installed")
    assert r.returncode == 0, r.stdout[-3000:]
    return exe


def test_planner_survives_random_and_damaged_specs(driver):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([driver, "1", "250"], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    assert r.returncode == 0, r.stdout[-4000:]
    last = r.stdout.strip().splitlines()[-1]
    assert last.startswith("host_fuzz: 250 seeds") and last.endswith(" 0 failed checks"), last
    compiled = int(last.split(" seeds, ")[1].split(" ")[0])
    rejected = int(last.split(" compiled, ")[1].split(" ")[0])
    assert compiled >= 200 and rejected >= 500, last   # the generator really produces valid graphs, the damage really bites


def test_request_aggregator_under_thread_sanitizer(tmp_path):
    """tests/server_sim.cpp: the server's queueing, batching, waiting and member swaps with the device replaced
    by host stand-ins, four client threads against the worker while the main thread swaps members, compiled with
    ThreadSanitizer.  Every request must receive the row of its own image and member; any race report fails."""
    gxx = shutil.which("g++")
    if gxx is None or not os.path.exists(os.path.join(ROCM, "include", "hip", "hip_runtime.h")):
        pytest.skip("needs g++ and the HIP headers")
    exe = str(tmp_path / "server_sim")
    cmd = [gxx, "-std=c++17", "-g", "-O1", "-fsanitize=thread", "-static-libtsan", "-D__HIP_PLATFORM_AMD__", "-w",
           "-I" + os.path.join(ROCM, "include"), "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
           os.path.join(CSRC, "fi_server.cpp"), os.path.join(ROOT, "tests", "server_sim.cpp"), "-lpthread", "-o", exe]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0 and "tsan" in r.stdout.lower() and "cannot find" in r.stdout.lower():
        pytest.skip("static ThreadSanitizer runtime is not installed")
    assert r.returncode == 0, r.stdout[-3000:]
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=0:exitcode=66")
    r = subprocess.run([exe, "4", "2500"], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    if "unexpected memory mapping" in r.stdout:
        pytest.skip("ThreadSanitizer cannot map its shadow memory on this kernel")
    assert r.returncode == 0 and "ThreadSanitizer" not in r.stdout, r.stdout[-4000:]
    last = r.stdout.strip().splitlines()[-1]
    assert last.startswith("server_sim: ") and last.endswith(" 0 wrong"), last
    served = int(last.split()[1])
    assert served >= 5000 and " swaps," in last   # most requests get through between the swaps
