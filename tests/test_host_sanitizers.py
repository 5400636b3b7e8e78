"""Host code under AddressSanitizer + UBSan (CPU only): the layer-spec planner of the HIP library
(csrc/ae_plan.cpp, with stand-ins for the kernel-geometry predicates it asks of the GPU translation units) and the
CPU oracle (oracle/ae_oracle.cpp) are compiled with g++ -fsanitize=address,undefined into one program
(tests/host_sanitize/driver.cpp) that drives them with the workload specs, hostile specs and a small network."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_planner_and_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    src = [os.path.join(ROOT, "tests", "host_sanitize", "driver.cpp"),
           os.path.join(ROOT, "tests", "host_sanitize", "plan_stubs.cpp"),
           os.path.join(ROOT, "paper_2602_17681_amd", "csrc", "ae_plan.cpp"),
           os.path.join(ROOT, "oracle", "ae_oracle.cpp")]
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-w",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan", "-static-libubsan",
           "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"),
           "-I" + os.path.join(ROOT, "paper_2602_17681_amd", "csrc")] + src + ["-o", exe]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "sanitize-ok" in r.stdout, r.stdout[-3000:] + r.stderr[-3000:]
