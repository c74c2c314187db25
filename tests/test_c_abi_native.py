"""The boundary is a C ABI: the header must be valid C, and a plain C program (no Python, no
torch) must be able to drive the library and match the oracle."""
import os
import subprocess

import pytest

import oracle
from paper_2511_09557_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "native", "c_abi_parity.c")


def test_header_is_plain_c(tmp_path):
    c = tmp_path / "use_header.c"
    c.write_text('#include "rar.h"\nint main(void) { rar_plan_t *p = 0; return rar_plan(8, 4, 64, RAR_BF16, &p) != RAR_OK; }\n')
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-c", "-I", os.path.join(ROOT, "include"),
                    "-o", str(tmp_path / "use_header.o"), str(c)], check=True)


def build_native(tmp_path) -> str:
    exe = str(tmp_path / "c_abi_parity")
    lib_dir = os.path.dirname(binding.LIB_PATH)
    oracle_dir = os.path.dirname(oracle.build())
    subprocess.run(["gcc", "-std=c11", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"),
                    "-I", "/opt/rocm/include", SRC, "-o", exe,
                    "-L", lib_dir, "-lrar", "-L", oracle_dir, "-lnvrar_oracle", "-L", "/opt/rocm/lib", "-lamdhip64",
                    f"-Wl,-rpath,{lib_dir}", f"-Wl,-rpath,{oracle_dir}", "-Wl,-rpath,/opt/rocm/lib"], check=True)
    return exe


def test_native_program_builds(tmp_path):
    assert os.path.exists(build_native(tmp_path))


@pytest.mark.gpu
@pytest.mark.parametrize("P,G,n,dtype", [(8, 4, 65536, 0), (16, 4, 100003, 1), (64, 4, 1048576, 0), (12, 3, 4099, 0),
                                          (12, 4, 4099, 0), (40, 8, 100003, 1)])
def test_native_program_matches_oracle(tmp_path, P, G, n, dtype):
    exe = build_native(tmp_path)
    print(f"[gpu] native C program P={P} G={G} n={n} dtype={dtype}", flush=True)
    r = subprocess.run([exe, str(P), str(G), str(n), str(dtype)], capture_output=True, text=True, timeout=100)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "c abi parity ok" in r.stdout


def test_planner_and_oracle_under_sanitizers(tmp_path):
    """plan.cpp (host-only) and the C oracle, built with AddressSanitizer and UBSan, run through
    every shape and tuning the launchers can see; the program checks that all index ranges the
    kernels derive from the plan stay inside the buffers the plan sizes."""
    exe = str(tmp_path / "host_checks")
    csrc = os.path.join(ROOT, "paper_2511_09557_amd", "csrc")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                    "-Wall", "-Wextra", "-I", os.path.join(ROOT, "include"), "-I", csrc,
                    os.path.join(ROOT, "tests", "native", "host_checks.cpp"), os.path.join(csrc, "plan.cpp"),
                    "-x", "c", os.path.join(ROOT, "oracle", "nvrar_oracle.c"), "-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1", LD_PRELOAD="")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host checks ok" in r.stdout
