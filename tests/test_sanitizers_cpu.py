"""Host-side code under sanitizers (CPU only): the C oracle and the input generator are rebuilt
with -fsanitize=address,undefined together with a C driver that walks all their entry points
(tests/c/sanitized_cpu_side.c), and the C program of the ABI's host-side argument checks
(tests/c/abi_host_checks.c) is rebuilt the same way and run against the library."""
import os
import subprocess
from pathlib import Path

ROOT = Path(__file__).resolve().parent.parent
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="2")


def _run(cmd, **kw):
    out = subprocess.run(cmd, capture_output=True, text=True, timeout=300, **kw)
    assert out.returncode == 0 and out.stdout.strip().endswith("ok"), (cmd, out.stdout[-2000:], out.stderr[-4000:])


def test_oracle_and_generator_under_address_and_ub_sanitizers(tmp_path):
    gen_o = tmp_path / "graphgen.o"
    subprocess.check_call(["g++", "-std=c++17", "-fopenmp", *SAN, "-c", str(ROOT / "graphgen" / "graphgen.cpp"),
                           "-o", str(gen_o)])
    exe = tmp_path / "sanitized_cpu_side"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-fopenmp", *SAN,
                           str(ROOT / "tests" / "c" / "sanitized_cpu_side.c"), str(ROOT / "oracle" / "epp_oracle.c"),
                           str(gen_o), "-o", str(exe), "-lstdc++", "-lm"])
    _run([str(exe)], env=ENV)


def test_abi_host_checks_under_sanitizers(tmp_path):
    import paper_2204_02662_amd as epp

    epp.load_library()
    so_dir = epp.SO.parent
    exe = tmp_path / "abi_host_checks_san"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", *SAN, "-I", str(ROOT / "include"),
                           str(ROOT / "tests" / "c" / "abi_host_checks.c"), "-o", str(exe),
                           "-L", str(so_dir), "-lepp", f"-Wl,-rpath,{so_dir}"])
    # (the HIP runtime the library pulls in keeps process-lifetime allocations: leak checking is for our own driver above)
    _run([str(exe)], env=dict(ENV, ASAN_OPTIONS="detect_leaks=0"))
