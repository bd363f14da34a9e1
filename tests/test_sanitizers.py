"""Sanitizer runs of the CPU-side code (no GPU).

1. oracle/sanitize_check.c + the oracle's sources under AddressSanitizer and
   UndefinedBehaviorSanitizer: every oracle entry point on small and degenerate
   inputs with exactly-sized buffers.
2. The oracle's pin tests (the tests that tie the oracle to definitions, closed forms and the
   paper's worked examples) once more against a build of the oracle with
   UndefinedBehaviorSanitizer, in a child interpreter."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE = os.path.join(ROOT, "oracle")
SOURCES = ["fastgl_oracle.c", "update_oracle.c", "idmap_oracle.c", "match_oracle.c", "edge_oracle.c"]


def test_oracle_entry_points_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_check")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-static-libasan", "-o", exe, os.path.join(ORACLE, "sanitize_check.c"),
           *[os.path.join(ORACLE, s) for s in SOURCES], "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "clean" in res.stdout


def test_oracle_pin_tests_under_ubsan():
    pins = ["tests/test_oracle_pins.py", "tests/test_update_oracle_pins.py", "tests/test_idmap_oracle_pins.py",
            "tests/test_match_oracle_pins.py", "tests/test_edge_oracle_pins.py"]
    env = dict(os.environ, FASTGL_ORACLE_UBSAN="1")
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *pins], cwd=ROOT,
                         capture_output=True, text=True, env=env, timeout=900)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]
    assert os.path.exists(os.path.join(ORACLE, "libfastgl_oracle_ubsan.so"))


def test_host_side_of_the_c_abi_under_asan_and_ubsan(tmp_path):
    """api.hip, bookkeeping.hip and aggregate.hip with sanitizers on their HOST code (device code
    is compiled as usual), driven by tests/abi_host_driver.cpp: refused calls, and - only where no GPU
    is present - the host-side carving and job-building code up to the first launch."""
    hipcc, clang = "/opt/rocm/bin/hipcc", "/opt/rocm/llvm/bin/clang++"
    csrc = os.path.join(ROOT, "paper_2409_14939_amd", "csrc")
    lib = str(tmp_path / "libfastgl_agg_asan.so")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-omit-frame-pointer"]
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-shared",
                    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *san,
                    "-I" + os.path.join(ROOT, "include"), "-I" + csrc,
                    *[os.path.join(csrc, f) for f in ("api.hip", "bookkeeping.hip", "aggregate.hip")], "-o", lib],
                   check=True, capture_output=True)
    exe = str(tmp_path / "abi_host_driver")
    subprocess.run([clang, "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-omit-frame-pointer",
                    "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "abi_host_driver.cpp"), "-L" + str(tmp_path), "-lfastgl_agg_asan",
                    "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath," + str(tmp_path), "-Wl,-rpath,/opt/rocm/lib", "-o", exe],
                   check=True, capture_output=True)
    # the HIP runtime keeps its own allocations until exit: leak reports are about it, not about the library
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "clean" in res.stdout
