"""Host code under AddressSanitizer and UBSan (CPU only).

1. The library's planner (csrc/plan.cpp holds no GPU code) and the whole oracle are compiled
   with -fsanitize=address,undefined into tests/sanitize/host_sweep.cpp, which walks K <= 7,
   every r, both schedules, c, m in {1, 2}, seven value lengths and all five payload algebras
   on exact-size heap buffers and compares the two sides' tables on the way.
2. The kernels themselves, compiled for the host against the stand-in for HIP under
   tests/hip_cpu_shim (one thread per lane, heap-backed device memory and LDS), run every entry
   point on small shapes under the same sanitizers; and a call that falls back to one-element
   packs on a shape bound for four-element packs is refused before anything is launched.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1805_01993_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def test_planner_and_oracle_under_sanitizers(tmp_path):
    objs = []
    for cmd in (["gcc", "-std=c11", "-c", os.path.join(ROOT, "oracle", "ccdc_oracle.c"), "-o", str(tmp_path / "oracle.o")],
                ["g++", "-std=c++17", "-c", os.path.join(CSRC, "plan.cpp"), "-o", str(tmp_path / "plan.o")],
                ["g++", "-std=c++17", "-c", os.path.join(ROOT, "tests", "sanitize", "host_sweep.cpp"),
                 "-o", str(tmp_path / "sweep.o")]):
        inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-I", os.path.join(ROOT, "oracle")]
        subprocess.run(cmd[:2] + SAN + ["-Wall", "-Wextra"] + inc + cmd[2:], check=True)
        objs.append(cmd[-1])
    exe = str(tmp_path / "host_sweep")
    subprocess.run(["g++"] + SAN + objs + ["-lm", "-o", exe], check=True)
    res = subprocess.run([exe, "7"], capture_output=True, text=True, env=ENV, timeout=600)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.startswith("clean:"), res.stdout


@pytest.fixture(scope="module")
def kernel_driver(tmp_path_factory):
    cxx = "/opt/rocm/lib/llvm/bin/clang++"
    if not os.path.exists(cxx):
        cxx = shutil.which("clang++")
    if not cxx:
        pytest.skip("no clang++ to build the kernels for the host")
    out = tmp_path_factory.mktemp("shim")
    res = subprocess.run([os.path.join(ROOT, "tests", "hip_cpu_shim", "build.sh"), CSRC, str(out)],
                         capture_output=True, text=True, env=dict(os.environ, SHIM_CXX=cxx), timeout=900)
    assert res.returncode == 0, res.stdout + res.stderr
    return str(out / "driver")


# K, r, Q, N, T, mode (0 f32, 1 u32, 2 h32, 3 bf16, 4 f16), jobs, compute units, workgroups per unit
KERNEL_CASES = [
    (4, 2, 4, 12, 256, 0, 0, 8, 4),       # the tiny workload: m = 2, rounds cut into chunks
    (4, 2, 4, 12, 256, 1, 0, 1, 1),       # same, one chunk
    (5, 3, 10, 20, 100, 2, 0, 8, 4),      # c = 2, m = 2, r does not divide W: short last segment
    (4, 2, 4, 12, 7, 1, 0, 8, 4),         # one-element packs, ragged tail
    (4, 3, 4, 4, 1, 0, 0, 8, 4),          # W = 1: all but the first segment empty
    (6, 1, 6, 12, 72, 3, 0, 8, 4),        # r = 1, bfloat16 with eight-element packs
    (7, 5, 7, 21, 40, 4, 0, 8, 4),        # r = 5, binary16
    (10, 8, 10, 45, 36, 1, 0, 8, 4),      # r = 8: one-pass kernel refuses, fused kernel unrolled
    (4, 2, 4, 6, 64, 0, 1, 8, 4),         # the paper's four-job schedule
    (5, 2, 10, 6, 30, 1, 1, 8, 4),        # ten jobs, c = 2, two-element alignment only
    (4, 2, 4, 240, 12, 0, 0, 8, 4),       # 40 files a batch: wavefront-wide combiner
    (10, 3, 10, 120, 512, 0, 0, 256, 5),  # the 10-node plan, ragged split, chunked as on the device
    (8, 2, 8, 28, 4096, 3, 0, 1, 1),      # the gradient shape's plan, bfloat16, a single chunk, several column tiles
    (8, 4, 8, 70, 2048, 1, 0, 256, 3),    # r = 4 with the many-node shape's value length: two-element packs
]


@pytest.mark.parametrize("case", KERNEL_CASES, ids=lambda c: "-".join(map(str, c)))
def test_kernels_compiled_for_the_host_under_sanitizers(kernel_driver, case):
    res = subprocess.run([kernel_driver] + [str(v) for v in case], capture_output=True, text=True, env=ENV, timeout=600)
    assert res.returncode == 0, res.stdout + res.stderr
    assert " 0 mismatches" in res.stdout, res.stdout


def test_narrow_pack_fallback_is_refused_before_launch(kernel_driver):
    res = subprocess.run([kernel_driver, "limits"], capture_output=True, text=True, env=ENV, timeout=600)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "limits ok" in res.stdout, res.stdout
