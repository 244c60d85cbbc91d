"""Host-side sanitizer legs (CPU only): native code of this repository that runs on the host is
compiled with -fsanitize=address,undefined and exercised; a memory error or undefined behaviour
makes the sanitized program exit non-zero with a report."""
import os
import struct
import subprocess

import numpy as np
import pytest

from oracle import svgear_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1", UBSAN_OPTIONS="halt_on_error=1",
           OMP_NUM_THREADS="4")
ENV.pop("LD_PRELOAD", None)  # the sanitizer runtime must come first in the sanitized child process


@pytest.fixture(scope="module")
def assign_exe(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("san") / "assign_sanitized")
    cmd = ["gcc", "-O1", "-ffp-contract=off", "-fopenmp", *SAN, os.path.join(ROOT, "oracle", "assign_f32.c"),
           os.path.join(ROOT, "tests", "native", "assign_sanitize_main.c"), "-o", out, "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return out


@pytest.mark.parametrize("n,d,C", [(1, 64, 1), (257, 64, 37), (1000, 128, 65), (33, 16, 500)])
def test_oracle_assignment_is_clean_under_address_and_ub_sanitizers(assign_exe, tmp_path, n, d, C):
    rng = np.random.default_rng(n + C)
    X = rng.standard_normal((n, d)).astype(np.float32)
    Cent = rng.standard_normal((C, d)).astype(np.float32)
    if C > 2:
        Cent[C // 2] = Cent[0]  # a tie
    inp, outp = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(inp, "wb") as f:
        f.write(struct.pack("<qii", n, d, C))
        f.write(X.tobytes())
        f.write(Cent.tobytes())
    r = subprocess.run([assign_exe, inp, outp], capture_output=True, text=True, env=ENV, timeout=120)
    assert r.returncode == 0, f"sanitizer report:\n{r.stderr[-3000:]}"
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]
    raw = open(outp, "rb").read()
    labels = np.frombuffer(raw[: 4 * n], np.int32)
    best = np.frombuffer(raw[4 * n:], np.float32)
    # the sanitized build decides the same labels, bit for bit, as the library the other tests use
    lab_ref, best_ref = orc.kmeans_assign(X, Cent, return_scores=True)
    assert np.array_equal(labels, lab_ref)
    assert np.array_equal(best.view(np.uint32), best_ref.view(np.uint32))


def test_abi_argument_checks_are_clean_under_host_sanitizers(tmp_path_factory):
    """The library's HOST code (argument checks, workspace arithmetic) compiled with
    -fsanitize=address,undefined (device code unchanged) and driven by a C program through every
    entry point's rejection paths and the workspace queries at extreme sizes. No GPU is needed:
    every call is refused before anything touches the device."""
    from paper_2603_08982_amd.build import HIPCC, build

    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not present")
    work = str(tmp_path_factory.mktemp("abi_san"))
    lib = build(lib=os.path.join(work, "libsvgear_san.so"), objdir=os.path.join(work, "obj"), host_sanitize=True)
    exe = os.path.join(work, "abi_argcheck")
    clang = os.path.join(os.path.dirname(os.path.realpath(HIPCC)), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang"
    cmd = [clang, *SAN, "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "native", "abi_argcheck_main.c"),
           lib, "-Wl,-rpath," + work, "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    env = dict(ENV, ASAN_OPTIONS="detect_leaks=0:halt_on_error=1")  # the HIP runtime's own start-up allocations are not ours
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, f"{r.stdout[-3000:]}\n{r.stderr[-3000:]}"
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]
    assert "0 wrong status code(s)" in r.stdout
