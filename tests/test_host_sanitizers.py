"""Host-side sanitizer pass (CPU, no device): the oracle, and the host code of the library's C ABI, each built
with -fsanitize=address,undefined and driven by a small program that runs every function on exactly-sized heap
buffers / through every refusal path.  Passing = the programs run to the end with nothing reported."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
OUT = os.path.join(ROOT, "tests", "sanitize", "_build")
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"]


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, (" ".join(cmd), r.stdout[-2000:], r.stderr[-4000:])
    return r.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "oracle_san")
    src = [os.path.join(ROOT, "oracle", f) for f in ("qpo.c", "qpo_encode.c", "qpo_kmeans.c")]
    run(["gcc", "-std=c99", "-O1", "-g", "-fopenmp"] + SAN + ["-Wall", "-Wextra", "-o", exe,
         os.path.join(HERE, "oracle_san.c")] + src + ["-lm"])
    assert "oracle: clean" in run([exe], env={**os.environ, "ASAN_OPTIONS": "detect_leaks=1", "OMP_NUM_THREADS": "4"})


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="no hipcc")
def test_library_host_side_under_address_and_undefined_behaviour_sanitizers():
    """Only the host pass of the two files that hold host logic (the C ABI and the solvers) is instrumented;
    the kernels' files come from the regular build (their host side only launches)."""
    from paper_2509_20214_amd import build as hip_build
    os.makedirs(OUT, exist_ok=True)
    regular = {s: os.path.join(hip_build.OBJ, s[:-4] + ".o") for s in hip_build.sources()}
    if not all(os.path.exists(o) for o in regular.values()):
        hip_build.build()
    objs = []
    for s in hip_build.sources():
        if s in ("qp_api.hip", "qp_msq.hip"):
            o = os.path.join(OUT, s[:-4] + "_san.o")
            flags = [f for f in hip_build.FLAGS if f != "-O3"] + ["-O1", "-g"]
            for f in SAN:
                flags += ["-Xarch_host", f]
            run([hip_build.HIPCC] + flags + ["-c", os.path.join(hip_build.CSRC, s), "-o", o])
            objs.append(o)
        else:
            objs.append(regular[s])
    drv = os.path.join(OUT, "abi_san.o")
    run([hip_build.HIPCC, "-std=c++17", "-O1", "-g", "-fno-gpu-sanitize"] + SAN + ["-I", os.path.join(ROOT, "include"), "-x", "c++", "-c",
         os.path.join(HERE, "abi_san.cpp"), "-o", drv])
    exe = os.path.join(OUT, "abi_san")
    run([hip_build.HIPCC, "--offload-arch=gfx950", "-fno-gpu-sanitize"] + SAN + ["-o", exe, drv] + objs)
    # (leak checking off: the HIP runtime keeps its own allocations until the process ends)
    assert "host side: clean" in run([exe], env={**os.environ, "ASAN_OPTIONS": "detect_leaks=0"})
