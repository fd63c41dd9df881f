"""CPU-only: the oracle, and the host side of the C-ABI library (shape planning and argument validation),
built and run under -fsanitize=address,undefined.  No GPU is touched: the drivers only make calls that
return before any HIP call."""
import concurrent.futures
import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANGXX = "/opt/rocm/llvm/bin/clang++"
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"]


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, "%s\n%s" % (" ".join(cmd), r.stdout[-4000:])
    return r.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    _run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-Wall"] + SAN +
         ["-o", exe, os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
          os.path.join(ROOT, "oracle", "dropit_oracle.c"), "-lm"])
    assert "OK" in _run([exe], env=dict(os.environ, OMP_NUM_THREADS="4"))


@pytest.mark.skipif(not (os.path.exists(HIPCC) and os.path.exists(CLANGXX)), reason="needs the ROCm compilers")
def test_host_side_of_the_library_under_sanitizers(tmp_path):
    """Every HIP source with its HOST code instrumented (the device code is compiled as usual and never runs),
    linked with a driver that walks the planning and validation paths."""
    host_san = []
    for f in SAN:
        host_san += ["-Xarch_host", f]
    common = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2202_13808_amd", "csrc")]
    sources = sorted(glob.glob(os.path.join(ROOT, "paper_2202_13808_amd", "csrc", "*.hip")))
    objs = [str(tmp_path / (os.path.basename(s)[:-4] + ".o")) for s in sources]
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 2)) as pool:
        list(pool.map(lambda so: _run([HIPCC] + common + host_san + ["-c", so[0], "-o", so[1]]), zip(sources, objs)))
    main_o = str(tmp_path / "abi_driver.o")
    _run([CLANGXX, "-O1", "-g", "-std=c++17"] + SAN + ["-I", os.path.join(ROOT, "include"), "-c",
          os.path.join(ROOT, "tests", "sanitize", "abi_driver.cpp"), "-o", main_o])
    exe = str(tmp_path / "abi_driver")
    _run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize"] + objs +
         [main_o, "-o", exe])
    assert "OK" in _run([exe])
    shutil.rmtree(str(tmp_path), ignore_errors=True)
