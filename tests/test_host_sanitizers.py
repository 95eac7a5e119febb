"""The CPU side under AddressSanitizer + UndefinedBehaviorSanitizer: the oracle (plain C) and the host
half of the library (roast_tile_index and the argument validation of every entry point, compiled from
csrc/roast_api.hip with host-side sanitizers; device code is never sanitised or run here)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
           OMP_NUM_THREADS="4")
ENV.pop("LD_PRELOAD", None)    # ASan must be the first runtime in the executable


def run_clean(exe):
    r = subprocess.run([exe], env=ENV, capture_output=True, text=True, timeout=300)
    text = r.stdout + r.stderr
    assert r.returncode == 0, text[-3000:]
    assert "runtime error" not in text and "AddressSanitizer" not in text, text[-3000:]
    assert "0 failures" in r.stdout, text[-3000:]


def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-Wall", "-Wextra",
                    os.path.join(ROOT, "oracle", "roast_oracle.c"), os.path.join(SAN, "oracle_driver.c"),
                    "-o", exe, "-lm"], check=True)
    run_clean(exe)


def test_library_host_half_under_address_and_undefined_sanitizers(tmp_path):
    from paper_2207_10702_amd import build as hb
    hipcc = hb._hipcc()
    if shutil.which(hipcc) is None and not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    objs = [os.path.join(hb.OBJ, os.path.splitext(s)[0] + ".o") for s in hb.SOURCES if s != "roast_api.hip"]
    if not all(os.path.exists(o) for o in objs):
        hb.build()          # the kernels' objects (unsanitised; none of their code runs here)
    san_host = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                "-Xarch_host", "-fno-sanitize-recover=undefined"]
    api_o, drv_o, exe = str(tmp_path / "api_san.o"), str(tmp_path / "drv.o"), str(tmp_path / "host_san")
    common = ["-O1", "-g", "-std=c++17", "-fPIC", "-I" + os.path.join(ROOT, "include"), "-I" + hb.CSRC]
    subprocess.run([hipcc, *common, "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                    *san_host, "-c", os.path.join(hb.CSRC, "roast_api.hip"), "-o", api_o],
                   check=True, stderr=subprocess.DEVNULL)
    subprocess.run([hipcc, *common, *san_host, "-c", os.path.join(SAN, "host_api_driver.cpp"), "-o", drv_o],
                   check=True, stderr=subprocess.DEVNULL)
    subprocess.run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                    "-o", exe, drv_o, api_o, *objs], check=True, stderr=subprocess.DEVNULL)
    run_clean(exe)
