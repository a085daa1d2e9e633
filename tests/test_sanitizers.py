"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no GPU work):
the oracle's C++ on small inputs with the edge cases, and the library's host-side argument validation."""
import concurrent.futures
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"]


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-3000:]}\n{r.stderr[-3000:]}"
    return r


@pytest.mark.skipif(shutil.which("g++") is None, reason="no g++")
def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["g++", "-std=c++17", "-O1", "-g", *SAN, "-static-libasan", os.path.join(ROOT, "oracle", "sanitize_main.cpp"),
          "-o", exe])
    r = _run([exe])
    assert "ok" in r.stdout


@pytest.mark.skipif(shutil.which("hipcc") is None or shutil.which("g++") is None, reason="no hipcc / g++")
def test_library_argument_validation_under_asan_and_ubsan(tmp_path):
    # the library's translation units with the sanitizers on their host code only (device code is cross-compiled
    # as usual), linked with a driver that walks the validation paths; nothing here touches a device
    csrc = os.path.join(ROOT, "paper_2310_02409_amd", "csrc")
    srcs = sorted(f for f in os.listdir(csrc) if f.endswith(".hip"))
    host_san = [x for flag in SAN for x in ("-Xarch_host", flag)]

    def compile_one(f):
        obj = str(tmp_path / (f[:-4] + ".o"))
        _run(["hipcc", "--offload-arch=gfx950", "-O1", "-std=c++17", "-fPIC", "-Wno-unused-function", "-Xclang",
              "-target-feature", "-Xclang", "-packed-fp32-ops", *host_san, "-I", os.path.join(ROOT, "include"), "-I", csrc,
              "-c", os.path.join(csrc, f), "-o", obj])
        return obj
    with concurrent.futures.ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(compile_one, srcs))
    main_o = str(tmp_path / "main.o")
    _run(["g++", "-std=c++17", "-O1", "-g", *SAN, "-I", os.path.join(ROOT, "include"), "-c",
          os.path.join(ROOT, "tests", "abi_sanitize_main.cpp"), "-o", main_o])
    exe = str(tmp_path / "abi_san")
    _run(["hipcc", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", main_o, *objs,
          "-o", exe])
    r = _run([exe])
    assert "ok" in r.stdout
