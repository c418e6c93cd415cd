"""The library's host code (argument validation, memory layouts, error paths, the once-per-device helpers) built with
AddressSanitizer and UndefinedBehaviorSanitizer on the CPU and driven through its validation paths by
tests/host_sanitize_main.cpp, from one thread and from four at once.  Device code is not sanitized (and not run)."""
import os
import shutil
import subprocess

import pytest

from paper_2409_15241_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/llvm/bin/clang++"
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


@pytest.mark.skipif(not (os.path.exists(CLANG) and shutil.which(B.hipcc())), reason="needs the ROCm compilers")
def test_host_code_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    os.makedirs(B.BUILD, exist_ok=True)
    objs = []
    for src in B.SOURCES:
        if src == "api.hip":
            continue
        obj = os.path.join(B.BUILD, src.replace(".hip", ".o"))
        if not os.path.exists(obj) or os.path.getmtime(obj) < os.path.getmtime(os.path.join(B.CSRC, src)):
            obj = B._compile(src)
        objs.append(obj)
    api = str(tmp_path / "api_san.o")
    host_flags = [f for s in SAN for f in ("-Xarch_host", s)]
    flags = [f for f in B.FLAGS if f != "-O3"]
    r = subprocess.run([B.hipcc(), *flags, "-O1", "-g", *host_flags, "-c", os.path.join(B.CSRC, "api.hip"), "-o", api],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    main = str(tmp_path / "main_san.o")
    r = subprocess.run([CLANG, *SAN, "-std=c++17", "-O1", "-g", "-c", os.path.join(ROOT, "tests", "host_sanitize_main.cpp"),
                        "-o", main], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    exe = str(tmp_path / "host_sanitize")
    r = subprocess.run([CLANG, *SAN[:2], main, api, *objs, "-o", exe, "-L/opt/rocm/lib", "-lamdhip64", "-lpthread",
                        "-Wl,-rpath,/opt/rocm/lib"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    out = r.stdout + r.stderr
    assert r.returncode == 0 and "host sanitize driver: ok" in r.stdout, out[-3000:]
    assert "runtime error" not in out and "AddressSanitizer" not in out, out[-3000:]
