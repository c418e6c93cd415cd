"""The library's host code built with AddressSanitizer and UndefinedBehaviorSanitizer on the CPU.  Device code is not
sanitized (and not run).  Two drivers:

* tests/host_sanitize_main.cpp links the real HIP runtime and walks the validation and error paths (argument checks,
  memory layouts, the once-per-device helpers), from one thread and from four at once;
* tests/host_schedule_main.cpp links neither the runtime nor the kernels: its stand-ins record every launch, event and
  wait that the layer and stack entry points enqueue, for every slicing and stream-pool size, and check the schedule
  itself: forks and joins, that no two launches that touch the same memory run unordered, the fixed accumulation
  order of the gradients, and that a captured call records no event twice."""
import os
import shutil
import subprocess

import pytest

from paper_2409_15241_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/llvm/bin/clang++"
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
needs_compilers = pytest.mark.skipif(not (os.path.exists(CLANG) and shutil.which(B.hipcc())), reason="needs the ROCm compilers")


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, (" ".join(cmd) + "\n" + r.stderr[-3000:])
    return r


@pytest.fixture(scope="module")
def api_san(tmp_path_factory):
    """api.hip with its host half under the sanitizers."""
    obj = str(tmp_path_factory.mktemp("san") / "api_san.o")
    host_flags = [f for s in SAN for f in ("-Xarch_host", s)]
    flags = [f for f in B.FLAGS if f != "-O3"]
    run([B.hipcc(), *flags, "-O1", "-g", *host_flags, "-c", os.path.join(B.CSRC, "api.hip"), "-o", obj])
    return obj


def driver(tmp_path, name):
    obj = str(tmp_path / (name + ".o"))
    run([CLANG, *SAN, "-std=c++17", "-O1", "-g", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-c",
         os.path.join(ROOT, "tests", name + ".cpp"), "-o", obj])
    return obj


@needs_compilers
def test_host_code_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path, api_san):
    os.makedirs(B.BUILD, exist_ok=True)
    objs = []
    for src in B.SOURCES:
        if src == "api.hip":
            continue
        obj = os.path.join(B.BUILD, src.replace(".hip", ".o"))
        if not os.path.exists(obj) or os.path.getmtime(obj) < os.path.getmtime(os.path.join(B.CSRC, src)):
            obj = B._compile(src)
        objs.append(obj)
    main = driver(tmp_path, "host_sanitize_main")
    exe = str(tmp_path / "host_sanitize")
    run([CLANG, *SAN[:2], main, api_san, *objs, "-o", exe, "-L/opt/rocm/lib", "-lamdhip64", "-lpthread", "-Wl,-rpath,/opt/rocm/lib"])
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)
    out = r.stdout + r.stderr
    assert r.returncode == 0 and "host sanitize driver: ok" in r.stdout, out[-3000:]
    assert "runtime error" not in out and "AddressSanitizer" not in out, out[-3000:]


@needs_compilers
def test_every_schedule_the_library_enqueues_is_ordered_and_race_free(tmp_path, api_san):
    main = driver(tmp_path, "host_schedule_main")
    exe = str(tmp_path / "host_schedule")
    run([CLANG, *SAN[:2], main, api_san, "-o", exe, "-lpthread"])
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)
    out = r.stdout + r.stderr
    assert r.returncode == 0 and "host schedule driver: ok" in r.stdout, out[-4000:]
    assert "planted race" in r.stdout                      # the race check showed that it can fail
    assert "runtime error" not in out and "AddressSanitizer" not in out, out[-3000:]
