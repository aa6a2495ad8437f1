"""AddressSanitizer + UndefinedBehaviorSanitizer over the host code: the fp64 C oracle (against its
pins) and the C-ABI library's argument validation (against tests/test_abi.py).  CPU only.

Each leg compiles a sanitized copy into a temporary folder, then runs the existing tests in a child
interpreter that has the matching sanitizer runtime preloaded and is pointed at that copy:

  * the oracle with gcc (-fsanitize=address,undefined; gcc's libasan preloaded);
  * the library with hipcc, each -fsanitize= behind -Xarch_host so that only the host side is instrumented
    (the device code is compiled as usual and never runs: every call in test_abi.py returns from a
    host-side check), clang's runtime preloaded.

The two runtimes cannot share a process, hence two children.  Leak checking is off (the interpreter itself
never frees everything); any other report makes the child exit non-zero.
"""
import glob
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2601_10155_amd", "csrc")


def _child_env(runtime):
    env = dict(os.environ)
    # the sanitizer runtime goes first; whatever was preloaded already stays
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=99"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:exitcode=98"
    env["PYTHONPATH"] = ROOT + (os.pathsep + env["PYTHONPATH"] if env.get("PYTHONPATH") else "")
    return env


def _run_child(code, runtime):
    p = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=_child_env(runtime),
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)
    assert p.returncode == 0, f"sanitized run failed (exit {p.returncode}):\n{p.stdout[-6000:]}"
    assert "runtime error:" not in p.stdout and "AddressSanitizer" not in p.stdout, p.stdout[-6000:]
    return p.stdout


def test_oracle_pins_under_asan_ubsan(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("gcc not found")
    runtime = subprocess.run([gcc, "-print-file-name=libasan.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("gcc has no shared libasan")
    lib = str(tmp_path / "liblookat_oracle_san.so")
    subprocess.run([gcc, "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
                    "-shared", "-fPIC", "-o", lib, os.path.join(ROOT, "oracle", "lookat_oracle.c"), "-lm"], check=True)
    code = f"""
import sys
import oracle
oracle._LIB = {lib!r}
oracle.build = lambda force=False: oracle._LIB
import pytest
sys.exit(pytest.main(["-x", "-q", "-p", "no:cacheprovider", "tests/test_oracle_pins.py", "tests/test_fidelity_metrics.py"]))
"""
    out = _run_child(code, runtime)
    assert " passed" in out, out[-2000:]


def test_library_host_validation_under_asan_ubsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    found = sorted(glob.glob("/opt/rocm*/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    if not found:
        pytest.skip("clang's shared AddressSanitizer runtime not found")
    runtime = found[-1]
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    objs, procs = [], []
    for src in sorted(f for f in os.listdir(CSRC) if f.endswith(".hip")):
        obj = str(tmp_path / src.replace(".hip", ".o"))
        objs.append(obj)
        procs.append((src, subprocess.Popen(
            [hipcc, "--offload-arch=gfx950", "-O1", "-std=c++17", "-fPIC", "-fno-omit-frame-pointer", *san,
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", os.path.join(CSRC, src), "-o", obj],
            stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate()
        assert p.returncode == 0, f"sanitized build of {src} failed:\n{out[-3000:]}"
    lib = str(tmp_path / "liblookat_host_san.so")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *san, "-o", lib, *objs], check=True,
                   stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    code = f"""
import sys
from paper_2601_10155_amd import binding
binding._LIB_PATH = {lib!r}
import pytest
rc = pytest.main(["-x", "-q", "-p", "no:cacheprovider", "tests/test_abi.py"])
assert binding.load_library()._name == {lib!r}
sys.exit(rc)
"""
    out = _run_child(code, runtime)
    assert " passed" in out, out[-2000:]
