"""AddressSanitizer + UndefinedBehaviorSanitizer over the C oracle and over the host side of the
HIP library (index builders, size arithmetic, argument checks).  Both are CPU builds: the drivers in
tests/sanitize/ size every array exactly, call every entry point, and any report (or any return code
other than the documented one) fails the test.  Device code is not instrumented."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g"]
# hipcc: the host pass only (device code is never instrumented)
HOST_SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
            "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="4")


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-6000:]}"
    return r.stdout


def _sanitizers_usable(tmp_path):
    """False where the toolchain has no sanitizer runtime (the check itself must not fail the suite)."""
    src = tmp_path / "probe.c"
    src.write_text("int main(void) { return 0; }\n")
    exe = tmp_path / "probe"
    r = subprocess.run(["gcc", *SAN, "-o", str(exe), str(src)], capture_output=True)
    return r.returncode == 0 and subprocess.run([str(exe)], env=ENV).returncode == 0


def test_oracle_under_asan_ubsan(tmp_path):
    if not _sanitizers_usable(tmp_path):
        pytest.skip("no sanitizer runtime for gcc here")
    exe = str(tmp_path / "oracle_driver")
    _run(["gcc", "-O1", *SAN, "-fopenmp", "-o", exe, os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
          os.path.join(ROOT, "oracle", "lmk_ref.c"), "-lm"])
    out = _run([exe], env=ENV)
    assert "oracle driver done" in out and "runtime error" not in out and "AddressSanitizer" not in out, out[-4000:]


def test_library_host_code_under_asan_ubsan(tmp_path):
    from paper_2503_21364_amd import build as hip_build
    if not _sanitizers_usable(tmp_path):
        pytest.skip("no sanitizer runtime for gcc here")
    cc = hip_build.hipcc()
    host_units = ("api.hip", "index.hip")       # every extern "C" entry point and all host-only code
    objs = []
    for unit in host_units:
        obj = str(tmp_path / unit.replace(".hip", ".o"))
        _run([cc, *hip_build.COMMON, *hip_build.UNITS[unit], *HOST_SAN, "-c", os.path.join(hip_build.CSRC, unit), "-o", obj])
        objs.append(obj)
    # the kernels' translation units as the library build left them (their host side is launch code only)
    rest = [os.path.join(hip_build.OBJDIR, u.replace(".hip", ".o")) for u in hip_build.UNITS if u not in host_units]
    if not all(os.path.exists(o) for o in rest):
        hip_build.build()
    drv = str(tmp_path / "host_driver.o")
    _run(["gcc", "-O1", *SAN, "-I", hip_build.INCLUDE, "-c", os.path.join(ROOT, "tests", "sanitize", "host_driver.c"), "-o", drv])
    exe = str(tmp_path / "host_driver")
    _run([cc, f"--offload-arch={hip_build.ARCH}", "-fsanitize=address,undefined", "-fno-gpu-sanitize", "-o", exe, drv, *objs, *rest,
          "-Wl,-rpath,/opt/rocm/lib"])
    # leaks are not checked here: the HIP runtime keeps its own allocations until exit
    out = _run([exe], env=dict(ENV, ASAN_OPTIONS="detect_leaks=0"))
    assert "host driver done" in out and "runtime error" not in out and "AddressSanitizer" not in out, out[-4000:]
    shutil.rmtree(tmp_path, ignore_errors=True)
