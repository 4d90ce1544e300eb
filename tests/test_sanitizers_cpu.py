"""Host-side AddressSanitizer + UndefinedBehaviorSanitizer builds (CPU only, no GPU code runs):
the C oracle on small inputs, and the C ABI's validation / sizing paths of the HIP library with its
host pass instrumented (hipcc: each -fsanitize= directly after -Xarch_host)."""
import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=0", UBSAN_OPTIONS="halt_on_error=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    out = "\n".join(l for l in r.stdout.splitlines() if "is not a recognized feature" not in l)
    return r.returncode, out[-4000:]


def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "oracle_san")
        rc, out = _run(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-omit-frame-pointer",
                        "-std=c11", "-o", exe, os.path.join(SAN, "oracle_driver.c"),
                        os.path.join(ROOT, "oracle", "ns_oracle.c"), "-lm"])
        assert rc == 0, out
        rc, out = _run([exe], env=ENV)
        assert rc == 0 and "oracle sanitizer run ok" in out, out
        assert "ERROR: AddressSanitizer" not in out and "runtime error" not in out, out


def test_c_abi_validation_under_host_sanitizers():
    from paper_2601_12150_amd import build as hip_build
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-omit-frame-pointer"]
    flags = [f for f in hip_build.FLAGS if f != "-O3"] + ["-O1"]
    with tempfile.TemporaryDirectory() as tmp:
        def compile_one(src):
            obj = os.path.join(tmp, src.replace(".hip", ".o"))
            rc, out = _run([hip_build.HIPCC, *flags, *san, "-c", os.path.join(hip_build.CSRC, src), "-o", obj])
            assert rc == 0, out
            return obj
        with ThreadPoolExecutor(max_workers=8) as ex:
            objs = list(ex.map(compile_one, hip_build.SOURCES))
        exe = os.path.join(tmp, "abi_san")
        drv = os.path.join(tmp, "abi_driver.o")
        clang = os.path.join(os.path.dirname(hip_build.HIPCC), "amdclang++")
        rc, out = _run([clang, "-O1", "-g", "-std=c++17", "-fsanitize=address", "-fsanitize=undefined",
                        "-fno-omit-frame-pointer", "-c", os.path.join(SAN, "abi_driver.cpp"), "-o", drv])
        assert rc == 0, out
        rc, out = _run([hip_build.HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined",
                        "-fno-gpu-sanitize", "-o", exe, drv, *objs])
        assert rc == 0, out
        rc, out = _run([exe], env=ENV)
        assert rc == 0 and "C ABI sanitizer run ok" in out, out
        assert "ERROR: AddressSanitizer" not in out and "runtime error" not in out, out
