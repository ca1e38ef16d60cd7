"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU involved): the CPU
oracle, and the host-side logic of the HIP library (launch plans, workspace sizes, argument
checks).  The device side is not instrumented (GPU sanitizers are not available here)."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN_ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0:abort_on_error=0",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, "%s\n%s" % (" ".join(cmd), r.stdout[-4000:])
    return r.stdout


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
          "-fno-sanitize-recover=all", "-static-libasan", os.path.join(ROOT, "oracle", "sqp_oracle.c"),
          os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), "-o", exe, "-lm"])
    out = _run([exe], env=dict(SAN_ENV, OMP_NUM_THREADS="2"))
    assert "0 inconsistencies" in out, out


def test_library_host_logic_under_asan_ubsan(tmp_path):
    from paper_2312_03788_amd import build as b
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]
    flags = [f for f in b.FLAGS if f != "-O3"] + ["-O1", "-g"]
    objs = []
    procs = []
    for src in b.SOURCES:
        obj = str(tmp_path / (os.path.splitext(src)[0] + ".o"))
        objs.append(obj)
        procs.append((src, subprocess.Popen(["hipcc"] + flags + san + ["-c", os.path.join(b.CSRC, src), "-o", obj],
                                            stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate()
        assert p.returncode == 0, "%s\n%s" % (src, out[-4000:])
    drv = str(tmp_path / "driver.o")
    _run(["hipcc", "-std=c++17", "-O1", "-g", "-I" + os.path.join(ROOT, "include"), "-fsanitize=address", "-fsanitize=undefined",
          "-fno-gpu-sanitize", "-fno-sanitize-recover=all", "-c", os.path.join(ROOT, "tests", "sanitize", "host_plan_driver.cpp"),
          "-o", drv])
    exe = str(tmp_path / "host_plan_san")
    _run(["hipcc", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", drv] + objs + ["-o", exe])
    out = _run([exe], env=dict(SAN_ENV, ASAN_OPTIONS=SAN_ENV["ASAN_OPTIONS"].replace("detect_leaks=1", "detect_leaks=0")))
    assert "0 inconsistencies" in out, out
