"""Host-side sanitizer targets (no GPU): the CPU oracle and the argument-validation layer of libshiftadd run
under AddressSanitizer and UndefinedBehaviorSanitizer.

* The oracle is compiled whole, with a C driver that calls every one of its functions on small ragged inputs in
  buffers of exactly the documented sizes.
* The library is rebuilt with its HOST code instrumented (the device code is compiled as always; sanitizers do not
  apply to it), and a C driver calls every entry point with arguments the validation must refuse before any launch.
Both programs must finish without a sanitizer report.
"""
import glob
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g"]
ENV = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def run_clean(cmd, ok_line):
    r = subprocess.run(cmd, env=ENV, capture_output=True, text=True, timeout=300)
    report = r.stdout + r.stderr
    assert r.returncode == 0, report[-4000:]
    assert ok_line in r.stdout
    assert "AddressSanitizer" not in report and "runtime error" not in report and "LeakSanitizer" not in report, report[-4000:]


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    subprocess.check_call(["gcc", "-std=c11", "-O1", "-fopenmp", "-ffp-contract=off"] + SAN +
                          [os.path.join(ROOT, "oracle", "shiftadd_oracle.c"), os.path.join(HERE, "oracle_driver.c"),
                           "-o", exe, "-lm"])
    run_clean([exe], "oracle driver ok")


def test_library_argument_validation_under_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    csrc = os.path.join(ROOT, "paper_2306_06446_amd", "csrc")
    host_san = []
    for f in SAN:
        host_san += ["-Xarch_host", f]
    common = [hipcc, "--offload-arch=gfx950", "-O1", "-std=c++17", "-fPIC", "-ffp-contract=off",
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", csrc]
    procs = []
    for src in sorted(glob.glob(os.path.join(csrc, "*.hip"))):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        procs.append((obj, subprocess.Popen(common + host_san + ["-c", src, "-o", obj], stdout=subprocess.PIPE,
                                            stderr=subprocess.STDOUT, text=True)))
    objs = []
    for obj, p in procs:
        out, _ = p.communicate()
        assert p.returncode == 0, out[-3000:]
        objs.append(obj)
    lib = str(tmp_path / "libshiftadd_asan.so")
    link_san = ["-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"]
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + link_san + ["-o", lib] + objs)
    clang = os.path.join(os.path.dirname(os.path.realpath(hipcc)), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang"
    rt_dir = os.path.dirname(subprocess.check_output([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], text=True).strip())
    exe = str(tmp_path / "api_driver")
    subprocess.check_call([clang, "-std=c11", "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined",
                           "-fno-sanitize-recover=undefined", "-shared-libsan", "-I", os.path.join(ROOT, "include"),
                           os.path.join(HERE, "api_driver.c"), lib, "-o", exe, "-lm",
                           "-Wl,-rpath," + str(tmp_path), "-Wl,-rpath," + rt_dir, "-Wl,-rpath,/opt/rocm/lib"])
    # leak checking off here: the HIP runtime the library links keeps allocations of its own until exit
    env = dict(ENV, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=0")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    report = r.stdout + r.stderr
    assert r.returncode == 0, report[-4000:]
    assert "api driver ok" in r.stdout
    assert "AddressSanitizer" not in report and "runtime error" not in report, report[-4000:]
