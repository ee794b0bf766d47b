"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer, without a GPU.

hipcc compiles the host side of every source file alone (--offload-host-only: seconds, no device code), with the
sanitizers on the host compiler only.  The objects still refer to the device code bundle of their file; placeholder
symbols stand in for those (nothing is ever launched: the driver program only makes calls that return from the
argument checks, the size arithmetic, the naming calls or the planning code).  Device code is never built with a
sanitizer here."""
import glob
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1909_09927_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
       "-Xarch_host", "-fno-sanitize-recover=undefined"]


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="no hipcc")
def test_host_paths_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    flags = ["--offload-arch=gfx950", "--offload-host-only", "-O1", "-g", "-std=c++17", "-fPIC",
             "-I", os.path.join(ROOT, "include"), "-I", CSRC, *SAN]
    procs = []
    for src in sorted(glob.glob(os.path.join(CSRC, "*.hip"))):
        obj = tmp_path / (os.path.basename(src) + ".o")
        procs.append((src, obj, subprocess.Popen([HIPCC, *flags, "-c", src, "-o", str(obj)],
                                                 stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    objs = []
    for src, obj, pr in procs:
        out, _ = pr.communicate()
        assert pr.returncode == 0, f"{src}:\n{out}"
        objs.append(str(obj))
    # one placeholder per device code bundle the host objects refer to
    undefined = subprocess.run(["nm", "-u", *objs], check=True, capture_output=True, text=True).stdout
    bundles = sorted(set(re.findall(r"__hip_fatbin_[0-9a-f]+", undefined)))
    stubs = tmp_path / "bundles.cpp"
    stubs.write_text("".join(f'extern "C" {{ __attribute__((aligned(4096))) char {b}[4096] = {{0}}; }}\n' for b in bundles))
    exe = tmp_path / "host_sanitizer_driver"
    link = subprocess.run([HIPCC, "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", *objs,
                           "-x", "c++", "-std=c++17", "-g", os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"),
                           str(stubs), "-I", os.path.join(ROOT, "include"), "-o", str(exe)],
                          stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert link.returncode == 0, link.stdout
    env = dict(os.environ)
    # leaks of the HIP runtime's own start-up are not this library's; the link order check trips over preloads
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    for k in ("SCONV_VARIANT", "SCONV_TAP_GEOM", "SCONV_TAP_SPLIT", "SCONV_QUAD_GEOM", "SCONV_QUAD_SPLIT"):
        env.pop(k, None)
    run = subprocess.run([str(exe)], env=env, capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert run.stdout.strip().endswith("ok")
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr
