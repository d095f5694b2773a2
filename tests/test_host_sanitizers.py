"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer: kvcar_host.hip is compiled once more
with the sanitizers on its host side only (device code is untouched), linked with the kernels' objects and a C driver
(tests/host_sanitize_driver.c) that walks the host logic of the C ABI - contexts, reuse maps, autoencoder descriptors,
plans, sizes, every argument error that must come back before a launch - with fake device pointers.  No kernel is
launched and no GPU is needed; a finding of either sanitizer aborts the driver."""
import os
import shutil
import subprocess

import pytest

from paper_2512_06727_amd import build as B

HERE = os.path.dirname(os.path.abspath(__file__))
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
       "-Xarch_host", "-fno-omit-frame-pointer"]


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    hipcc = B.hipcc()
    bdir = os.path.join(B.PKG, "_build")
    others = [s for s in B.SOURCES if s != "kvcar_host.hip"]
    objs = [os.path.join(bdir, s.replace(".hip", ".o")) for s in others]
    if not all(os.path.exists(o) for o in objs):
        B.build()                                     # the kernels' objects (compiled as always, without sanitizers)
    flags = [f for f in B.HIP_FLAGS if f != "-O3"] + ["-O1", "-g"]
    host_o = str(tmp_path / "kvcar_host_san.o")
    r = subprocess.run([hipcc, *flags, *SAN, "-I", os.path.join(B.ROOT, "include"), "-I", B.CSRC, "-c", os.path.join(B.CSRC, "kvcar_host.hip"), "-o", host_o],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout
    drv_o = str(tmp_path / "driver.o")
    cc = shutil.which("amdclang") or "/opt/rocm/llvm/bin/clang"
    r = subprocess.run([cc, "-O1", "-g", "-fsanitize=address,undefined", "-fno-gpu-sanitize", "-fno-sanitize-recover=undefined", "-I", os.path.join(B.ROOT, "include"),
                        "-c", os.path.join(HERE, "host_sanitize_driver.c"), "-o", drv_o], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout
    exe = str(tmp_path / "host_sanitize_driver")
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize", "-o", exe, drv_o, host_o, *objs],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout
    env = dict(os.environ)
    # the HIP runtime keeps its own allocations until exit: leak checking would report those, not the library's
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    # the driver hands fake device pointers to the library: make sure nothing could ever be launched with them
    env["HIP_VISIBLE_DEVICES"] = ""
    env["ROCR_VISIBLE_DEVICES"] = ""
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "host sanitize driver: ok" in r.stdout, r.stdout[-4000:]
