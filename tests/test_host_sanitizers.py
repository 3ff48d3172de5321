"""The host-side validation layer of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer,
on the CPU: energon_api.hip is compiled once more with both sanitizers on its host pass (the device
pass is untouched), linked with the ordinary objects of the other sources into a second library, and
a small C driver (tests/host_driver/abi_driver.c, built with the same sanitizers) calls every entry
point with arguments that must be answered on the host.  Any out-of-bounds read of a host array, or
undefined arithmetic on the sizes, aborts the driver."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
       "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]


@pytest.mark.timeout(600)
def test_validation_layer_is_clean_under_asan_and_ubsan(tmp_path):
    from paper_2209_02341_amd import build as b
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc is not installed")
    objs = [os.path.join(b.OBJ_DIR, s.replace(".hip", ".o")) for s in b.SOURCES if s != "energon_api.hip"]
    if not all(os.path.exists(o) for o in objs):
        b.build()
    api_obj = str(tmp_path / "energon_api_san.o")
    lib = str(tmp_path / "libenergon_san.so")
    exe = str(tmp_path / "abi_driver")
    run = lambda cmd, **kw: subprocess.run(cmd, capture_output=True, text=True, **kw)
    r = run([HIPCC, *b.FLAGS, "-g", *SAN, "-c", os.path.join(b.CSRC, "energon_api.hip"), "-o", api_obj])
    assert r.returncode == 0, r.stderr[-3000:]
    r = run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
             "-o", lib, api_obj, *objs])
    assert r.returncode == 0, r.stderr[-3000:]
    r = run([HIPCC, "-x", "c", "-g", "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined",
             "-fno-gpu-sanitize", os.path.join(ROOT, "tests", "host_driver", "abi_driver.c"), "-x", "none", lib, "-o", exe,
             "-Wl,-rpath," + str(tmp_path)])
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = run([exe], env=env, timeout=120)
    assert r.returncode == 0 and "abi driver ok" in r.stdout, (r.stdout[-2000:], r.stderr[-4000:])
