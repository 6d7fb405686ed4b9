"""CPU-only sanitizer builds (AddressSanitizer + UndefinedBehaviorSanitizer): the oracle as a whole, driven over
ragged and strided inputs, and the host side of the C-ABI library, driven through calls that its argument
validation must refuse before anything is launched.  GPU code cannot be sanitized on this machine; these builds
cover everything that runs on the host."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    subprocess.check_call(["gcc", "-O1", "-g", "-ffp-contract=off", "-fopenmp", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-static-libasan", "-o", exe,
                           os.path.join(HERE, "oracle_driver.c"), os.path.join(ROOT, "oracle", "brq_oracle.c"), "-lm"])
    r = subprocess.run([exe], env=ENV, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert r.returncode == 0 and "oracle sanitizer driver ok" in r.stdout, r.stdout[-3000:]


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_host_api_validation_under_asan_and_ubsan(tmp_path):
    """The library's host code (argument validation, launch set-up) compiled with the sanitizers on the host pass
    only; the driver makes calls that must all be refused on the host, so no GPU is touched."""
    csrc = os.path.join(ROOT, "paper_2511_04214_amd", "csrc")
    from paper_2511_04214_amd.build import SOURCES, FLAGS
    objs = []
    for src in SOURCES:
        obj = str(tmp_path / src.replace(".hip", ".o"))
        # host pass sanitized; the device pass is compiled as always (each -fsanitize= directly after -Xarch_host)
        cmd = ["hipcc"] + [f for f in FLAGS if f != "-O3"] + ["-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
                                                               "-fsanitize=undefined", "-c", os.path.join(csrc, src), "-o", obj]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert r.returncode == 0, r.stdout[-3000:]
        objs.append(obj)
    exe = str(tmp_path / "host_api_driver")
    drv = str(tmp_path / "driver.o")
    subprocess.check_call(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-I",
                           os.path.join(ROOT, "include"), "-c", os.path.join(HERE, "host_api_driver.c"), "-o", drv])
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize", "-o", exe, drv] + objs,
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-3000:]
    r = subprocess.run([exe], env=ENV, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert r.returncode == 0 and "host api sanitizer driver ok" in r.stdout, r.stdout[-3000:]
