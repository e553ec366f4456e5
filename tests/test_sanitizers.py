"""Host-side sanitizer builds (AddressSanitizer + UndefinedBehaviorSanitizer; the GPU side cannot be
sanitized on the test machines): the oracle's C sources exercised on exactly sized heap buffers, and the C
ABI's argument checks (the host code of spin_api.hip) called with everything they must refuse.  Both are
separate programs, so the sanitizer runtime never has to be loaded into the Python process."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
FLAGS = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def run(exe):
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300, env=ENV)
    assert res.returncode == 0 and "run ok" in res.stdout and "runtime error" not in res.stdout \
        and "AddressSanitizer" not in res.stdout, res.stdout[-4000:]


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.run(["gcc", "-std=c11", "-Wall"] + FLAGS + ["-o", exe, os.path.join(SAN, "oracle_san.c"),
                    os.path.join(ROOT, "oracle", "spin_oracle.c"), os.path.join(ROOT, "oracle", "spin_oracle128.c"),
                    "-lm", "-Wno-unknown-pragmas"], check=True)
    run(exe)


def test_abi_argument_checks_under_sanitizers(tmp_path):
    from paper_2402_02320_amd import build
    hipcc = build.hipcc()
    if shutil.which(hipcc) is None and not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    host_san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                "-Xarch_host", "-fno-sanitize-recover=all"]
    obj_dir = os.path.join(os.path.dirname(build.LIB), "_build")
    others = [os.path.join(obj_dir, s.replace(".hip", ".o")) for s in build.SOURCES if s != "spin_api.hip"]
    if not all(os.path.exists(o) for o in others):
        build.build()
    api_o, drv_o, exe = (str(tmp_path / n) for n in ("spin_api_san.o", "abi_san.o", "abi_san"))
    quiet = dict(stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    res = subprocess.run([hipcc] + build.COMPILE_FLAGS + ["-O1", "-g"] + host_san +
                         ["-c", os.path.join(build.CSRC, "spin_api.hip"), "-o", api_o], **quiet)
    assert res.returncode == 0, res.stdout[-3000:]
    subprocess.run(["gcc", "-std=c99", "-Wall"] + FLAGS + ["-I", os.path.join(ROOT, "include"), "-c",
                    os.path.join(SAN, "abi_san.c"), "-o", drv_o], check=True)
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-Wno-unused-command-line-argument"] + host_san[:4] +
                         [drv_o, api_o] + others + ["-o", exe], **quiet)
    assert res.returncode == 0, res.stdout[-3000:]
    run(exe)
