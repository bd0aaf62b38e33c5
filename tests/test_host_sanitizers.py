"""AddressSanitizer + UndefinedBehaviorSanitizer over the host-side code: the library's host-only entry points
(size rules, Eq. 5-7, argument checks) and the whole CPU oracle, on small odd-sized inputs.  CPU only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIP_INCLUDE = "/opt/rocm/include"


CLANG = "/opt/rocm/lib/llvm/bin/clang"
HIPCC = "/opt/rocm/bin/hipcc"


@pytest.mark.skipif(not (os.path.exists(CLANG) and os.path.exists(HIPCC)), reason="needs the ROCm clang and hipcc")
def test_host_code_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
    inc = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2503_20354_amd", "csrc")]
    oracle_o, host_o, test_o, stubs_o = (str(tmp_path / n) for n in ("oracle.o", "host.o", "test.o", "stubs.o"))
    subprocess.run([CLANG, "-std=c11", "-ffp-contract=off", "-c", os.path.join(ROOT, "oracle", "surgeon_oracle.c"),
                    "-o", oracle_o] + san, check=True)
    # surgeon_host.cpp holds no kernel, but its headers are HIP headers: host pass of hipcc, sanitizers on the host only
    host_san = []
    for f in san:
        host_san += ["-Xarch_host", f]
    subprocess.run([HIPCC, "--offload-arch=gfx950", "--cuda-host-only", "-std=c++17", "-ffp-contract=off", "-x", "hip", "-c",
                    os.path.join(ROOT, "paper_2503_20354_amd", "csrc", "surgeon_host.cpp"), "-o", host_o] + inc + host_san,
                   check=True)
    for src, obj in ((os.path.join(ROOT, "tests", "native", "host_sanitize.cpp"), test_o),
                     (os.path.join(ROOT, "tests", "native", "host_stubs.cpp"), stubs_o)):
        subprocess.run([CLANG + "++", "-std=c++17", "-D__HIP_PLATFORM_AMD__", "-I", HIP_INCLUDE, "-c", src, "-o", obj] + inc + san,
                       check=True)
    subprocess.run([CLANG + "++", test_o, host_o, stubs_o, oracle_o, "-o", exe, "-lm"] + san, check=True)
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host sanitizer run ok" in r.stdout
