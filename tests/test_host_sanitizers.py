"""The library's HOST code under AddressSanitizer and UndefinedBehaviorSanitizer: every source is compiled with
the sanitizers on the host pass only (the device pass is untouched), linked into a library of its own in a
temporary folder, and the host-only C-ABI tests (tests/test_abi.py: plan construction, every validation path,
the coupling tables, all on a context without a device) run against it in a child process."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    from paper_2602_17698_amd import build as b
    if not os.path.exists(b.HIPCC):
        pytest.skip("needs hipcc")
    rt = subprocess.run([b.HIPCC, "-print-file-name=libclang_rt.asan-x86_64.so"], stdout=subprocess.PIPE,
                        text=True).stdout.strip()
    if not os.path.isabs(rt) or not os.path.exists(rt):
        pytest.skip("no shared AddressSanitizer runtime in this toolchain")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-g"]
    flags = [f for f in b.FLAGS if f != "-O3"] + ["-O1"] + san

    def compile_one(src):
        obj = str(tmp_path / src.replace(".hip", ".o"))
        r = subprocess.run([b.HIPCC, *flags, "-c", os.path.join(b.CSRC, src), "-o", obj],
                           stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert r.returncode == 0, r.stdout[-3000:]
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, b.SOURCES))
    lib = str(tmp_path / "libscalebits_hostsan.so")
    subprocess.run([b.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined", "-shared-libsan", "-o", lib, *objs],
                   check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)       # (host runtime only: no device code is instrumented)
    env = dict(os.environ)
    env["SBITS_LIB"] = lib
    # the sanitizer's runtime has to be in the process before the library is opened
    env["LD_PRELOAD"] = (env["LD_PRELOAD"] + ":" if env.get("LD_PRELOAD") else "") + rt
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_abi.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                       text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "passed" in r.stdout and "AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout
