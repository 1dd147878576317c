"""Host sanitizer job (CPU only): the oracle's C code, and the host side of the C ABI, built with
-fsanitize=address,undefined and driven by small C programs (tests/sanitize/).  The ABI driver covers what a call does
before it enqueues anything -- argument checks, descriptor checks, the workspace planner under both rules -- so no GPU
is needed; device code is not instrumented (hipcc takes the sanitizer flags for the host pass only)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]


def run(cmd, timeout=300, leaks=None):
    """Runs cmd; leaks = True / False runs it as a sanitized program with leak detection on / off."""
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=timeout, env=_sanitizer_env(leaks))
    if res.returncode != 0:
        pytest.fail("%s\n%s\n%s" % (" ".join(cmd), res.stdout[-4000:], res.stderr[-4000:]), pytrace=False)
    return res


def _sanitizer_env(leaks):
    if leaks is None:
        return None
    # the test harness may preload a library of its own in front of the sanitizer runtime; that order is harmless here
    return dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=%d" % int(leaks), UBSAN_OPTIONS="print_stacktrace=1")


def test_oracle_c_code_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    run(["gcc", "-std=c11", "-O1"] + SAN + ["-I" + os.path.join(ROOT, "oracle"), "-o", exe,
         os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), os.path.join(ROOT, "oracle", "relax_oracle.c"), "-lm"])
    res = run([exe], leaks=True)
    assert "oracle driver ok" in res.stdout and "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr


def test_abi_host_code_under_address_and_undefined_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    from paper_2311_02103_amd import build as b
    objs = {s: os.path.join(b.OBJ, s[:-4] + ".o") for s in b.sources()}
    if not all(os.path.exists(o) for o in objs.values()):
        b.build(verbose=False)                                   # the other translation units come from the normal build
    # api.hip holds every argument check and the planner: its host pass is the one that gets instrumented
    api_o = str(tmp_path / "api_san.o")
    host_san = []
    for f in SAN[:2]:
        host_san += ["-Xarch_host", f]
    run([hipcc] + b.FLAGS + host_san + ["-Xarch_host", "-fno-omit-frame-pointer", "-c", os.path.join(b.CSRC, "api.hip"), "-o", api_o], timeout=900)
    lib = str(tmp_path / "librelax_san.so")
    others = [o for s, o in objs.items() if s != "api.hip"]
    run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address,undefined", "-fno-gpu-sanitize", "-o", lib, api_o] + others, timeout=600)
    exe = str(tmp_path / "abi_san")
    cc = shutil.which("clang") or os.path.join(os.path.dirname(hipcc), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(cc):
        cc = "/opt/rocm/lib/llvm/bin/clang"
    # same compiler family as the library, so that driver and library share one sanitizer runtime
    run([cc, "-std=c11", "-O1"] + SAN + ["-I" + os.path.join(ROOT, "include"), "-o", exe, os.path.join(ROOT, "tests", "sanitize", "abi_driver.c"),
         lib, "-Wl,-rpath," + str(tmp_path), "-Wl,-rpath,/opt/rocm/lib"], timeout=300)
    # the HIP runtime the library links keeps allocations for the life of the process: leak checking is for the oracle
    res = run([exe], leaks=False)
    assert "abi driver ok" in res.stdout and "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr
