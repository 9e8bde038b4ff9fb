"""The library's host code (argument checks, dispatch, tuning knobs) under AddressSanitizer and
UndefinedBehaviorSanitizer -- CPU only.

api.hip and tuning.hip are rebuilt with the sanitizers on their host side and linked with the objects of
the regular build (the kernels are not touched); the host-side ABI tests then run again in a child process
against that library, with the sanitizer runtime preloaded after whatever the environment already preloads.
A read or write outside an argument array, a bad shift or a signed overflow in a size computation ends
the child with a report."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2604_12782_amd", "csrc")


def test_host_code_under_asan_and_ubsan(tmp_path):
    sys.path.insert(0, ROOT)
    from paper_2604_12782_amd import build as b
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    rts = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not os.path.exists(hipcc) or not rts:
        pytest.skip("hipcc or its sanitizer runtime is not installed")
    plain = [os.path.join(CSRC, s.replace(".hip", ".o")) for s in b.SOURCES if s not in ("api.hip", "tuning.hip")]
    if not all(os.path.exists(o) for o in plain):
        pytest.skip("the regular build's objects are not there (run __graft_entry__.build() first)")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined"]
    objs = []
    for s in ("api.hip", "tuning.hip"):
        o = str(tmp_path / s.replace(".hip", ".o"))
        flags = [f for f in b.FLAGS if f != "-O3"]
        subprocess.run([hipcc, *flags, "-O1", "-g", *san, "-I", os.path.join(ROOT, "include"), "-c",
                        os.path.join(CSRC, s), "-o", o], check=True, capture_output=True, timeout=600)
        objs.append(o)
    lib = str(tmp_path / "libosc_hostsan.so")
    # (host sanitizers only: the device code objects are those of the regular build)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-shared-libsan"]
    subprocess.run([*link, *objs, *plain, "-o", lib], check=True, capture_output=True, timeout=600)
    env = dict(os.environ)
    env["LD_PRELOAD"] = " ".join(x for x in (env.get("LD_PRELOAD", ""), rts[0]) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    runner = ("import sys, pytest\n"
              "import paper_2604_12782_amd.binding as b\n"
              f"b._LIB_PATH = {lib!r}\n"
              "b.lib()\n"
              "sys.exit(pytest.main(['-x', '-q', '-p', 'no:cacheprovider', 'tests/test_abi_host.py']))\n")
    p = subprocess.run([sys.executable, "-c", runner], cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    out = p.stdout + p.stderr
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert p.returncode == 0, out[-4000:]
    assert " passed" in out
