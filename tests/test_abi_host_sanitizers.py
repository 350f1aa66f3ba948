"""The host side of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer (host code only: the sanitizers
never see a GPU).  The translation unit with the entry points is compiled with -fsanitize=address,undefined on its
host pass, linked with the ordinary objects of the other sources, and the argument-validation cases of
test_library_abi.py are run against that library in a child process with the sanitizer runtime preloaded: fake
pointers, no GPU needed, every call must be answered on the host and neither sanitizer may report anything."""
import os
import shlex
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BUILD = os.path.join(ROOT, "_build")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CSRC = os.path.join(ROOT, "paper_2510_08431_amd", "csrc")
OTHER_SOURCES = tuple(sorted(f[:-4] for f in os.listdir(CSRC) if f.endswith(".hip") and f != "attn_jvp_api.hip"))

CHILD = r"""
import ctypes, sys
sys.path.insert(0, {root!r})
from paper_2510_08431_amd import binding
binding.LIB_PATH = {lib!r}
lib = binding.load_library()
import tests.test_library_abi as t
t.test_argument_validation_returns_codes_without_launching(lib)
t.test_rmsnorm_argument_validation_returns_codes_without_launching(lib)
t.test_rate_probe_argument_validation_returns_codes_without_launching(lib)
t.test_static_entry_point_rejects_on_the_host(lib)
t.test_version_and_strerror(lib)
t.test_workspace_bytes(lib)
print("sanitized validation cases passed")
"""


def test_validation_cases_under_host_sanitizers(tmp_path):
    if not all(os.path.exists(os.path.join(BUILD, s + ".o")) for s in OTHER_SOURCES):
        import __graft_entry__
        __graft_entry__.build()
    runtime = subprocess.run([HIPCC.replace("bin/hipcc", "llvm/bin/clang"), "-print-file-name=libclang_rt.asan-x86_64.so"],
                             capture_output=True, text=True).stdout.strip()
    if not os.path.exists(runtime):
        pytest.skip("no AddressSanitizer runtime in this toolchain")
    obj = str(tmp_path / "attn_jvp_api_san.o")
    lib = str(tmp_path / "libattn_jvp_san.so")
    # (each command is one line of text, so that a reader, or a tool, sees at a glance that only the HOST pass is
    # sanitized: every -fsanitize= of the compile line follows an -Xarch_host, the link line carries -fno-gpu-sanitize)
    inc, src = os.path.join(ROOT, "include"), os.path.join(ROOT, "paper_2510_08431_amd", "csrc", "attn_jvp_api.hip")
    compile_cmd = f"{HIPCC} --offload-arch=gfx950 -O1 -g -fPIC -std=c++17 -Wno-unused-command-line-argument -Xclang -target-feature -Xclang -packed-fp32-ops -Xarch_host -fsanitize=address -Xarch_host -fsanitize=undefined -Xarch_host -fno-sanitize-recover=undefined -I {inc} -c {src} -o {obj}"
    others = " ".join(os.path.join(BUILD, s + ".o") for s in OTHER_SOURCES)
    link_cmd = f"{HIPCC} --offload-arch=gfx950 -shared -fPIC -fno-gpu-sanitize -fsanitize=address -fsanitize=undefined -shared-libsan -o {lib} {obj} {others}"
    subprocess.run(shlex.split(compile_cmd), check=True, capture_output=True)
    subprocess.run(shlex.split(link_cmd), check=True, capture_output=True)
    env = dict(os.environ, LD_PRELOAD=runtime, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:exitcode=99",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    res = subprocess.run([sys.executable, "-c", CHILD.format(root=ROOT, lib=lib)], env=env, capture_output=True, text=True,
                         timeout=300)
    out = res.stdout + res.stderr
    assert res.returncode == 0, out[-4000:]
    assert "sanitized validation cases passed" in res.stdout
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
