"""AddressSanitizer + UndefinedBehaviorSanitizer builds (CPU only, no GPU code runs):
the naive C oracle on exact-size buffers with ragged shapes, and the host side of the C
ABI (argument checks and workspace planning of every kernel class) compiled with the
sanitizers on the host pass only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DRIVER = os.path.join(ROOT, "tests", "sanitize", "driver.c")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=0",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _run(cmd, **kw):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert p.returncode == 0, f"{' '.join(cmd)}\n{p.stdout[-4000:]}"
    return p.stdout


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-O1", "-std=c11", *SAN, "-o", exe, DRIVER,
          os.path.join(ROOT, "oracle", "forward_naive.c"), "-lm"])
    out = _run([exe], env=ENV)
    assert "oracle clean" in out


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not available")
def test_abi_host_layer_under_asan_ubsan(tmp_path):
    csrc = os.path.join(ROOT, "paper_2603_25385_amd", "csrc")
    host_san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                "-Xarch_host", "-fno-sanitize-recover=all"]
    objs, procs = [], []
    for src in ["api.hip", "prepare.hip", "proj.hip", "decode.hip", "prefill.hip", "probe.hip",
                "factorize.hip", "mx.hip"]:
        obj = str(tmp_path / (src + ".o"))
        extra = ["-mllvm", "-amdgpu-mfma-vgpr-form"] if src == "decode.hip" else []
        procs.append(subprocess.Popen(
            ["hipcc", "--offload-arch=gfx950", "-O1", "-std=c++17", "-fPIC", "-Xclang", "-target-feature",
             "-Xclang", "-packed-fp32-ops", *host_san, *extra, "-c", os.path.join(csrc, src), "-o", obj],
            stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True))
        objs.append(obj)
    for p in procs:
        out, _ = p.communicate()
        assert p.returncode == 0, out[-4000:]
    lib = str(tmp_path / "libglowq_san.so")
    _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
          "-o", lib, *objs])
    exe = str(tmp_path / "abi_san")
    # (the same compiler family as the library: the sanitizer run-times of gcc and clang
    # do not mix in one process)
    clang = shutil.which("amdclang") or "/opt/rocm/llvm/bin/clang"
    _run([clang, "-O1", "-std=c11", *SAN, "-DWITH_GLOWQ_ABI", "-o", exe, DRIVER,
          os.path.join(ROOT, "oracle", "forward_naive.c"), lib, "-lm", f"-Wl,-rpath,{tmp_path}"])
    out = _run([exe], env=ENV)
    assert "ABI host checks clean" in out
