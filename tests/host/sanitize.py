#!/usr/bin/env python3
"""Host sanitizer pass (AddressSanitizer + UndefinedBehaviorSanitizer), CPU only.

Builds (1) the C oracle with gcc -fsanitize=address,undefined, (2) libsdvg with the sanitizers
applied to its HOST code only (the argument validation of every entry point; device code is left
alone) and (3) the host replay of the attention kernel's index arithmetic, each into a temporary
directory, and runs the `-m "not gpu"` tests that exercise them (or the replay itself) under the
matching sanitizer runtime. Run from the repository root:

    python tests/host/sanitize.py

Exit code 0 = both test runs passed with no sanitizer report.
"""
import os
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)


def run(cmd, env):
    print("+", " ".join(cmd), flush=True)
    return subprocess.run(cmd, cwd=ROOT, env=env).returncode


def main():
    from oracle import build as oracle_build
    from paper_2604_17397_amd import build as sdvg_build
    tmp = tempfile.mkdtemp(prefix="sdvg_san_")
    base = dict(os.environ)
    base["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    base["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    rc = 0

    # (1) the oracle, gcc's runtime
    lib = oracle_build.build(force=True, extra_flags=["-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer"],
                             out=os.path.join(tmp, "libsdvg_oracle_san.so"))
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    env = dict(base, SDVG_ORACLE_LIBRARY=lib, LD_PRELOAD=asan)
    rc |= run([sys.executable, "-m", "pytest", "-x", "-q", "tests/test_oracle_attn.py", "tests/test_oracle_kv_route.py"],
              env)

    # (2) the library's host side, clang's runtime (each -fsanitize= directly after -Xarch_host)
    lib = sdvg_build.build(extra_flags=["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                                        "-Xarch_host", "-fno-omit-frame-pointer", "-shared-libsan"],
                           out=os.path.join(tmp, "libsdvg_san.so"))
    clang = os.path.join(os.path.dirname(os.path.realpath(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"))), "..", "lib",
                         "llvm", "bin", "clang")
    rt = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], stdout=subprocess.PIPE,
                        text=True).stdout.strip()
    env = dict(base, SDVG_LIBRARY=lib, LD_PRELOAD=rt)
    rc |= run([sys.executable, "-m", "pytest", "-x", "-q", "tests/test_abi.py"], env)
    # (3) the host replay of the attention kernel's index arithmetic (same header as the kernel)
    exe = os.path.join(tmp, "attn_index_replay_san")
    rc |= run(["g++", "-O1", "-g", "-std=c++17", "-fopenmp", "-fsanitize=address,undefined", "-fno-omit-frame-pointer",
               "-I", os.path.join(ROOT, "paper_2604_17397_amd", "csrc"),
               os.path.join(ROOT, "tests", "host", "attn_index_replay.cpp"), "-o", exe], base)
    rc |= run([exe], base)
    print("sanitizer pass:", "clean" if rc == 0 else "FAILED")
    return rc


if __name__ == "__main__":
    sys.exit(main())
