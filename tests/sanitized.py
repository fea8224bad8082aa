#!/usr/bin/env python3
"""CPU-only sanitizer run: AddressSanitizer + UndefinedBehaviorSanitizer over the checker and over the
host half of the library.  Not collected by pytest; run it by hand:

    python tests/sanitized.py            # both passes
    python tests/sanitized.py oracle     # pass 1 only
    python tests/sanitized.py host       # pass 2 only

Pass 1 builds oracle/absb_oracle.c with gcc -fsanitize=address,undefined and runs every `-m "not gpu"`
test against it.  Pass 2 builds the library with the sanitizers on its host code (hipcc -Xarch_host;
the device code is untouched) and runs the host ABI tests (argument validation, planning, workspace
carving, the block-size rule) against that build.  The two passes use different sanitizer runtimes
(gcc's and clang's), which cannot share a process; each is preloaded into its own pytest run, in
front of whatever the environment already preloads.  Exit status 0 = both suites green and no
sanitizer report.
"""
import glob
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def _preload(env, runtime):
    env = dict(env)
    env["LD_PRELOAD"] = runtime + ((" " + env["LD_PRELOAD"]) if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"      # Python itself leaks by design
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    return env


def oracle_pass():
    src = os.path.join(ROOT, "oracle", "absb_oracle.c")
    lib = os.path.join(ROOT, "oracle", "liboracle_san.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                           "-fno-fast-math", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-Wall", "-Wextra", src, "-o", lib, "-lm"])
    runtime = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    env = _preload(os.environ, runtime)
    env["ABSB_ORACLE_LIB"] = lib
    return subprocess.call([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests"), "-x", "-q", "-m", "not gpu",
                            "-p", "no:cacheprovider"], env=env, cwd=ROOT)


def host_pass():
    from paper_2605_12110_amd.build import build_sanitized, _hipcc
    lib = build_sanitized()
    clang = os.path.join(os.path.dirname(os.path.realpath(_hipcc())), "..", "llvm", "bin", "clang")
    runtime = subprocess.check_output([clang if os.path.exists(clang) else "/opt/rocm/llvm/bin/clang",
                                       "-print-file-name=libclang_rt.asan-x86_64.so"], text=True).strip()
    if not os.path.isabs(runtime):
        hits = glob.glob("/opt/rocm/**/libclang_rt.asan-x86_64.so", recursive=True)
        runtime = hits[0]
    env = _preload(os.environ, runtime)
    env["ABSB_LIB"] = lib
    return subprocess.call([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_abi_host.py"), "-x", "-q",
                            "-m", "not gpu", "-p", "no:cacheprovider"], env=env, cwd=ROOT)


if __name__ == "__main__":
    which = sys.argv[1] if len(sys.argv) > 1 else "both"
    rc = 0
    if which in ("both", "oracle"):
        rc |= oracle_pass()
    if which in ("both", "host"):
        rc |= host_pass()
    print("sanitized run:", "clean" if rc == 0 else f"FAILED ({rc})")
    sys.exit(rc)
