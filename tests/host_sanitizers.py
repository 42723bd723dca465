"""Host-side sanitizer run (CPU only, no GPU code is executed):

    python tests/host_sanitizers.py

1. the C oracle built with gcc -fsanitize=address,undefined, under the whole oracle pin suite (tests/test_oracle_pins.py);
2. libkla.so with the host code of the C ABI (csrc/kla_api.hip: validation, workspace plans, dispatch) built with
   clang's AddressSanitizer and UndefinedBehaviorSanitizer (device code is not instrumented), under tests/test_abi.py
   and the CPU part of tests/test_zz_no_alloc.py, i.e. every refusal path and every workspace query.

Python itself is not instrumented, so the sanitizer runtime is preloaded into the test process (leak checking off:
the interpreter's own allocations would drown it).  Any report makes the sanitizer abort the test run.
Exit status 0 = both suites passed with no report.  `pytest tests/test_host_sanitizers.py` runs this when
KLA_RUN_SANITIZERS=1 is set."""
import glob
import os
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def run(cmd, **kw):
    print("+", " ".join(cmd), flush=True)
    subprocess.check_call(cmd, **kw)


def main() -> int:
    from paper_2605_08587_amd import build as kbuild
    tmp = tempfile.mkdtemp(prefix="kla_sanitize_")
    env0 = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1:halt_on_error=1",
                UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    pre = env0.get("LD_PRELOAD", "")

    # ---- 1. the oracle
    olib = os.path.join(tmp, "libkla_oracle_san.so")
    run(["gcc", "-O1", "-g", "-std=c99", "-fPIC", "-shared", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         "-o", olib, os.path.join(ROOT, "oracle", "kla_oracle.c"), "-lm"])
    gcc_asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    env = dict(env0, KLA_ORACLE_LIBRARY=olib, LD_PRELOAD=gcc_asan + (":" + pre if pre else ""))
    run([sys.executable, "-m", "pytest", "-x", "-q", os.path.join(ROOT, "tests", "test_oracle_pins.py")], env=env, cwd=ROOT)

    # ---- 2. the host side of the C ABI
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in kbuild.FLAGS if f != "-shared"]
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all",
           "-Xarch_host", "-g"]
    objs = []
    procs = []
    for src in kbuild.SOURCES:
        obj = os.path.join(tmp, src + ".o")
        cmd = [hipcc, *flags, *(san if src == "kla_api.hip" else []), "-c", os.path.join(kbuild.CSRC, src), "-o", obj]
        print("+", " ".join(cmd), flush=True)
        procs.append(subprocess.Popen(cmd, stderr=subprocess.DEVNULL))
        objs.append(obj)
    for p in procs:
        if p.wait() != 0:
            raise SystemExit("compile failed")
    klib = os.path.join(tmp, "libkla_san.so")
    # host-only link of the sanitizer runtimes (no -Xarch_ option on this line, device sanitizers explicitly off)
    run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined",
         "-shared-libsan", "-o", klib, *objs])
    rt = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not rt:
        raise SystemExit("clang's shared AddressSanitizer runtime not found")
    env = dict(env0, KLA_LIBRARY=klib, LD_PRELOAD=rt[0] + (":" + pre if pre else ""))
    run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", os.path.join(ROOT, "tests", "test_abi.py"),
         os.path.join(ROOT, "tests", "test_zz_no_alloc.py")], env=env, cwd=ROOT)
    print("host sanitizers: both suites passed, no report")
    return 0


if __name__ == "__main__":
    sys.exit(main())
