"""Host code of the library and the C oracle under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

    python tests/sanitize_host.py

Builds, into a temporary directory, (1) libmamba_hip.so with its host side instrumented (argument validation,
plans, workspace layouts, the tree search; the device code is compiled as usual and never runs here) and
(2) oracle/mamba_oracle.c, both with the address and undefined-behaviour sanitizers (host code only) and the shared
sanitizer runtime, then runs the
host tests (tests/test_abi_host.py, tests/test_tree_search.py, tests/test_oracle_pins.py) in a child process that
loads those two libraries instead of the regular ones (MAMBA_HIP_LIB, MAMBA_ORACLE_LIB) with the runtime preloaded.
Exit status 0: tests green and no sanitizer report.  GPU code is not covered (no GPU sanitizer on this pool).
"""
import glob
import os
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANG = os.environ.get("MAMBA_CLANG", "/opt/rocm/lib/llvm/bin/clang")
# host code only: never the device code
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]
LINK_SAN = ["-fsanitize=address,undefined", "-fno-gpu-sanitize", "-shared-libasan"]


def runtime():
    found = sorted(glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    if not found:
        raise SystemExit("no shared AddressSanitizer runtime under /opt/rocm/lib/llvm")
    return found[-1]


def build(tmp):
    from paper_2506_01206_amd import build as hip_build
    csrc = os.path.join(ROOT, "paper_2506_01206_amd", "csrc")
    def one(src):
        obj = os.path.join(tmp, os.path.splitext(src)[0] + ".o")
        r = subprocess.run([HIPCC] + hip_build.FLAGS + ["-g", "-fno-omit-frame-pointer", "-w"] + SAN +
                           ["-c", os.path.join(csrc, src), "-o", obj], capture_output=True, text=True)
        if r.returncode != 0:
            raise SystemExit("hipcc failed for %s:\n%s" % (src, r.stdout + r.stderr))
        return obj
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(one, hip_build.SOURCES))
    hip_lib = os.path.join(tmp, "libmamba_hip_san.so")
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + LINK_SAN + ["-o", hip_lib] + objs)
    oracle_lib = os.path.join(tmp, "libmamba_oracle_san.so")
    subprocess.check_call([CLANG, "-O1", "-g", "-fno-omit-frame-pointer", "-std=c11", "-fPIC", "-shared"] + LINK_SAN +
                          ["-fno-sanitize-recover=undefined", "-ffp-contract=off", "-Wno-unused-command-line-argument",
                           "-o", oracle_lib, os.path.join(ROOT, "oracle", "mamba_oracle.c"), "-lm"])
    return hip_lib, oracle_lib


def main():
    with tempfile.TemporaryDirectory(prefix="mamba_san_") as tmp:
        hip_lib, oracle_lib = build(tmp)
        env = dict(os.environ)
        rt = runtime()
        env["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
        # the interpreter itself is not instrumented: no leak check, no complaint about its allocator use
        env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=66:verify_asan_link_order=0"
        env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:exitcode=67"
        env["MAMBA_HIP_LIB"] = hip_lib
        env["MAMBA_ORACLE_LIB"] = oracle_lib
        tests = [os.path.join(ROOT, "tests", t) for t in ("test_abi_host.py", "test_tree_search.py", "test_oracle_pins.py")]
        r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-s", "-p", "no:cacheprovider"] + tests, env=env, cwd=ROOT,
                           capture_output=True, text=True)
        out = r.stdout + r.stderr
        first = min([out.find(k) for k in ("runtime error:", "ERROR: AddressSanitizer") if k in out] or [max(len(out) - 3000, 0)])
        sys.stdout.write(out[max(first - 300, 0):first + 3000] + "\n")
        report = any(k in r.stdout + r.stderr for k in ("ERROR: AddressSanitizer", "runtime error:", "SUMMARY: UndefinedBehaviorSanitizer"))
        if r.returncode != 0 or report:
            raise SystemExit("sanitizer run failed (status %d, report %s)" % (r.returncode, report))
        print("sanitizer run clean: %s" % ", ".join(os.path.basename(t) for t in tests))


if __name__ == "__main__":
    main()
