#!/usr/bin/env python3
"""CPU-side sanitizer run: the host code of libkvs and the C oracle under AddressSanitizer and
UndefinedBehaviorSanitizer, exercised by the tests that need no GPU.

    python tests/sanitize_cpu.py            (from the repository root; a minute or two)

Builds, under _build/sanitize/ (not tracked):
  - libkvs.so with hipcc: the host side of every source is instrumented (each -fsanitize= behind
    -Xarch_host), the gfx950 device code is compiled as usual and never runs here;
  - libkvs_oracle.so with the same clang, without OpenMP (one runtime for both libraries),
and runs `pytest -m "not gpu"` with the two libraries in place of the regular ones (environment
variables KVS_LIBRARY and KVS_ORACLE_LIBRARY, which the binding and the oracle's loader honour)
and clang's sanitizer runtime preloaded into the interpreter.  Leak checking is off: the
interpreter itself never frees most of what it allocates.
"""
import glob
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OUT = os.path.join(ROOT, "_build", "sanitize")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANG = os.environ.get("KVS_CLANG", "/opt/rocm/lib/llvm/bin/clang")
SAN = ["address", "undefined"]


def main() -> int:
    sys.path.insert(0, ROOT)
    from paper_2410_18517_amd import build as kvs_build
    os.makedirs(OUT, exist_ok=True)
    host_san = []
    for s in SAN:
        host_san += ["-Xarch_host", f"-fsanitize={s}"]
    objs = []
    for src in kvs_build.sources():
        obj = os.path.join(OUT, os.path.basename(src) + ".o")
        cmd = [HIPCC] + kvs_build.FLAGS + ["-g", "-fno-omit-frame-pointer"] + host_san + ["-x", "hip", "-c", src, "-o", obj]
        print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        objs.append(obj)
    lib = os.path.join(OUT, "libkvs.so")
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-shared-libsan"] + [f"-fsanitize={s}" for s in SAN] +
                   ["-o", lib] + objs, check=True)
    oracle = os.path.join(OUT, "libkvs_oracle.so")
    subprocess.run([CLANG, "-O1", "-g", "-fno-omit-frame-pointer", "-std=c11", "-fPIC", "-shared", "-shared-libsan", "-Wall", "-Wextra"] +
                   [f"-fsanitize={s}" for s in SAN] + ["-o", oracle, os.path.join(ROOT, "oracle", "kvs_oracle.c"), "-lm"], check=True)
    runtime = subprocess.run([CLANG, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True, check=True).stdout.strip()
    if not os.path.exists(runtime):
        found = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
        if not found:
            print("clang's AddressSanitizer runtime was not found", file=sys.stderr)
            return 2
        runtime = found[0]
    env = dict(os.environ)
    env.update({"KVS_LIBRARY": lib, "KVS_ORACLE_LIBRARY": oracle, "LD_PRELOAD": runtime,
                "ASAN_OPTIONS": "detect_leaks=0:abort_on_error=1:halt_on_error=1",
                "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1"})
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests"), "-x", "-q", "-m", "not gpu",
                           "-p", "no:cacheprovider"], env=env, cwd=ROOT).returncode


if __name__ == "__main__":
    sys.exit(main())
