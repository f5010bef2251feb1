"""CPU sanitizer mode (AddressSanitizer + UndefinedBehaviorSanitizer), no GPU needed.

  oracle   mustdrop_ref.c + oracle/sanitize_main.c under gcc sanitizers: every oracle entry point on
           small ragged inputs with exactly sized buffers.
  abi      the HIP library's HOST pass under clang sanitizers (the device pass is compiled as usual)
           + tests/sanitize/abi_errors_main.cpp: the argument checks of every entry point and the
           workspace arithmetic.

    python tests/sanitize/build_and_run.py [oracle|abi|all]

Builds go to _build/sanitize/ (not committed) and are reused while the sources are older.
"""
from __future__ import annotations

import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
OUT = os.path.join(ROOT, "_build", "sanitize")
CSRC = os.path.join(ROOT, "paper_2411_10803_amd", "csrc")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _stale(target, sources):
    return not os.path.exists(target) or any(os.path.getmtime(s) > os.path.getmtime(target) for s in sources)


def _run(exe):
    r = subprocess.run([exe], env=ENV, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    return r.returncode, r.stdout


def oracle():
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "oracle_sanitize")
    src = [os.path.join(ROOT, "oracle", "mustdrop_ref.c"), os.path.join(ROOT, "oracle", "sanitize_main.c")]
    if _stale(exe, src):
        subprocess.check_call(["gcc", "-O1", "-g", "-std=c99", "-Wall", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                               "-static-libasan", "-static-libubsan", *src, "-o", exe, "-lm"])
    return _run(exe)


def abi():
    os.makedirs(OUT, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    exe = os.path.join(OUT, "abi_sanitize")
    units = ["api.hip", "encode.hip", "prefill.hip", "decode.hip"]
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hpp")] + \
              [os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include"))]
    flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-function", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=all"]
    objs, procs = [], []
    for u in units:                                   # the four translation units side by side
        src, obj = os.path.join(CSRC, u), os.path.join(OUT, u.replace(".hip", ".o"))
        objs.append(obj)
        if _stale(obj, [src] + headers):
            procs.append(subprocess.Popen([hipcc, *flags, "-c", src, "-o", obj], stderr=subprocess.PIPE, text=True))
    for p in procs:
        _, err = p.communicate()
        if p.returncode != 0:
            raise RuntimeError(err)
    main = os.path.join(ROOT, "tests", "sanitize", "abi_errors_main.cpp")
    if _stale(exe, objs + [main] + headers):
        subprocess.check_call([hipcc, *flags, *objs, main, "-o", exe], stderr=subprocess.DEVNULL)
    return _run(exe)


if __name__ == "__main__":
    which = sys.argv[1] if len(sys.argv) > 1 else "all"
    rc = 0
    for name, fn in (("oracle", oracle), ("abi", abi)):
        if which in (name, "all"):
            code, out = fn()
            print(out, end="")
            rc |= code
    sys.exit(rc)
