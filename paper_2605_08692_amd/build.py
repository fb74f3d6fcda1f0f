"""Builds libaaac.so (hipcc, gfx950 only) next to this file.

    python -m paper_2605_08692_amd.build            # compile every source, link
    python -m paper_2605_08692_amd.build --changed  # recompile only sources older objects do not cover

The sources are compiled one hipcc process each, side by side, into _build/ and then linked.
"""
import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libaaac.so")
SOURCES = ["aaac_api.hip", "aaac_kernels.hip", "aaac_lloyd.hip", "aaac_small.hip", "aaac_quantile.hip", "aaac_gemv.hip", "aaac_gemm.hip"]

# -ffp-contract=off: every fp32 operation that decides a code or a selection bit
# must stay a single IEEE operation.  Packed fp32 instructions are switched off.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-munsafe-fp-atomics",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]
NOISE = "packed-fp32-ops"  # the host pass does not know the target feature and says so


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if NOISE not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)


def _headers_mtime():
    files = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    files.append(os.path.join(ROOT, "include", "aaac.h"))
    return max(os.path.getmtime(f) for f in files)


def build(verbose=False, only_changed=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    base = [hipcc] + FLAGS + ["-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
    newest_header = _headers_mtime()
    jobs = []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ, s + ".o")
        fresh = os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header)
        if not (only_changed and fresh):
            jobs.append(base + ["-c", src, "-o", obj])
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as pool:
        for f in [pool.submit(_run, cmd, verbose) for cmd in jobs]:
            f.result()
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + [os.path.join(OBJ, s + ".o") for s in SOURCES] +
         ["-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, only_changed="--changed" in sys.argv[1:]))
