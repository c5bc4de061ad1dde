"""Build librt_hip.so (hipcc, gfx950) in-tree next to this file."""
from __future__ import annotations

import glob
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "librt_hip.so")
INCLUDE = os.path.join(os.path.dirname(_HERE), "include")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # MFMA results go to ordinary VGPRs: the softmax arithmetic reads them directly (no v_accvgpr copies)
    "-mllvm", "-amdgpu-mfma-vgpr-form",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(INCLUDE, "*.h"))
    return any(os.path.getmtime(p) > t for p in deps)


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    return r.returncode, out


def build_hip(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source (one hipcc process per file, side by side) and link them into one shared library.
    Cross-compiles without a GPU."""
    if not force and not is_stale():
        return LIB
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(_HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    srcs = sources()
    objs = [os.path.join(objdir, os.path.basename(p)[:-4] + ".%d.o" % os.getpid()) for p in srcs]
    jobs = [[hipcc] + flags + ["-I", INCLUDE, "-c", src, "-o", obj] for src, obj in zip(srcs, objs)]
    try:
        with ThreadPoolExecutor(max_workers=min(len(jobs), int(os.environ.get("MAX_JOBS", "8")))) as pool:
            results = list(pool.map(_run, jobs))
        log = "\n".join(out for _, out in results if out.strip())
        if any(rc != 0 for rc, _ in results):
            raise RuntimeError("hipcc failed:\n" + log)
        tmp = LIB + ".tmp%d" % os.getpid()
        rc, out = _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", tmp])
        if rc != 0:
            if os.path.exists(tmp):
                os.remove(tmp)
            raise RuntimeError("hipcc link failed:\n" + out)
        if verbose and (log + out).strip():
            print(log + out)
        os.replace(tmp, LIB)
    finally:
        for o in objs:
            if os.path.exists(o):
                os.remove(o)
    return LIB


if __name__ == "__main__":
    print(build_hip(True, verbose=True))
