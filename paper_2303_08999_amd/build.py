"""Builds libsrdict.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsrdict.so")
SOURCES = ["sr_api.hip", "sr_generic.hip", "sr_list.hip", "sr_mfma.hip", "sr_mfma_k3.hip", "sr_mfma_k5.hip", "sr_mfma_k5_big.hip", "sr_mfma_k5_ps.hip", "sr_mfma_k5_pm.hip", "sr_mfma_k5_lg.hip", "sr_mfma_k5_blk.hip", "sr_mfma_list.hip", "sr_mfma_k5_f32.hip", "sr_mfma_k5_f8.hip", "sr_mfma_k7.hip", "sr_mfma_k7_f8.hip", "sr_mfma_bf16.hip", "sr_probe.hip", "sr_select.hip"]
HEADERS = ["sr_device.h", "sr_launch.h", "sr_mfma_kernel.h", os.path.join("..", "..", "include", "sr_dict.h"),
           os.path.join("..", "..", "include", "sr_probe.h"),
           os.path.join("..", "..", "include", "sr_select.h")]
OBJDIR = os.path.join(HERE, "_build")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off", "-fvisibility=hidden", "-fno-gpu-rdc",
    # packed-fp32 VALU forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.abspath(__file__)]
    return any(os.path.getmtime(d) > t for d in deps)


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        sys.stderr.write(err + "\n")
        raise RuntimeError("hipcc failed: " + " ".join(cmd[-3:]))
    if verbose and err.strip():
        sys.stderr.write(err + "\n")


def build_library(force: bool = True, verbose: bool = False, extra=(), out: str = LIB) -> str:
    """Compile every HIP source (in parallel) and link one shared library.  Returns its path."""
    if not force and out == LIB and not stale():
        return LIB
    from concurrent.futures import ThreadPoolExecutor
    objdir = OBJDIR + ("" if out == LIB else "_" + os.path.basename(out))
    os.makedirs(objdir, exist_ok=True)
    cc = hipcc()
    objs = [os.path.join(objdir, s.replace(".hip", ".o")) for s in SOURCES]
    cmds = [[cc] + FLAGS + list(extra) + ["-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(8, len(cmds))) as pool:
        list(pool.map(lambda c: _run(c, verbose), cmds))
    tmp = out + ".tmp%d" % os.getpid()
    _run([cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fvisibility=hidden", "-o", tmp] + objs, verbose)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    # python -m paper_2303_08999_amd.build [-o other.so] [extra hipcc flags ...]
    args = sys.argv[1:]
    target = LIB
    if args[:1] == ["-o"]:
        target, args = os.path.abspath(args[1]), args[2:]
    print(build_library(force=True, verbose=False, extra=args, out=target))
