"""Build libbinattn.so (HIP, gfx950) in-tree with hipcc.

    python -m paper_2603_09582_amd.build [--force]

Every translation unit under csrc/ is compiled to an object in csrc/_build/ (in
parallel) and linked into paper_2603_09582_amd/libbinattn.so.
"""
from __future__ import annotations

import concurrent.futures as cf
import glob
import json
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libbinattn.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 VALU forms are kept out of every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
    # per-kernel register / scratch / LDS figures as compiler remarks (collected below)
    "-Rpass-analysis=kernel-resource-usage",
] + os.environ.get("HIPCC_FLAGS", "").split()


def _sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _headers():
    return glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))


RES_KEYS = {"VGPRs": "vgprs", "AGPRs": "agprs", "ScratchSize [bytes/lane]": "scratch_bytes",
            "Occupancy [waves/SIMD]": "waves_per_simd", "LDS Size [bytes/block]": "lds_bytes"}


def _resources(stderr: str):
    """(kernel symbol -> figures, the other compiler output) from the resource-usage remarks."""
    table, rest, cur = {}, [], None
    for l in stderr.splitlines():
        if "[-Rpass-analysis=kernel-resource-usage]" in l:
            body = l.split("remark:", 1)[1].replace("[-Rpass-analysis=kernel-resource-usage]", "").strip()
            key, _, val = body.partition(":")
            if key.strip() == "Function Name":
                cur = table.setdefault(val.strip(), {})
            elif cur is not None and key.strip() in RES_KEYS:
                cur[RES_KEYS[key.strip()]] = int(val.strip())
        elif "remark:" not in l and not (rest and rest[-1] is None):
            rest.append(l)
    # drop the source excerpts that follow each remark (a line of code and a caret line)
    keep = [l for l in rest if l is not None and not l.lstrip().startswith(("|", "^", "In file included from"))
            and " | " not in l[:12]]
    return table, "\n".join(keep)


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")
    res = obj[:-2] + ".resources.json"
    newest = max(os.path.getmtime(p) for p in [src, __file__] + _headers())
    if not force and os.path.exists(obj) and os.path.exists(res) and os.path.getmtime(obj) >= newest:
        return obj
    cmd = [HIPCC, *FLAGS, "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    table, other = _resources(r.stderr)
    err = "\n".join(l for l in other.splitlines()
                    if "not a recognized feature for this target" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    with open(res, "w") as f:
        json.dump(table, f, indent=0, sort_keys=True)
    return obj


def kernel_resources() -> dict:
    """Registers, scratch bytes per lane, waves per SIMD and LDS bytes of every kernel of the last
    build, by mangled name (from the compiler's resource-usage remarks)."""
    out = {}
    for p in glob.glob(os.path.join(OBJ, "*.resources.json")):
        with open(p) as f:
            out.update(json.load(f))
    return out


def build(force: bool = False, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = _sources()
    with cf.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), srcs))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
