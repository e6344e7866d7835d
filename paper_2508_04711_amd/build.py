"""Builds libhstu_attn.so (the gfx950 HIP library) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhstu_attn.so")
SOURCES = ["hstu_api.hip", "hstu_plan.hip", "hstu_fwd.hip", "hstu_dkdv.hip", "hstu_dkdv2.hip", "hstu_dq.hip", "hstu_f32.hip", "hstu_probe.hip"]
FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
    # packed fp32 VALU forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    # the compiler's per-kernel register and LDS figures, kept beside the library (RESOURCES)
    "-Rpass-analysis=kernel-resource-usage",
]
# Per kernel: registers, spills, scratch, LDS, as the compiler reports them ("name: key value ..." lines).
RESOURCES = os.path.join(HERE, "kernel_resources.txt")


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc()] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, res.stderr[-4000:]))
    return obj, _resource_lines(res.stderr)


def _resource_lines(stderr: str):
    """One line per kernel from the compiler's resource-usage remarks."""
    out, cur = [], None
    for line in stderr.splitlines():
        if "remark:" not in line:
            continue
        text = line.split("remark:", 1)[1].split("[-Rpass")[0].strip()
        if text.startswith("Function Name:"):
            cur = [text.split(":", 1)[1].strip()]
            out.append(cur)
        elif cur is not None and ":" in text:
            key, val = text.rsplit(":", 1)
            cur.append("%s=%s" % (key.strip().replace(" ", "_"), val.strip()))
    return [" ".join(c) for c in out]


def build(verbose: bool = False) -> str:
    """Compiles every source for gfx950 and links the shared library; returns its path."""
    with ThreadPoolExecutor(max_workers=8) as ex:
        done = list(ex.map(_compile, SOURCES))
    objs = [d[0] for d in done]
    with open(RESOURCES, "w") as f:
        for d in done:
            f.write("\n".join(d[1]) + ("\n" if d[1] else ""))
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n%s" % res.stderr[-4000:])
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
