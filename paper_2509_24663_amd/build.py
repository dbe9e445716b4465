"""Build libinfllmv2.so (HIP kernels + C ABI) for gfx950, in-tree, with hipcc."""
from __future__ import annotations

import json
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libinfllmv2.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffast-math", "-fno-finite-math-only",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option", "-Wno-inline-asm",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]

# Per-file additions.  The backward kernels keep 64 accumulator registers plus short-lived ones; with the default
# split of the register file the compiler parks accumulators in AGPRs and then shuffles them through VGPRs around
# every temporary MFMA (a hundred v_accvgpr moves per token).  Keeping MFMA results in VGPRs avoids that.
EXTRA_FLAGS = {
    "attn_bwd_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
}


def kernel_resources() -> dict:
    """Resource usage of every kernel of the last build: {source file: {mangled kernel name: {...}}}."""
    res = {}
    for src in sources():
        path = os.path.join(OBJ, src[:-4] + ".resources.json")
        if os.path.exists(path):
            with open(path) as f:
                res[src] = json.load(f)
    return res


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ, src[:-4] + ".o")
    deps = [os.path.join(CSRC, src), os.path.join(ROOT, "include", "infllmv2.h")] + [
        os.path.join(CSRC, h) for h in os.listdir(CSRC) if h.endswith(".h")]
    if not force and os.path.exists(obj) and all(os.path.getmtime(obj) >= os.path.getmtime(d) for d in deps):
        return obj
    cmd = [HIPCC, *FLAGS, *EXTRA_FLAGS.get(src, []), "-Rpass-analysis=kernel-resource-usage",
           "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    usage, rest = _split_resource_remarks(r.stdout)
    # the host pass warns that it does not know the packed-fp32 target feature: harmless
    out = "\n".join(l for l in rest if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    if out.strip():
        sys.stderr.write(out + "\n")
    with open(obj[:-2] + ".resources.json", "w") as f:
        json.dump(usage, f, indent=1)
    for name, u in usage.items():
        if u.get("ScratchSize", 0) or u.get("VGPRs Spill", 0):
            sys.stderr.write(f"note: {src}: kernel {name} uses {u.get('ScratchSize', 0)} B/lane of private-segment memory "
                             f"({u.get('VGPRs Spill', 0)} spilled VGPRs)\n")
    return obj


_REMARK = re.compile(r"remark:\s+(.*?)\s+\[-Rpass-analysis=kernel-resource-usage\]")


def _split_resource_remarks(text: str):
    """Separate the compiler's per-kernel resource remarks from the rest of its output.

    Returns ({mangled kernel name: {"VGPRs": n, "ScratchSize": bytes per lane, "VGPRs Spill": n, ...}}, other lines).
    A prefetch array that ends up in private-segment memory costs a kernel tens of percent and shows nowhere in the
    source, so the numbers are kept next to the objects (tests read them) and non-zero scratch is reported.
    """
    usage, rest, cur = {}, [], None
    skip = 0
    for line in text.splitlines():
        m = _REMARK.search(line)
        if m:
            body = m.group(1)
            if body.startswith("Function Name:"):
                cur = body.split(":", 1)[1].strip()
                usage[cur] = {}
            elif cur is not None and ":" in body:
                key, val = body.rsplit(":", 1)
                key = key.split("[")[0].strip()
                val = val.strip()
                usage[cur][key] = int(val) if val.lstrip("-").isdigit() else val
            skip = 2          # the source line and the caret line that follow a remark
            continue
        if skip and (re.match(r"\s*\d+ \|", line) or re.match(r"\s*\|\s*\^", line)):
            skip -= 1
            continue
        skip = 0
        rest.append(line)
    return usage, rest


def build(force: bool = True, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), sources()))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.check_call(cmd)
    return LIB


def build_probes() -> str:
    """The measurement program behind the roofline model (probes/unit_limits.hip): a stand-alone executable."""
    src = os.path.join(HERE, "probes", "unit_limits.hip")
    exe = os.path.join(HERE, "probes", "unit_limits")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-inline-asm", "-Wno-unused-command-line-argument", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", exe, src]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on unit_limits.hip:\n{r.stdout}")
    return exe


def build_variant(name: str, defines) -> str:
    """libinfllmv2_<name>.so: the library with extra -D flags, for timing experiments (bench.py --lib <name>).  The
    timing switches of attn_mfma.hip (ATTN_TIMING_NO_LOADS, ATTN_TIMING_NO_BARRIER) give wrong results by design."""
    out_dir = os.path.join(OBJ, "variant_" + name)
    os.makedirs(out_dir, exist_ok=True)
    objs = []
    for src in sources():
        obj = os.path.join(out_dir, src[:-4] + ".o")
        cmd = [HIPCC, *FLAGS, *EXTRA_FLAGS.get(src, []), *[f"-D{d}" for d in defines], "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}")
        objs.append(obj)
    lib = os.path.join(HERE, f"libinfllmv2_{name}.so")
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs])
    return lib


if __name__ == "__main__":
    if "--probes" in sys.argv:
        print(build_probes())
    elif "--variant" in sys.argv:          # build.py --variant NAME DEFINE [DEFINE ...]
        i = sys.argv.index("--variant")
        print(build_variant(sys.argv[i + 1], sys.argv[i + 2:]))
    else:
        print(build(force="--force" in sys.argv))
