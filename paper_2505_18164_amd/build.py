"""Builds libmdi.so (gfx950) in-tree with hipcc.  `python -m paper_2505_18164_amd.build`."""
from __future__ import annotations

import glob
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmdi.so")
SOURCES = ["mdi_api.hip", "decode.hip", "prefill.hip", "step_w4.hip", "step_w8.hip", "step2.hip", "attn_prefill.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wall", "-Wno-unused-function"]


RING_SOURCE = "step2.hip"


def check_ring_kernels(asm_files):
    """The persistent decode kernel keeps its prefetch ring in accumulation registers that only its own
    asm statements name, and validates them with its own waits.  Verified on the generated code: the
    compiler put nothing of its own there (no accumulation register is written except by the ring's
    loads), no scratch memory, no spilled registers."""
    if not asm_files:
        raise RuntimeError("device assembly of " + RING_SOURCE + " not found; cannot verify its register ring")
    text = open(asm_files[0]).read()
    bodies = re.findall(r"^(_ZN\w*k_step2\w*):[^\n]*\n(.*?)^\.Lfunc_end", text, flags=re.S | re.M)
    if not bodies:
        raise RuntimeError("no k_step2 kernel in " + asm_files[0])
    for name, body in bodies:
        if not re.search(r"global_load_dwordx4 a\[\d+:\d+\]", body):
            raise RuntimeError(f"{name}: no ring loads found")
        for line in body.split("\n"):
            ins = line.split(";")[0].strip()
            if not ins or ins.startswith("."):
                continue
            ops = ins.split(None, 1)
            if len(ops) == 2 and re.match(r"a(\[|\d)", ops[1].strip()) and not ins.startswith("global_load_dwordx4 a["):
                raise RuntimeError(f"{name}: the compiler writes an accumulation register: {ins}")
            if re.match(r"scratch_(load|store)", ins):
                raise RuntimeError(f"{name}: uses scratch memory")
    for m in re.finditer(r"\.name:\s+(\S*k_step2\S*)\n(?:.*\n)*?\s+\.private_segment_fixed_size:\s+(\d+)\n(?:.*\n)*?\s+\.vgpr_spill_count:\s+(\d+)", text):
        if int(m.group(2)) or int(m.group(3)):
            raise RuntimeError(f"{m.group(1)}: private segment {m.group(2)} bytes, {m.group(3)} spilled registers")


def _hipcc():
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build(verbose=False):
    os.makedirs(OBJ, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(OBJ, src.replace(".hip", ".o"))
        cmd = [_hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if src == RING_SOURCE:
            cmd.insert(1, "--save-temps=obj")          # keeps the device assembly next to the object
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    check_ring_kernels(glob.glob(os.path.join(OBJ, RING_SOURCE.replace(".hip", "") + "-hip-amdgcn-*.s")))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
