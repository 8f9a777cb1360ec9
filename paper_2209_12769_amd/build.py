"""Builds libdisco.so (HIP, gfx950) in-tree next to this file."""
from __future__ import annotations

import glob
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
LIB_PATH = os.path.join(_HERE, "libdisco.so")


def sources():
    return sorted(glob.glob(os.path.join(_HERE, "csrc", "*.hip")))


COMPILE_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                 "-packed-fp32-ops", "-Wno-unused-result", "-I", os.path.join(_ROOT, "include"),
                 "-I", os.path.join(_HERE, "csrc")]


def _spilling_layer_kernels(report: str):
    """Layer kernels of the resource report that keep registers in scratch memory (they run several times
    slower: a restructuring that pushes one over its register budget must not pass unnoticed)."""
    bad, name = [], None
    for line in report.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split()[0]
        elif "ScratchSize [bytes/lane]:" in line and name and "layer256" in name:
            n = int(line.split("ScratchSize [bytes/lane]:")[1].split()[0])
            if n:
                bad.append((name, n))
    return bad


def build_lib(verbose: bool = False, checks: bool = True) -> str:
    """Compiles the library.  With `checks`, the build fails if a bulk layer kernel spills registers or if
    the listing of the kernels that wait by hand for untracked loads shows an instruction touching a
    load's destination while the load is in flight (isa_check)."""
    cmd = ["hipcc", *COMPILE_FLAGS, "-fPIC", "-shared", "-Rpass-analysis=kernel-resource-usage", "-o", LIB_PATH] + sources()
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    import re
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops" not in l and "remark:" not in l and not re.match(r"^\s*\d*\s*\|", l))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out, flush=True)
    if checks:
        bad = _spilling_layer_kernels(res.stdout)
        if bad:
            os.remove(LIB_PATH)
            raise RuntimeError(f"layer kernels spill registers to scratch memory: {bad}")
        from . import isa_check
        hazards = {k: h for k, h in isa_check.check_layer256().items() if h}
        if hazards:
            os.remove(LIB_PATH)
            raise RuntimeError(f"loads in flight touched by compiler-generated instructions: "
                               f"{ {k: h[:3] for k, h in hazards.items()} }")
    return LIB_PATH


if __name__ == "__main__":
    build_lib(verbose=True)
