"""Build step: compiles the HIP sources into the C-ABI shared library, in-tree.

    python -m paper_2505_21487_amd.build            # build the library
    python -m paper_2505_21487_amd.build --check    # code-generation check (see check_register_windows)
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgla_decode.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Wall", "-Wno-unused-function",
    # packed-fp32 VALU ops are not to be generated on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return [os.path.join(CSRC, "gla_decode.hip")]


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    deps.append(os.path.join(os.path.dirname(HERE), "include", "gla_decode.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose: bool = True, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + ["-o", tmp] + sources()
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


def check_register_windows(verbose: bool = True) -> list:
    """Code-generation check for the kernels that keep page-id windows in registers
    (pages of 8 tokens or fewer with the 512-dim latent).  Those registers are
    loaded asynchronously by one inline-assembly statement and must stay where
    they are until the load has landed: any copy the compiler makes of them in
    between would carry stale page ids.  Compiles those kernels to assembly and
    verifies, per kernel, that every load site names the same registers and that
    nothing else in the kernel writes them after the first site (before it they
    are set to zero).  Returns one description per kernel; raises on a violation."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    with tempfile.TemporaryDirectory() as tmp:
        asm = os.path.join(tmp, "check.s")
        cmd = [hipcc] + flags + ["--cuda-device-only", "-S", "-o", asm, os.path.join(CSRC, "check_register_windows.hip")]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
        text = open(asm).read()
    found = []
    for fn in re.split(r"\n(?=_ZN3gla17tuned_main_kernel\S*: ; @)", text):
        m = re.match(r"(_ZN3gla17tuned_main_kernel\S*):", fn)
        if not m or "gla_win_skip" not in fn:
            continue
        lines = fn.split(".Lfunc_end")[0].split("\n")
        sites, in_site = [], set()
        for i, line in enumerate(lines):
            if "s_cbranch_scc1 .Lgla_win_skip" not in line:
                continue
            regs, j = [], i + 1
            while "global_load_dword" in lines[j]:
                regs.append(int(re.search(r"global_load_dword v(\d+),", lines[j]).group(1)))
                in_site.add(j)
                j += 1
            sites.append((i, regs))
        first = sorted(set(tuple(r) for k, (_, r) in enumerate(sites) if k % 2 == 0))
        second = sorted(set(tuple(r) for k, (_, r) in enumerate(sites) if k % 2 == 1))
        if not sites or len(first) != 1 or len(second) != 1:
            raise RuntimeError(f"{m.group(1)}: load sites disagree on the window registers: {first} {second}")
        window = set(first[0]) | set(second[0])
        for k, line in enumerate(lines):
            t = line.strip()
            if k in in_site or not t or t[0] in ";." or t.endswith(":"):
                continue
            op, _, rest = t.partition(" ")
            if op.startswith(("s_", "ds_write", "global_store", "scratch_store", "buffer_store")):
                continue
            dst = rest.split(",")[0].strip()
            one, many = re.fullmatch(r"v(\d+)", dst), re.fullmatch(r"v\[(\d+):(\d+)\]", dst)
            written = {int(one.group(1))} if one else set(range(int(many.group(1)), int(many.group(2)) + 1)) if many else set()
            zeroed = re.fullmatch(r"v_mov_b32_e32 v\d+, 0", t) or (k < sites[0][0] and op == "v_mov_b32_e32")
            if written & window and not zeroed:
                raise RuntimeError(f"{m.group(1)}: window register written outside the load statement: {t}")
        found.append(f"{m.group(1)}: windows {first[0]} {second[0]}, {len(sites)} load sites")
    if len(found) != 2:
        raise RuntimeError(f"expected two kernels with register windows, found {len(found)}")
    if verbose:
        print("\n".join(found))
    return found


if __name__ == "__main__":
    if sys.argv[1:] == ["--check"]:
        check_register_windows()
    else:
        build(extra_flags=sys.argv[1:])
