"""Builds libnntile_mi.so (the C-ABI library of HIP kernels for gfx950) in-tree.

    python -m paper_2504_13236_amd.build

Every .hip file under csrc/ is compiled with hipcc for gfx950 and linked into
paper_2504_13236_amd/libnntile_mi.so.  Works without a GPU (cross-compilation).
"""
from __future__ import annotations

import concurrent.futures
import json
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libnntile_mi.so")

FLAGS = [
    "-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-fvisibility=hidden",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
    # packed fp32 VALU forms are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    # per-kernel register, scratch and LDS figures on stderr (parsed below)
    "-Rpass-analysis=kernel-resource-usage",
]

# Sources whose kernels keep LDS reads in flight across statements (the reads are issued by
# inline assembly and waited for later by hand): a register the compiler spills or reloads
# between a read and its wait would hold stale data, so inside their loops these kernels
# must not touch scratch memory.  (Spills in the prologue or after the last wait are harmless.)
# Their assembly is also scanned for any instruction that names a register between the LDS read that
# targets it and the next full wait (registers_touched_in_flight): a copy or move the compiler
# places there would read stale data just the same.
IN_FLIGHT_SOURCES = ("gemm_bf16_dl.hip", "gemm_f32_dl.hip")


def scratch_in_loops(asm_text: str) -> list:
    """[(kernel, line number)] of scratch instructions inside loop blocks of a device assembly listing.

    The listing marks each basic block that belongs to a loop in the comment on its label."""
    hits = []
    kernel, in_loop = None, False
    for no, line in enumerate(asm_text.splitlines(), 1):
        t = line.strip()
        if t.startswith("_Z") and t.split(":")[0].isidentifier() and ":" in t:
            kernel, in_loop = t.split(":")[0], False
        elif t.startswith(".LBB") or t.startswith("; %bb."):
            in_loop = "Loop" in t
        elif in_loop and t.startswith("scratch_"):
            hits.append((kernel, no))
    return hits


_VREG = re.compile(r"\bv(\d+)\b|\bv\[(\d+):(\d+)\]")


def _vregs(text: str) -> set:
    out = set()
    for m in _VREG.finditer(text):
        if m.group(1) is not None:
            out.add(int(m.group(1)))
        else:
            out.update(range(int(m.group(2)), int(m.group(3)) + 1))
    return out


def registers_touched_in_flight(asm_text: str) -> list:
    """[(kernel, line number, register, line of the read)]: instructions of a device assembly listing that name a
    vector register while an LDS read into it is still in flight, i.e. between the ds_read that targets it and
    the next `s_waitcnt lgkmcnt(0)`.

    The compiler believes such a register holds its value from the read's asm statement on, so a copy, a move to
    an accumulation register or any other use it schedules before the hand-placed wait would see stale data.
    The scan is linear per kernel (listing order); only a full wait clears the reads in flight."""
    hits = []
    kernel, pending = None, {}
    for no, line in enumerate(asm_text.splitlines(), 1):
        t = line.split(";")[0].strip()
        if not t:
            continue
        if t.startswith("_Z") and t.endswith(":"):
            kernel, pending = t[:-1], {}
            continue
        if t.endswith(":") or t.startswith("."):
            continue
        op, _, rest = t.partition(" ")
        if op == "s_waitcnt":
            if "lgkmcnt(0)" in rest:
                pending = {}
            continue
        if op == "s_endpgm":
            pending = {}
            continue
        if op.startswith("ds_read"):
            ops = [o.strip() for o in rest.split(",")]
            for o in ops[1:]:                       # the address is read now
                for r in _vregs(o):
                    if r in pending:
                        hits.append((kernel, no, "v%d" % r, pending[r]))
            for r in _vregs(ops[0]):
                pending[r] = no
            continue
        for r in _vregs(rest):
            if r in pending:
                hits.append((kernel, no, "v%d" % r, pending[r]))
    return hits


_NAME = re.compile(r"remark: Function Name: (\S+)")
_FIELD = re.compile(r"remark:\s+(TotalSGPRs|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|Occupancy \[waves/SIMD\]"
                    r"|VGPRs Spill|LDS Size \[bytes/block\]): (\d+)")


def resource_usage(stderr: str) -> dict:
    """{mangled kernel name: {field: value}} from hipcc's kernel-resource-usage remarks."""
    out: dict = {}
    cur = None
    for line in stderr.splitlines():
        m = _NAME.search(line)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        m = _FIELD.search(line)
        if m and cur is not None:
            cur[m.group(1).split(" [")[0]] = int(m.group(2))
    return out


def _newest_header() -> float:
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hpp")]
    hs += [os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include"))]
    return max(os.path.getmtime(h) for h in hs)


def _compile(src: str, only_if_stale: bool = False) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    if only_if_stale and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), _newest_header(),
                                                                              os.path.getmtime(__file__)):
        return obj
    in_flight = os.path.basename(src) in IN_FLIGHT_SOURCES
    cmd = ["hipcc", *FLAGS, *(["-save-temps=obj"] if in_flight else []), "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, r.stderr[-4000:]))
    usage = resource_usage(r.stderr)
    if in_flight:
        stem = os.path.splitext(os.path.basename(src))[0]
        with open(os.path.join(OBJ, stem + "-hip-amdgcn-amd-amdhsa-gfx950.s")) as f:
            hits = scratch_in_loops(f.read())
        if hits:
            raise RuntimeError("%s: scratch access inside a loop of %s (assembly line %d, %d in all): "
                               "in-flight fragment registers do not survive a spill"
                               % (os.path.basename(src), hits[0][0], hits[0][1], len(hits)))
        with open(os.path.join(OBJ, stem + "-hip-amdgcn-amd-amdhsa-gfx950.s")) as f:
            early = registers_touched_in_flight(f.read())
        if early:
            raise RuntimeError("%s: %s, assembly line %d, uses %s before the wait for the LDS read of line %d (%d such uses in all)"
                               % (os.path.basename(src), early[0][0], early[0][1], early[0][2], early[0][3], len(early)))
    with open(obj + ".usage.json", "w") as f:
        json.dump(usage, f, indent=1, sort_keys=True)
    return obj


def build_library(jobs: int | None = None, verbose: bool = True, only_stale: bool = False) -> str:
    """Compiles every source (or, with only_stale, those older than their object file) and links."""
    os.makedirs(OBJ, exist_ok=True)
    srcs = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))
    jobs = jobs or min(8, len(srcs), os.cpu_count() or 1)
    with concurrent.futures.ThreadPoolExecutor(jobs) as ex:
        objs = list(ex.map(lambda f: _compile(f, only_stale), srcs))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr[-4000:])
    if verbose:
        print("built", LIB, "from", len(srcs), "sources")
    return LIB


if __name__ == "__main__":
    build_library(only_stale="--stale" in sys.argv[1:])
    sys.exit(0)
