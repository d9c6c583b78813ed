"""Build the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librnn_mi355x.so")
SOURCES = ["wavefront_ll.hip", "wavefront_ll_b.hip", "wavefront_ll_c.hip", "wavefront_ll_d.hip", "wavefront_ll_e.hip",
           "wavefront_ll_f.hip", "wavefront_x.hip", "wavefront_x_b.hip", "wavefront.hip", "wavefront_b.hip",
           "rnn_api.hip", "gemm.hip", "cellwise.hip", "schedule.hip", "probe.hip", "rnn_stack.hip"]   # the slowest first
HEADERS = ["common.h", "kernels.h", "wf_traits.h", "wavefront_ll.hip", "wavefront_x.hip", "wavefront.hip",
           os.path.join("..", "..", "include", "rnn.h"),
           os.path.join("..", "..", "include", "rnn_schedule.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function", "-Wno-unused-const-variable",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


# Kernels that issue matrix instructions from inline assembly, with operands in the accumulation registers
# (the interleaved-chain variants of the inside-product kernel).  The compiler cannot see those operands'
# hazards, and a register spill would put memory operations and register copies of its own between the
# hand-spaced instructions: such a kernel must not spill.  The build reads the compiler's resource remarks,
# and fails as well when no kernel name matches any more (a renamed kernel or a new template parameter would
# otherwise pass the check unseen).
NO_SPILL = {"wavefront_x.hip": ("wavefront_x_kernel", "ELi2ELb"),     # file: (kernel name, piece of the name that says two chains)
            "wavefront_x_b.hip": ("wavefront_x_kernel", "ELi2ELb"),
            "gemm.hip": ("gemm_bf16_nt_wide_kernel", "")}               # 256 accumulation + 244 vector registers of 512


def _check_no_spill(src: str, remarks: str) -> None:
    kernel, piece = NO_SPILL[src]
    name = None
    seen = 0
    for line in remarks.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split()[0]
        elif "ScratchSize [bytes/lane]:" in line and name and kernel in name and piece in name:
            seen += 1
            if int(line.split("ScratchSize [bytes/lane]:")[1].split()[0]) != 0:
                raise RuntimeError("%s: %s spills registers to memory" % (src, name))
    if seen == 0:
        raise RuntimeError("%s: no kernel named like %s...%s in the compiler's remarks: the spill check checks nothing"
                           % (src, kernel, piece))


def _compile(src: str, obj: str) -> None:
    extra = ["-Rpass-analysis=kernel-resource-usage"] if src in NO_SPILL else []
    cmd = [_hipcc()] + FLAGS + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if src in NO_SPILL and r.returncode == 0:
        _check_no_spill(src, r.stdout)
    lines = [l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l]
    if src in NO_SPILL and r.returncode == 0:   # the remarks come with source excerpts: keep the diagnostics only
        lines = [l for l in lines if "warning:" in l or "error:" in l]
    out = "\n".join(lines)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, out))
    if out.strip():
        sys.stderr.write(out + "\n")


def build(force: bool = True, jobs: int = 8) -> str:
    """Compile every kernel source and link librnn_mi355x.so.  With force=False nothing is
    done when the library is newer than all sources."""
    deps = [os.path.join(CSRC, s) for s in SOURCES] + [os.path.normpath(os.path.join(CSRC, h)) for h in HEADERS]
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    objs = [os.path.join(bdir, s.replace(".hip", ".o")) for s in SOURCES]
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        list(ex.map(lambda so: _compile(*so), zip(SOURCES, objs)))
    tmp = LIB + ".tmp%d" % os.getpid()
    r = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs,
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
