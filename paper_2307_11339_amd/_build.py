"""Build the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import re
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


# Sources whose kernels issue matrix instructions by hand (inline asm with the A operand and the accumulator in the
# accumulation registers): the compiler neither sees the instruction nor inserts the waits it inserts for its own.
HAND_ISSUED = ("wavefront_x.hip", "wavefront_x_b.hip")
HAND_MIN_APART = 5        # a hand-issued matrix instruction and the next one on the same accumulator: four others between
                          # (a 4-pass instruction has delivered its result by then; the tiles rotate over >= 4 accumulators)
HAND_MIN_BEFORE_READ = 16  # wait states between a hand-issued matrix instruction and any other reader of its result
HAND_MIN_AFTER_WRITE = 2   # wait states between v_accvgpr_write and a hand-issued matrix instruction that reads it

_AGPR = re.compile(r"\ba\[(\d+):(\d+)\]|\ba(\d+)\b")


def _agprs(operand: str):
    out = []
    for m in _AGPR.finditer(operand):
        if m.group(3) is not None:
            out.append(int(m.group(3)))
        else:
            out += list(range(int(m.group(1)), int(m.group(2)) + 1))
    return out


def _check_hand_issued(src: str, asm: str) -> int:
    """Walks the generated code of every kernel in program order (branches ignored: a guard, not a proof) and
    raises when a hand-issued matrix instruction (between #ASMSTART and #ASMEND) follows another one on the same
    accumulator by fewer than HAND_MIN_APART instructions, when anything but a matrix instruction reads an
    accumulation register fewer than HAND_MIN_BEFORE_READ wait states after a hand-issued instruction wrote it,
    or when such an instruction reads a register fewer than HAND_MIN_AFTER_WRITE wait states after
    v_accvgpr_write set it.  Returns the number of hand-issued instructions seen; none at all is an error too."""
    seen = 0
    in_asm = False
    kernel = None
    count = ws = 0
    hand_at = {}      # register -> (instruction count, wait states) of the last hand-issued writer
    set_at = {}       # register -> wait states at the last v_accvgpr_write
    for raw in asm.splitlines():
        t = raw.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            continue
        if not t or t[0] in ";." or t.startswith("//"):
            continue
        if t.endswith(":") or (":" in t.split()[0] and not t.startswith("s_") and not t.startswith("v_")):
            if not t.startswith(".L"):                    # a function label: a new kernel
                kernel, count, ws, hand_at, set_at = t.split(":")[0], 0, 0, {}, {}
            continue
        t = t.split(";")[0].strip()
        parts = t.split(None, 1)
        op, args = parts[0], [a.strip() for a in (parts[1].split(",") if len(parts) > 1 else [])]
        count += 1
        if op == "s_nop":
            ws += int(args[0], 0) + 1
            continue
        ws += 1
        if op.startswith("v_mfma"):
            dst = _agprs(args[0])
            if in_asm:
                seen += 1
                for r in dst:
                    if r in hand_at and count - hand_at[r][0] < HAND_MIN_APART:
                        raise RuntimeError("%s: %s: hand-issued matrix instructions on a%d only %d instructions apart"
                                           % (src, kernel, r, count - hand_at[r][0]))
                for a in args[1:]:
                    for r in _agprs(a):
                        if r in set_at and ws - set_at[r] < HAND_MIN_AFTER_WRITE + 1:
                            raise RuntimeError("%s: %s: a%d read by a hand-issued matrix instruction %d wait states "
                                               "after v_accvgpr_write" % (src, kernel, r, ws - set_at[r] - 1))
                for r in dst:
                    hand_at[r] = (count, ws)
            else:
                for r in dst:
                    hand_at.pop(r, None)                  # the compiler's own instruction: its waits are the compiler's
            continue
        writes_first = op.startswith(("global_load", "buffer_load", "ds_read", "flat_load", "scratch_load",
                                      "v_accvgpr_write", "v_accvgpr_mov"))
        for i, a in enumerate(args):
            for r in _agprs(a):
                if i == 0 and writes_first:
                    hand_at.pop(r, None)
                    if op.startswith("v_accvgpr_write"):
                        set_at[r] = ws
                elif r in hand_at and ws - hand_at[r][1] < HAND_MIN_BEFORE_READ + 1:
                    raise RuntimeError("%s: %s: %s reads a%d %d wait states after a hand-issued matrix instruction"
                                       % (src, kernel, op, r, ws - hand_at[r][1] - 1))
    if seen == 0:
        raise RuntimeError("%s: no hand-issued matrix instruction found in the generated code: the check checks nothing" % src)
    return seen


def _compile(src: str, obj: str) -> None:
    if src in HAND_ISSUED:
        asm = obj[:-2] + ".s"
        r = subprocess.run([_hipcc()] + FLAGS + ["--cuda-device-only", "-S", os.path.join(CSRC, src), "-o", asm],
                           stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc -S failed for %s:\n%s" % (src, r.stdout))
        _check_hand_issued(src, open(asm).read())
        os.remove(asm)
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
