"""Builds libdsbd.so (HIP, gfx950) in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdsbd.so")
SOURCES = ["attention.hip", "verify.hip", "select.hip", "commit.hip", "draft.hip", "timing.hip", "knobs.hip"]
# Per-file flags.  attention.hip: scores come out of the matrix units and go through max / exp2 only; without
# -fno-honor-nans every fmaxf operand is first canonicalised (v_max x, x), which triples the instructions of the
# row-maximum checks.  (verify.hip must keep NaN semantics: it detects non-finite logits.)
# verify.hip: the layer kernel is held to 240 registers (an attribute in the source) and its warped build uses them
# all; hoisting loop-invariant address arithmetic out of its layer loop (machine LICM) made it spill 84-120 bytes per
# lane, with reloads in front of stores on the critical path.
# (-Rpass-analysis: the compiler's per-kernel register report, checked below)
FILE_FLAGS = {"attention.hip": os.environ.get("DSBD_ATTN_FLAGS", "-fno-honor-nans").split(),
              "verify.hip": os.environ.get("DSBD_VERIFY_FLAGS", "-mllvm -disable-machine-licm").split()
              + ["-Rpass-analysis=kernel-resource-usage"]}
# The statistics pass runs beside the layer kernel, one workgroup (a wave of 32 registers per SIMD) per compute unit:
# that needs the layer kernel's two waves per SIMD to leave 32 of the 512 registers of a SIMD lane free (handed out in
# eights): at most 240 each.
LAYER_KERNEL_VGPR_BUDGET = 240
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fgpu-rdc-", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def hipcc():
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def check_registers(report, verbose):
    """Reads the compiler's resource report: warns when a layer kernel outgrows the register budget that lets the
    statistics pass share its compute units, or spills.  Returns what is left of the compiler's output."""
    import re
    rest, name = [], None
    for line in report.splitlines():
        if "-Rpass-analysis=kernel-resource-usage" not in line:
            if "remark:" not in line and not (name and (line.strip().startswith(("|", "^")) or re.match(r"\s*\d+ \|", line))):
                rest.append(line)
            continue
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"\bVGPRs: (\d+)", line)
        if m and name and "verify_layers_kernel" in name:
            if verbose:
                print("%s: %s vector registers" % (name, m.group(1)))
            if int(m.group(1)) > LAYER_KERNEL_VGPR_BUDGET:
                print("WARNING: %s uses %s vector registers (budget %d): the statistics pass will no longer fit beside it"
                      % (name, m.group(1), LAYER_KERNEL_VGPR_BUDGET))
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and name and "verify_layers_kernel" in name and int(m.group(1)) > 0:
            print("WARNING: %s spills %s bytes per lane" % (name, m.group(1)))
    return "\n".join(rest)


def build(verbose=True):
    """Compile every translation unit and link the shared library. Always rebuilds."""
    flags = [f for f in FLAGS if f != "-fgpu-rdc-"] + os.environ.get("DSBD_EXTRA_HIPCC_FLAGS", "").split()
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [hipcc()] + flags + FILE_FLAGS.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        if "-Rpass-analysis=kernel-resource-usage" in FILE_FLAGS.get(src, []):
            out = check_registers(out, verbose)
        if verbose and out.strip():
            print(out)
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
