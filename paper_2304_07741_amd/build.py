"""Builds libcanvas_dag.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
import glob
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcanvas_dag.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-mllvm", "-amdgpu-mfma-vgpr-form", "-Wall", "-Wno-unused-command-line-argument"]
# every kernel must fit the architectural register file without spilling: at most MAX_VGPRS vector registers
# (VGPRs + AGPRs) and no scratch memory; the compiler's per-kernel report is checked after each compilation
RESOURCE_FLAG = "-Rpass-analysis=kernel-resource-usage"
MAX_VGPRS = 256
# kernels that are known to spill a few vector registers and were measured that way (substrings of the mangled name);
# anything else that starts to use scratch memory fails the build
SCRATCH_ALLOWED = (
    r"sgfc.*5k_bwdILi1ELi1ELi2E",            # shift/FC backward, two tiles per wavefront under a 128-register cap (4 waves per SIMD)
    r"gfctm.*5k_fwdILi[12]ELi5ELi5ELb1ELi[24]ELb0E",  # 5x5 windows, fp32 destination, split K: 36 bytes of SGPR spill slots
    r"chain.*7k_chainILi9ELi2ELi1E",          # 9 lanes x 2 pixels under its 128-register cap (4 waves per SIMD): one register, stored and reloaded once per work item, outside the channel loop
)


def check_resources(src, remarks):
    """Parse the kernel-resource-usage remarks of one compilation; returns (kernels seen, list of violations)."""
    bad = []
    name, regs, n = None, {}, 0
    for line in remarks.splitlines():
        m = re.search(r"remark:\s+(Function Name|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|VGPRs Spill|SGPRs Spill): (\S+)", line)
        if not m:
            continue
        key, val = m.group(1), m.group(2)
        if key == "Function Name":
            name, regs = val, {}
            n += 1
            continue
        regs[key] = int(val)
        if key == "VGPRs Spill":  # (the last of the fields this check reads)
            total = regs.get("VGPRs", 0) + regs.get("AGPRs", 0)
            if total > MAX_VGPRS:
                bad.append(f"{os.path.basename(src)}: {name}: {total} vector registers (> {MAX_VGPRS})")
            if (regs.get("ScratchSize [bytes/lane]", 0) or regs.get("VGPRs Spill", 0)) and not any(re.search(a, name) for a in SCRATCH_ALLOWED):
                bad.append(f"{os.path.basename(src)}: {name}: spills vector registers to scratch memory ({regs})")
    return n, bad


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.cpp")))


def build(verbose=True):
    """Compile every source under csrc/ and link the shared library.  Always recompiles."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        objs.append(obj)
        cmd = [HIPCC, *FLAGS, RESOURCE_FLAG, "-x", "hip", "-c", src, "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    violations = []
    kernels = 0
    for src, p in procs:
        out, _ = p.communicate()
        n, bad = check_resources(src, out)
        kernels += n
        violations += bad
        # drop the resource report itself (a remark line, the source line it quotes and the caret line below it)
        kept, skip = [], 0
        for l in out.splitlines():
            if RESOURCE_FLAG in l:
                skip = 2
                continue
            if skip and (re.match(r"\s*\d+ \| ", l) or re.match(r"\s*\| +\^", l)):
                skip -= 1
                continue
            skip = 0
            kept.append(l)
        out = "\n".join(kept)
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if p.returncode != 0:
            failed = True
            sys.stderr.write(f"--- {src}\n{out}\n")
        elif verbose and out:
            sys.stderr.write(f"--- {src}\n{out}\n")
    if failed:
        raise RuntimeError("hipcc failed")
    if violations:
        raise RuntimeError("kernel register budget exceeded:\n  " + "\n  ".join(violations))
    if verbose:
        sys.stderr.write(f"register budget: {kernels} kernels within {MAX_VGPRS} vector registers, no unlisted kernel uses scratch memory\n")
    subprocess.check_call([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build())
