"""Build libpf.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpf.so")
SOURCES = ["pf_host.hip", "pf_pool.hip", "pf_index.hip", "pf_attn.hip", "pf_classify.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# Packed-FP32 code generation is switched off for every device translation unit.
# Vector registers are never spilled into accumulation registers: the 64-row attention kernel keeps operands in
# accumulation registers the compiler does not know about (see pf_attn.hip).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
         "-mllvm", "-amdgpu-spill-vgpr-to-agpr=0"]


W64_KERNEL = "_Z17pf_attn_pp_kernelILi128ELi4EEv10AttnParams"
W64_FIRST_HIDDEN = 32     # the kernel's asm statements own a64..a255; the compiler's own code must stay below a32


def check_hidden_registers(listing):
    """The 64-row attention kernel keeps operands in accumulation registers behind the compiler's back (pf_attn.hip).
    That is sound only while no instruction the COMPILER emitted for that kernel touches those registers: read the
    device listing and raise if one does.  Returns the highest accumulation register the compiler used (-1: none)."""
    import re
    lines = listing.split("\n")
    try:
        start = next(i for i, ln in enumerate(lines) if ln.startswith(W64_KERNEL + ":"))
    except StopIteration:
        raise RuntimeError("listing has no 64-row attention kernel")
    end = next(i for i in range(start, len(lines)) if lines[i].strip().startswith("s_endpgm"))
    in_asm, highest = False, -1
    for ln in lines[start:end]:
        st = ln.strip()
        if st == ";;#ASMSTART":
            in_asm = True
        elif st == ";;#ASMEND":
            in_asm = False
        elif not in_asm:
            for m in re.finditer(r"\ba(\d+)\b|\ba\[(\d+):(\d+)\]", ln.split(";")[0]):
                highest = max(highest, int(m.group(1) or m.group(3)))
    if highest >= W64_FIRST_HIDDEN:
        raise RuntimeError("the compiler uses accumulation register a%d in the 64-row attention kernel: its hidden "
                           "operands are not safe (see pf_attn.hip)" % highest)
    return highest


def build(verbose=False, extra=()):
    """extra: more hipcc flags; PF_HIPCC_FLAGS in the environment adds to them (e.g. -DPF_STRICT_FENCES=1: release
    fences in front of the cross-workgroup arrival counters, the form the memory model asks for)."""
    extra = list(extra) + os.environ.get("PF_HIPCC_FLAGS", "").split()
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [HIPCC] + FLAGS + list(extra) + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    # device listing of the attention kernels, for the register check above (compiled next to the objects)
    lst = subprocess.Popen([HIPCC] + FLAGS + list(extra) + ["--cuda-device-only", "-S", os.path.join(CSRC, "pf_attn.hip"), "-o", "-"],
                           stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        lines = [ln for ln in out.splitlines() if "packed-fp32-ops" not in ln]   # host pass does not know the feature
        if p.returncode != 0:
            failed = True
        if lines and (verbose or p.returncode != 0):
            print("\n".join(lines), file=sys.stderr)
    listing, _ = lst.communicate()
    if failed or lst.returncode != 0:
        raise RuntimeError("hipcc failed")
    highest = check_hidden_registers(listing)
    if verbose:
        print("64-row attention kernel: highest accumulation register used by the compiler: a%d" % highest, flush=True)
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
