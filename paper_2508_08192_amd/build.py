"""Build libtreeattn.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2508_08192_amd.build
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtreeattn.so")
SOURCES = ["ta_api.hip", "ta_generic.hip", "ta_mfma.hip", "ta_host.cpp"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # hipcc must not form packed-fp32 instructions on these machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def generate_blocks(verbose=False):
    """ta_sp_block.inc is written by csrc/gen_sp_block.py; keep the file in step with its generator."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("gen_sp_block", os.path.join(CSRC, "gen_sp_block.py"))
    gen = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(gen)
    text = gen.generate()
    path = os.path.join(CSRC, "ta_sp_block.inc")
    if not os.path.exists(path) or open(path).read() != text:
        with open(path, "w") as f:
            f.write(text)
        if verbose:
            print("regenerated " + path)


def build_library(verbose=False, extra_flags=()):
    """Compile every HIP source for gfx950 and link the C-ABI shared library; returns its path."""
    generate_blocks(verbose)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc] + FLAGS + list(extra_flags) + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the packed-fp32 feature and says so once per source: harmless
    noise = "is not a recognized feature for this target"
    log = "\n".join(l for l in proc.stdout.splitlines() if noise not in l)
    if proc.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise RuntimeError("hipcc failed:\n" + log)
    if verbose and log.strip():
        print(log)
    try:
        verify_register_partition(verbose)
    except Exception:
        os.remove(tmp)
        raise
    os.replace(tmp, LIB)
    return LIB


HOST_CHECKED_LIB = os.path.join(HERE, "libtreeattn_hostcheck.so")


def build_host_checked(verbose=False):
    """The host logic alone (validation, planning, dispatch table) as a shared library built by g++ with
    AddressSanitizer and UndefinedBehaviorSanitizer; its launching entry points stop with TA_ERR_HIP.  The CPU
    tests load it through TREEATTN_LIB, with the sanitizer runtime preloaded.  Returns (library, runtime)."""
    gxx = os.environ.get("CXX", "g++")
    tmp = HOST_CHECKED_LIB + ".tmp%d" % os.getpid()
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fPIC", "-shared", "-Wall", "-Wextra", "-Werror",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           os.path.join(CSRC, "ta_host.cpp"), os.path.join(CSRC, "ta_host_only.cpp"), "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise RuntimeError("g++ failed:\n" + proc.stdout)
    os.replace(tmp, HOST_CHECKED_LIB)
    runtime = subprocess.run([gxx, "-print-file-name=libasan.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    return HOST_CHECKED_LIB, runtime


def verify_register_partition(verbose=False):
    """ta_mfma_sp_kernel keeps its large operands in v32..v255, which only its asm blocks may touch: the compiler
    is confined to v0..v31 by amdgpu_num_vgpr.  That contract is checked here on the generated ISA rather than
    trusted: outside the asm blocks no VGPR above v31 may appear, and the kernel must be sized for 256 VGPRs."""
    import re
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in FLAGS if f not in ("-fPIC", "-shared")]
    cmd = [hipcc] + flags + ["-S", "--cuda-device-only", "-o", "-", os.path.join(CSRC, "ta_mfma.hip")]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc -S failed for ta_mfma.hip")
    lines = proc.stdout.split("\n")
    starts = [i for i, l in enumerate(lines) if re.match(r"_Z17ta_mfma_sp_kernel\w*:", l)]
    if len(starts) != 2:
        raise RuntimeError("expected the two instances of ta_mfma_sp_kernel in the ISA, found %d" % len(starts))
    for start in starts:
        name = lines[start].split(":")[0]
        end = next(i for i in range(start, len(lines)) if ".end_amdhsa_kernel" in lines[i])
        in_asm, worst = False, -1
        for l in lines[start:end]:
            if "#ASMSTART" in l:
                in_asm = True
            elif "#ASMEND" in l:
                in_asm = False
            elif not in_asm and not l.lstrip().startswith((";", ".")):
                for mm in re.finditer(r"\bv(\d+)\b|\bv\[(\d+):(\d+)\]", l):
                    worst = max(worst, int(mm.group(1) or mm.group(3)))
        sized = any(".amdhsa_next_free_vgpr 256" in l for l in lines[start:end])
        if worst > 31 or not sized:
            raise RuntimeError("register partition of %s broken: compiler code uses v%d (limit v31), "
                               "kernel sized for 256 VGPRs: %s" % (name, worst, sized))
        if verbose:
            print("%s: compiler code stays in v0..v%d; kernel sized for 256 VGPRs" % (name, worst))


if __name__ == "__main__":
    print(build_library(verbose=True))
    sys.exit(0)
