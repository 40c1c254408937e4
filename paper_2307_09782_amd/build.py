"""Build libzqfp.so (HIP kernels + C ABI) for gfx950 with hipcc.

Run as ``python -m paper_2307_09782_amd.build``; ``__graft_entry__.build()``
calls :func:`build_lib`.  The library is placed next to this file so that it
travels with the source tree; objects go to ``_build/`` (not committed).
"""
import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

from . import check_lds_waits

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libzqfp.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-FP32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


# Kernels that issue LDS reads by hand (inline asm) and wait for them by count: a register spill
# between such a read and its wait would save a value that has not arrived yet, so these must
# compile without scratch memory.  The compiler's resource remarks are checked after every build.
NO_SCRATCH_KERNELS = ("k_gemm_tile",)
# The same kernels' device assembly is kept by the compile and checked for another thing the compiler may do to
# such reads: copy their destination register before the wait (see check_lds_waits).
HAND_WAIT_SOURCES = {"gemm_tile.hip": "k_gemm_tile"}


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd) + "\n" + out)
    return out


def _check_no_scratch(remarks):
    """Raise if a kernel named in NO_SCRATCH_KERNELS uses scratch memory or spills registers."""
    name = None
    for line in remarks.splitlines():
        if "remark:" not in line:
            continue
        text = line.split("remark:", 1)[1].strip()
        if text.startswith("Function Name:"):
            name = text.split(":", 1)[1].split("[")[0].strip()
        elif name and any(k in name for k in NO_SCRATCH_KERNELS):
            for key in ("ScratchSize [bytes/lane]:", "VGPRs Spill:"):
                if text.startswith(key) and int(text[len(key):].split("[")[0]) != 0:
                    raise RuntimeError(f"{name}: '{text}' -- this kernel must not spill (hand-scheduled LDS reads)")


def build_lib(verbose=False, jobs=8):
    """Compile every csrc/*.hip and link libzqfp.so (always recompiles)."""
    os.makedirs(OBJDIR, exist_ok=True)
    srcs = sources()
    objs = [os.path.join(OBJDIR, os.path.basename(s)[:-4] + ".o") for s in srcs]
    cmds = [[HIPCC, *FLAGS, "-Rpass-analysis=kernel-resource-usage",
             *(["-save-temps=obj"] if os.path.basename(s) in HAND_WAIT_SOURCES else []), "-c", s, "-o", o] for s, o in zip(srcs, objs)]
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        outs = list(ex.map(_run, cmds))
    for o in outs:
        _check_no_scratch(o)
    for src, kernel in HAND_WAIT_SOURCES.items():
        listing = os.path.join(OBJDIR, src[:-4] + "-hip-amdgcn-amd-amdhsa-gfx950.s")
        with open(listing) as f:
            check_lds_waits.check_text(f.read(), kernel)
    outs = ["\n".join(l for l in o.splitlines() if "kernel-resource-usage" not in l and not l.lstrip().startswith(("|", "^")) and not l.strip().split(" ", 1)[0].isdigit()) for o in outs]
    outs.append(_run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]))
    if verbose:
        text = "\n".join(o for o in outs if o.strip())
        if text:
            print(text)
    return LIB


def sanitizer_runtime():
    """Path of the AddressSanitizer runtime of the compiler that hipcc drives (to be preloaded by a process
    that loads a library built by build_host_sanitized)."""
    clang = os.path.join(os.path.dirname(os.path.realpath(HIPCC)), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/llvm/bin/clang"
    return _run([clang, "--print-file-name=libclang_rt.asan-x86_64.so"]).strip()


def build_host_sanitized(out):
    """libzqfp with the HOST side of the C ABI (csrc/zqfp_api.hip: argument checks, dispatch, the header check)
    compiled under AddressSanitizer + UndefinedBehaviorSanitizer; device code and the kernels' launchers are the
    ordinary objects of the last build_lib().  For CPU-side tests only."""
    objs = [os.path.join(OBJDIR, os.path.basename(s)[:-4] + ".o") for s in sources()]
    if not all(os.path.exists(o) for o in objs):
        build_lib()
    api = os.path.join(CSRC, "zqfp_api.hip")
    api_o = os.path.join(os.path.dirname(out), "zqfp_api.san.o")
    flags = [f for f in FLAGS if f != "-O3"]
    _run([HIPCC, *flags, "-O1", "-g", "-fno-omit-frame-pointer", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
          "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined", "-c", api, "-o", api_o])
    others = [o for o in objs if os.path.basename(o) != "zqfp_api.o"]
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
          "-o", out, api_o, *others])
    return out


if __name__ == "__main__":
    print(build_lib(verbose=True))
