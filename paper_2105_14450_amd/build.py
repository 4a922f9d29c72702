"""Build ``libcube3d.so`` (the C-ABI library) for gfx950 with hipcc, in-tree."""
import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
# CUBE3D_OUT: another file name for the library (a variant build, e.g. with CUBE3D_EXTRA_FLAGS=-DCUBE3D_PROFILE,
# beside the product's libcube3d.so); its objects go to a folder of their own
LIB = os.path.join(HERE, os.environ.get("CUBE3D_OUT", "libcube3d.so"))
OBJDIR = os.path.join(HERE, "_build" if "CUBE3D_OUT" not in os.environ else "_build_" + os.environ["CUBE3D_OUT"].replace(".", "_"))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", INCLUDE, "-I", CSRC,
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option", "-Wno-inline-asm"] + \
    os.environ.get("CUBE3D_EXTRA_FLAGS", "").split()


SCRATCH_LIMIT = 1024   # bytes per lane
MFMA_BLOCK = 8         # a basic block with at least this many MFMAs belongs to a K loop


def _spills_in_k_loops(asm_path):
    """Names of the kernels whose device assembly has a scratch access in a K loop: a basic block
    with many MFMAs that branches back to its own label."""
    bad, func, label, mfma, scratch, loops = [], None, None, 0, 0, False

    def close_block():
        if func and loops and mfma >= MFMA_BLOCK and scratch:
            bad.append(func)

    with open(asm_path) as f:
        for line in f:
            head = line.split(";")[0].strip()
            if head.endswith(":") and not head.startswith("."):
                close_block()
                func, label, mfma, scratch, loops = head[:-1], None, 0, 0, False
            elif head.startswith(".LBB") and head.endswith(":"):
                close_block()
                label, mfma, scratch, loops = head[:-1], 0, 0, False
            elif head.startswith("v_mfma") or head.startswith("v_smfmac"):
                mfma += 1
            elif head.startswith("scratch_"):
                scratch += 1
            elif head.startswith("s_cbranch") or head.startswith("s_branch"):
                if label and head.split()[-1] == label:
                    loops = True
    close_block()
    return sorted(set(bad))


def _compile(src):
    """Compile one source; refuse kernels that spill registers inside a K loop (the tuned kernels
    are sized to live in the register file: a spill there is a performance bug) or that spill
    wholesale.  What the persistent kernel parks between two work items (lane-constant addresses,
    a few dozen registers, reloaded once per item) is accepted."""
    base = os.path.basename(src)
    obj = os.path.join(OBJDIR, base + ".o")
    res = subprocess.run([HIPCC, *FLAGS, "-Rpass-analysis=kernel-resource-usage", "-save-temps=obj", "-c", src, "-o", obj],
                         stderr=subprocess.PIPE, text=True)
    name, spilled, keep = None, [], []
    for line in res.stderr.splitlines():
        if "kernel-resource-usage" in line:
            if "Function Name:" in line:
                name = line.split("Function Name:")[1].split()[0]
            elif "ScratchSize" in line:
                if int(line.split(":")[-1].split()[0]) > SCRATCH_LIMIT:
                    spilled.append(name)
            continue
        if "packed-fp32-ops" in line and "not a recognized feature" in line:
            continue
        keep.append(line)
    # the remark lines come with source excerpts; print diagnostics only when the compile failed
    if res.returncode != 0:
        sys.stderr.write("\n".join(keep) + "\n")
        raise subprocess.CalledProcessError(res.returncode, HIPCC)
    asm = glob.glob(os.path.join(OBJDIR, base + "-hip-amdgcn-amd-amdhsa-gfx950.s")) + \
        glob.glob(os.path.join(OBJDIR, os.path.splitext(base)[0] + "-hip-amdgcn-amd-amdhsa-gfx950.s"))
    for path in asm:
        spilled += _spills_in_k_loops(path)
    # (a profiling build carries the time stamps' registers as well: its spills are reported, not refused)
    if spilled and ("-DCUBE3D_PROFILE" in FLAGS or os.environ.get("CUBE3D_ALLOW_SPILLS")):
        sys.stderr.write("note: register spills in %s: %d kernels\n" % (base, len(set(spilled))))
    elif spilled:
        raise RuntimeError("register spills in %s: %s" % (base, sorted(set(spilled))))
    return obj


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(force: bool = True, jobs: int = 8) -> str:
    srcs = sources()
    deps = srcs + glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(INCLUDE, "*.h"))
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    os.makedirs(OBJDIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, srcs))
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs,
                    "-Wl,-rpath,/opt/rocm/lib"], check=True)
    os.replace(tmp, LIB)
    return LIB


def build_sanitized(outdir: str, jobs: int = 8) -> str:
    """The library with its HOST code under AddressSanitizer and UndefinedBehaviorSanitizer (the device
    code is compiled as usual), for the host-only check of the argument-validation layer.  Returns the
    path of ``libcube3d_san.so`` in `outdir`."""
    os.makedirs(outdir, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]

    def one(src):
        obj = os.path.join(outdir, os.path.basename(src) + ".o")
        res = subprocess.run([HIPCC, *FLAGS, *san, "-c", src, "-o", obj], stderr=subprocess.PIPE, text=True)
        if res.returncode != 0:
            sys.stderr.write(res.stderr)
            raise subprocess.CalledProcessError(res.returncode, HIPCC)
        return obj
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(one, sources()))
    lib = os.path.join(outdir, "libcube3d_san.so")
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                    "-fno-gpu-sanitize", "-o", lib, *objs, "-Wl,-rpath,/opt/rocm/lib"], check=True)
    return lib


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
