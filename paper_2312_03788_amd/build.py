"""Build the HIP library (gfx950 only) in-tree: paper_2312_03788_amd/libsqp.so."""
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsqp.so")

SOURCES = ["sqp_api.hip", "sqp_companion.hip", "sqp_gemm_decode.hip", "sqp_gemm_prefill.hip", "sqp_gemm_slice.hip", "sqp_loss.hip", "sqp_mlp.hip", "sqp_static.hip"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-I" + os.path.join(ROOT, "include"),
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


# The GEMM kernels issue loads whose destination registers are written asynchronously and wait
# for them by hand (inline assembly): a register the compiler spilled or copied to scratch memory
# between issue and wait would silently hold stale data.  The build therefore checks the
# compiler's output for these kernels and fails otherwise:
#   decode kernel: no scratch memory and no spilled vector register at all (resource-usage remarks);
#   tiled kernel:  the compiler spills some store addresses of the epilogue; every scratch access
#                  must come after the kernel's last barrier, i.e. after the main loop and its
#                  final wait for all outstanding loads (checked in the generated assembly).
GUARDED_KERNELS = {"sqp_gemm_decode.hip": ("w4a16_decode_kernel", "none"),
                   "sqp_gemm_slice.hip": ("w4a16_decode_slice_kernel", "none"),
                   "sqp_gemm_prefill.hip": ("w4a16_prefill_kernel", "after-last-barrier")}


def _check_no_spills(src, remarks):
    """remarks: compiler output with -Rpass-analysis=kernel-resource-usage."""
    want, rule = GUARDED_KERNELS[src]
    name, seen, spilling = None, 0, set()
    for line in remarks.splitlines():
        if "[-Rpass-analysis=kernel-resource-usage]" not in line:
            continue
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            seen += want in name
            continue
        m = re.search(r"(ScratchSize \[bytes/lane\]|VGPRs Spill): (\d+)", line)
        if m and name and want in name and int(m.group(2)) != 0:
            if rule == "none":
                raise RuntimeError("%s: kernel %s has %s = %s; its hand-written waits assume none" % (src, name, m.group(1), m.group(2)))
            spilling.add(name)
    if seen == 0:
        raise RuntimeError("%s: no resource-usage remark for %s (compiler output changed?)" % (src, want))
    return spilling


def _check_scratch_after_last_barrier(src, asm_path, kernels):
    text = open(asm_path).read().splitlines()
    for k in kernels:
        start = next((i for i, l in enumerate(text) if l.startswith(k + ":")), None)
        if start is None:
            raise RuntimeError("%s: kernel %s not found in %s" % (src, k, asm_path))
        end = next(i for i in range(start, len(text)) if "s_endpgm" in text[i])
        body = text[start:end]
        barriers = [i for i, l in enumerate(body) if re.match(r"\s*s_barrier", l)]
        scratch = [i for i, l in enumerate(body) if re.match(r"\s*scratch_", l)]
        if not barriers or (scratch and min(scratch) < max(barriers)):
            raise RuntimeError("%s: kernel %s touches scratch memory inside its main loop; its hand-written waits "
                               "assume spills only in the epilogue" % (src, k))


def _compile(src):
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    guard = ["-Rpass-analysis=kernel-resource-usage", "-save-temps=obj"] if src in GUARDED_KERNELS else []
    cmd = ["hipcc"] + FLAGS + guard + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = [l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l]
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, "\n".join(lines)))
    if guard:
        spilling = _check_no_spills(src, r.stdout)
        if spilling:
            stem = os.path.splitext(src)[0]
            _check_scratch_after_last_barrier(src, os.path.join(OBJ, stem + "-hip-amdgcn-amd-amdhsa-gfx950.s"), spilling)
        keep, skip = [], 0
        for l in lines:  # drop the remarks (and the source excerpt lines that follow the first of each kernel)
            if "[-Rpass-analysis=kernel-resource-usage]" in l:
                skip = 2 if "Function Name" in l else 0
                continue
            if skip and re.match(r"\s+\d* *\|", l):
                skip -= 1
                continue
            keep.append(l)
        lines = keep
    out = "\n".join(lines)
    if out.strip():
        print(out, file=sys.stderr)
    return obj


def build(verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.run(cmd, check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
