"""Compile the HIP kernels and the C ABI into paper_2510_08055_amd/libmoe_lp.so (gfx950 only).

hipcc cross-compiles without a GPU.  Objects go to paper_2510_08055_amd/_build/ (not committed);
the shared library is built in-tree so that it travels with the source tree.
"""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmoe_lp.so")
SOURCES = ["api.hip", "router.hip", "permute.hip", "ffn.hip", "ffn_w4.hip", "combine.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


# Kernels in these files issue loads from inline asm whose results are picked up after an explicit wait.
# The register allocator takes such a result for ready at once: if it ever spilled one, it would save a
# register the load has not written yet, and the load would later land on whatever the register holds by
# then (an address, say).  So these kernels must compile without any scratch memory; the build checks it.
NO_SCRATCH = {"router.hip": ("router_logits_kernel",), "ffn_w4.hip": ("grouped_gemm_w4_stream_kernel",),
              "ffn.hip": ("grouped_gemm_bf16_pipe_kernel",)}


def _scratch_users(log, names):
    """Kernels (mangled names containing one of `names`) whose resource remarks report scratch or spills."""
    bad, cur = [], None
    for line in log.splitlines():
        if "Function Name:" in line:       # "remark: <file>:<line>:<col>: Function Name: ..." or "<file>:<line>:<col>: remark: Function Name: ..."
            cur = line.split("Function Name:")[1].split()[0]
        elif cur and any(n in cur for n in names):
            for key in ("ScratchSize [bytes/lane]:", "VGPRs Spill:"):
                if key in line and int(line.split(key)[1].split()[0]) != 0:
                    bad.append(f"{cur}: {key} {line.split(key)[1].split()[0]}")
    return bad


# Files whose kernels issue their direct-to-LDS loads from inline asm that writes M0 (the LDS base of such a
# load).  The compiler does not honour an M0 clobber on an asm statement, so these files must hold no other
# use of M0; the build reads the device assembly (a by-product of the same compile) and checks that M0
# only ever appears as  s_mov_b32 m0, <sgpr> ; s_nop 0 ; global_load_lds_<size>.
M0_ONLY_FOR_LDS_LOADS = ("ffn.hip", "ffn_w4.hip")


def _foreign_m0_uses(asm):
    """Lines of the device assembly that touch M0 in any way other than the asm-issued LDS loads."""
    code = [l.strip() for l in asm.splitlines()]
    code = [l for l in code if l and not l.startswith((";", ".", "//")) and not l.endswith(":")]
    bad = []
    for i, l in enumerate(code):
        if "m0" not in l.split(";")[0].replace(",", " ").split():
            continue
        nxt = [c.split(";")[0].split() for c in code[i + 1:i + 3]]
        ok = (l.split(";")[0].replace(",", " ").split()[:2] == ["s_mov_b32", "m0"] and len(nxt) == 2
              and nxt[0] == ["s_nop", "0"] and nxt[1][0].startswith("global_load_lds_"))
        if not ok:
            bad.append(l)
    return bad


# Kernels of these files load single dwords into registers from inline asm (`global_load_dword vN, ...`
# between the compiler's #ASMSTART / #ASMEND markers) and pick the value up after an explicit
# `s_waitcnt vmcnt`.  In the assembly, nothing between such a load and the next vmcnt wait may name vN.
ASYNC_DWORD_LOADS = {"ffn.hip": "grouped_gemm_bf16_pipe_kernel", "ffn_w4.hip": "grouped_gemm_w4_stream_kernel"}


def _early_uses_of_async_loads(asm, kernel):
    """Instructions that name the destination of an asm-issued global_load_dword before the next vmcnt wait,
    in every function whose (mangled) name contains `kernel`; the scan follows the listing, not the branches."""
    import re
    bad, cur, in_asm, pending = [], None, False, {}
    for line in asm.splitlines():
        m = re.match(r"^(_Z\S+):", line)
        if m:
            cur, in_asm, pending = (m.group(1) if kernel in m.group(1) else None), False, {}
            continue
        if cur is None:
            continue
        if "#ASMSTART" in line:
            in_asm = True
            continue
        if "#ASMEND" in line:
            in_asm = False
            continue
        code = line.split(";")[0].strip()
        if not code or code.startswith(".") or code.endswith(":"):
            continue
        if "s_waitcnt" in code and "vmcnt" in code:
            pending = {}
            continue
        named = set(int(r) for r in re.findall(r"\bv(\d+)\b", code))
        for lo, hi in re.findall(r"\bv\[(\d+):(\d+)\]", code):
            named.update(range(int(lo), int(hi) + 1))
        hit = sorted(named & set(pending))
        m = re.match(r"global_load_dword v(\d+), v\[", code) if in_asm else None
        if m:
            hit = [r for r in hit if r != int(m.group(1))]
        if hit:
            bad.append(f"{cur[:60]}...: v{hit[0]} (loaded asynchronously) named by: {code}")
        if m:
            pending[int(m.group(1))] = True
    return bad


def _compile(src, verbose):
    out = os.path.join(OBJ, src.replace(".hip", ".o"))
    extra = ["-Rpass-analysis=kernel-resource-usage"] if src in NO_SCRATCH else []
    if src in M0_ONLY_FOR_LDS_LOADS:
        extra.append("-save-temps=obj")
    cmd = ["hipcc", *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}")
    if src in NO_SCRATCH:
        bad = _scratch_users(r.stdout, NO_SCRATCH[src])
        if bad:
            raise RuntimeError(f"{src}: kernels with asynchronous register loads must not use scratch memory:\n  "
                               + "\n  ".join(bad))
    if src in M0_ONLY_FOR_LDS_LOADS:
        asm_path = os.path.join(OBJ, src.replace(".hip", "-hip-amdgcn-amd-amdhsa-gfx950.s"))
        with open(asm_path) as f:
            bad = _foreign_m0_uses(f.read())
        if bad:
            raise RuntimeError(f"{src}: M0 is used outside the asm-issued direct-to-LDS loads:\n  " + "\n  ".join(bad[:10]))
        if src in ASYNC_DWORD_LOADS:
            with open(asm_path) as f:
                bad = _early_uses_of_async_loads(f.read(), ASYNC_DWORD_LOADS[src])
            if bad:
                raise RuntimeError(f"{src}: an asynchronously loaded register is used before its wait:\n  "
                                   + "\n  ".join(bad[:10]))
    # the host pass does not know the GPU-only target feature (that warning is expected); the resource
    # remarks are only read by the check above
    log = "\n".join(l for l in r.stdout.splitlines()
                    if "packed-fp32-ops" not in l and "kernel-resource-usage" not in l)
    if verbose and log.strip():
        print(log, flush=True)
    return out


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, verbose), SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
