"""Build libvq.so (the HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

try:
    from . import check_async
except ImportError:                      # run as a script
    import check_async

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libvq.so")
SOURCES = ["vq_api.hip", "vq_dequant.hip", "vq_dequant_fast.hip", "vq_gemv.hip", "vq_gemv_fast.hip", "vq_gemv_res8.hip", "vq_gemv_mfma.hip", "vq_gemm.hip", "vq_gemm_fused.hip", "vq_assign.hip", "vq_gemv_down.hip", "vq_gemv_down_mfma.hip", "vq_gemv_v8.hip", "vq_colperm.hip", "vq_quantize.hip", "vq_gemm_v6.hip", "vq_gemv_lds.hip", "vq_dequant_lds.hip", "vq_gemv_down_lds.hip"]
# packed-FP32 VALU forms are switched off for every device compile (they are not trusted on the test machines)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument"]
# Kernels in these files load registers asynchronously from inline assembly and wait for them with counted
# s_waitcnt.  The compiler does not know such a register is pending: if it spilled one, it would save the old
# contents.  Their kernels must therefore not spill at all; the build reads the compiler's resource remarks.
NO_SPILL = {"vq_gemv_mfma.hip", "vq_gemm_fused.hip", "vq_gemv_down.hip", "vq_gemv_down_mfma.hip", "vq_gemv_fast.hip", "vq_gemv_res8.hip", "vq_quantize.hip", "vq_gemm_v6.hip"}
# One exception, checked in the generated code of this image's compiler (ROCm 7.2): the 512-token GEMM tile saves
# five address registers at kernel entry, before its first asynchronous load, and reloads them in the epilogue.
SPILLS_ALLOWED = {"gemm_v8_kernelILi512E": 5}
REMARKS = ["-Rpass-analysis=kernel-resource-usage"]
# The same files, and the dot-product GEMV with its hand-issued LDS reads, get their device assembly audited for
# instructions that touch a register while an inline-assembly load into it is pending (check_async.py).
AUDITED = ["vq_gemv_mfma.hip", "vq_gemm_fused.hip", "vq_gemv_fast.hip", "vq_gemv_res8.hip", "vq_gemv_down.hip", "vq_gemv_down_mfma.hip", "vq_quantize.hip", "vq_gemm_v6.hip"]


# Files whose control-flow graphs hold paths that no run takes (two branches on the same loop-invariant value, taken
# differently) and on which the audit's queues therefore come up short: the number of cross-block findings when those paths
# were last read.  Their single-block findings still fail the build; every other file must come out clean across blocks.
# vq_gemv_mfma.hip: the variants with two 16-row blocks per chunk, whose unrolled pass loop tests "this wave has vectors in
# this group" and "chunks left" once per copy of its body.  vq_gemm_fused.hip: the dense kernel's loop exit, which the
# compiler tests separately from the "last step" branch that collects the reads in flight.
CROSS_BLOCK_KNOWN = {"vq_gemv_mfma.hip": 1472, "vq_gemm_fused.hip": 1}
# The compiler whose generated code the counted waits were last checked against (first line of `hipcc --version`).
VERIFIED_HIPCC = "HIP version: 7.2.26015-fc0010cf6a"


def hipcc_version(hipcc: str) -> str:
    try:
        return subprocess.run([hipcc, "--version"], stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True).stdout.splitlines()[0].strip()
    except (OSError, IndexError):
        return "unknown"


def check_no_spills(src: str, remarks: str) -> None:
    name = None
    for line in remarks.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].strip()
        elif "VGPRs Spill:" in line:
            n = int(line.split("Spill:")[1].split()[0])
            allowed = max([v for k, v in SPILLS_ALLOWED.items() if name and k in name] + [0])
            if n > allowed:
                raise RuntimeError("%s: kernel %s spills %d vector registers; it must not (asynchronous loads)" % (src, name, n))
        elif "ScratchSize" in line and "bytes/lane" in line:
            # arrays the compiler keeps in scratch memory (a run-time choice among registers does that) travel through the same
            # counters as the asynchronous loads and cost a trip to memory each
            n = int(line.split(":")[-1].split()[0])
            allowed = max([4 * v + 4 for k, v in SPILLS_ALLOWED.items() if name and k in name] + [0])
            if n > allowed:
                raise RuntimeError("%s: kernel %s uses %d bytes of scratch memory per lane; it must not" % (src, name, n))


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(HERE, "_build", src.replace(".hip", ".o"))
        cmd = [hipcc] + FLAGS + (REMARKS if src in NO_SPILL else []) + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        if src in NO_SPILL:
            check_no_spills(src, out)
            out = "\n".join(l for l in out.splitlines() if "remark:" not in l)
        if verbose and out.strip():
            print(out)
    def audit(src):
        asm = check_async.device_asm(hipcc, FLAGS, os.path.join(CSRC, src))
        return src, check_async.audit_blocks(asm), check_async.audit(asm)
    with ThreadPoolExecutor(max_workers=len(AUDITED)) as pool:
        for src, in_block, cross_block in pool.map(audit, AUDITED):
            findings = in_block if src in CROSS_BLOCK_KNOWN else cross_block
            if findings:
                name, label, text, regs = findings[0]
                raise RuntimeError("%s: %d instruction(s) touch a register with an asynchronous load pending, e.g. in %s %s: %s"
                                   % (src, len(findings), name, label, text))
            if src in CROSS_BLOCK_KNOWN and len(cross_block) != CROSS_BLOCK_KNOWN[src]:
                print("note: %s: %d cross-block findings of the asynchronous-load audit, %d when its paths were last read; "
                      "read the new ones (python check_async.py on the device assembly)" % (src, len(cross_block), CROSS_BLOCK_KNOWN[src]))
    if hipcc_version(hipcc) != VERIFIED_HIPCC:
        print("note: hipcc is '%s'; the counted waits of the kernels in %s were read against the code generated by '%s': "
              "run the GPU tests before relying on this build" % (hipcc_version(hipcc), ", ".join(AUDITED), VERIFIED_HIPCC))
    # no rpath: inside a PyTorch process the already-loaded HIP runtime (same soname) is the one used
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
