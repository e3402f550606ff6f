"""Build libbcq.so (HIP, gfx950 only) in-tree with hipcc."""
import glob
import os
import re
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libbcq.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


TRACE_LIB = os.path.join(HERE, "libbcq_trace.so")


def sources():
    """Sources of libbcq.so: every .hip file except the tracing build's entry points."""
    return sorted(f for f in glob.glob(os.path.join(CSRC, "*.hip")) if not f.endswith("bcq_trace_api.hip"))


def build_trace(verbose=False):
    """libbcq_trace.so: the GEMV compiled with per-wave time stamps (-DBCQ_TRACE), for trace_gemv.py."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    srcs = [os.path.join(CSRC, f) for f in ("bcq_gemv.hip", "bcq_gemv2.hip", "bcq_skinny.hip", "bcq_lut4.hip", "bcq_pack.hip", "bcq_trace_api.hip")]
    cmd = [hipcc] + HIPCC_FLAGS + ["-DBCQ_TRACE"] + srcs + ["-o", TRACE_LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True, stderr=subprocess.DEVNULL if not verbose else None)
    return TRACE_LIB


def build_probes(verbose=False):
    """Compile the stand-alone hardware probes under probes/ (diagnostics; nothing in the library uses them)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = []
    pdir = os.path.join(HERE, "probes")
    for f in sorted(os.listdir(pdir)):
        if not f.endswith(".hip"):
            continue
        exe = os.path.join(pdir, f[:-4])
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               os.path.join(pdir, f), "-o", exe]
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True, stderr=subprocess.DEVNULL if not verbose else None)
        out.append(exe)
    return out


def kernel_resources(stderr_text):
    """Parse the compiler's kernel-resource-usage remarks: {mangled name: {field: int}}."""
    res, cur = {}, None
    for line in stderr_text.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            cur = res.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z ]+?)(?: \[[^\]]*\])?: (\d+) \[-Rpass", line)
        if m and cur is not None:
            cur[m.group(1).strip()] = int(m.group(2))
    return res


def build(verbose=False, extra_flags=()):
    """Compile every kernel for gfx950 and link libbcq.so.  Fails if a compute kernel (GEMV,
    skinny GEMM) needs scratch memory or spills registers: those kernels are sized to keep
    everything in registers, and a spill would silently cost HBM traffic."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-Rpass-analysis=kernel-resource-usage"] + list(extra_flags) + sources() \
        + ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    proc = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    noise = ("-Rpass-analysis=kernel-resource-usage", "packed-fp32-ops", "warning generated", "warnings generated")
    other, skip = [], 0
    for line in proc.stderr.splitlines():
        if skip:  # the two source-excerpt lines that follow a located remark
            skip -= 1
            if re.match(r"\s+\d* *\|", line):
                continue
        if any(n in line for n in noise):
            skip = 2 if "Function Name" in line else 0
            continue
        other.append(line)
    if other:
        print("\n".join(other))
    if proc.returncode != 0:
        raise subprocess.CalledProcessError(proc.returncode, cmd)
    res = kernel_resources(proc.stderr)
    hot = {k: v for k, v in res.items() if "bcq_gemv" in k or "bcq_skinny" in k or "bcq_lut4" in k}
    if not hot:
        raise RuntimeError("no resource remarks for the compute kernels: cannot check for spills")
    bad = {k: v for k, v in hot.items()
           if v.get("ScratchSize", 0) or v.get("VGPRs Spill", 0) or v.get("SGPRs Spill", 0)}
    if bad:
        raise RuntimeError(f"compute kernels use scratch or spill registers: {bad}")
    if verbose:
        for k, v in sorted(hot.items()):
            print(f"{k}: VGPRs {v.get('VGPRs')} AGPRs {v.get('AGPRs')} occupancy {v.get('Occupancy')}")
    return LIB


if __name__ == "__main__":
    import sys
    if "--probes" in sys.argv:
        print(build_probes(verbose=True))
    else:
        print(build_trace(verbose=True) if "--trace" in sys.argv else build(verbose=True))
