"""Compile libs3kv.so (HIP kernels + host bookkeeping) for gfx950, in-tree."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libs3kv.so")
# (source, extra defines, object name); the multi-head attention kernels are one object per head dimension
HEAD_DIMS = (64, 96, 128, 256)
UNITS = [("s3kv_attn_inst.hip", [f"-DS3_INST_D={d}"], f"s3kv_attn_d{d}.o") for d in HEAD_DIMS] + [
    (s, [], s + ".o") for s in ("s3kv_kernels.hip", "s3kv_gqa.hip", "s3kv_gqa_mfma.hip", "s3kv_fp8.hip", "s3kv_alloc.cpp",
                                "s3kv_sched.cpp")]
HEADERS = ["s3kv_internal.h", "s3kv_device.h", "s3kv_attn.h"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build_lib(force: bool = True, verbose: bool = False) -> str:
    """Compile every source to an object (in parallel, one hipcc each), then link the shared library."""
    from concurrent.futures import ThreadPoolExecutor

    srcs = sorted({os.path.join(CSRC, u[0]) for u in UNITS})
    deps = srcs + [os.path.join(CSRC, h) for h in HEADERS] + [os.path.join(ROOT, "include", "s3kv.h")]
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
             # keep the compiler from forming packed-fp32 instructions
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             # fuse a*b+c only inside one expression: the max-subtracted exponent s - max(s) must stay
             # an exact zero for the largest score (cross-statement fusing would turn it into a residual)
             "-ffp-contract=on",
             "-Wall", "-Wno-unused-function",
             "-I", os.path.join(ROOT, "include"), "-I", CSRC]

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + out)
        if verbose and out.strip():
            print(out, flush=True)

    objs = [os.path.join(objdir, u[2]) for u in UNITS]
    with ThreadPoolExecutor(max_workers=min(len(UNITS), int(os.environ.get("MAX_JOBS", "8")))) as pool:
        list(pool.map(lambda u: run([_hipcc()] + flags + u[1] + ["-c", "-x", "hip", os.path.join(CSRC, u[0]), "-o",
                                                              os.path.join(objdir, u[2])]), UNITS))
    tmp = LIB + ".tmp"
    run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", tmp])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
