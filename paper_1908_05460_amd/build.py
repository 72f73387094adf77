"""Builds libwgrad.so (the HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libwgrad.so")
ROOFS_LIB = os.path.join(HERE, "libwgrad_roofs.so")   # bench-only kernels that measure the machine's ceilings
SOURCES = ["api.hip", "exact_mfma.hip", "exact_stream.hip", "exact_stream_w1.hip", "exact_stream_w2.hip",
           "exact_stream_w4.hip", "exact_multi.hip", "exact_bf16.hip", "exact_bf16_planes.hip", "exact_direct.hip", "exact_plane2.hip", "approx.hip", "approx_topk.hip", "combine.hip",
           "fill.hip", "layouts.hip"]
# packed fp32 VALU forms are switched off on purpose (they have misbehaved on the test machines)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build(extra_flags=(), out=LIB, objdir=None, verbose=False):
    objdir = objdir or os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    cc = hipcc()

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [cc, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                         if "packed-fp32-ops" not in l or "error" in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{msgs}")
        if verbose and msgs.strip():
            print(msgs, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    # -no-hip-rt: the library does not name a HIP runtime of its own; it binds to the one the
    # host process has already loaded (a process must never run two HIP runtimes side by side,
    # and PyTorch wheels bundle theirs).  A plain C program links -lamdhip64 itself.
    subprocess.run([cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-no-hip-rt", "-o", out, *objs], check=True)
    if out == LIB:
        roofs = compile_one("roofs.hip")
        subprocess.run([cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-no-hip-rt", "-o", ROOFS_LIB, roofs], check=True)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
