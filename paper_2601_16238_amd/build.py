"""Build libmi355attn.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libmi355attn.so")
# (source, extra flags, object): the kernel sources are built once per element type
SOURCES = [("attn_api.hip", [], "attn_api.o"),
           ("attn_fwd.hip", [], "attn_fwd.o"), ("attn_bwd.hip", [], "attn_bwd.o"),
           ("attn_fwd_wide.hip", [], "attn_fwd_wide.o"),
           ("attn_bwd_small.hip", [], "attn_bwd_small.o"),
           ("attn_bwd_small.hip", ["-DATTN_F16"], "attn_bwd_small_f16.o"),
           ("attn_fwd_wide.hip", ["-DATTN_F16"], "attn_fwd_wide_f16.o"),
           ("attn_fwd.hip", ["-DATTN_F16"], "attn_fwd_f16.o"),
           ("attn_bwd.hip", ["-DATTN_F16"], "attn_bwd_f16.o"),
           ("rowops.hip", [], "rowops.o"), ("probe.hip", [], "probe.o")]
# -packed-fp32-ops: never let the compiler form v_pk_*_f32 instructions.
# -fno-honor-nans (device only): fmaxf lowers to bare v_max/v_max3 without canonicalising
# moves; the kernels never produce or test NaNs.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=fast",
         "-Xarch_device", "-fno-honor-nans",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def _hipcc():
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    raise RuntimeError("hipcc not found")


def build(verbose=False, resource_usage=False, extra_flags=(), lib_path=LIB):
    """Compile every HIP source and link the shared library.  Always recompiles.
    `extra_flags` (e.g. a -D switch of an experiment) and `lib_path` serve development builds
    that must not replace the in-tree library."""
    os.makedirs(OBJ, exist_ok=True)
    cc = _hipcc()

    def one(job):
        src, extra, objname = job
        obj = os.path.join(OBJ, objname)
        cmd = [cc] + FLAGS + list(extra_flags) + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
        if resource_usage:
            cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(ln for ln in res.stdout.splitlines()
                        if "packed-fp32-ops" not in ln)  # host pass does not know the feature
        if res.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s" % (src, out))
        if (verbose or resource_usage) and out.strip():
            print(out)
        return obj

    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(one, SOURCES))
    tmp = lib_path + ".tmp%d" % os.getpid()
    subprocess.check_call([cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
    os.replace(tmp, lib_path)
    return lib_path


if __name__ == "__main__":
    build(verbose=True, resource_usage="--usage" in sys.argv)
    print("built", LIB)
