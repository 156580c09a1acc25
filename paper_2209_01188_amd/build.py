"""Compile the HIP sources into paper_2209_01188_amd/libpetals_span.so (gfx950 only)."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpetals_span.so")
OBJ = os.path.join(HERE, "_build")
SOURCES = ["api.hip", "api_backward.hip", "quant.hip", "gemv.hip", "gemm.hip", "gemm_lds.hip", "attn.hip", "client.hip", "backward.hip", "microbench.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 ops are disabled on the test machines.
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
# the quantizers' fp32 expressions decide int8 codes: never let the compiler fuse them
EXTRA = {"quant.hip": ["-ffp-contract=off"]}


def _stale(dst, deps):
    return not os.path.exists(dst) or any(os.path.getmtime(d) > os.path.getmtime(dst) for d in deps)


def build(force=True, verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers.append(os.path.join(os.path.dirname(HERE), "include", "petals_span.h"))
    headers.append(os.path.join(os.path.dirname(HERE), "include", "petals_client.h"))
    jobs = []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ, s.replace(".hip", ".o"))
        if force or _stale(obj, [src] + headers):
            jobs.append([HIPCC] + FLAGS + EXTRA.get(s, []) + ["-c", src, "-o", obj])

    def run(cmd):
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), err))
        if verbose and err.strip():
            print(err)

    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as ex:
        list(ex.map(run, jobs))
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]
    if force or jobs or _stale(LIB, objs):
        run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
