"""Build libmixllm_hip.so (gfx950) in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.environ.get("MIXLLM_LIB_OUT", os.path.join(HERE, "libmixllm_hip.so"))
PROBE_LIB = os.path.join(HERE, "libmixllm_probe.so")
SOURCES = ["api.hip", "quant_act.hip", "quant_weights.hip", "linear_generic.hip",
           "linear_decode.hip", "linear_prefill.hip"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # correctly rounded fp32 division: the quantizers must match IEEE division bit for bit
         "-fhip-fp32-correctly-rounded-divide-sqrt", "-ffp-contract=off",
         # no compiler-generated packed fp32 arithmetic
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-I", INCLUDE, "-I", CSRC] + os.environ.get("MIXLLM_EXTRA_FLAGS", "").split()


def _hipcc():
    for c in ("/opt/rocm/bin/hipcc", "hipcc"):
        if c == "hipcc" or os.path.exists(c):
            return c


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source and link the shared library.  Objects are cached per source
    by modification time unless force is set."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    deps = [os.path.join(CSRC, "internal.h"), os.path.join(INCLUDE, "mixllm.h"), __file__]
    dep_m = max(os.path.getmtime(p) for p in deps)
    objs, procs = [], []
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(o)
        if force or not os.path.exists(o) or os.path.getmtime(o) < max(os.path.getmtime(s), dep_m):
            cmd = [_hipcc(), *FLAGS, "-c", s, "-o", o]
            if verbose:
                print(" ".join(cmd))
            procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            failed = True
            print(f"--- {src} FAILED\n{out}", file=sys.stderr)
        elif out.strip() and verbose:
            print(f"--- {src}\n{out}")
    if failed:
        raise RuntimeError("hipcc failed")
    subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    # the ceiling probes of the benchmark: a separate small library
    r = subprocess.run([_hipcc(), *FLAGS, "-shared", "-o", PROBE_LIB, os.path.join(CSRC, "probe.hip")],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        print(r.stdout, file=sys.stderr)
        raise RuntimeError("hipcc failed on probe.hip")
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
