"""Build libmixllm_hip.so (gfx950) in-tree with hipcc."""
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.environ.get("MIXLLM_LIB_OUT", os.path.join(HERE, "libmixllm_hip.so"))
PROBE_LIB = os.path.join(HERE, "libmixllm_probe.so")
SOURCES = ["api.hip", "quant_act.hip", "quant_weights.hip", "linear_generic.hip",
           "linear_decode.hip", "linear_decode_split.hip", "linear_mid.hip", "linear_prefill.hip", "salience.hip"]

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


# sources with hand-issued loads -> the kernels in them that must not spill
NO_SPILL = {"linear_prefill.hip": lambda n: "linear_prefill_kernel" in n and "ELb0ELb1ELb1EEEv" in n,
            "linear_decode_split.hip": lambda n: "linear_decode_split_kernel" in n,
            "linear_mid.hip": lambda n: "linear_mid_kernel" in n}


def _check_no_scratch(src: str, compile_log: str) -> None:
    """Kernels that issue their loads by hand (the prefill variant with template flags DUMP=0,
    ACT_PT=1, W8PC=1; every evenly split decode kernel) must not spill: a register saved to
    scratch between such a load and its wait would be saved before the data has arrived.  Their
    sources are compiled with -Rpass-analysis=kernel-resource-usage; fail the build if one of
    those kernels reports scratch."""
    found = 0
    for m in re.finditer(r"Function Name: (\S+).*?ScratchSize \[bytes/lane\]: (\d+)", compile_log, re.S):
        name, scratch = m.group(1), int(m.group(2))
        if NO_SPILL[src](name):
            found += 1
            if scratch != 0:
                raise RuntimeError(f"{name} spills {scratch} bytes: hand-issued loads are unsafe in it")
    if found == 0:
        raise RuntimeError(f"no resource-usage remark for the hand-issued-load kernels of {src}")


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source and link the shared library.  Objects are cached per source
    by modification time unless force is set."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    deps = [os.path.join(CSRC, "internal.h"), os.path.join(CSRC, "async_loads.h"), os.path.join(INCLUDE, "mixllm.h"), __file__]
    dep_m = max(os.path.getmtime(p) for p in deps)
    objs, procs = [], []
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(o)
        if force or not os.path.exists(o) or os.path.getmtime(o) < max(os.path.getmtime(s), dep_m):
            cmd = [_hipcc(), *FLAGS, "-c", s, "-o", o]
            if src in NO_SPILL:
                cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
            if verbose:
                print(" ".join(cmd))
            procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, pr in procs:
        out, _ = pr.communicate()
        if src in NO_SPILL and pr.returncode == 0:
            _check_no_scratch(src, out)
            out = "\n".join(l for l in out.splitlines() if "kernel-resource-usage" not in l and not l.lstrip().startswith(("|", "^")) and not re.match(r"\s*\d+ \|", l))
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
