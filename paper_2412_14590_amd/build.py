"""Build libmixllm_hip.so (gfx950) in-tree with hipcc."""
import os
import re
import subprocess
import sys

try:
    from . import asm_scan
except ImportError:   # run as a plain script
    import asm_scan

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
         # (the direct-to-LDS load names m0, a register the compiler reserves, among its clobbers)
         "-Wall", "-Wno-unused-function", "-Wno-inline-asm", "-I", INCLUDE, "-I", CSRC] + os.environ.get("MIXLLM_EXTRA_FLAGS", "").split()


def _hipcc():
    for c in ("/opt/rocm/bin/hipcc", "hipcc"):
        if c == "hipcc" or os.path.exists(c):
            return c


# sources with hand-issued loads -> the kernels in them that must not spill
NO_SPILL = {"linear_prefill.hip": lambda n: "linear_prefill_kernel" in n,
            "linear_decode_split.hip": lambda n: "linear_decode_split_kernel" in n,
            "linear_mid.hip": lambda n: "linear_mid_kernel" in n}


def _check_no_scratch(src: str, compile_log: str) -> None:
    """Kernels that issue their loads by hand (every tiled kernel, every evenly split decode kernel,
    every kernel for a few dozen tokens, the debug variants included) must not spill: a register saved to
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


def _vregs(text: str) -> set:
    out = set()
    for a, b in re.findall(r"\bv\[(\d+):(\d+)\]", text):
        out |= set(range(int(a), int(b) + 1))
    out |= {int(a) for a in re.findall(r"\bv(\d+)\b", text)}
    return out


def check_hand_issued_loads(asm_text: str, name: str) -> None:
    """Scan the gfx950 assembly of a source with hand-issued loads: inside a basic block, between a
    load written in inline asm and the next inline-asm `s_waitcnt vmcnt`, no instruction of the
    compiler's may read or write the load's destination registers - the data is not there yet.
    (This is what happens when a hand-loaded variable is reinterpreted through memory: the compiler
    keeps it in pieces, splits the register right after the load and reassembles it for the wait.)
    Limits of the scan: it judges straight-line code only.  The set of pending registers is dropped
    at every label and branch, so a load issued before a loop's back edge and awaited after it is
    not followed around the edge; the kernels are written so that every wait that ties a register
    (await_loads / await_slot / tie_slot) sits in the same unrolled body as the first use, and the
    no-spill check above covers the other way a register could be touched early."""
    pending, in_asm, bad = {}, False, []
    for i, line in enumerate(asm_text.split("\n"), 1):
        t = line.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            continue
        if not t or t.startswith(";"):
            continue
        if t.startswith(".") or t.endswith(":") or t.startswith(("s_cbranch", "s_branch", "s_endpgm", "s_setpc")):
            pending = {}                      # basic block boundary: only straight-line code is judged
            continue
        if in_asm:
            if t.startswith("global_load_") and "_lds_" not in t:
                for r in _vregs(t.split(",")[0]):
                    pending[r] = i
            elif t.startswith("s_waitcnt vmcnt"):
                pending = {}
            continue
        hit = _vregs(t) & set(pending)
        if hit:
            bad.append(f"{name}.s:{i}: `{t[:70]}` touches v{sorted(hit)}, hand-loaded at line {pending[min(hit)]}")
    if bad:
        raise RuntimeError("registers of hand-issued loads are used before their wait:\n  " + "\n  ".join(bad[:10]))


# Sources whose kernels pass the path-following scan of asm_scan.py (every path through the control-flow
# graph, loop back edges included).  The others issue or await some loads under conditions the scan cannot
# relate to each other (the same uniform test before the load and before its wait), which it reports as
# paths without a wait; they get the straight-line scan above and the tripwire below.
FULL_SCAN = {"linear_prefill.hip"}
# Kernels that keep a ring of hand-issued loads in flight around a rolled loop: registers of the ring must
# stay where they are.  Where the loop nest makes the compiler rotate them (seen with the chunk loop of
# the evenly split decode kernel nested in a loop over activation windows: 80 to 220 copies, at the loop
# latch, of registers whose loads were still in flight; the late data then landed in registers that
# held addresses by then) the kernel has dozens of register-to-register copies of them; as built it
# has none, or a handful that copy a thread index into a register the ring used earlier.
RING_COPY_LIMIT = {"linear_decode_split.hip": ("linear_decode_split_kernel", 8)}


def check_ring_copies(asm_text: str, src: str) -> None:
    """Tripwire: count, per kernel, the VGPR-to-VGPR copies that name a destination register of a
    hand-issued load of the ring (the activation loads are consumed before the loop and their
    registers reused); fail above RING_COPY_LIMIT."""
    kernel, limit = RING_COPY_LIMIT[src]
    lines = asm_text.split("\n")
    for st in [i for i, l in enumerate(lines) if re.match(r"^_Z\S*" + kernel + r"\S*:", l)]:
        end = next((i for i in range(st, len(lines)) if "s_endpgm" in lines[i]), len(lines))
        hand, copies, in_asm = set(), [], False
        for l in lines[st:end]:
            t = l.strip()
            if t.startswith(";;#ASMSTART"):
                in_asm = True
            elif t.startswith(";;#ASMEND"):
                in_asm = False
            elif in_asm and (re.match(r"global_load_dwordx4 .* nt$", t) or t.startswith(("global_load_dwordx2", "global_load_ushort"))):
                hand |= _vregs(t.split(",")[0])   # weights (non-temporal) and their scales and zero points: the ring
            elif re.match(r"v_(mov_b(32|64)_e32|swap_b32) v[\[\d][^,]*, v[\[\d]", t):
                copies.append(t)
        n = sum(1 for c in copies if _vregs(c) & hand)
        if n > limit:
            raise RuntimeError(f"{lines[st].split(':')[0]}: {n} register copies of hand-loaded registers (limit {limit}): "
                               "the compiler is moving a ring of loads that may be in flight")


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source and link the shared library.  Objects are cached per source
    by modification time unless force is set."""
    # a build with extra flags (other launch constants, for measurements) keeps its objects apart from
    # the default build's and is always compiled afresh
    variant = bool(os.environ.get("MIXLLM_EXTRA_FLAGS", "").strip())
    objdir = os.path.join(HERE, "_build", "variant") if variant else os.path.join(HERE, "_build")
    force = force or variant
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
            try:
                _check_no_scratch(src, out)
            except RuntimeError:
                os.remove(os.path.join(objdir, src.replace(".hip", ".o")))   # a later build must not take it for up to date
                raise
            out = "\n".join(l for l in out.splitlines() if "kernel-resource-usage" not in l and not l.lstrip().startswith(("|", "^")) and not re.match(r"\s*\d+ \|", l))
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            failed = True
            print(f"--- {src} FAILED\n{out}", file=sys.stderr)
        elif out.strip() and verbose:
            print(f"--- {src}\n{out}")
    if failed:
        raise RuntimeError("hipcc failed")
    # second safety net for the sources with hand-issued loads: their device assembly is scanned
    asm_procs = []
    for src in NO_SPILL:
        a = os.path.join(objdir, src.replace(".hip", ".s"))
        o = os.path.join(objdir, src.replace(".hip", ".o"))
        if force or not os.path.exists(a) or os.path.getmtime(a) < os.path.getmtime(o):
            cmd = [_hipcc(), *FLAGS, "--cuda-device-only", "-S", os.path.join(CSRC, src), "-o", a]
            asm_procs.append((src, a, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, a, pr in asm_procs:
        out, _ = pr.communicate()
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc -S failed for {src}:\n{out}")
        try:
            text = open(a).read()
            check_hand_issued_loads(text, src)
            if src in FULL_SCAN:
                asm_scan.check_hand_issued_loads(text, src)
            if src in RING_COPY_LIMIT:
                check_ring_copies(text, src)
        except RuntimeError:
            for stale in (a, os.path.join(objdir, src.replace(".hip", ".o"))):   # a later build must check again
                if os.path.exists(stale):
                    os.remove(stale)
            raise
    subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    if variant:
        return LIB
    # the ceiling probes of the benchmark: a separate small library
    r = subprocess.run([_hipcc(), *FLAGS, "-shared", "-o", PROBE_LIB, os.path.join(CSRC, "probe.hip")],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        print(r.stdout, file=sys.stderr)
        raise RuntimeError("hipcc failed on probe.hip")
    return LIB


def build_sanitized_host(driver_cpp: str, exe: str) -> str:
    """Link `driver_cpp` with the library's sources compiled so that their HOST code carries
    AddressSanitizer and UndefinedBehaviorSanitizer (device code is compiled as always; the GPU
    sanitizers are not used).  For the CPU test that runs the host-side validation, size accounting
    and launch planning under the sanitizers."""
    objdir = os.path.join(HERE, "_build", "san")
    os.makedirs(objdir, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    procs, objs = [], []
    for src in SOURCES:
        s, o = os.path.join(CSRC, src), os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(o)
        if not os.path.exists(o) or os.path.getmtime(o) < max(os.path.getmtime(p) for p in (s, os.path.join(CSRC, "internal.h"),
                                                                                          os.path.join(CSRC, "async_loads.h"),
                                                                                          os.path.join(INCLUDE, "mixllm.h"), __file__)):
            procs.append((src, subprocess.Popen([_hipcc(), *FLAGS, *san, "-c", s, "-o", o], stdout=subprocess.PIPE,
                                                stderr=subprocess.STDOUT, text=True)))
    for src, pr in procs:
        out, _ = pr.communicate()
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc (host sanitizers) failed on {src}:\n{out}")
    clang = "/opt/rocm/lib/llvm/bin/clang++"
    drv = os.path.join(objdir, "driver.o")
    san_host = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]
    for cmd in ([clang, "-std=c++17", "-O1", *san_host, "-I", INCLUDE, "-c", driver_cpp, "-o", drv],
                [_hipcc(), "--offload-arch=gfx950", "-fno-gpu-sanitize", *san_host, "-o", exe, drv, *objs]):
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"{' '.join(cmd[:3])} ... failed:\n{r.stdout}")
    return exe


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
