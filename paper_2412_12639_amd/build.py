"""Compile the HIP library for gfx950, in-tree (hipcc cross-compiles without a GPU).

The kernels are instantiated per (element type, head size) pair in csrc/fv_step.hip, compiled four
times with different -D settings; those objects and csrc/falcon_verify.hip (the C ABI) are built in
parallel into _build/ and linked into libfalcon_verify.so."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libfalcon_verify.so")
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
DEPS = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC)) + \
    [os.path.join(os.path.dirname(HERE), "include", "falcon_verify.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
UNITS = [("falcon_verify", "falcon_verify.hip", []), ("fv_draft", "fv_draft.hip", [])] + \
    [(f"fv_step_{el.lower()}_d{d}", "fv_step.hip", [f"-DFV_INST_EL={el}", f"-DFV_INST_D={d}"])
     for el in ("BF16", "F32") for d in (128, 64)]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if err.strip():
        sys.stderr.write(err + "\n")


def build(force: bool = True, verbose: bool = False, extra_flags=()) -> str:
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in DEPS):
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    objs = [os.path.join(OBJ, name + ".o") for name, _, _ in UNITS]
    jobs = [[hipcc, *FLAGS, *extra_flags, *defs, "-c", os.path.join(CSRC, src), "-o", obj]
            for (_, src, defs), obj in zip(UNITS, objs)]
    with ThreadPoolExecutor(min(len(jobs), os.cpu_count() or 1)) as ex:
        list(ex.map(lambda c: _run(c, verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], verbose)
    return LIB


def build_probe(verbose: bool = False):
    """The stand-alone GEMM timing aid (probe/fv_gemm_probe.hip): plain, with per-wavefront time stamps, and with the
    activation and/or weight requests taken out of the streaming loop."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    src = os.path.join(HERE, "probe", "fv_gemm_probe.hip")
    variants = [("", []), ("_stamps", ["-DFV_PROBE_STAMPS"]), ("_no_x", ["-DFV_PROBE_NO_X"]), ("_no_w", ["-DFV_PROBE_NO_W"]),
                ("_no_loads", ["-DFV_PROBE_NO_X", "-DFV_PROBE_NO_W"]), ("_no_loads_stamps", ["-DFV_PROBE_NO_X", "-DFV_PROBE_NO_W", "-DFV_PROBE_STAMPS"]),
                # the same for a 32-token step (one block of tokens instead of two)
                ("_t32", ["-DFV_PROBE_TB=1"]), ("_t32_no_x", ["-DFV_PROBE_TB=1", "-DFV_PROBE_NO_X"]),
                ("_t32_no_loads", ["-DFV_PROBE_TB=1", "-DFV_PROBE_NO_X", "-DFV_PROBE_NO_W"])]
    outs = [(os.path.join(HERE, "probe", "fv_gemm_probe" + suffix), defs) for suffix, defs in variants]
    flags = [f for f in FLAGS if f != "-fPIC"]
    with ThreadPoolExecutor(min(len(outs), os.cpu_count() or 1)) as ex:
        list(ex.map(lambda o: _run([hipcc, *flags, *o[1], src, "-o", o[0]], verbose), outs))
    return [o[0] for o in outs]


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
    if "probe" in sys.argv:
        print(build_probe(verbose="-v" in sys.argv))
