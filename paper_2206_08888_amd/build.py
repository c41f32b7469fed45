"""Build the HIP library in-tree: python -m paper_2206_08888_amd.build [--trace] [extra hipcc flags]

Every source under csrc/ is compiled for gfx950 with hipcc and linked into
paper_2206_08888_amd/libpop.so.  Packed fp32 VALU ops are switched off for all
device code.  --trace also builds libpop_trace.so, the same library as one
translation unit with the timeline instrumentation compiled in (csrc/trace_unity.hip;
paper_2206_08888_amd/timeline.py uses it).
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libpop.so")
TRACE_LIB = os.path.join(HERE, "libpop_trace.so")
SOURCES = ["pop_api.hip", "k_replay.hip", "k_init.hip", "k_chain.hip", "k_wgrad_adam.hip", "k_step.hip", "k_sac.hip", "k_wgrad_shared.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wno-unused-command-line-argument", "-Wno-pass-failed",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines()
                    if "packed-fp32-ops' is not a recognized feature" not in l)
    if p.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose=False, extra_flags=(), trace=False):
    os.makedirs(OBJ, exist_ok=True)
    cc = _hipcc()
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]

    def one(pair):
        src, obj = pair
        if src is None:                                    # the traced library: one translation unit, compiled and linked at once
            return _run([cc, *FLAGS, *extra_flags, "-shared", os.path.join(CSRC, "trace_unity.hip"), "-o", TRACE_LIB])
        return _run([cc, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj])

    jobs = ([(None, None)] if trace else []) + list(zip(SOURCES, objs))      # the long job first
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        logs = list(ex.map(one, jobs))
    logs.append(_run([cc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs]))
    if verbose:
        print("\n".join(l for l in logs if l.strip()))
    return LIB


if __name__ == "__main__":
    flags = [a for a in sys.argv[1:] if a != "--trace"]
    print(build(verbose=True, extra_flags=flags, trace="--trace" in sys.argv[1:]))
