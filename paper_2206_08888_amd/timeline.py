"""Where the time of an update step goes, from block timestamps: python -m paper_2206_08888_amd.timeline [--config N] [--P n] ...

Runs the traced build of the library (libpop_trace.so: `python -m paper_2206_08888_amd.build --trace`), in which
every workgroup of the update step's kernels records the constant-rate clock (100 MHz) when it starts and when it
ends, on a synthetic population of the chosen workload, and prints per launch and per part of a launch: number of
workgroups, first start, last end, and the spread of the workgroups' own durations, in microseconds from the start
of the step's first workgroup.  The summaries under profiles/ named *_timeline.txt are its output.

The traced library is the product's sources as one translation unit with a few clock reads per workgroup added: the
arithmetic is unchanged, the times are some per cent above those of the library proper.
"""
import argparse
import ctypes as C
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

KINDS = ("step (single launch)", "target + critic chains", "critic weight-gradient tiles", "actor chains",
         "actor weight-gradient tiles", "target chains", "critic chains")
TICK_US = 0.01


def _stats(start, end, t0):
    run = end > 0
    if not run.any():
        return None
    s, e = (start[run] - t0) * TICK_US, (end[run] - t0) * TICK_US
    d = e - s
    return dict(n=int(run.sum()), first=float(s.min()), last_start=float(s.max()), end=float(e.max()),
                d_min=float(d.min()), d_med=float(np.median(d)), d_max=float(d.max()))


def _line(name, st):
    return ("  %-34s %6d workgroups  start %7.1f .. %7.1f  last end %7.1f  |  own duration min %6.1f  median %6.1f  max %6.1f"
            % (name, st["n"], st["first"], st["last_start"], st["end"], st["d_min"], st["d_med"], st["d_max"]))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--P", type=int, default=None)
    ap.add_argument("--capacity", type=int, default=50_000, help="replay rows per agent (the timeline does not depend on it)")
    ap.add_argument("--launch", type=int, default=0, help="pop_tuning.launch (0: the library's choice)")
    ap.add_argument("--steps", type=int, default=4, help="steps traced one by one after the warm-up")
    ap.add_argument("--marks", type=int, default=None, metavar="BLOCK",
                    help="also print the phase marks (POP_MARK sites of the kernels) that workgroup BLOCK of each launch passed")
    args = ap.parse_args()
    import torch
    import paper_2206_08888_amd as pp
    from paper_2206_08888_amd import build
    import workloads
    assert torch.cuda.is_available(), "the timeline needs a GPU"
    lib = pp.load_library(build.TRACE_LIB)
    kinds, blocks = C.c_int32(), C.c_int32()
    lib.pop_trace_dims(C.byref(kinds), C.byref(blocks))
    K, N = kinds.value, blocks.value
    c = dict(workloads.CONFIGS[args.config])
    P = c["P"] if args.P is None else args.P
    algo = {"sac": pp.POP_ALGO_SAC, "td3": pp.POP_ALGO_TD3, "td3_shared": pp.POP_ALGO_TD3_SHARED}[c["algo"]]
    cfg = pp.make_config(P, c["obs_dim"], c["act_dim"], c["hidden"], c["batch"], args.capacity, algo=algo, launch=args.launch)
    pop = pp.Population(cfg, workloads.hparams(args.config, P))
    gen = torch.Generator(device="cuda"); gen.manual_seed(1)
    O, A, n = c["obs_dim"], c["act_dim"], args.capacity
    pop.insert(-1, obs=torch.randn((P, n, O), generator=gen, device="cuda"), act=torch.rand((P, n, A), generator=gen, device="cuda") * 2 - 1,
               rew=torch.randn((P, n), generator=gen, device="cuda"), done=(torch.rand((P, n), generator=gen, device="cuda") < 0.01).float(),
               next_obs=torch.randn((P, n, O), generator=gen, device="cuda"))
    pop.update(20)
    pop.sync()
    print("timeline of one update step: config %d (%s), P = %d, obs %d, act %d; times in us from the step's first workgroup"
          % (args.config, c["algo"], P, O, A))
    buf = np.zeros((K, 2, N), dtype=np.uint64)
    parts = (C.c_int32 * 6)()
    marks = np.zeros(64, dtype=np.uint64)
    if args.marks is not None:
        lib.pop_trace_select_block(args.marks)
    for s in range(args.steps):
        lib.pop_trace_reset()
        t = pop.step_count()
        pop.update(1)
        pop.sync()
        assert lib.pop_trace_block_times(buf.ctypes.data_as(C.c_void_p)) == 0
        ran = buf[:, 1, :] > 0
        t0 = int(buf[:, 0, :][ran].min())
        print("step %d (%s):" % (t, "with the delayed actor part" if t % 2 == 0 or c["algo"] == "sac" else "critics only"))
        for k in range(K):
            st = _stats(buf[k, 0].astype(np.int64), buf[k, 1].astype(np.int64), t0)
            if st is None:
                continue
            print(_line(KINDS[k] if k < len(KINDS) else "kind %d" % k, st))
            if k == 0:                                     # the single launch: its parts are ranges of block ids
                lib.pop_trace_step_parts(parts)
                lo = 0
                for name, cnt in zip(("target chains", "critic chains", "critic weight-gradient tiles", "actor chains",
                                      "actor weight-gradient tiles", "gather of the next step"), list(parts)):
                    if cnt:
                        sp = _stats(buf[0, 0, lo:lo + cnt].astype(np.int64), buf[0, 1, lo:lo + cnt].astype(np.int64), t0)
                        if sp:
                            print(_line("    " + name, sp))
                    lo += cnt
        if args.marks is not None:
            lib.pop_trace_marks(marks.ctypes.data_as(C.c_void_p))
            seen = sorted((int(v), i) for i, v in enumerate(marks) if v)
            print("  marks passed by workgroups with block id %d (mark: us from the step's first workgroup; the kernels of a step share "
                  "the mark numbers): %s" % (args.marks, "  ".join("%d: %.1f" % (i, (v - t0) * TICK_US) for v, i in seen)))
    pop.close()


if __name__ == "__main__":
    main()
