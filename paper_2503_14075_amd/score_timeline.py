"""Diagnostics of the register-resident pruning-score kernel on the bench launch (cfg1 x 128), from
the diagnostic build of the library (`python -m paper_2503_14075_amd.build --trace`, which writes
libtwigpath_trace.so):

    python -m paper_2503_14075_amd.score_timeline [--ladder]

Timeline: lane 0 of every wavefront records the 100 MHz wall clock at eight points of each of its
first 16 (sequence, head) pairs; the report gives the mean and the spread of every phase over all
workgroups, wavefronts and pairs 2..14, and one workgroup's pair wavefront by wavefront.
With --ladder: the launch timed with parts of its work switched off at run time (TW_SCORE_DRY of
the diagnostic build: 1 no matrix products / row maxima, 2 also no exponentials, 3 also no column
sums, 4 also no Q traffic = the bare K stream with its staging and barrier), each level in a child
process, with the compaction and verification launches of a step between the timed launches.
Nothing here is part of the method; it exists so that what is said about where this kernel's
time goes can be re-measured from the tree.
"""
import ctypes
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
os.environ["TWIGPATH_LIB"] = os.path.join(HERE, "libtwigpath_trace.so")
sys.path.insert(0, os.path.dirname(HERE))

import numpy as np  # noqa: E402
import torch  # noqa: E402

from paper_2503_14075_amd import binding as tw, runner, workloads as W  # noqa: E402

WAVES, PAIRS, MARKS = 8, 16, 8


def workload(dev):
    cfg = W.replicate(W.CONFIGS["cfg1"], 128)
    return runner.DeviceWorkload(W.make_workload(cfg, device=dev, with_compact=True), dev)


def timed(dw, n=40):
    """Sorted event times (us) of the score launch, a step's other two large launches before each."""
    for _ in range(5):
        dw.run_score()
    ev = []
    for _ in range(n):
        dw.run_compact()
        dw.run_verify()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        dw.run_score()
        b.record()
        ev.append((a, b))
    torch.cuda.synchronize()
    return sorted(x.elapsed_time(y) * 1e3 for x, y in ev)


def ladder_level():
    dw = workload("cuda:0")
    ts = timed(dw)
    print(f"TW_SCORE_DRY={os.environ.get('TW_SCORE_DRY', '0')}: median {ts[len(ts) // 2]:.1f} us  "
          f"p10 {ts[len(ts) // 10]:.1f} us  min {ts[0]:.1f} us", flush=True)


def ladder():
    for level in range(5):
        env = dict(os.environ, TW_SCORE_DRY=str(level))
        rc = subprocess.call([sys.executable, "-m", "paper_2503_14075_amd.score_timeline", "--ladder-level"], env=env)
        if rc:
            sys.exit(rc)


def timeline():
    dev = "cuda:0"
    dw = workload(dev)
    lib = tw.raw()
    lib.tw_debug_set_trace.argtypes = [ctypes.c_void_p]
    n_wg = torch.cuda.get_device_properties(0).multi_processor_count
    trace = torch.zeros(n_wg * WAVES * PAIRS * MARKS, dtype=torch.int64, device=dev)
    for _ in range(3):
        dw.run_score()
    dw.run_compact()
    dw.run_verify()
    torch.cuda.synchronize()
    lib.tw_debug_set_trace(ctypes.c_void_p(trace.data_ptr()))
    dw.run_score()
    torch.cuda.synchronize()
    lib.tw_debug_set_trace(None)
    t = trace.cpu().numpy().reshape(n_wg, WAVES, PAIRS, MARKS).astype(np.float64) * 0.01   # us
    print(f"{n_wg} workgroups x {WAVES} wavefronts; first mark to last recorded mark: "
          f"{t[:, :, PAIRS - 1, 7].max() - t[:, :, 0, 0].min():.1f} us for {PAIRS} pairs per workgroup")
    it = slice(2, PAIRS - 1)
    phases = (
        ("top of the pair -> chunk 0 staged", t[:, :, it, 1] - t[:, :, it, 0]),
        ("-> logits of chunk 0 done", t[:, :, it, 2] - t[:, :, it, 1]),
        ("-> chunk 1 staged", t[:, :, it, 3] - t[:, :, it, 2]),
        ("-> chunk 2 staged (logits of chunk 1 between)", t[:, :, it, 4] - t[:, :, it, 3]),
        ("-> pass 1 done (logits of chunk 2)", t[:, :, it, 5] - t[:, :, it, 4]),
        ("exponentials, publish statistics", t[:, :, it, 6] - t[:, :, it, 5]),
        ("wait at the workgroup barrier", t[:, :, it, 7] - t[:, :, it, 6]),
        ("factors, column sums -> top of the next pair", t[:, :, 3:PAIRS, 0] - t[:, :, 2:PAIRS - 1, 7]),
    )
    total = 0.0
    for name, s in phases:
        print(f"  {name:48s} mean {s.mean():5.2f}  p10 {np.percentile(s, 10):5.2f}  p50 {np.percentile(s, 50):5.2f}  "
              f"p90 {np.percentile(s, 90):5.2f} us")
        total += s.mean()
    per = t[:, :, 3:PAIRS, 0] - t[:, :, 2:PAIRS - 1, 0]
    print(f"  sum of the means {total:.2f} us; pair period mean {per.mean():.2f}  p10 {np.percentile(per, 10):.2f}  "
          f"p90 {np.percentile(per, 90):.2f} us")
    wg, pr = n_wg // 2, 5
    print(f"workgroup {wg}, its pair {pr}: marks of every wavefront in us after wavefront 0's top of the pair")
    for wv in range(WAVES):
        print(f"  wavefront {wv}: " + " ".join(f"{t[wg, wv, pr, k] - t[wg, 0, pr, 0]:5.2f}" for k in range(MARKS))
              + f" | next top {t[wg, wv, pr + 1, 0] - t[wg, 0, pr, 0]:5.2f}")


if __name__ == "__main__":
    if "--ladder-level" in sys.argv:
        ladder_level()
    elif "--ladder" in sys.argv:
        ladder()
    else:
        timeline()
