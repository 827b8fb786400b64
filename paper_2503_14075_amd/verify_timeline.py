"""Diagnostics of tree_verify_attn on small launches, from the diagnostic build of the library
(`python -m paper_2503_14075_amd.build --trace`, which writes libtwigpath_trace.so):

    python -m paper_2503_14075_amd.verify_timeline [cfg2_p0 cfg2_p256 cfg2_p1024 cfg3 cfg4 cfg1x128 cfg1_T61x128] [--floor]

For every named configuration: thread 0 of each workgroup of the verification kernel records the
100 MHz wall clock at five points of its life (start, first loads issued, masks and Q ready, first
chunk done, loop done, end) plus its XCD; the report gives the launch's span, the distribution of
starts, ends and phase lengths, and the ends by XCD and by dispatch order.  Launches are made cold
(1 GiB streamed through the caches before each).  With --floor: what a bare read-only stream over as
many bytes reaches on the same box, cold and warm (the ceiling for a kernel of that size).
Nothing here is part of the method; it exists so that what is said about the ramp-up and the tail of
these launches can be re-measured from the tree.
"""
import collections
import ctypes
import dataclasses
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
os.environ["TWIGPATH_LIB"] = os.path.join(HERE, "libtwigpath_trace.so")
sys.path.insert(0, os.path.dirname(HERE))

import torch  # noqa: E402

from paper_2503_14075_amd import binding as tw, runner, workloads as W  # noqa: E402


def q(xs, p):
    xs = sorted(xs)
    return xs[min(len(xs) - 1, int(p * len(xs)))]


def verify_bytes(cfg, w):
    row = cfg.H * cfg.d_h * 2
    return sum(2 * (c + t) * row + t * cfg.H * cfg.d_h * 6 + 8 * t for c, t in zip(w.ctx_len, w.n_nodes))


def main():
    args = [a for a in sys.argv[1:] if not a.startswith("--")]
    floor = "--floor" in sys.argv
    names = args or ["cfg2_p0", "cfg2_p256", "cfg2_p1024", "cfg3", "cfg4"]
    lib = tw.raw()
    lib.tw_debug_set_trace.argtypes = [ctypes.c_void_p]
    lib.tw_debug_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
    lib.tw_debug_stream_read.restype = ctypes.c_int32
    dev = "cuda:0"
    flush_a = torch.empty(1 << 29, dtype=torch.bfloat16, device=dev)
    flush_b = torch.empty_like(flush_a)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    for name in names:
        if name == "cfg1x128":
            cfg = W.replicate(W.CONFIGS["cfg1"], 128)
        elif name == "cfg1_T61x128":    # the bench batch with the paper's default tree: 60 candidates + the root
            cfg = dataclasses.replace(W.replicate(W.CONFIGS["cfg1"], 128), name=name, T=61, tree=("random", 6))
        else:
            cfg = W.CONFIGS[name]
        wo = W.make_workload(cfg, device=dev, with_compact=False, with_score=False)
        do = runner.DeviceWorkload(wo, dev)
        trace = torch.zeros((1 << 16) * 8, dtype=torch.int64, device=dev)
        for _ in range(3):
            do.run_verify()
        torch.cuda.synchronize()
        evt = []
        for _ in range(4):
            trace.zero_()
            flush_b.copy_(flush_a)
            lib.tw_debug_set_trace(ctypes.c_void_p(trace.data_ptr()))
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            do.run_verify()
            e1.record()
            torch.cuda.synchronize()
            lib.tw_debug_set_trace(None)
            evt.append(e0.elapsed_time(e1) * 1e3)
        t = trace.cpu().view(-1, 8)
        t = t[t[:, 0] != 0]
        t0 = int(t[:, 0].min())
        us = lambda x: (int(x) - t0) / 100.0
        start, end = [us(v) for v in t[:, 0]], [us(v) for v in t[:, 5]]
        phases = (("start -> first loads issued", 0, 1), ("-> masks and Q ready", 1, 2), ("-> first chunk done", 2, 3),
                  ("masks and Q ready -> loop done", 2, 4), ("loop done -> end", 4, 5), ("whole life", 0, 5))
        nbytes = verify_bytes(cfg, wo)
        print(f"== {name}: {t.shape[0]} workgroups, {nbytes / 1e6:.1f} MB ({nbytes / 8e6:.1f} us at 8 TB/s), "
              f"event times of the cold launches {[round(x, 1) for x in sorted(evt)]} us")
        print(f"   span first start -> last end {max(end):.2f} us; starts p50 {q(start, .5):.2f} max {max(start):.2f}; "
              f"ends p10 {q(end, .1):.2f} p50 {q(end, .5):.2f} p90 {q(end, .9):.2f}")
        for lab, i, j in phases:
            d = [(int(r[j]) - int(r[i])) / 100.0 for r in t if int(r[j]) and int(r[i])]
            if d:
                print(f"   {lab:32s} p10 {q(d, .1):6.2f} p50 {q(d, .5):6.2f} p90 {q(d, .9):6.2f} max {max(d):6.2f}")
        byx = collections.defaultdict(list)
        for r, e in zip(t, end):
            byx[int(r[7]) & 0xF].append(e)
        print("   ends by XCD (mean / max): " + "  ".join(f"{x}: {sum(v) / len(v):.1f} / {max(v):.1f}"
                                                          for x, v in sorted(byx.items())))
        half = len(end) // 2
        print(f"   ends by dispatch order: first half of the workgroups mean {sum(end[:half]) / max(half, 1):.1f}, "
              f"second half {sum(end[half:]) / max(len(end) - half, 1):.1f}")
        if floor:
            src = torch.empty(max(nbytes, 1 << 20) // 2, dtype=torch.bfloat16, device=dev).normal_()
            for cold in (True, False):
                ts = []
                for _ in range(10):
                    if cold:
                        flush_b.copy_(flush_a)
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    lib.tw_debug_stream_read(src.data_ptr(), nbytes, 512, sink.data_ptr(), None)
                    e1.record()
                    torch.cuda.synchronize()
                    ts.append(e0.elapsed_time(e1) * 1e3)
                m = sorted(ts)[len(ts) // 2]
                print(f"   bare read stream of the same bytes, {'cold' if cold else 'warm'}: {m:.1f} us by events "
                      f"= {nbytes / m / 1e3:.0f} GB/s ({nbytes / m / 8e6 * 100:.0f} % of 8 TB/s)")
        sys.stdout.flush()
        del do, wo


if __name__ == "__main__":
    main()
