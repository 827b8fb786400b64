#!/usr/bin/env python3
"""Benchmark of the TwigVLM decode hot path on one MI355X.

A step is one pass of the whole path -- ttp_score -> ttp_select -> ttp_compact
-> tree_verify_attn -> tree_accept -- over a batch of independent sequences at
the LLaVA-1.5-7B shape (576 visual + 64 text tokens pruned to 64 visual, 128
generated tokens -> 256 cache rows, 26-node draft tree, one layer, bf16).  The
batch (default 128 sequences) is what makes the working set larger than the
on-die caches, so every launch streams its K/V from HBM.

Prints ONE JSON line: whole-step throughput in verified tree tokens per second,
the HBM roofline of the kernel the metric is named for (tree_verify_attn) from
HIP-event timings taken inside the timed steps, per-stage times and bandwidths of
all five calls (extras.stages), and the CPU oracle timed on a bounded sample of
the same inputs on this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def verify_bytes(cfg, w):
    """Algorithmic bytes of one tree_verify_attn launch: K and V rows once per
    (sequence, layer), Q in, O out, parent/length arrays."""
    row = cfg.H * cfg.d_h * 2
    total = 0
    for c, t in zip(w.ctx_len, w.n_nodes):
        total += 2 * (c + t) * row + t * cfg.H * cfg.d_h * (2 + 4) + 8 * t
    return total


def verify_sources_hash():
    """sha256 over the sources the verification kernel is built from; printed with --sources-hash for
    the profile summaries, which record it."""
    import hashlib
    h = hashlib.sha256()
    for f in ("tree_verify_mfma.hip", "twig_internal.h", "index_math.h", "mfma_util.h"):
        h.update(open(os.path.join(ROOT, "paper_2503_14075_amd", "csrc", f), "rb").read())
    return h.hexdigest()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=128, help="independent sequences per step")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget of the CPU oracle leg (0 = skip)")
    ap.add_argument("--other-configs", type=int, default=1,
                    help="also time tree_verify_attn on cfg2 (three prefix lengths), cfg3 and cfg4 (0 = skip)")
    ap.add_argument("--next-rows", type=int, default=1,
                    help="also time the calls around the hot path (P-Head score, commit, draft side; 0 = skip)")
    ap.add_argument("--bf16-out-iters", type=int, default=25,
                    help="launches of the bf16-output leg of tree_verify_attn (0 = skip)")
    ap.add_argument("--graph-iters", type=int, default=50,
                    help="replays of the HIP-graph leg (0 = skip)")
    ap.add_argument("--single-iters", type=int, default=200,
                    help="launches of the single-sequence latency leg (0 = skip)")
    ap.add_argument("--sources-hash", action="store_true", help="print the hash of the verification kernel's sources and exit")
    args = ap.parse_args()
    if args.sources_hash:
        print(verify_sources_hash())
        return
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 (no multi-GPU path exists)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2503_14075_amd import runner, workloads as W

    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = W.replicate(W.CONFIGS["cfg1"], args.batch)
    w = W.make_workload(cfg, device=dev)
    dw = runner.DeviceWorkload(w, dev)
    tokens = sum(w.n_nodes)

    for _ in range(args.warmup):
        dw.step()
    torch.cuda.synchronize()

    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        dw.run_score_select()
        dw.run_compact()
        ev[i][0].record()
        dw.run_verify()
        ev[i][1].record()
        dw.run_accept()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    ker_ms = sorted(a.elapsed_time(b) for a, b in ev)
    ker_avg = sum(ker_ms) / len(ker_ms)
    vbytes = verify_bytes(cfg, w)
    achieved = vbytes / (ker_avg * 1e-3) / 1e9

    # per-stage times of the same step (a separate, untimed pass: events around every call)
    stage_names = ("ttp_score", "ttp_select", "ttp_compact", "tree_verify_attn", "tree_accept")
    calls = (dw.run_score, dw.run_select, dw.run_compact, dw.run_verify, dw.run_accept)
    stage_ev = []
    for _ in range(20):
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)]
        marks[0].record()
        for call, m in zip(calls, marks[1:]):
            call()
            m.record()
        stage_ev.append(marks)
    torch.cuda.synchronize()
    row = cfg.H * cfg.d_h * 2
    stage_bytes = {
        # K of every sequence once, the scoring rows of Q, the scores
        "ttp_score": sum(n * row + q * row + 4 * cfg.M for n, q in zip(w.n_tot, w.n_q)),
        # every kept row of every tensor read once and written once
        "ttp_compact": sum(2 * (cfg.R + n) * t.shape[1:].numel() * t.element_size()
                           for n in w.n_text for t in w.compact_src),
        "tree_verify_attn": vbytes,
    }
    stages = {}
    for i, name in enumerate(stage_names):
        ts = sorted(m[i].elapsed_time(m[i + 1]) for m in stage_ev)
        med = ts[len(ts) // 2]
        stages[name] = {"us_median": med * 1e3}
        if name in stage_bytes:
            gbs = stage_bytes[name] / (med * 1e-3) / 1e9
            stages[name].update(algorithmic_MB=stage_bytes[name] / 1e6, GBps=gbs, frac_of_8TBps=gbs / HBM_PEAK_GBS)

    # the pruning score again with only the last 8 text rows scoring (the configurations that name a
    # row count use 8 or 16; the timed step scores with all 64 text rows, as Eq. 3 of the paper sums)
    from paper_2503_14075_amd import binding as tw
    q8 = dw.q_sel[:, -8:].contiguous()
    n8 = torch.full((args.batch,), 8, dtype=torch.int32, device=dev)
    pos8 = (dw.q_pos0 + dw.n_q - 8).to(torch.int32)
    ev8 = []
    for i in range(12):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        tw.ttp_score(q8, dw.k_score_view, n8, pos8, dw.n_tot, dw.n_tot_max, 0, cfg.M, cfg.scale, True, dw.scores,
                     dw.score_ws)
        e1.record()
        ev8.append((e0, e1))
    torch.cuda.synchronize()
    t8 = sorted(x.elapsed_time(y) for x, y in ev8[2:])
    b8 = sum(n * row + 8 * row + 4 * cfg.M for n in w.n_tot)
    stages["ttp_score_last_8_rows"] = {"us_median": t8[len(t8) // 2] * 1e3, "algorithmic_MB": b8 / 1e6,
                                       "GBps": b8 / (t8[len(t8) // 2] * 1e-3) / 1e9}
    dw.run_score()   # leave the scores of the timed configuration in place
    # score + select as the timed step issues them: one call, the head reduction and the select in one launch
    evf = []
    for i in range(12):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        dw.run_score_select()
        e1.record()
        evf.append((e0, e1))
    torch.cuda.synchronize()
    tf = sorted(x.elapsed_time(y) for x, y in evf[2:])
    stages["ttp_score_select_one_call"] = {"us_median": tf[len(tf) // 2] * 1e3}

    # tree_verify_attn with bf16 output (what a following bf16 projection consumes; half the bytes
    # written).  The headline and the parity bar use the fp32 output.
    verify_bf16_us = None
    if args.bf16_out_iters > 0:
        from paper_2503_14075_amd import binding as tw
        out16 = torch.empty(dw.out.shape, dtype=torch.bfloat16, device=dev)
        ev16 = []
        for _ in range(args.bf16_out_iters + 5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            tw.tree_verify_attn(dw.q_tree, dw.k_view, dw.v_view, dw.ctx_len, dw.max_ctx_len, dw.parent,
                                dw.n_nodes, cfg.scale, out16, dw.verify_ws)
            e1.record()
            ev16.append((e0, e1))
        torch.cuda.synchronize()
        t16 = sorted(x.elapsed_time(y) for x, y in ev16[5:])
        verify_bf16_us = t16[len(t16) // 2] * 1e3
        del out16

    # the same step replayed from a HIP graph (the library only enqueues kernels, so a step can be
    # captured once); reported beside the eager figure, which stays the headline
    graph_ms = None
    if args.graph_iters > 0:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            dw.step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            dw.step()
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        tg = time.perf_counter()
        for _ in range(args.graph_iters):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - tg) * 1e3 / args.graph_iters

    # the same step with its two independent chains (verify -> accept, score -> select -> compact) on two
    # streams; beside the serial figure, which stays the headline because the per-kernel durations of
    # the roofline are only meaningful when the kernels run alone
    two_streams_ms = None
    if args.graph_iters > 0:
        side2 = torch.cuda.Stream()
        for _ in range(3):
            dw.step_two_streams(side2)
        torch.cuda.synchronize()
        t2s = time.perf_counter()
        for _ in range(args.graph_iters):
            dw.step_two_streams(side2)
        torch.cuda.synchronize()
        two_streams_ms = (time.perf_counter() - t2s) * 1e3 / args.graph_iters

    # single-instance latency of the graded kernel (one sequence, one layer: what batch-1 decoding
    # issues 32 times per step), launched eagerly and as 32 back-to-back launches of a HIP graph
    single_us = single_graph_us = None
    if args.single_iters > 0:
        w1 = W.make_workload(W.CONFIGS["cfg1"], device=dev, with_compact=False, with_score=False)
        d1 = runner.DeviceWorkload(w1, dev)
        for _ in range(10):
            d1.run_verify()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(args.single_iters):
            d1.run_verify()
        torch.cuda.synchronize()
        single_us = (time.perf_counter() - t2) / args.single_iters * 1e6
        if args.graph_iters > 0:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            g1 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g1, stream=side):
                for _ in range(32):
                    d1.run_verify()
            for _ in range(3):
                g1.replay()
            torch.cuda.synchronize()
            t3 = time.perf_counter()
            for _ in range(args.graph_iters):
                g1.replay()
            torch.cuda.synchronize()
            single_graph_us = (time.perf_counter() - t3) / (32 * args.graph_iters) * 1e6
            del g1

    # the graded kernel on the other configurations (parity-tested elsewhere); each launch is made
    # cold by streaming 1 GiB through the caches between timed launches
    others = {}
    if args.other_configs:
        flush_a = torch.empty(1 << 29, dtype=torch.bfloat16, device=dev)
        flush_b = torch.empty_like(flush_a)
        import dataclasses
        # the bench batch again with the paper's default tree: N_max = 60 candidates + the root (App. A)
        t61 = dataclasses.replace(W.replicate(W.CONFIGS["cfg1"], args.batch), name=f"cfg1_T61x{args.batch}", T=61,
                                  tree=("random", 6))
        named = [(n, W.CONFIGS[n]) for n in ("cfg2_p0", "cfg2_p256", "cfg2_p1024", "cfg3", "cfg4")] + [(t61.name, t61)]
        for name, ocfg in named:
            wo = W.make_workload(ocfg, device=dev, with_compact=False, with_score=False)
            do = runner.DeviceWorkload(wo, dev)
            for _ in range(2):
                do.run_verify()
            # back-to-back launches first (caches and address translation warm from the launch before:
            # what a decode loop sees), then cold ones
            evw = []
            for _ in range(10):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                do.run_verify()
                e1.record()
                evw.append((e0, e1))
            torch.cuda.synchronize()
            tw_ = sorted(x.elapsed_time(y) for x, y in evw)
            warm_med = tw_[len(tw_) // 2]
            evs = []
            for _ in range(10):
                flush_b.copy_(flush_a)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                do.run_verify()
                e1.record()
                evs.append((e0, e1))
            torch.cuda.synchronize()
            ts = sorted(x.elapsed_time(y) for x, y in evs)
            med = ts[len(ts) // 2]
            nbytes = verify_bytes(wo.cfg, wo)
            others[name] = {"kernel_us_median": med * 1e3, "algorithmic_MB": nbytes / 1e6,
                            "GBps": nbytes / (med * 1e-3) / 1e9,
                            "frac_of_8TBps": nbytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBS,
                            "kernel_us_median_back_to_back": warm_med * 1e3,
                            "frac_of_8TBps_back_to_back": nbytes / (warm_med * 1e-3) / 1e9 / HBM_PEAK_GBS,
                            "tree_tokens": sum(wo.n_nodes),
                            "tokens_per_s": sum(wo.n_nodes) / (med * 1e-3),
                            # one launch covers every layer cache of the config: tree rows of one
                            # sequence per full sweep over its layers
                            "sweep_tokens_per_s": sum(wo.n_nodes) / wo.cfg.L / (med * 1e-3)}
            del do, wo
        del flush_a, flush_b

    # the calls around the timed step, on the same batch: the P-Head form of the pruning score (an
    # HBM stream over the keys and their gates), the commit of the accepted paths, and the draft
    # side (top-E of a 32000-wide distribution per expanded node, pruning of the drafted tree)
    next_rows = {}
    if args.next_rows:
        from paper_2503_14075_amd import binding as twb

        def med_us(fn, n=12):
            ev = []
            for _ in range(n):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                fn()
                e1.record()
                ev.append((e0, e1))
            torch.cuda.synchronize()
            ts = sorted(x.elapsed_time(y) for x, y in ev[2:])
            return ts[len(ts) // 2] * 1e3

        Bn = args.batch
        gk = torch.empty_like(dw.k_score).normal_()
        qp = dw.q_sel[:, -1].contiguous()
        gq = torch.empty_like(qp).normal_()
        gview = twb.kv_view(gk, row_off=dw.score_row_off)
        t_ph = med_us(lambda: twb.ttp_score_phead(qp, gq, dw.k_score_view, gview, 0, cfg.M, cfg.scale, dw.scores,
                                                  dw.score_ws))
        b_ph = 2 * Bn * cfg.M * cfg.H * cfg.d_h * 2
        next_rows["ttp_score_phead"] = {"us_median": t_ph, "algorithmic_MB": b_ph / 1e6, "GBps": b_ph / t_ph / 1e3,
                                        "frac_of_8TBps": b_ph / t_ph / 1e3 / HBM_PEAK_GBS}
        del gk, gview
        dw.run_score()   # the scores of the timed configuration back in place
        new_len = torch.empty(Bn, dtype=torch.int32, device=dev)
        ctx_seq = dw.ctx_len[:Bn].contiguous()
        kc, vc = dw.k_pool.clone(), dw.v_pool.clone()      # the commit moves rows in place: not on the timed caches
        cviews = [twb.kv_view(kc, dw.row_off, dw.page_table, cfg.page_rows),
                  twb.kv_view(vc, dw.row_off, dw.page_table, cfg.page_rows)]
        next_rows["kv_commit_us_median"] = med_us(lambda: twb.kv_commit(dw.path, dw.n_acc, cviews, ctx_seq, new_len))
        del kc, vc, cviews
        probs = torch.rand(Bn * 10, 32000, device=dev)
        ids = torch.empty((Bn * 10, 10), dtype=torch.int32, device=dev)
        vals = torch.empty((Bn * 10, 10), dtype=torch.float32, device=dev)
        t_tk = med_us(lambda: twb.draft_topk(probs, 10, ids, vals))
        next_rows["draft_topk_us_median"] = t_tk
        tk_bytes = probs.numel() * 4 + ids.numel() * 8       # the rows read once, ids and values written
        next_rows["draft_topk"] = {"rows": Bn * 10, "V": 32000, "E": 10, "algorithmic_MB": tk_bytes / 1e6,
                                   "GBps": tk_bytes / t_tk / 1e3, "frac_of_8TBps": tk_bytes / t_tk / 1e3 / 8000.0}
        # the same expansion from logits (softmax on the way): the rows read once, ids and probabilities written
        t_tl = med_us(lambda: twb.draft_topk_logits(probs, 10, ids, vals))
        next_rows["draft_topk_logits"] = {"rows": Bn * 10, "V": 32000, "E": 10, "us_median": t_tl,
                                          "algorithmic_MB": tk_bytes / 1e6, "GBps": tk_bytes / t_tl / 1e3,
                                          "frac_of_8TBps": tk_bytes / t_tl / 1e3 / 8000.0}
        del probs
        N = 310                                     # 10 expanded nodes x 10 tokens on each of 3 levels + 10
        cp = (torch.arange(N, device=dev, dtype=torch.int32) // 10 - 1).clamp(min=-1).repeat(Bn, 1).contiguous()
        ct = torch.randint(0, 32000, (Bn, N), device=dev, dtype=torch.int32)
        pb = torch.rand(Bn, N, device=dev)
        nc = torch.full((Bn,), N, dtype=torch.int32, device=dev)
        root = torch.zeros(Bn, dtype=torch.int32, device=dev)
        outs = [torch.empty((Bn, 61), dtype=torch.int32, device=dev) for _ in range(3)]
        nn = torch.empty(Bn, dtype=torch.int32, device=dev)
        tws = torch.empty(twb.tree_build_workspace_bytes(Bn, N, 61) // 4 + 1, dtype=torch.float32, device=dev)
        next_rows["tree_build_us_median"] = med_us(lambda: twb.tree_build(cp, ct, pb, nc, root, 61, outs[0], outs[1],
                                                                          outs[2], nn, tws))
        # sequence-based speculative decoding with the paper's delta = 5, theta = 0.6: chain tree from the
        # draft probabilities (early exit), then the accepted prefix -- latency work on KB-sized inputs
        c_prob = torch.rand(Bn, 5, device=dev)
        c_par = torch.empty((Bn, 6), dtype=torch.int32, device=dev)
        c_nn = torch.empty(Bn, dtype=torch.int32, device=dev)
        c_dr = torch.randint(0, 4, (Bn, 6), device=dev, dtype=torch.int32)
        c_am = torch.randint(0, 4, (Bn, 6), device=dev, dtype=torch.int32)
        c_out = [torch.empty(Bn, dtype=torch.int32, device=dev), torch.empty((Bn, 6), dtype=torch.int32, device=dev),
                 torch.empty(Bn, dtype=torch.int32, device=dev)]

        def chain_calls():
            twb.chain_tree(c_prob, 0.6, 5, c_par, c_nn)
            twb.chain_accept(c_dr, c_am, c_nn, c_out[0], c_out[1], c_out[2])
        next_rows["chain_tree_plus_chain_accept_us_median"] = med_us(chain_calls)

        # grouped-query attention at the head layout of Qwen2.5-VL-7B (28 query heads over 4 key/value
        # heads of 128), cfg1's lengths, the same 128 sequences: the verification attention and the score
        Hq, Hkv, dh = 28, 4, 128
        n_txt, C_g = cfg.N[1], cfg.R + cfg.N[1] + cfg.P[1]     # cfg1: 64 text rows, 256 cache rows
        rows_g, n_tot_g = C_g + cfg.T, cfg.M + n_txt
        gen = torch.Generator(device=dev).manual_seed(7)
        qg = (torch.randn(Bn, cfg.T, Hq, dh, device=dev, generator=gen) / dh ** 0.5).to(torch.bfloat16)
        kg = (torch.randn(Bn * rows_g, Hkv, dh, device=dev, generator=gen) * 0.5).to(torch.bfloat16)
        vg = (torch.randn(Bn * rows_g, Hkv, dh, device=dev, generator=gen) * 0.5).to(torch.bfloat16)
        ro_g = torch.arange(Bn, device=dev, dtype=torch.int32) * rows_g
        kvg, vvg = twb.kv_view(kg, ro_g, None, 16), twb.kv_view(vg, ro_g, None, 16)
        ctx_g = torch.full((Bn,), C_g, dtype=torch.int32, device=dev)
        out_g = torch.empty(Bn, cfg.T, Hq, dh, dtype=torch.float32, device=dev)
        nb_g = twb.workspace_bytes(twb.TW_CALL_TREE_VERIFY_ATTN, Bn, cfg.T, Hq, dh, rows_g)
        ws_g = torch.zeros(max(nb_g, 4) // 4, dtype=torch.float32, device=dev) if nb_g else None
        t_vg = med_us(lambda: twb.tree_verify_attn_gqa(qg, kvg, vvg, Hq // Hkv, ctx_g, C_g, dw.parent, dw.n_nodes,
                                                       cfg.scale, out_g, ws_g))
        b_vg = 2 * Bn * rows_g * Hkv * dh * 2 + Bn * cfg.T * Hq * dh * (2 + 4)
        qs_g = torch.randn(Bn, n_txt, Hq, dh, device=dev, generator=gen).to(torch.bfloat16)
        ks_g = torch.randn(Bn * n_tot_g, Hkv, dh, device=dev, generator=gen).to(torch.bfloat16)
        ro_s = torch.arange(Bn, device=dev, dtype=torch.int32) * n_tot_g
        ksv = twb.kv_view(ks_g, row_off=ro_s)
        i32 = lambda v: torch.full((Bn,), v, dtype=torch.int32, device=dev)
        nq_g, pos_g, nt_g = i32(n_txt), i32(n_tot_g - n_txt), i32(n_tot_g)
        ws_s = torch.empty(twb.workspace_bytes(twb.TW_CALL_TTP_SCORE, Bn, n_txt, Hq, dh, n_tot_g) // 4,
                           dtype=torch.float32, device=dev)
        sc_g = torch.empty(Bn, cfg.M, dtype=torch.float32, device=dev)
        t_sg = med_us(lambda: twb.ttp_score_gqa(qs_g, ksv, Hq // Hkv, nq_g, pos_g, nt_g, n_tot_g, 0, cfg.M,
                                                cfg.scale, True, sc_g, ws_s))
        b_sg = Bn * n_tot_g * Hkv * dh * 2 + Bn * n_txt * Hq * dh * 2 + Bn * cfg.M * 4
        next_rows["grouped_query_28q_4kv_heads"] = {
            "tree_verify_attn_gqa": {"us_median": t_vg, "algorithmic_MB": b_vg / 1e6, "GBps": b_vg / t_vg / 1e3},
            "ttp_score_gqa": {"us_median": t_sg, "algorithmic_MB": b_sg / 1e6, "GBps": b_sg / t_sg / 1e3}}
        del qg, kg, vg, out_g, qs_g, ks_g

    # what plain library kernels reach on this machine in this run (context for the roofline fraction):
    # a 1 GiB device-to-device copy (read + write) and a 1 GiB reduction (read only)
    ctx_a = torch.empty(1 << 29, dtype=torch.bfloat16, device=dev).normal_()
    ctx_b = torch.empty_like(ctx_a)
    box = {}
    for name, fn, nbytes in (("torch_copy_1GiB_GBps_read_plus_write", lambda: ctx_b.copy_(ctx_a), 2 << 30),
                             ("torch_sum_1GiB_GBps_read", lambda: ctx_a.sum(), 1 << 30)):
        for _ in range(3):
            fn()
        evs = []
        for _ in range(10):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
        ts = sorted(x.elapsed_time(y) for x, y in evs)
        box[name] = nbytes / (ts[len(ts) // 2] * 1e-3) / 1e9
    del ctx_a, ctx_b

    cpu = None
    if args.cpu_seconds > 0:
        import oracle
        n_done, t_cpu = 0, 0.0
        # sequences are taken in order and the batch is walked again until the time budget is used,
        # so the sample is 10-15 s of CPU work whatever the speed of the host
        def one_sequence(b):
            """Seconds the oracle takes for the whole path of sequence b (inputs copied out beforehand)."""
            n_tot, off = w.n_tot[b], w.score_row_off[b]
            q_sel = w.q_sel[b:b + 1].cpu()
            k_sc = w.k_score[off:off + n_tot].cpu()
            srcs = [t[off:off + n_tot].cpu() for t in w.compact_src]
            r0, nr = w.row_off[b], w.ctx_len[b] + w.n_nodes[b]
            kp, vp = w.k_pool[r0:r0 + nr].cpu(), w.v_pool[r0:r0 + nr].cpu()
            qt = w.q_tree[b:b + 1].cpu()
            s = time.perf_counter()
            sc = oracle.ttp_score(q_sel, k_sc, [w.n_q[b]], [w.q_pos0[b]], [n_tot], [0], 0, cfg.M,
                                  cfg.scale, True)
            kept = oracle.ttp_select(sc.float(), cfg.R)
            for t in srcs:
                oracle.ttp_compact(kept[0], 0, cfg.M, t)
            oracle.tree_verify_attn(qt, kp, vp, [w.ctx_len[b]], [w.n_nodes[b]], [w.parent[b]], cfg.scale,
                                    row_off=[0])
            oracle.tree_accept([w.draft[b]], [w.argmax[b]], [w.tree_seq[b]], [cfg.T])
            return time.perf_counter() - s

        while t_cpu < args.cpu_seconds:
            t_cpu += one_sequence(n_done % cfg.B)
            n_done += 1
        # the same whole path with the oracle held to one thread, a quarter of the budget
        n_thr = oracle.max_threads()
        oracle.set_threads(1)
        n1, t1_cpu = 0, 0.0
        while t1_cpu < args.cpu_seconds / 4:
            t1_cpu += one_sequence(n1 % cfg.B)
            n1 += 1
        oracle.set_threads(n_thr)
        model = ""
        try:
            for ln in open("/proc/cpuinfo"):
                if ln.startswith("model name"):
                    model = ln.split(":", 1)[1].strip()
                    break
        except OSError:
            pass
        cpu = {"value": n_done * cfg.T / t_cpu, "unit": "tokens/s", "cores": n_thr,
               "kind": "oracle", "cpu_model": model,
               "single_thread_tokens_per_s": n1 * cfg.T / t1_cpu,
               "single_thread_sample": f"whole path on {n1} sequences, one thread ({t1_cpu:.1f} s)",
               "sample": f"whole path on {n_done} sequences drawn in order (with wrap-around) from the "
                         f"{cfg.B} of the same batch ({t_cpu:.1f} s of fp64 C, OpenMP over heads/rows)"}

    # HBM bytes per launch: taken from the committed rocprofv3 counter summary, and only when that summary
    # was made from the very kernel sources of this build (it records their hash) and the same batch;
    # otherwise null -- the counters are not measured inside this run
    traffic, traffic_src = None, None
    tpath = os.path.join(ROOT, "profiles", "verify_mfma_cfg1x128_hbm_traffic.md")
    if os.path.exists(tpath):
        rec = dict(ln.split("=", 1) for ln in open(tpath) if ln.count("=") == 1 and ln[0].isalpha())
        rec = {k.strip(): v.strip() for k, v in rec.items()}
        if (rec.get("batch") == str(args.batch) and "hbm_bytes_per_launch" in rec
                and rec.get("verify_kernel_sources_sha256") == verify_sources_hash()):
            traffic = int(rec["hbm_bytes_per_launch"])
            traffic_src = "profiles/verify_mfma_cfg1x128_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, same sources)"

    out = {
        "metric": "tree-verify attention tokens/s (whole hot-path step), LLaVA-7B shape",
        "value": tokens / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"cfg1 LLaVA-1.5-7B shape x {cfg.B} independent sequences per step: "
                               f"M=576 N=64 R=64 C=256 T=26 H=32 d_h=128, one layer",
                   "batch": cfg.B, "tree_tokens_per_step": tokens},
        "roofline": {"bound": "hbm", "kernel": "void tw::verify_mfma_kernel<128, false, true>(tw::VerifyArgs)",
                     "traffic_source": traffic_src,
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "algorithmic_bytes_per_launch": vbytes, "kernel_ms_avg": ker_avg,
                     "kernel_ms_min": ker_ms[0], "kernel_ms_median": ker_ms[len(ker_ms) // 2]},
        "cpu_baseline": cpu,
        "extras": {"stages": stages, "ms_per_step_hip_graph": graph_ms, "ms_per_step_two_streams": two_streams_ms,
                   "verify_bf16_output_us_median": verify_bf16_us,
                   "same_box_library_kernels": box,
                   "verify_tokens_per_s_kernel_only": tokens / (ker_avg * 1e-3),
                   "verify_single_sequence_latency_us": single_us,
                   "verify_single_sequence_latency_us_hip_graph": single_graph_us,
                   "verify_other_configs": others,
                   "next_rows": next_rows},
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
