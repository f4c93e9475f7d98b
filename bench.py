#!/usr/bin/env python3
"""Benchmark of the phrase-boosting-tree hot path on one MI355X.

A "step" is one greedy shallow-fusion decode of the 20K-phrase workload (config 3: V = 1024,
B = 128 hypotheses, T = 1000 frames of fp32 log-probs resident in HBM): the whole hot path --
failure-chain resolution, boost row, Eq. 1 fusion, arg-max and state advance -- for every hypothesis
and frame, through pb_fuse_frames_ws (the multi-frame call with a caller workspace).  `value` is
hypothesis-frames per second over the K timed steps (wall clock, bracketed by device synchronisation);
`roofline` prices the call by its algorithmic bytes against the 8 TB/s HBM peak, with the kernel time
taken from HIP events on the launch stream.  The other regimes (the same call without a workspace, the
selection rules, structured inputs, one launch per frame, HIP-graph replay of the per-frame launches,
config 5 with its 8192-token rows), the dense pb_score sweep, the EOS rule and the beam step are reported
beside it under "extra", every regime labelled.  The CPU oracle is timed on the same arrays as
"cpu_baseline".
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
ROTATE_BYTES = 5 << 28  # 1.25 GiB: buffers a sweep rotates over, so that no launch finds its data in a cache


def _events(torch, fn, reps):
    """Mean milliseconds per call of `fn` over `reps` calls, from events on the current stream."""
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(reps):
        fn()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / reps


def _load_probe():
    """The bench-only probe library (dependent-load latency); built beforehand like the product library."""
    import ctypes as C

    from paper_2508_07014_amd import build as B
    if not os.path.exists(B.PROBE_LIB):
        B.build_probe(force=True)
    lib = C.CDLL(B.PROBE_LIB)
    lib.pb_probe_chase.restype = C.c_int
    lib.pb_probe_chase.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]

    lib.pb_probe_rowmax.restype = C.c_int
    lib.pb_probe_rowmax.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]

    def chase(d_table, n, start, hops, d_out, stream):
        rc = lib.pb_probe_chase(d_table.data_ptr(), n, start, hops, d_out.data_ptr(), stream or None)
        if rc != 0:
            raise RuntimeError(f"pb_probe_chase: {rc}")

    def rowmax(d_logp, row_stride, V, d_prev, d_out, B, stream):
        rc = lib.pb_probe_rowmax(d_logp.data_ptr(), row_stride, V, d_prev.data_ptr(), d_out.data_ptr(), B, stream or None)
        if rc != 0:
            raise RuntimeError(f"pb_probe_rowmax: {rc}")

    chase.rowmax = rowmax
    return chase


def _rate(byts, ms):
    gbs = byts / (ms * 1e-3) / 1e9
    return {"us": ms * 1e3, "GBps": gbs, "frac_hbm": gbs / HBM_PEAK_GBS}


def _same(got, want):
    """Tokens and states bit-exact, scores too (uniform weights and alpha = 0.5 make every boost dyadic)."""
    return bool(all(np.array_equal(g.cpu().numpy(), w) for g, w in zip(got, want)))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-extra", action="store_true", help="skip the side measurements")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing and the parity checks")
    ap.add_argument("--config5-only", action="store_true",
                    help="run only the config 5 greedy decode (V=8192, B=256, 200 steps) and print its block: the "
                         "command behind the config 5 profile")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (reference for hardware-counter runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; the path shards by utterance with no collective "
              "(every GPU holds the tree), so --gpus must be 1", file=sys.stderr)
        return 2

    import torch

    import paper_2508_07014_amd as pb
    import pb_workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    dev = "cuda:0"
    torch.cuda.set_device(0)
    stream = int(torch.cuda.current_stream().cuda_stream)

    if args.config5_only:
        cfg5 = W.CONFIGS[5]
        t5, o5 = W.make_phrases(cfg5)
        tree5 = pb.pb_build(t5, o5, cfg5.vocab_size, cfg5.blank_id, device=0)
        if args.calibrate_copy:
            src = torch.ones(64 << 20, dtype=torch.float32, device=dev)
            dst = torch.empty_like(src)
            for _ in range(3):
                dst.copy_(src)
            torch.cuda.synchronize()
            del src, dst
        print(json.dumps({"config5_greedy": config5_greedy(torch, pb, W, dev, stream, tree5, t5, o5, not args.no_cpu,
                                                           reps=args.steps)}))
        return 0

    cfg = W.CONFIGS[3]
    T, B, V = cfg.steps, cfg.batch, cfg.vocab_size
    toks, offs = W.make_phrases(cfg)
    t0 = time.perf_counter()
    tree = pb.pb_build(toks, offs, V, cfg.blank_id, device=0)
    build_ms = (time.perf_counter() - t0) * 1e3
    info = pb.pb_info(tree)
    logp = W.make_logp(cfg)
    d_logp = torch.from_numpy(logp).to(dev)
    d_s0 = torch.zeros(B, dtype=torch.int32, device=dev)
    d_tok = torch.empty((T, B), dtype=torch.int32, device=dev)
    d_st = torch.empty((T, B), dtype=torch.int32, device=dev)
    d_sc = torch.empty((T, B), dtype=torch.float32, device=dev)
    ws_bytes = pb.pb_fuse_frames_workspace_bytes(tree, T, B)
    d_ws = torch.empty(max(ws_bytes, 4) // 4, dtype=torch.int32, device=dev)  # caller-owned, allocated once

    def step():
        pb.pb_fuse_frames_ws(tree, d_logp, B * V, V, d_s0, None, cfg.alpha, T, B, pb.PB_SELECT_FUSED, d_tok, d_st, d_sc,
                             d_ws, ws_bytes, stream)

    if args.calibrate_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    w0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - w0
    kernel_ms = ev0.elapsed_time(ev1) / args.steps
    ms_per_step = wall * 1e3 / args.steps
    value = B * T / (wall / args.steps)

    bytes_per_launch = T * B * (4 * V + 12) + 4 * B
    achieved = bytes_per_launch / (kernel_ms * 1e-3) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f).get("pb_fuse_frames_ws/config3")

    out = {
        "metric": "greedy hyp-frames/s at 20K phrases (V=1024, B=128, T=1000)",
        "value": value,
        "unit": "hyp-frames/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "config 3: greedy, 20000 phrases of 2-12 Zipf(1.1) tokens, V=1024, blank=0, "
                               "w=1.0, alpha=0.5, B=128, T=1000, N(0,2) log-softmax logits",
                   "entry_point": "pb_fuse_frames_ws (all T frames in one call, caller workspace of "
                                  f"{ws_bytes} bytes)",
                   "num_states": info["num_states"], "tree_bytes": info["device_bytes"]},
        "roofline": {"bound": "hbm", "kernel": "frames_spec_kernel + frames_fix_kernel (one pb_fuse_frames_ws call)",
                     "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "bytes_per_launch": bytes_per_launch, "kernel_ms": kernel_ms},
        "scores_per_s": value * V,
        "build_ms": build_ms,
    }

    # ---- parity + oracle timing on the same arrays ---------------------------------------------------
    ot = None
    if not args.no_cpu:
        from oracle import OracleTree, oracle_threads, set_oracle_threads
        ot = OracleTree(toks, offs, V, cfg.blank_id)
        c0 = time.perf_counter()
        want = ot.fuse_frames(logp, np.zeros(B, np.int32), cfg.alpha)
        cpu_s = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": B * T / cpu_s, "unit": "hyp-frames/s", "cores": oracle_threads(),
                               "kind": "oracle", "sample": f"the whole workload: {T} frames x {B} hypotheses, "
                               f"{cpu_s:.2f} s wall"}
        out["parity"] = _same((d_tok, d_st, d_sc), want)
        nthreads = oracle_threads()
        set_oracle_threads(1)   # the same oracle on one thread, on the first 100 frames
        c0 = time.perf_counter()
        ot.fuse_frames(logp[:100], np.zeros(B, np.int32), cfg.alpha)
        out["cpu_baseline"]["one_thread_value"] = B * 100 / (time.perf_counter() - c0)
        set_oracle_threads(nthreads)

    if not args.no_extra:
        out["extra"] = side_measurements(torch, pb, W, dev, stream, cfg, toks, offs, tree, info, logp, d_logp, ot,
                                         achieved, bytes_per_launch, (d_tok, d_st, d_sc, d_s0, d_ws, ws_bytes))
    print(json.dumps(out))
    return 0


def config5_greedy(torch, pb, W, dev, stream, tree5, t5, o5, with_oracle, reps=5):
    """Config 5 greedy decode (V = 8192, blank-free, B = 256, 200 steps), the per-step shape that moves 8 MiB:
    the multi-frame call, one launch per step and HIP-graph replay of those launches."""
    cfg5 = W.CONFIGS[5]
    V5, T5, B5 = cfg5.vocab_size, cfg5.steps, cfg5.batch
    logp5 = W.make_logp(cfg5)
    d_lp5 = torch.from_numpy(logp5).to(dev)
    z5 = torch.zeros(B5, dtype=torch.int32, device=dev)
    o5b = [torch.empty((T5, B5), dtype=torch.int32, device=dev) for _ in range(2)] + \
        [torch.empty((T5, B5), dtype=torch.float32, device=dev)]
    bytes5 = T5 * B5 * (4 * V5 + 12) + 4 * B5

    def rate5(ms):
        return {"ms": ms, "us_per_frame": ms * 1e3 / T5, "hyp_frames_per_s": B5 * T5 / (ms * 1e-3),
                "GBps": bytes5 / (ms * 1e-3) / 1e9, "frac_hbm": bytes5 / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}

    c5 = {"workload": "config 5: greedy, 20000 phrases of 2-8 Zipf(1.1) tokens, V=8192, blank-free, alpha=0.5, "
                      "B=256, 200 steps, N(0,3) log-softmax logits (1.6 GiB of log-probs, read once per decode)"}
    fn = lambda: pb.pb_fuse_frames(tree5, d_lp5, B5 * V5, V5, z5, cfg5.alpha, T5, B5, o5b[0], o5b[1], o5b[2], stream)
    fn()
    c5["pb_fuse_frames"] = rate5(_events(torch, fn, reps))
    w5 = None
    if with_oracle:
        from oracle import OracleTree
        ot5 = OracleTree(t5, o5, V5, cfg5.blank_id)
        w5 = ot5.fuse_frames(logp5, np.zeros(B5, np.int32), cfg5.alpha)
        c5["pb_fuse_frames"]["parity"] = _same(o5b, w5)

    def per_launch5(sp):
        prev = z5
        for t in range(T5):
            pb.pb_fuse_step(tree5, d_lp5[t], V5, prev, cfg5.alpha, B5, o5b[0][t], o5b[1][t], o5b[2][t], sp)
            prev = o5b[1][t]

    o5b[0].fill_(-9)
    per_launch5(stream)
    torch.cuda.synchronize()
    c5["per_launch"] = rate5(_events(torch, lambda: per_launch5(stream), 3))
    if w5 is not None:
        c5["per_launch"]["parity"] = _same(o5b, w5)
    try:
        g5 = torch.cuda.CUDAGraph()
        side5 = torch.cuda.Stream()
        side5.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side5):
            with torch.cuda.graph(g5, stream=side5):
                per_launch5(int(side5.cuda_stream))
        torch.cuda.current_stream().wait_stream(side5)
        g5.replay()
        torch.cuda.synchronize()
        c5["graph_replay"] = rate5(_events(torch, g5.replay, reps))
    except Exception as e:
        c5["graph_replay"] = {"error": repr(e)}
    return c5


def side_measurements(torch, pb, W, dev, stream, cfg, toks, offs, tree, info, logp, d_logp, ot, achieved,
                      bytes_per_launch, bufs):
    d_tok, d_st, d_sc, d_s0, d_ws, ws_bytes = bufs
    T, B, V = cfg.steps, cfg.batch, cfg.vocab_size
    if ot is not None:
        from oracle import OracleTree
    extra = {}
    # ---- what a plain device copy reaches on this machine (read + write bytes), and the headline against it
    src = torch.ones(64 << 20, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    ms = _events(torch, lambda: dst.copy_(src), 10)
    copy_gbs = 2 * src.numel() * 4 / (ms * 1e-3) / 1e9
    del src, dst
    extra["copy_256MiB"] = {"GBps": copy_gbs, "frac_hbm": copy_gbs / HBM_PEAK_GBS,
                            "headline_frac_of_copy": achieved / copy_gbs}
    # ---- latency of one dependent load i = table[i] through a random cyclic permutation.  Every timed launch
    # starts at a fresh place of the cycle, so its lines are touched for the first time since the preparation
    # step: "L2" = small table read beforehand, "MALL" = 64 MiB table read beforehand, "HBM" = 1 GiB table after
    # 512 MiB of unrelated traffic.
    chase = _load_probe()
    lat = {}
    d_one = torch.zeros(1, dtype=torch.int32, device=dev)
    hops = 20000
    for label, n in (("L2_256KiB_table", 1 << 16), ("MALL_64MiB_table", 1 << 24), ("HBM_1GiB_table", 1 << 28)):
        rng = np.random.Generator(np.random.PCG64(n))
        order = rng.permutation(n).astype(np.int32)
        table = np.empty(n, np.int32)
        table[order] = np.roll(order, -1)
        d_table = torch.from_numpy(table).to(dev)
        chase(d_table, n, 0, 10, d_one, stream)
        if n <= (1 << 24):
            d_table.sum()
        else:
            junk = torch.ones(64 << 20, dtype=torch.float32, device=dev)
            junk2 = junk.clone()
            del junk, junk2
        torch.cuda.synchronize()
        starts = [int(order[(k + 1) * (n // 4)]) for k in range(3)]
        it = iter(starts)
        ms = _events(torch, lambda: chase(d_table, n, next(it), hops, d_one, stream), 3)
        lat[label] = {"ns_per_hop": ms * 1e6 / hops}
        del d_table, table, order
    extra["dependent_load_latency"] = lat
    # ---- structured variants of config 3 under the three selection rules (single-stage, two-stage, two-stage
    # with the CTC repeat rule): the multi-frame call with a workspace ("ws") and without, each checked
    # against the oracle.  512 MiB of log-probs per call: every call reads them from HBM.
    variants = {"as_written": {}, "planted_20pct": dict(planting=W.Planting(toks, offs)),
                "blank_dominated_75pct": dict(blank_bias=8.0, blank_frac=0.75)}
    modes = {"fused": pb.PB_SELECT_FUSED, "two_stage": pb.PB_SELECT_TWO_STAGE,
             "two_stage_ctc": pb.PB_SELECT_TWO_STAGE_CTC}
    results = {}
    for name, kw in variants.items():
        lp = logp if not kw else W.make_logp(cfg, **kw)
        d_lp = d_logp if not kw else torch.from_numpy(lp).to(dev)
        results[name] = {}
        for mname, mode in modes.items():
            rec = {}
            w = None if ot is None else ot.fuse_frames_select(lp, np.zeros(B, np.int32), None, cfg.alpha, mode)
            calls = {"ws": lambda: pb.pb_fuse_frames_ws(tree, d_lp, B * V, V, d_s0, None, cfg.alpha, T, B, mode, d_tok,
                                                        d_st, d_sc, d_ws, ws_bytes, stream),
                     "no_workspace": lambda: pb.pb_fuse_frames_select(tree, d_lp, B * V, V, d_s0, None, cfg.alpha, T, B,
                                                                      mode, d_tok, d_st, d_sc, stream)}
            for cname, fn in calls.items():
                d_tok.fill_(-9)
                fn()
                ms = _events(torch, fn, 5)
                r = {"ms": ms, "hyp_frames_per_s": B * T / (ms * 1e-3), "GBps": bytes_per_launch / (ms * 1e-3) / 1e9,
                     "frac_hbm": bytes_per_launch / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
                if w is not None:
                    r["parity"] = _same((d_tok, d_st, d_sc), w)
                rec[cname] = r
            if w is not None:
                rec["blank_frac"] = float(np.mean(w[0] == cfg.blank_id))
                rec["depth_ge2_frac"] = float(np.mean(w[1] > info["root_degree"]))
            results[name][mname] = rec
        if kw:
            del d_lp, lp
    extra["config3_variants"] = results
    # ---- one launch per frame (the RNN-T / AED shaped loop, the regime the 50 % target names: B = 128 rows of
    # 4 KiB per step; latency-bound by construction): states ping through a [T,B] buffer
    frames = min(T, 200)

    def per_launch(sp):
        prev = d_s0
        for t in range(frames):
            pb.pb_fuse_step(tree, d_logp[t], V, prev, cfg.alpha, B, d_tok[t], d_st[t], d_sc[t], sp)
            prev = d_st[t]

    step_bytes = frames * B * (4 * V + 16)
    per_launch(stream)
    torch.cuda.synchronize()
    ms = _events(torch, lambda: per_launch(stream), 3)
    extra["per_launch"] = {"us_per_frame": ms * 1e3 / frames, "hyp_frames_per_s": B * frames / (ms * 1e-3),
                           "GBps": step_bytes / (ms * 1e-3) / 1e9,
                           "frac_hbm": step_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    # HIP-graph replay of the same launches, and the floor of that regime: as many dependent, nearly empty kernels
    try:
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                per_launch(int(side.cuda_stream))
        torch.cuda.current_stream().wait_stream(side)
        g.replay()
        torch.cuda.synchronize()
        ms = _events(torch, g.replay, 5)
        extra["graph_replay"] = {"us_per_frame": ms * 1e3 / frames, "hyp_frames_per_s": B * frames / (ms * 1e-3),
                                 "GBps": step_bytes / (ms * 1e-3) / 1e9,
                                 "frac_hbm": step_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        g0 = torch.cuda.CUDAGraph()
        side.wait_stream(torch.cuda.current_stream())
        tiny = torch.zeros(4, dtype=torch.int32, device=dev)
        with torch.cuda.stream(side):
            with torch.cuda.graph(g0, stream=side):
                for t in range(frames):
                    chase(tiny, 4, 0, 0, d_one, int(side.cuda_stream))
        torch.cuda.current_stream().wait_stream(side)
        g0.replay()
        torch.cuda.synchronize()
        extra["graph_replay"]["empty_kernel_us_per_node"] = _events(torch, g0.replay, 5) * 1e3 / frames
        # ... and the least a greedy step can do: the same rows, one wave per row, arg-max without a tree, every
        # launch reading what the one before it wrote
        g1 = torch.cuda.CUDAGraph()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g1, stream=side):
                prev = d_s0
                for t in range(frames):
                    chase.rowmax(d_logp[t], V, V, prev, d_tok[t], B, int(side.cuda_stream))
                    prev = d_tok[t]
        torch.cuda.current_stream().wait_stream(side)
        g1.replay()
        torch.cuda.synchronize()
        extra["graph_replay"]["row_argmax_without_tree_us_per_node"] = _events(torch, g1.replay, 5) * 1e3 / frames
    except Exception as e:  # the graph regime is a side measurement; say why it is missing
        extra["graph_replay"] = {"error": repr(e)}
    # ---- the single-step kernel at growing batch (config 3 tree): where it leaves the latency-bound regime.
    # Every launch reads a different slice of a 1.25 GiB pool, so none of them finds its rows in a cache.
    gen = torch.Generator(device=dev).manual_seed(7)
    step_sweep = {"note": "inputs rotate over 1.25 GiB: every launch reads its rows from HBM"}
    pool = torch.randn(ROTATE_BYTES // 4, device=dev, generator=gen) * cfg.sigma
    for Bs in (1024, 4096, 16384, 65536):
        n = ROTATE_BYTES // (Bs * V * 4)
        lp = pool[: n * Bs * V].view(n, Bs, V)
        o_tok = torch.empty(Bs, dtype=torch.int32, device=dev)
        o_st = torch.empty(Bs, dtype=torch.int32, device=dev)
        o_sc = torch.empty(Bs, dtype=torch.float32, device=dev)
        rec = {}
        for kind in ("depth1_states", "uniform_states"):
            if kind == "depth1_states":   # what a greedy trajectory sits in
                stn = (1 + np.arange(Bs) % info["root_degree"]).astype(np.int32)
            else:
                stn = W.sample_states(info["num_states"], Bs, 300 + Bs)
            d_stn = torch.from_numpy(stn).to(dev)
            k = [0]

            def fn():
                pb.pb_fuse_step(tree, lp[k[0] % n], V, d_stn, cfg.alpha, Bs, o_tok, o_st, o_sc, stream)
                k[0] += 1

            fn()
            rec[kind] = _rate(Bs * (4 * V + 16), _events(torch, fn, max(20, n)))
        step_sweep[f"B{Bs}"] = rec
    del pool, lp
    extra["pb_fuse_step_batch_sweep"] = step_sweep
    # ---- dense rows: config 5 sweep (V = 8192, 20K phrases).  Outputs rotate over 1.25 GiB.
    cfg5 = W.CONFIGS[5]
    V5 = cfg5.vocab_size
    t5, o5 = W.make_phrases(cfg5)
    tree5 = pb.pb_build(t5, o5, V5, cfg5.blank_id, device=0)
    n5 = pb.pb_info(tree5)["num_states"]
    eos5 = V5 - 1
    t5e = np.where(t5 == eos5, 1, t5).astype(np.int32)
    tree5e = pb.pb_build(t5e, o5, V5, cfg5.blank_id, device=0, eos_id=eos5, final_eos_score=1.0)
    pool_sc = torch.empty(ROTATE_BYTES // 8, dtype=torch.float32, device=dev)
    pool_nx = torch.empty(ROTATE_BYTES // 8, dtype=torch.int32, device=dev)

    def score_rate(tr, st, Bs):
        n = (ROTATE_BYTES // 8) // (Bs * V5)
        sc = pool_sc[: n * Bs * V5].view(n, Bs, V5)
        nx = pool_nx[: n * Bs * V5].view(n, Bs, V5)
        k = [0]

        def fn():
            pb.pb_score(tr, st, Bs, sc[k[0] % n], nx[k[0] % n], stream)
            k[0] += 1

        for _ in range(5):  # (the launches before may have been of another kernel: let the clocks settle)
            fn()
        ms = _events(torch, fn, max(20, n))
        r = _rate(Bs * V5 * 8 + 4 * Bs, ms)
        r["scores_per_s"] = Bs * V5 / (ms * 1e-3)
        return r

    sweep = {"note": "outputs rotate over 1.25 GiB: every launch writes to HBM"}
    for Bs in (64, 256, 1024, 4096):
        st = torch.from_numpy(W.sample_states(n5, Bs, 100 + Bs)).to(dev)
        sweep[f"B{Bs}"] = score_rate(tree5, st, Bs)
    extra["pb_score_v8192_uniform_states"] = sweep
    # the same call on states of a greedy trajectory (mostly the root and depth 1), and with the EOS rule
    lp5 = torch.from_numpy(W.make_logp(cfg5, steps=8, batch=1024)).to(dev)
    tr_o = [torch.empty((8, 1024), dtype=torch.int32, device=dev) for _ in range(2)] + \
        [torch.empty((8, 1024), dtype=torch.float32, device=dev)]
    pb.pb_fuse_frames(tree5, lp5, 1024 * V5, V5, torch.zeros(1024, dtype=torch.int32, device=dev), cfg5.alpha, 8, 1024,
                      tr_o[0], tr_o[1], tr_o[2], stream)
    st_traj = tr_o[1][7].contiguous()
    extra["pb_score_v8192_trajectory_states"] = {"B1024": score_rate(tree5, st_traj, 1024)}
    st_uni = torch.from_numpy(W.sample_states(n5, 1024, 100 + 1024)).to(dev)
    extra["pb_score_v8192_with_eos"] = {"B1024_uniform_states": score_rate(tree5e, st_uni, 1024),
                                        "B1024_trajectory_states": score_rate(tree5e, st_traj, 1024)}
    del lp5, pool_sc, pool_nx
    extra["config5_greedy"] = config5_greedy(torch, pb, W, dev, stream, tree5, t5, o5, ot is not None)
    # ---- the EOS rule on the step calls (Sec. II-C, the AED decoder's shape): V = 1024, greedy and beam 3
    eos = V - 1
    toks_e = np.where(toks == eos, 1, toks).astype(np.int32)
    tree_e = pb.pb_build(toks_e, offs, V, cfg.blank_id, device=0, eos_id=eos, final_eos_score=1.0)
    frames_e = 100
    eos_rec = {}

    def greedy_loop(tr):
        prev = d_s0
        for t in range(frames_e):
            pb.pb_fuse_step(tr, d_logp[t], V, prev, cfg.alpha, B, d_tok[t], d_st[t], d_sc[t], stream)
            prev = d_st[t]

    for label, tr in (("greedy_step_B128_no_eos", tree), ("greedy_step_B128_eos", tree_e)):
        greedy_loop(tr)
        eos_rec[label] = {"us_per_step": _events(torch, lambda: greedy_loop(tr), 3) * 1e3 / frames_e}
    U3, K3 = 32, 3
    hyp3 = torch.full((U3 * K3,), float("-inf"), device=dev)
    hyp3[::K3] = 0
    bufs3 = [[torch.zeros(U3 * K3, dtype=torch.int32, device=dev) for _ in range(3)] +
             [torch.zeros(U3 * K3, device=dev)] for _ in range(2)]
    st3 = torch.zeros(U3 * K3, dtype=torch.int32, device=dev)

    def beam_loop(tr):
        h, s = hyp3, st3
        for t in range(frames_e):
            o = bufs3[t & 1]
            pb.pb_fuse_step_beam(tr, d_logp[t][: U3 * K3], V, h, s, cfg.alpha, U3, K3, o[0], o[1], o[2], o[3], stream)
            h, s = o[3], o[2]

    for label, tr in (("beam3_step_32utt_no_eos", tree), ("beam3_step_32utt_eos", tree_e)):
        beam_loop(tr)
        eos_rec[label] = {"us_per_step": _events(torch, lambda: beam_loop(tr), 3) * 1e3 / frames_e}
    extra["eos_rule_steps_v1024"] = eos_rec
    # ---- beam step: config 4 shape (32 utterances x 4 beams, 5K phrases)
    cfg4 = W.CONFIGS[4]
    t4, o4 = W.make_phrases(cfg4)
    tree4 = pb.pb_build(t4, o4, cfg4.vocab_size, cfg4.blank_id, device=0)
    U, K = cfg4.batch // cfg4.beam, cfg4.beam
    lp4 = torch.from_numpy(W.make_logp(cfg4, steps=50)).to(dev)
    hyp = torch.full((U * K,), float("-inf"), device=dev)
    hyp[::K] = 0
    bufs4 = [[torch.zeros(U * K, dtype=torch.int32, device=dev) for _ in range(3)] +
             [torch.zeros(U * K, device=dev)] for _ in range(2)]
    st_in = torch.zeros(U * K, dtype=torch.int32, device=dev)

    def beam_run():
        h, s = hyp, st_in
        for t in range(50):
            o = bufs4[t & 1]
            pb.pb_fuse_step_beam(tree4, lp4[t], cfg4.vocab_size, h, s, cfg4.alpha, U, K, o[0], o[1], o[2], o[3], stream)
            h, s = o[3], o[2]

    beam_run()
    ms = _events(torch, beam_run, 3)
    extra["beam_step_config4"] = {"us_per_step": ms * 1e3 / 50, "steps_per_s": 50 / (ms * 1e-3),
                                  "GBps": U * K * (4 * cfg4.vocab_size + 20) / (ms / 50 * 1e-3) / 1e9}
    return extra


if __name__ == "__main__":
    sys.exit(main())
