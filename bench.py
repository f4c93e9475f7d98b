#!/usr/bin/env python3
"""Benchmark of the phrase-boosting-tree hot path on one MI355X.

A "step" is one greedy shallow-fusion decode of the 20K-phrase workload (config 3: V = 1024,
B = 128 hypotheses, T = 1000 frames of fp32 log-probs resident in HBM): the whole hot path --
failure-chain resolution, boost row, Eq. 1 fusion, arg-max and state advance -- for every hypothesis
and frame.  `value` is hypothesis-frames per second over the K timed steps (wall clock, bracketed by
device synchronisation); `roofline` prices the dominant kernel by its algorithmic bytes against the
8 TB/s HBM peak, with the kernel time taken from HIP events on the launch stream.  The other
regimes (one launch per frame, HIP-graph replay of the per-frame launches), the dense pb_score
sweep and the beam step are reported beside it under "extra".  The CPU oracle is timed on the same
arrays as "cpu_baseline".
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

    def chase(d_table, n, start, hops, d_out, stream):
        rc = lib.pb_probe_chase(d_table.data_ptr(), n, start, hops, d_out.data_ptr(), stream or None)
        if rc != 0:
            raise RuntimeError(f"pb_probe_chase: {rc}")

    return chase


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-extra", action="store_true", help="skip the side measurements")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
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

    def step():
        pb.pb_fuse_frames(tree, d_logp, B * V, V, d_s0, cfg.alpha, T, B, d_tok, d_st, d_sc, stream)

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
            traffic = json.load(f).get("pb_fuse_frames/config3")

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
                   "entry_point": "pb_fuse_frames (all T frames in one launch)",
                   "num_states": info["num_states"], "tree_bytes": info["device_bytes"]},
        "roofline": {"bound": "hbm", "kernel": "frames_spec_kernel + frames_fix_kernel (one pb_fuse_frames call)",
                     "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "bytes_per_launch": bytes_per_launch, "kernel_ms": kernel_ms},
        "scores_per_s": value * V,
        "build_ms": build_ms,
    }

    # ---- parity spot check + oracle timing on the same arrays -------------------------------------
    if not args.no_cpu:
        from oracle import OracleTree, oracle_threads
        ot = OracleTree(toks, offs, V, cfg.blank_id)
        c0 = time.perf_counter()
        want = ot.fuse_frames(logp, np.zeros(B, np.int32), cfg.alpha)
        cpu_s = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": B * T / cpu_s, "unit": "hyp-frames/s", "cores": oracle_threads(),
                               "kind": "oracle", "sample": f"the whole workload: {T} frames x {B} hypotheses, "
                               f"{cpu_s:.2f} s wall"}
        # tokens and states bit-exact; scores exact too (uniform weights and alpha = 0.5 make every boost dyadic)
        out["parity"] = bool(np.array_equal(d_tok.cpu().numpy(), want[0]) and
                             np.array_equal(d_st.cpu().numpy(), want[1]) and
                             np.array_equal(d_sc.cpu().numpy(), want[2]))
        # the same oracle on one thread, on the first 100 frames
        from oracle import set_oracle_threads
        nthreads = oracle_threads()
        set_oracle_threads(1)
        c0 = time.perf_counter()
        ot.fuse_frames(logp[:100], np.zeros(B, np.int32), cfg.alpha)
        out["cpu_baseline"]["one_thread_value"] = B * 100 / (time.perf_counter() - c0)
        set_oracle_threads(nthreads)

    # ---- side measurements ---------------------------------------------------------------------------
    if not args.no_extra:
        extra = {}
        # what a plain device copy reaches on this machine (read + write bytes), and the headline against it
        src = torch.ones(64 << 20, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        ms = _events(torch, lambda: dst.copy_(src), 10)
        copy_gbs = 2 * src.numel() * 4 / (ms * 1e-3) / 1e9
        del src, dst
        extra["copy_256MiB"] = {"GBps": copy_gbs, "frac_hbm": copy_gbs / HBM_PEAK_GBS,
                                "headline_frac_of_copy": achieved / copy_gbs}
        # latency of one dependent load i = table[i] through a random cyclic permutation.  Every timed
        # launch starts at a fresh place of the cycle, so its lines are touched for the first time since
        # the preparation step: "L2" = small table read beforehand, "MALL" = 64 MiB table read beforehand,
        # "HBM" = 1 GiB table after 512 MiB of unrelated traffic.
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
        # structured variants of config 3 through the same entry point, under the three selection rules
        # (single-stage, two-stage, two-stage with the CTC repeat rule), each checked against the oracle
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
                fn = lambda: pb.pb_fuse_frames_select(tree, d_lp, B * V, V, d_s0, None, cfg.alpha, T, B, mode, d_tok,
                                                      d_st, d_sc, stream)
                fn()
                ms = _events(torch, fn, 5)
                rec = {"ms": ms, "hyp_frames_per_s": B * T / (ms * 1e-3),
                       "GBps": bytes_per_launch / (ms * 1e-3) / 1e9,
                       "frac_hbm": bytes_per_launch / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
                if not args.no_cpu:
                    w = ot.fuse_frames_select(lp, np.zeros(B, np.int32), None, cfg.alpha, mode)
                    rec["parity"] = bool(np.array_equal(d_tok.cpu().numpy(), w[0]) and
                                         np.array_equal(d_st.cpu().numpy(), w[1]) and
                                         np.array_equal(d_sc.cpu().numpy(), w[2]))
                    rec["blank_frac"] = float(np.mean(w[0] == cfg.blank_id))
                    rec["depth_ge2_frac"] = float(np.mean(w[1] > info["root_degree"]))
                results[name][mname] = rec
            if kw:
                del d_lp, lp
        extra["config3_variants"] = results
        # one launch per frame (the RNN-T / AED shaped loop): states ping through a [T,B] buffer
        frames = min(T, 200)

        def per_launch():
            prev = d_s0
            for t in range(frames):
                pb.pb_fuse_step(tree, d_logp[t], V, prev, cfg.alpha, B, d_tok[t], d_st[t], d_sc[t], stream)
                prev = d_st[t]

        per_launch()
        torch.cuda.synchronize()
        w0 = time.perf_counter()
        ms = _events(torch, per_launch, 3)
        torch.cuda.synchronize()
        extra["per_launch"] = {"us_per_frame": ms * 1e3 / frames, "hyp_frames_per_s": B * frames / (ms * 1e-3),
                               "GBps": frames * B * (4 * V + 12) / (ms * 1e-3) / 1e9}
        # HIP-graph replay of the same launches
        try:
            g = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                with torch.cuda.graph(g, stream=side):
                    sp = int(side.cuda_stream)
                    prev = d_s0
                    for t in range(frames):
                        pb.pb_fuse_step(tree, d_logp[t], V, prev, cfg.alpha, B, d_tok[t], d_st[t], d_sc[t], sp)
                        prev = d_st[t]
            torch.cuda.current_stream().wait_stream(side)
            g.replay()
            torch.cuda.synchronize()
            ms = _events(torch, g.replay, 5)
            extra["graph_replay"] = {"us_per_frame": ms * 1e3 / frames, "hyp_frames_per_s": B * frames / (ms * 1e-3),
                                     "GBps": frames * B * (4 * V + 12) / (ms * 1e-3) / 1e9}
            # the floor of that regime: the same number of dependent, nearly empty kernels in a graph
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
        except Exception as e:  # the graph regime is a side measurement; say why it is missing
            extra["graph_replay"] = {"error": repr(e)}
        # the single-step kernel at growing batch (config 3 tree): where it leaves the latency-bound regime
        gen = torch.Generator(device=dev).manual_seed(7)
        step_sweep = {}
        for Bs in (1024, 4096, 16384, 65536):
            lp = torch.log_softmax(torch.randn((Bs, V), device=dev, generator=gen) * cfg.sigma, dim=-1)
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
                fn = lambda: pb.pb_fuse_step(tree, lp, V, d_stn, cfg.alpha, Bs, o_tok, o_st, o_sc, stream)
                fn()
                ms = _events(torch, fn, 20)
                byts = Bs * (4 * V + 16)
                rec[kind] = {"us": ms * 1e3, "GBps": byts / (ms * 1e-3) / 1e9,
                             "frac_hbm": byts / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
            step_sweep[f"B{Bs}"] = rec
            del lp
        extra["pb_fuse_step_batch_sweep"] = step_sweep
        # dense rows: config 5 sweep (V = 8192, 20K phrases), states drawn from all states
        cfg5 = W.CONFIGS[5]
        t5, o5 = W.make_phrases(cfg5)
        tree5 = pb.pb_build(t5, o5, cfg5.vocab_size, cfg5.blank_id, device=0)
        n5 = pb.pb_info(tree5)["num_states"]
        sweep = {}
        for Bs in (64, 256, 1024, 4096):
            st = torch.from_numpy(W.sample_states(n5, Bs, 100 + Bs)).to(dev)
            sc = torch.empty((Bs, cfg5.vocab_size), dtype=torch.float32, device=dev)
            nx = torch.empty((Bs, cfg5.vocab_size), dtype=torch.int32, device=dev)
            fn = lambda: pb.pb_score(tree5, st, Bs, sc, nx, stream)
            fn()
            ms = _events(torch, fn, 20)
            byts = Bs * cfg5.vocab_size * 8 + 4 * Bs
            sweep[f"B{Bs}"] = {"us": ms * 1e3, "scores_per_s": Bs * cfg5.vocab_size / (ms * 1e-3),
                               "GBps": byts / (ms * 1e-3) / 1e9, "frac_hbm": byts / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        extra["pb_score_v8192_uniform_states"] = sweep
        # the same call on states of a greedy trajectory (mostly the root and depth 1)
        lp5 = torch.from_numpy(W.make_logp(cfg5, steps=8, batch=1024)).to(dev)
        tr_tok = torch.empty((8, 1024), dtype=torch.int32, device=dev)
        tr_st = torch.empty((8, 1024), dtype=torch.int32, device=dev)
        tr_sc = torch.empty((8, 1024), dtype=torch.float32, device=dev)
        pb.pb_fuse_frames(tree5, lp5, 1024 * cfg5.vocab_size, cfg5.vocab_size,
                          torch.zeros(1024, dtype=torch.int32, device=dev), cfg5.alpha, 8, 1024, tr_tok, tr_st, tr_sc,
                          stream)
        st = tr_st[7].contiguous()
        fn = lambda: pb.pb_score(tree5, st, 1024, sc, nx, stream)
        fn()
        ms = _events(torch, fn, 20)
        byts = 1024 * cfg5.vocab_size * 8 + 4 * 1024
        extra["pb_score_v8192_trajectory_states"] = {"B1024": {
            "us": ms * 1e3, "scores_per_s": 1024 * cfg5.vocab_size / (ms * 1e-3), "GBps": byts / (ms * 1e-3) / 1e9,
            "frac_hbm": byts / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}}
        del lp5
        # config 5 greedy decode (V = 8192, blank-free, B = 256, 200 steps): the per-step shape that moves 8 MiB
        cfg5 = W.CONFIGS[5]
        T5, B5, V5 = cfg5.steps, cfg5.batch, cfg5.vocab_size
        logp5 = W.make_logp(cfg5)
        d_lp5 = torch.from_numpy(logp5).to(dev)
        z5 = torch.zeros(B5, dtype=torch.int32, device=dev)
        o5_tok = torch.empty((T5, B5), dtype=torch.int32, device=dev)
        o5_st = torch.empty((T5, B5), dtype=torch.int32, device=dev)
        o5_sc = torch.empty((T5, B5), dtype=torch.float32, device=dev)
        bytes5 = T5 * B5 * (4 * V5 + 12) + 4 * B5

        def rate5(ms):
            return {"ms": ms, "us_per_frame": ms * 1e3 / T5, "hyp_frames_per_s": B5 * T5 / (ms * 1e-3),
                    "GBps": bytes5 / (ms * 1e-3) / 1e9, "frac_hbm": bytes5 / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}

        c5 = {"workload": "config 5: greedy, 20000 phrases of 2-8 Zipf(1.1) tokens, V=8192, blank-free, alpha=0.5, "
                          "B=256, 200 steps, N(0,3) log-softmax logits (1.6 GiB of log-probs, read once per decode)"}
        fn = lambda: pb.pb_fuse_frames(tree5, d_lp5, B5 * V5, V5, z5, cfg5.alpha, T5, B5, o5_tok, o5_st, o5_sc, stream)
        fn()
        c5["pb_fuse_frames"] = rate5(_events(torch, fn, 5))
        if not args.no_cpu:
            ot5 = OracleTree(t5, o5, V5, cfg5.blank_id)
            w5 = ot5.fuse_frames(logp5, np.zeros(B5, np.int32), cfg5.alpha)
            c5["pb_fuse_frames"]["parity"] = bool(np.array_equal(o5_tok.cpu().numpy(), w5[0]) and
                                                  np.array_equal(o5_st.cpu().numpy(), w5[1]) and
                                                  np.array_equal(o5_sc.cpu().numpy(), w5[2]))

        def per_launch5(sp):
            prev = z5
            for t in range(T5):
                pb.pb_fuse_step(tree5, d_lp5[t], V5, prev, cfg5.alpha, B5, o5_tok[t], o5_st[t], o5_sc[t], sp)
                prev = o5_st[t]

        per_launch5(stream)
        torch.cuda.synchronize()
        c5["per_launch"] = rate5(_events(torch, lambda: per_launch5(stream), 3))
        if not args.no_cpu:
            c5["per_launch"]["parity"] = bool(np.array_equal(o5_tok.cpu().numpy(), w5[0]) and
                                              np.array_equal(o5_st.cpu().numpy(), w5[1]) and
                                              np.array_equal(o5_sc.cpu().numpy(), w5[2]))
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
            c5["graph_replay"] = rate5(_events(torch, g5.replay, 5))
        except Exception as e:
            c5["graph_replay"] = {"error": repr(e)}
        extra["config5_greedy"] = c5
        del d_lp5, logp5
        # beam step: config 4 shape (32 utterances x 4 beams, 5K phrases)
        cfg4 = W.CONFIGS[4]
        t4, o4 = W.make_phrases(cfg4)
        tree4 = pb.pb_build(t4, o4, cfg4.vocab_size, cfg4.blank_id, device=0)
        U, K = cfg4.batch // cfg4.beam, cfg4.beam
        lp4 = torch.from_numpy(W.make_logp(cfg4, steps=50)).to(dev)
        hyp = torch.full((U * K,), float("-inf"), device=dev)
        hyp[::K] = 0
        bufs = [[torch.zeros(U * K, dtype=torch.int32, device=dev) for _ in range(3)] +
                [torch.zeros(U * K, device=dev)] for _ in range(2)]
        st_in = torch.zeros(U * K, dtype=torch.int32, device=dev)

        def beam_run():
            h, s = hyp, st_in
            for t in range(50):
                o = bufs[t & 1]
                pb.pb_fuse_step_beam(tree4, lp4[t], cfg4.vocab_size, h, s, cfg4.alpha, U, K, o[0], o[1], o[2], o[3],
                                     stream)
                h, s = o[3], o[2]

        beam_run()
        ms = _events(torch, beam_run, 3)
        extra["beam_step_config4"] = {"us_per_step": ms * 1e3 / 50, "steps_per_s": 50 / (ms * 1e-3),
                                      "GBps": U * K * (4 * cfg4.vocab_size + 20) / (ms / 50 * 1e-3) / 1e9}
        out["extra"] = extra

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
