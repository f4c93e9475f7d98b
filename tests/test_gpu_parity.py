"""GPU parity: libpb.so (through the C ABI) against the CPU oracle, element by element, on the same
seeded inputs.  States, tokens and parents must match bit-exact; scores within 1e-5 absolute (fp32).
"""
import numpy as np
import pytest

import pb_workloads as W
from oracle import OracleTree
from oracle.pb_oracle import W_LOGDEPTH, W_UNIFORM

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import paper_2508_07014_amd as pb  # noqa: E402
from gpu_helpers import (DEV, assert_scores, build_both, config_trees, dev, gpu_beam_step, gpu_fuse_frames,  # noqa: E402
                         gpu_fuse_step, gpu_score, stream_ptr)

# ---------------------------------------------------------------------------------------- pb_score

@pytest.mark.parametrize("seed", range(12))
def test_score_tiny_trees_all_states(seed):
    """Odd vocabulary sizes (scalar path, ragged tail), blank / blank-free, c_unk != 0, both weight modes."""
    V = [5, 6, 7, 9, 13, 66, 130, 257][seed % 8]
    blank = 0 if seed % 2 else -1
    toks, offs, wts = W.tiny_case(7000 + seed, vocab_size=min(V, 9), blank_id=blank, max_phrases=10, max_len=6)
    mode = W_LOGDEPTH if seed % 3 == 0 else W_UNIFORM
    ot, tr = build_both(toks, offs, V, blank, weights=wts, weight_mode=mode, unk_score=0.25 * (seed % 3),
                        final_zero_backoff=seed % 4 != 0)
    states = np.arange(ot.num_states, dtype=np.int32)
    want_s, want_n = ot.score(states)
    got_s, got_n = gpu_score(tr, states, V)
    assert np.array_equal(got_n, want_n)
    assert_scores(got_s, want_s)
    got_s2, none = gpu_score(tr, states, V, want_next=False)
    assert none is None and np.array_equal(got_s2, got_s)


@pytest.mark.parametrize("idx,mode", [(1, W_UNIFORM), (1, W_LOGDEPTH), (2, W_UNIFORM), (2, W_LOGDEPTH), (2, 2)])
def test_score_small_configs_all_or_many_states(idx, mode):
    cfg, toks, offs, ot, tr = config_trees(idx, mode)
    states = np.arange(min(ot.num_states, 3000), dtype=np.int32)
    if ot.num_states > 3000:
        states = np.concatenate([states, W.sample_states(ot.num_states, 1000, 17)])
    want_s, want_n = ot.score(states)
    got_s, got_n = gpu_score(tr, states, cfg.vocab_size)
    assert np.array_equal(got_n, want_n)
    assert_scores(got_s, want_s)
    if mode == W_UNIFORM:
        assert np.array_equal(got_s, want_s)      # integer boosts are exact in fp32


@pytest.mark.parametrize("idx,B", [(3, 128), (3, 1024), (5, 64), (5, 256), (5, 1024)])
def test_score_full_size_uniformly_sampled_states(idx, B):
    """Full-size trees, launch shapes of the benchmark; states drawn from all states (deep chains)."""
    cfg, toks, offs, ot, tr = config_trees(idx)
    states = W.sample_states(ot.num_states, B, 100 + B)
    got_s, got_n = gpu_score(tr, states, cfg.vocab_size)
    rows = np.arange(B) if B * cfg.vocab_size <= 1 << 20 else np.random.default_rng(B).choice(B, 96, replace=False)
    want_s, want_n = ot.score(states[rows])
    assert np.array_equal(got_n[rows], want_n)
    assert np.array_equal(got_s[rows], want_s)
    # properties that hold for every row: blank column, next-state range, root row for state 0
    assert got_n.min() >= 0 and got_n.max() < ot.num_states
    if cfg.blank_id >= 0:
        assert np.all(got_s[:, cfg.blank_id] == 0) and np.array_equal(got_n[:, cfg.blank_id], states)


def test_score_invalid_state_and_empty_batch():
    cfg, toks, offs, ot, tr = config_trees(1)
    states = np.array([0, ot.num_states, -3, 1], np.int32)
    got_s, got_n = gpu_score(tr, states, cfg.vocab_size)
    want_s, want_n = ot.score(states[[0, 3]])
    assert np.array_equal(got_n[[0, 3]], want_n) and np.array_equal(got_s[[0, 3]], want_s)
    assert np.all(got_n[[1, 2]] == -1) and np.all(np.isnan(got_s[[1, 2]]))
    pb.pb_score(tr, 0, 0, 0, None, stream_ptr())      # B = 0: no-op, pointers untouched


def test_score_root_only_tree():
    tr = pb.pb_build(np.zeros(0, np.int32), np.zeros(1, np.int64), 12, 3, unk_score=0.5, device=0)
    got_s, got_n = gpu_score(tr, np.zeros(2, np.int32), 12)
    want = np.full((2, 12), 0.5, np.float32)
    want[:, 3] = 0
    assert np.array_equal(got_s, want) and np.all(got_n == 0)


# ------------------------------------------------------------------------------------ pb_fuse_step

def run_steps(tr, logp, alpha, states0=None, in_place=False):
    T, B, V = logp.shape
    d_logp = dev(logp)
    d_states = dev(np.zeros(B, np.int32) if states0 is None else states0)
    toks, sts, scs = [], [], []
    for t in range(T):
        tk, d_states, sc = gpu_fuse_step(tr, d_logp[t], d_states, alpha, in_place=in_place)
        toks.append(tk.clone()); sts.append(d_states.clone()); scs.append(sc)
    torch.cuda.synchronize()
    return (torch.stack(toks).cpu().numpy(), torch.stack(sts).cpu().numpy(), torch.stack(scs).cpu().numpy())


@pytest.mark.parametrize("idx,planted", [(1, False), (1, True), (2, False), (2, True)])
def test_fuse_step_chained_over_all_frames(idx, planted):
    cfg, toks, offs, ot, tr = config_trees(idx)
    logp = W.make_logp(cfg, planting=W.Planting(toks, offs, cover=0.5) if planted else None)
    want = ot.fuse_frames(logp, np.zeros(cfg.batch, np.int32), cfg.alpha)
    got = run_steps(tr, logp, cfg.alpha, in_place=planted)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
    assert_scores(got[2], want[2])
    if planted:
        depth = max(ot.node(int(s))["depth"] for s in np.unique(want[1]))
        assert depth >= 4                                 # deep states and failure exits were exercised
    got_f = gpu_fuse_frames(tr, dev(logp), dev(np.zeros(cfg.batch, np.int32)), cfg.alpha)
    assert np.array_equal(got_f[0], want[0]) and np.array_equal(got_f[1], want[1])
    assert_scores(got_f[2], want[2])


@pytest.mark.parametrize("seed", range(10))
def test_fuse_step_tiny_random_states_logdepth_and_strides(seed):
    V = [5, 7, 9, 66, 130][seed % 5]
    blank = 0 if seed % 2 else -1
    toks, offs, wts = W.tiny_case(8000 + seed, vocab_size=min(V, 8), blank_id=blank, max_phrases=10, max_len=6)
    ot, tr = build_both(toks, offs, V, blank, weights=wts, weight_mode=W_LOGDEPTH, unk_score=0.5 * (seed % 2))
    rng = np.random.default_rng(seed)
    B = 37
    stride = V + 3
    buf = np.full((B, stride), 99.0, np.float32)          # padding must never be read as a token
    raw = rng.standard_normal((B, V)) * 2
    buf[:, :V] = W.log_softmax_rows(raw)
    states = rng.integers(0, ot.num_states, B).astype(np.int32)
    alpha = 0.7
    want = ot.fuse_step(buf[:, :V], states, alpha)
    tk, st, sc = gpu_fuse_step(tr, dev(buf), dev(states), alpha, row_stride=stride)
    torch.cuda.synchronize()
    assert np.array_equal(tk.cpu().numpy(), want[0]) and np.array_equal(st.cpu().numpy(), want[1])
    assert_scores(sc.cpu().numpy(), want[2])


def test_fuse_step_ties_minus_inf_rows_and_invalid_state():
    cfg, toks, offs, ot, tr = config_trees(1)
    V = cfg.vocab_size
    logp = np.full((4, V), -3.0, np.float32)              # all equal: lowest boosted token wins
    logp[1] = -np.inf                                     # dead row: token 0 by the first-max rule
    logp[2, 100:] = -1.0
    states = np.array([0, 0, 5, ot.num_states + 4], np.int32)
    want = ot.fuse_step(logp[:3], states[:3], cfg.alpha)
    tk, st, sc = gpu_fuse_step(tr, dev(logp), dev(states), cfg.alpha)
    torch.cuda.synchronize()
    tk, st, sc = tk.cpu().numpy(), st.cpu().numpy(), sc.cpu().numpy()
    assert np.array_equal(tk[:3], want[0]) and np.array_equal(st[:3], want[1]) and np.array_equal(sc[:3], want[2])
    assert tk[3] == -1 and st[3] == -1 and np.isnan(sc[3])


def test_fuse_frames_config3_full_size():
    """Headline shape: 20K phrases, V = 1024, B = 128, T = 1000, every output against the oracle."""
    cfg, toks, offs, ot, tr = config_trees(3)
    logp = W.make_logp(cfg)
    want = ot.fuse_frames(logp, np.zeros(cfg.batch, np.int32), cfg.alpha)
    got = gpu_fuse_frames(tr, dev(logp), dev(np.zeros(cfg.batch, np.int32)), cfg.alpha)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
    assert np.array_equal(got[2], want[2])
    # the per-step entry point on a sample of frames, fed with the oracle's states
    d_logp = dev(logp[:40])
    for t in range(0, 40, 3):
        prev = np.zeros(cfg.batch, np.int32) if t == 0 else want[1][t - 1]
        tk, st, sc = gpu_fuse_step(tr, d_logp[t], dev(prev), cfg.alpha)
        assert np.array_equal(tk.cpu().numpy(), want[0][t]) and np.array_equal(st.cpu().numpy(), want[1][t])


def test_fuse_frames_config3_planted_logdepth():
    cfg, toks, offs, ot, tr = config_trees(3, W_LOGDEPTH)
    logp = W.make_logp(cfg, steps=300, planting=W.Planting(toks, offs, cover=0.4))
    want = ot.fuse_frames(logp, np.zeros(cfg.batch, np.int32), 0.3)
    got = gpu_fuse_frames(tr, dev(logp), dev(np.zeros(cfg.batch, np.int32)), 0.3)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
    assert_scores(got[2], want[2])
    assert max(ot.node(int(s))["depth"] for s in np.unique(want[1])) >= 6


def test_fuse_config5_large_vocab_blank_free():
    cfg, toks, offs, ot, tr = config_trees(5)
    T = 40
    logp = W.make_logp(cfg, steps=T, planting=W.Planting(toks, offs, cover=0.3))
    want = ot.fuse_frames(logp, np.zeros(cfg.batch, np.int32), cfg.alpha)
    got = gpu_fuse_frames(tr, dev(logp), dev(np.zeros(cfg.batch, np.int32)), cfg.alpha)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
    assert np.array_equal(got[2], want[2])
    got_s = run_steps(tr, logp[:5], cfg.alpha)
    assert np.array_equal(got_s[0], want[0][:5]) and np.array_equal(got_s[1], want[1][:5])


# ------------------------------------------------------------------------------- pb_fuse_step_beam

def run_beam(ot, tr, logp, alpha, U, K):
    """Chained beam decoding on both sides; returns the per-step outputs of each."""
    T = logp.shape[0]
    hyp = np.full(U * K, -np.inf, np.float32)
    hyp[::K] = 0.0
    st = np.zeros(U * K, np.int32)
    d_logp = dev(logp)
    d_hyp, d_st = dev(hyp), dev(st)
    out_o, out_g = [], []
    for t in range(T):
        o = ot.fuse_step_beam(logp[t], hyp, st, alpha, U, K)
        g = gpu_beam_step(tr, d_logp[t], d_hyp, d_st, alpha, U, K)
        out_o.append(o)
        out_g.append(tuple(x.clone() for x in g))
        hyp, st = o[3], o[2]
        d_hyp, d_st = g[3], g[2]
    torch.cuda.synchronize()
    return out_o, [tuple(x.cpu().numpy() for x in g) for g in out_g]


def check_beam(out_o, out_g):
    for t, (o, g) in enumerate(zip(out_o, out_g)):
        assert np.array_equal(g[0], o[0]), t
        assert np.array_equal(g[1], o[1]), t
        assert np.array_equal(g[2], o[2]), t
        assert_scores(g[3], o[3])


def test_beam_config4_full():
    cfg, toks, offs, ot, tr = config_trees(4)
    U, K = cfg.batch // cfg.beam, cfg.beam
    logp = W.make_logp(cfg, planting=W.Planting(toks, offs, cover=0.3))
    out_o, out_g = run_beam(ot, tr, logp, cfg.alpha, U, K)
    check_beam(out_o, out_g)
    assert max(ot.node(int(s))["depth"] for s in np.unique(out_o[-1][2])) >= 1


@pytest.mark.parametrize("K,V,U", [(1, 128, 5), (2, 128, 3), (3, 66, 4), (8, 1024, 4), (5, 130, 3), (16, 128, 2),
                                    (32, 128, 2), (32, 7, 3)])
def test_beam_various_widths(K, V, U):
    cfg = W.CONFIGS[1]
    toks, offs, wts = W.tiny_case(9000 + K + V, vocab_size=min(V, 9), blank_id=0, max_phrases=10, max_len=6)
    ot, tr = build_both(toks, offs, V, 0, weights=wts, weight_mode=W_LOGDEPTH)
    rng = np.random.default_rng(K * 1000 + V)
    T = 12
    logp = W.log_softmax_rows(rng.standard_normal((T, U * K, V)) * 2)
    out_o, out_g = run_beam(ot, tr, logp, 0.6, U, K)
    check_beam(out_o, out_g)


def test_beam_ties_dead_beams_and_k1_is_greedy():
    cfg, toks, offs, ot, tr = config_trees(1)
    V = cfg.vocab_size
    U, K = 3, 4
    rng = np.random.default_rng(4)
    logp = W.log_softmax_rows(rng.standard_normal((U * K, V)) * 2)
    logp[5] = logp[4]                                      # identical beams: ties broken by flat index
    states = rng.integers(0, ot.num_states, U * K).astype(np.int32)
    states[5] = states[4]
    hyp = rng.standard_normal(U * K).astype(np.float32)
    hyp[5] = hyp[4]
    hyp[8:12] = -np.inf                                    # a fully dead utterance
    hyp[1] = -np.inf
    o = ot.fuse_step_beam(logp, hyp, states, cfg.alpha, U, K)
    g = gpu_beam_step(tr, dev(logp), dev(hyp), dev(states), cfg.alpha, U, K)
    torch.cuda.synchronize()
    g = tuple(x.cpu().numpy() for x in g)
    for a, b in zip(g, o):
        assert np.array_equal(a, b)
    # K = 1 with zero hypothesis scores is the greedy step
    g1 = gpu_beam_step(tr, dev(logp), dev(np.zeros(U * K, np.float32)), dev(states), cfg.alpha, U * K, 1)
    tk, st, sc = gpu_fuse_step(tr, dev(logp), dev(states), cfg.alpha)
    torch.cuda.synchronize()
    assert torch.equal(g1[0], tk) and torch.equal(g1[2], st) and torch.all(g1[1] == 0)


def test_beam_rejects_bad_arguments():
    cfg, toks, offs, ot, tr = config_trees(1)
    x = torch.zeros(8, dtype=torch.int32, device=DEV)
    lp = torch.zeros((8, cfg.vocab_size), device=DEV)
    hyp = torch.zeros(8, device=DEV)
    for K, code in [(0, pb.PB_EINVAL), (33, pb.PB_EUNSUPPORTED)]:
        with pytest.raises(pb.PbError) as e:
            pb.pb_fuse_step_beam(tr, lp, cfg.vocab_size, hyp, x, 0.5, 1, K, x, x, x.clone(), hyp)
        assert e.value.code == code
    with pytest.raises(pb.PbError):                       # aliasing of state buffers
        pb.pb_fuse_step_beam(tr, lp, cfg.vocab_size, hyp, x, 0.5, 2, 4, x.clone(), x.clone(), x, hyp)
    with pytest.raises(pb.PbError):                       # stride smaller than V
        pb.pb_fuse_step(tr, lp, cfg.vocab_size - 1, x, 0.5, 8, x, x, hyp)


def test_results_are_deterministic_run_to_run():
    cfg, toks, offs, ot, tr = config_trees(2)
    logp = dev(W.make_logp(cfg, steps=60, planting=W.Planting(toks, offs, cover=0.5)))
    s0 = dev(np.zeros(cfg.batch, np.int32))
    a = gpu_fuse_frames(tr, logp, s0, cfg.alpha)
    b = gpu_fuse_frames(tr, logp, s0, cfg.alpha)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


# ------------------------------------------------------------------- rare paths of the wave kernels

def _adversarial_tree(seed, V):
    """Tiny vocabulary, mixed-sign phrase weights and a large unknown-token score: overriding arcs often
    score *below* the root row they shadow, so the base winner is regularly an overridden token."""
    rng = np.random.default_rng(seed)
    toks, offs, _ = W.tiny_case(12000 + seed, vocab_size=min(V, 7), blank_id=0, max_phrases=12, max_len=6)
    wts = rng.choice(np.array([-2.0, -1.0, -0.5, 0.25, 1.0, 2.0], np.float32), size=len(offs) - 1)
    mode = W_LOGDEPTH if seed % 2 else W_UNIFORM
    kw = dict(weights=wts, weight_mode=mode, beta=float(rng.choice([-1.0, 0.5, 2.0])),
              unk_score=float(rng.choice([0.0, 1.5, -0.75])), final_zero_backoff=bool(seed % 3))
    return build_both(toks, offs, V, 0, **kw)


@pytest.mark.parametrize("seed", range(16))
def test_fuse_overridden_base_winner_and_shadowed_arcs(seed):
    V = [8, 12, 64, 1024][seed % 4]
    ot, tr = _adversarial_tree(seed, V)
    rng = np.random.default_rng(seed)
    B, T = 24, 40
    # flat logits: the boost decides; the few live tokens are where the phrases are
    raw = rng.standard_normal((T, B, V)) * 0.3
    raw[:, :, 7:] -= 6.0
    logp = W.log_softmax_rows(raw)
    alpha = float(rng.choice([0.5, 1.0, 2.0]))
    # every state as a start state, step by step
    states = np.arange(ot.num_states, dtype=np.int32)
    lp = np.repeat(logp[0, :1], len(states), axis=0)
    want = ot.fuse_step(lp, states, alpha)
    tk, st, sc = gpu_fuse_step(tr, dev(lp), dev(states), alpha)
    torch.cuda.synchronize()
    assert np.array_equal(tk.cpu().numpy(), want[0]) and np.array_equal(st.cpu().numpy(), want[1])
    assert_scores(sc.cpu().numpy(), want[2])
    # and chained over frames, from random start states
    s0 = rng.integers(0, ot.num_states, B).astype(np.int32)
    wantf = ot.fuse_frames(logp, s0, alpha)
    gotf = gpu_fuse_frames(tr, dev(logp), dev(s0), alpha)
    assert np.array_equal(gotf[0], wantf[0]) and np.array_equal(gotf[1], wantf[1])
    assert_scores(gotf[2], wantf[2])


@pytest.mark.parametrize("idx,T,B", [(2, 200, 4), (3, 260, 8), (1, 97, 3), (5, 64, 8)])
def test_fuse_frames_long_phrases_across_segment_boundaries(idx, T, B):
    """Few hypotheses: many short speculative segments.  Almost every frame follows a listed phrase, so
    a segment started from the root keeps disagreeing with the true state for longer than a segment
    lasts and the ordered repair pass has to run."""
    cfg, toks, offs, ot, tr = config_trees(idx)
    logp = W.make_logp(cfg, steps=T, batch=B, planting=W.Planting(toks, offs, cover=0.92, truncate=0.1, bump=6.0 * cfg.sigma))
    want = ot.fuse_frames(logp, np.zeros(B, np.int32), cfg.alpha)
    got = gpu_fuse_frames(tr, dev(logp), dev(np.zeros(B, np.int32)), cfg.alpha)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
    assert_scores(got[2], want[2])
    depth = np.array([ot.node(int(s))["depth"] for s in want[1][:, 0]])
    assert depth.max() >= min(6, ot.max_depth) and (depth >= 2).mean() > 0.3


def test_fuse_frames_invalid_start_state_marks_whole_hypothesis():
    cfg, toks, offs, ot, tr = config_trees(2)
    T, B = 120, 6
    logp = W.make_logp(cfg, steps=T, batch=B)
    s0 = np.zeros(B, np.int32)
    s0[2] = ot.num_states + 7
    s0[4] = -1
    got = gpu_fuse_frames(tr, dev(logp), dev(s0), cfg.alpha)
    ok = [0, 1, 3, 5]
    want = ot.fuse_frames(logp[:, ok], s0[ok], cfg.alpha)
    assert np.array_equal(got[0][:, ok], want[0]) and np.array_equal(got[1][:, ok], want[1])
    for b in (2, 4):
        assert np.all(got[0][:, b] == -1) and np.all(got[1][:, b] == -1) and np.all(np.isnan(got[2][:, b]))


def test_fuse_frames_strided_rows_and_frames():
    cfg, toks, offs, ot, tr = config_trees(2)
    T, B, V = 50, 5, cfg.vocab_size
    logp = W.make_logp(cfg, steps=T, batch=B, planting=W.Planting(toks, offs, cover=0.5))
    rs, fs = V + 8, B * (V + 8) + 16
    buf = np.full(T * fs, 50.0, np.float32)
    for t in range(T):
        for b in range(B):
            buf[t * fs + b * rs: t * fs + b * rs + V] = logp[t, b]
    d_buf = dev(buf)
    d_tok = torch.zeros((T, B), dtype=torch.int32, device=DEV)
    d_st = torch.zeros((T, B), dtype=torch.int32, device=DEV)
    d_sc = torch.zeros((T, B), dtype=torch.float32, device=DEV)
    pb.pb_fuse_frames(tr, d_buf, fs, rs, dev(np.zeros(B, np.int32)), cfg.alpha, T, B, d_tok, d_st, d_sc, stream_ptr())
    torch.cuda.synchronize()
    want = ot.fuse_frames(logp, np.zeros(B, np.int32), cfg.alpha)
    assert np.array_equal(d_tok.cpu().numpy(), want[0]) and np.array_equal(d_st.cpu().numpy(), want[1])


def test_fuse_exact_ties_between_arcs_in_different_lanes():
    """Flat log-probs: all children of a state tie exactly, and so do all root arcs; lowest token wins."""
    cfg, toks, offs, ot, tr = config_trees(2)
    V = cfg.vocab_size
    deg = [(ot.node(s)["depth"], s) for s in range(1, 300)]
    states = np.array([0] + [s for d, s in deg if d == 1][:40] + [s for d, s in deg if d == 2][:20], np.int32)
    for const, alpha in [(-4.0, 0.5), (-np.inf, 0.5), (-4.0, 0.0)]:
        logp = np.full((len(states), V), const, np.float32)
        want = ot.fuse_step(logp, states, alpha)
        tk, st, sc = gpu_fuse_step(tr, dev(logp), dev(states), alpha)
        torch.cuda.synchronize()
        assert np.array_equal(tk.cpu().numpy(), want[0]) and np.array_equal(st.cpu().numpy(), want[1])
        assert np.array_equal(sc.cpu().numpy(), want[2])


def test_fuse_frames_config5_full_size():
    """Large-vocabulary shape as written: V = 8192 (rows in eight chunks), blank-free, B = 256, 200 steps."""
    cfg, toks, offs, ot, tr = config_trees(5)
    logp = W.make_logp(cfg)
    want = ot.fuse_frames(logp, np.zeros(cfg.batch, np.int32), cfg.alpha)
    got = gpu_fuse_frames(tr, dev(logp), dev(np.zeros(cfg.batch, np.int32)), cfg.alpha)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
    assert np.array_equal(got[2], want[2])


def test_step_calls_replay_correctly_from_a_hip_graph():
    """The step calls allocate nothing and synchronise nothing, so a decoding loop can be captured.  The
    graph is replayed several times, with eager work and synchronisation in between and fresh inputs
    copied into the captured buffers, and every replay is compared with the oracle."""
    cfg, toks, offs, ot, tr = config_trees(2)
    T, B, V = 24, cfg.batch, cfg.vocab_size
    U, K = B // 4, 4
    d_logp = torch.zeros((T, B, V), dtype=torch.float32, device=DEV)
    d_s0 = torch.zeros(B, dtype=torch.int32, device=DEV)
    d_tok = torch.zeros((T, B), dtype=torch.int32, device=DEV)
    d_st = torch.zeros((T, B), dtype=torch.int32, device=DEV)
    d_sc = torch.zeros((T, B), dtype=torch.float32, device=DEV)
    f_tok, f_st, f_sc = torch.zeros_like(d_tok), torch.zeros_like(d_st), torch.zeros_like(d_sc)
    d_hyp = torch.zeros(B, dtype=torch.float32, device=DEV)
    beam = [torch.zeros(B, dtype=torch.int32, device=DEV) for _ in range(3)] + [torch.zeros(B, device=DEV)]
    d_rows = torch.zeros((B, V), dtype=torch.float32, device=DEV)
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            sp = int(side.cuda_stream)
            prev = d_s0
            for t in range(T):
                pb.pb_fuse_step_select(tr, d_logp[t], V, prev, d_tok[t - 1] if t else None, cfg.alpha, B,
                                       pb.PB_SELECT_TWO_STAGE_CTC, d_tok[t], d_st[t], d_sc[t], sp)
                prev = d_st[t]
            pb.pb_fuse_frames(tr, d_logp, B * V, V, d_s0, cfg.alpha, T, B, f_tok, f_st, f_sc, sp)
            pb.pb_fuse_step_beam(tr, d_logp[0], V, d_hyp, d_s0, cfg.alpha, U, K, beam[0], beam[1], beam[2], beam[3], sp)
            pb.pb_score(tr, d_st[T - 1], B, d_rows, None, sp)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        logp = W.sticky_logp(50 + rep, T, B, V, cfg.blank_id, grid=None, bump=10.0)
        s0 = W.sample_states(ot.num_states, B, 60 + rep)
        hyp = np.random.default_rng(rep).standard_normal(B).astype(np.float32)
        d_logp.copy_(dev(logp)); d_s0.copy_(dev(s0)); d_hyp.copy_(dev(hyp))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        want = ot.fuse_frames_select(logp, s0, None, cfg.alpha, 2)
        assert np.array_equal(d_tok.cpu().numpy(), want[0]) and np.array_equal(d_st.cpu().numpy(), want[1])
        assert_scores(d_sc.cpu().numpy(), want[2])
        wf = ot.fuse_frames(logp, s0, cfg.alpha)
        assert np.array_equal(f_tok.cpu().numpy(), wf[0]) and np.array_equal(f_st.cpu().numpy(), wf[1])
        wb = ot.fuse_step_beam(logp[0], hyp, s0, cfg.alpha, U, K)
        for got, w in zip(beam[:3], wb[:3]):
            assert np.array_equal(got.cpu().numpy(), w)
        assert_scores(d_rows.cpu().numpy(), ot.score(want[1][T - 1])[0])
        (d_rows * 2).sum().item()      # eager work between the replays


@pytest.mark.parametrize("T,B", [(1, 1), (2, 1), (3000, 2), (700, 1), (65, 130)])
def test_fuse_frames_extreme_shapes(T, B):
    """One frame, one hypothesis, segments longer than 64 frames, more hypotheses than chains per segment."""
    cfg, toks, offs, ot, tr = config_trees(2)
    logp = W.make_logp(cfg, steps=T, batch=B, planting=W.Planting(toks, offs, cover=0.5))
    s0 = W.sample_states(ot.num_states, B, T + B)
    for mode in (0, 2):
        want = ot.fuse_frames_select(logp, s0, None, cfg.alpha, mode)
        d_tok = torch.full((T, B), -5, dtype=torch.int32, device=DEV)
        d_st = torch.full((T, B), -5, dtype=torch.int32, device=DEV)
        d_sc = torch.zeros((T, B), dtype=torch.float32, device=DEV)
        pb.pb_fuse_frames_select(tr, dev(logp), B * cfg.vocab_size, cfg.vocab_size, dev(s0), None, cfg.alpha, T, B, mode,
                                 d_tok, d_st, d_sc, stream_ptr())
        torch.cuda.synchronize()
        assert np.array_equal(d_tok.cpu().numpy(), want[0]) and np.array_equal(d_st.cpu().numpy(), want[1])
        assert_scores(d_sc.cpu().numpy(), want[2])


def test_root_only_tree_is_plain_argmax_in_every_fused_call():
    """No phrases at all: one state, no arcs (the kernels' clamped arc reads then touch the dense root row)."""
    V, B, T = 1024, 9, 40
    empty_t, empty_o = np.zeros(0, np.int32), np.zeros(1, np.int64)
    ot, tr = build_both(empty_t, empty_o, V, 0, unk_score=0.5)
    logp = W.make_logp(W.CONFIGS[2], steps=T, batch=B)
    want = ot.fuse_frames(logp, np.zeros(B, np.int32), 0.7)
    got = gpu_fuse_frames(tr, dev(logp), dev(np.zeros(B, np.int32)), 0.7)
    assert np.array_equal(got[0], want[0]) and np.all(got[1] == 0)
    assert_scores(got[2], want[2])
    tk, st, sc = gpu_fuse_step(tr, dev(logp[0]), dev(np.zeros(B, np.int32)), 0.7)
    torch.cuda.synchronize()
    assert np.array_equal(tk.cpu().numpy(), want[0][0])
    hyp = np.zeros(8, np.float32)
    wb = ot.fuse_step_beam(logp[0][:8], hyp, np.zeros(8, np.int32), 0.7, 2, 4)
    gb = gpu_beam_step(tr, dev(logp[0][:8]), dev(hyp), dev(np.zeros(8, np.int32)), 0.7, 2, 4)
    torch.cuda.synchronize()
    for g, w in zip(gb[:3], wb[:3]):
        assert np.array_equal(g.cpu().numpy(), w)
