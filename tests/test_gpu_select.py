"""GPU parity of the two-stage token selection (Sec. II-C): pb_fuse_step_select / pb_fuse_frames_select
through the C ABI against the CPU oracle on the same seeded inputs.  Tokens and states bit-exact,
scores within 1e-5 absolute (they are in fact bit-identical: both sides evaluate the same fp32 tree).
"""
import numpy as np
import pytest

import pb_workloads as W
from oracle.pb_oracle import SELECT_FUSED, SELECT_TWO_STAGE, SELECT_TWO_STAGE_CTC, W_LOGDEPTH, W_UNIFORM

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import paper_2508_07014_amd as pb  # noqa: E402
from gpu_helpers import DEV, assert_scores, build_both, config_trees, dev, stream_ptr  # noqa: E402

MODES = [SELECT_TWO_STAGE, SELECT_TWO_STAGE_CTC]


def gpu_step_select(tr, d_logp, d_states, d_last, alpha, mode, row_stride=None):
    B = d_states.shape[0]
    d_tokens = torch.full((B,), -5, dtype=torch.int32, device=DEV)
    d_out = torch.full((B,), -5, dtype=torch.int32, device=DEV)
    d_scores = torch.zeros(B, dtype=torch.float32, device=DEV)
    pb.pb_fuse_step_select(tr, d_logp, d_logp.shape[-1] if row_stride is None else row_stride, d_states, d_last, alpha,
                           B, mode, d_tokens, d_out, d_scores, stream_ptr())
    torch.cuda.synchronize()
    return d_tokens.cpu().numpy(), d_out.cpu().numpy(), d_scores.cpu().numpy()


def gpu_frames_select(tr, logp, states0, last0, alpha, mode):
    T, B, V = logp.shape
    d_logp = dev(logp)
    d_tokens = torch.full((T, B), -5, dtype=torch.int32, device=DEV)
    d_states = torch.full((T, B), -5, dtype=torch.int32, device=DEV)
    d_scores = torch.zeros((T, B), dtype=torch.float32, device=DEV)
    pb.pb_fuse_frames_select(tr, d_logp, B * V, V, dev(states0), None if last0 is None else dev(last0), alpha, T, B,
                             mode, d_tokens, d_states, d_scores, stream_ptr())
    torch.cuda.synchronize()
    return d_tokens.cpu().numpy(), d_states.cpu().numpy(), d_scores.cpu().numpy()


def check(got, want, exact=False):
    assert np.array_equal(got[0], want[0])
    assert np.array_equal(got[1], want[1])
    if exact:
        assert np.array_equal(got[2], want[2])
    else:
        assert_scores(got[2], want[2])


@pytest.mark.parametrize("seed", range(16))
@pytest.mark.parametrize("mode", MODES)
def test_step_select_tiny_trees_random_states_and_previous_labels(seed, mode):
    """Every row shape: V % 4 != 0 and padded strides (workgroup-per-row kernel), V % 4 == 0 (wave kernel)."""
    V = [5, 8, 7, 12, 9, 64, 66, 130][seed % 8]
    blank = 0 if seed % 3 else -1
    toks, offs, wts = W.tiny_case(9000 + seed, vocab_size=min(V, 8), blank_id=blank, max_phrases=10, max_len=6)
    ot, tr = build_both(toks, offs, V, blank, weights=wts, weight_mode=W_LOGDEPTH if seed % 2 else W_UNIFORM,
                        unk_score=0.5 * (seed % 2))
    rng = np.random.default_rng(seed)
    B = 53
    stride = V + (4 if V % 4 == 0 else 3)
    buf = np.full((B, stride), 99.0, np.float32)           # padding must never be read as a token
    buf[:, :V] = W.sticky_logp(seed, 1, B, V, blank, grid=None)[0]
    states = rng.integers(0, ot.num_states, B).astype(np.int32)
    last = rng.integers(-1, min(V, 9), B).astype(np.int32)
    for b in range(0, B, 3):                                # "arg-max is the previous label" made frequent
        if last[b] >= 0:
            buf[b, last[b]] = np.float32(1.0)           # above every log-probability
    want = ot.fuse_step_select(buf[:, :V], states, last, 0.7, mode)
    got = gpu_step_select(tr, dev(buf), dev(states), dev(last), 0.7, mode, row_stride=stride)
    check(got, want)
    if mode == SELECT_TWO_STAGE_CTC:
        assert np.any((want[0] == last) & (last != blank))   # the repeat rule fired
    # no previous labels at all
    want = ot.fuse_step_select(buf[:, :V], states, None, 0.7, mode)
    got = gpu_step_select(tr, dev(buf), dev(states), None, 0.7, mode, row_stride=stride)
    check(got, want)


@pytest.mark.parametrize("seed", range(12))
def test_previous_label_that_would_win_the_reselection_is_excluded(seed):
    """Tiny vocabulary with doubled tokens inside phrases: the boosted previous label regularly beats the
    unboosted winner, so the frame has to be decided again without it."""
    V = [8, 12, 64, 1024][seed % 4]
    rng = np.random.default_rng(seed)
    n = 10
    lens = rng.integers(2, 6, n)
    offs = np.zeros(n + 1, np.int64)
    np.cumsum(lens, out=offs[1:])
    toks = rng.integers(1, 5, int(offs[-1])).astype(np.int32)
    for i in range(n):                                       # double a token in most phrases
        if rng.random() < 0.8:
            j = int(rng.integers(offs[i], offs[i + 1] - 1))
            toks[j + 1] = toks[j]
    wts = np.full(n, 2.0, np.float32)
    ot, tr = build_both(toks, offs, V, 0, weights=wts)
    B, T = 32, 60
    raw = rng.standard_normal((T, B, V)) * 0.4
    raw[:, :, 5:] -= 8.0
    logp = W.log_softmax_rows(raw)
    s0 = rng.integers(0, ot.num_states, B).astype(np.int32)
    last0 = rng.integers(-1, 5, B).astype(np.int32)
    want = ot.fuse_frames_select(logp, s0, last0, 1.0, SELECT_TWO_STAGE_CTC)
    got = gpu_frames_select(tr, logp, s0, last0, 1.0, SELECT_TWO_STAGE_CTC)
    check(got, want)
    # count the frames where the exclusion mattered: the single-step oracle without a previous label
    # would have emitted exactly that label
    hits = 0
    for t in range(1, T):
        free = ot.fuse_step_select(logp[t], want[1][t - 1], None, 1.0, SELECT_TWO_STAGE_CTC)
        hits += int(np.sum((free[0] == want[0][t - 1]) & (want[0][t] != want[0][t - 1])))
    assert hits > 0
    # the single-step entry point on the same frames, chained through its own outputs
    d_logp = dev(logp)
    d_s, d_last = dev(s0), dev(last0)
    for t in range(T):
        d_tok = torch.empty(B, dtype=torch.int32, device=DEV)
        d_sc = torch.empty(B, dtype=torch.float32, device=DEV)
        pb.pb_fuse_step_select(tr, d_logp[t], V, d_s, d_last, 1.0, B, SELECT_TWO_STAGE_CTC, d_tok, d_s, d_sc,
                               stream_ptr())
        d_last = d_tok
        torch.cuda.synchronize()
        assert np.array_equal(d_tok.cpu().numpy(), want[0][t]) and np.array_equal(d_s.cpu().numpy(), want[1][t])


@pytest.mark.parametrize("idx", [1, 2])
@pytest.mark.parametrize("mode", MODES)
def test_frames_select_small_configs_ctc_shaped_rows(idx, mode):
    cfg, toks, offs, ot, tr = config_trees(idx)
    B, T, V = cfg.batch, cfg.steps, cfg.vocab_size
    logp = W.sticky_logp(cfg.seed + mode, T, B, V, cfg.blank_id, grid=None, bump=12.0)
    want = ot.fuse_frames_select(logp, np.zeros(B, np.int32), None, cfg.alpha, mode)
    got = gpu_frames_select(tr, logp, np.zeros(B, np.int32), None, cfg.alpha, mode)
    check(got, want, exact=True)
    assert np.mean(want[0] == cfg.blank_id) > 0.1
    if mode == SELECT_TWO_STAGE_CTC:
        assert np.mean((want[0][1:] == want[0][:-1]) & (want[0][1:] != cfg.blank_id)) > 0.05


@pytest.mark.parametrize("mode", MODES)
def test_frames_select_config3_full_size_blank_dominated(mode):
    """Headline shape (20K phrases, V = 1024, B = 128, T = 1000) with 75 % blank frames and planted
    phrases: every output against the oracle."""
    cfg, toks, offs, ot, tr = config_trees(3)
    logp = W.make_logp(cfg, planting=W.Planting(toks, offs, cover=0.3), blank_bias=10.0, blank_frac=0.75)
    want = ot.fuse_frames_select(logp, np.zeros(cfg.batch, np.int32), None, cfg.alpha, mode)
    got = gpu_frames_select(tr, logp, np.zeros(cfg.batch, np.int32), None, cfg.alpha, mode)
    check(got, want, exact=True)
    assert 0.6 < np.mean(want[0] == cfg.blank_id) < 0.9
    assert max(ot.node(int(s))["depth"] for s in np.unique(want[1])) >= 4


@pytest.mark.parametrize("mode", MODES)
def test_frames_select_config3_as_written(mode):
    cfg, toks, offs, ot, tr = config_trees(3)
    logp = W.make_logp(cfg, steps=400)
    want = ot.fuse_frames_select(logp, np.zeros(cfg.batch, np.int32), None, cfg.alpha, mode)
    got = gpu_frames_select(tr, logp, np.zeros(cfg.batch, np.int32), None, cfg.alpha, mode)
    check(got, want, exact=True)


@pytest.mark.parametrize("mode", MODES)
def test_frames_select_config5_large_vocab(mode):
    """V = 8192 (rows in eight chunks), blank-free: the two-stage rule only differs through repeats."""
    cfg, toks, offs, ot, tr = config_trees(5)
    T, B, V = 48, 64, cfg.vocab_size
    logp = W.sticky_logp(77 + mode, T, B, V, -1, sigma=cfg.sigma, bump=20.0, grid=None)
    s0 = W.sample_states(ot.num_states, B, 5)
    last0 = np.argmax(logp[0], axis=-1).astype(np.int32)
    last0[::2] = -1
    want = ot.fuse_frames_select(logp, s0, last0, cfg.alpha, mode)
    got = gpu_frames_select(tr, logp, s0, last0, cfg.alpha, mode)
    check(got, want, exact=True)
    if mode == SELECT_TWO_STAGE_CTC:
        assert np.mean(want[0][1:] == want[0][:-1]) > 0.1
        assert np.all(want[0][0, 1::2] == last0[1::2])       # frame 0 repeats the caller's previous label
    got1 = gpu_step_select(tr, dev(logp[0]), dev(s0), dev(last0), cfg.alpha, mode)
    assert np.array_equal(got1[0], want[0][0]) and np.array_equal(got1[1], want[1][0])


@pytest.mark.parametrize("idx,T,B", [(2, 230, 4), (1, 97, 3), (3, 300, 6)])
def test_frames_select_ctc_across_segment_boundaries(idx, T, B):
    """Few hypotheses: many short speculative segments, each started without a previous label; repeats
    and long planted phrases straddle the boundaries, so the re-run and the ordered repair both work on
    (state, label) pairs."""
    cfg, toks, offs, ot, tr = config_trees(idx)
    V = cfg.vocab_size
    base = W.make_logp(cfg, steps=T, batch=B, planting=W.Planting(toks, offs, cover=0.9, truncate=0.1, bump=6.0 * cfg.sigma))
    # stretch time: every frame is followed by a copy of itself or by a blank-dominated frame
    logp = np.empty((2 * T, B, V), np.float32)
    logp[0::2] = base
    logp[1::2] = base
    rng = np.random.default_rng(idx)
    blanks = rng.random((T, B)) < 0.4
    odd = logp[1::2]
    odd[blanks, cfg.blank_id] = 0.0
    logp[1::2] = odd
    for mode in MODES:
        want = ot.fuse_frames_select(logp, np.zeros(B, np.int32), None, cfg.alpha, mode)
        got = gpu_frames_select(tr, logp, np.zeros(B, np.int32), None, cfg.alpha, mode)
        check(got, want)
    depth = np.array([ot.node(int(s))["depth"] for s in want[1][:, 0]])
    assert depth.max() >= min(5, ot.max_depth)


def test_select_mode_zero_and_bad_arguments():
    cfg, toks, offs, ot, tr = config_trees(1)
    B, V = cfg.batch, cfg.vocab_size
    logp = W.make_logp(cfg, steps=20)
    want = ot.fuse_frames(logp, np.zeros(B, np.int32), cfg.alpha)
    got = gpu_frames_select(tr, logp, np.zeros(B, np.int32), None, cfg.alpha, SELECT_FUSED)
    check(got, want, exact=True)
    d = dev(logp[0])
    z = dev(np.zeros(B, np.int32))
    o = torch.zeros(B, dtype=torch.int32, device=DEV)
    sc = torch.zeros(B, dtype=torch.float32, device=DEV)
    with pytest.raises(pb.PbError) as e:
        pb.pb_fuse_step_select(tr, d, V, z, None, 0.5, B, 3, o, o, sc, stream_ptr())
    assert e.value.code == pb.PB_EINVAL
    with pytest.raises(pb.PbError) as e:
        pb.pb_fuse_frames_select(tr, d, B * V, V, z, None, 0.5, 1, B, -1, o, o, sc, stream_ptr())
    assert e.value.code == pb.PB_EINVAL
    # invalid state: marked, no fault
    bad = dev(np.array([0, ot.num_states, -3, 1], np.int32))
    got = gpu_step_select(tr, d, bad, None, 0.5, SELECT_TWO_STAGE_CTC)
    assert got[0][1] == -1 and got[1][2] == -1 and np.isnan(got[2][1])
