"""Pins for the oracle's two-stage greedy token selection (Sec. II-C), independent of its code.

  * the rule restated on the dense rows (themselves pinned by brute force) with numpy's argmax over
    the allowed index set;
  * CTC semantics: the labels the tree consumes are exactly the CTC collapse (merge repeats, drop
    blanks) of the emitted frame labels, so the final tree state must be the brute-force state of the
    collapsed sequence and the boost collected over the frames must be the brute-force cumulative
    boost of that sequence -- a repeat that was boosted, a blank that moved the state or a previous
    label that was not excluded from the re-selection each break one of the two;
  * transducer semantics: the same with "drop blanks" only;
  * degenerate cases: alpha = 0 is plain argmax of the acoustic row; a blank-free vocabulary makes
    the two-stage rule the single-stage one; hand-made rows around a phrase with a doubled token.
"""
import numpy as np
import pytest

import pb_workloads as W
from brute import BruteTree
from oracle import OracleTree
from oracle.pb_oracle import SELECT_FUSED, SELECT_TWO_STAGE, SELECT_TWO_STAGE_CTC, W_LOGDEPTH, W_UNIFORM


def _phrases(tokens, offsets):
    return [tuple(int(x) for x in tokens[offsets[i]:offsets[i + 1]]) for i in range(len(offsets) - 1)]


def _sticky_rows(seed, T, B, V, blank):
    """Acoustic rows on a dyadic grid whose arg-max path has blanks and repeated labels."""
    return W.sticky_logp(seed, T, B, V, blank)


def _collapse(labels, blank, ctc):
    out, prev = [], None
    for v in labels:
        v = int(v)
        if v == blank:
            prev = v
            continue
        if ctc and v == prev:
            continue
        out.append(v)
        prev = v
    return tuple(out)


def _numpy_select(ot, logp, states, last, alpha, mode):
    """The rule of Sec. II-C on dense rows: numpy argmax over the allowed indices."""
    sc, nx = ot.score(states)
    B, V = logp.shape
    toks, sts, vals = np.empty(B, np.int32), np.empty(B, np.int32), np.empty(B, np.float32)
    for b in range(B):
        v0 = int(np.argmax(logp[b]))
        if v0 == ot.blank_id or (mode == SELECT_TWO_STAGE_CTC and last is not None and v0 == last[b]):
            toks[b], sts[b], vals[b] = v0, states[b], logp[b, v0]
            continue
        allowed = np.ones(V, bool)
        if ot.blank_id >= 0:
            allowed[ot.blank_id] = False
        if mode == SELECT_TWO_STAGE_CTC and last is not None and 0 <= last[b] < V:
            allowed[last[b]] = False
        idx = np.flatnonzero(allowed)
        fused = (logp[b, idx] + (np.float32(alpha) * sc[b, idx]).astype(np.float32)).astype(np.float32)
        k = int(np.argmax(fused))
        toks[b], sts[b], vals[b] = idx[k], nx[b, idx[k]], fused[k]
    return toks, sts, vals


@pytest.mark.parametrize("seed", range(30))
@pytest.mark.parametrize("mode", [SELECT_TWO_STAGE, SELECT_TWO_STAGE_CTC])
def test_selection_is_numpy_argmax_over_the_allowed_set(seed, mode):
    V = 6 + seed % 4
    blank = 0 if seed % 3 else -1
    toks, offs, wts = W.tiny_case(4000 + seed, vocab_size=V, blank_id=blank, max_phrases=8)
    wm = W_LOGDEPTH if seed % 2 else W_UNIFORM
    ot = OracleTree(toks, offs, V, blank, weights=wts, weight_mode=wm, unk_score=0.25 * (seed % 3))
    rng = np.random.Generator(np.random.PCG64(seed))
    B = 64
    states = rng.integers(0, ot.num_states, B).astype(np.int32)
    last = rng.integers(-1, V, B).astype(np.int32)
    logp = _sticky_rows(seed, 1, B, V, blank)[0]
    # make "arg-max is the previous label" frequent
    for b in range(0, B, 3):
        if last[b] >= 0:
            logp[b, last[b]] += np.float32(3.0)
    got = ot.fuse_step_select(logp, states, last, 0.5, mode)
    want = _numpy_select(ot, logp, states, last, 0.5, mode)
    for g, w in zip(got, want):
        assert np.array_equal(g, w)


@pytest.mark.parametrize("seed", range(40))
@pytest.mark.parametrize("ctc", [True, False])
def test_consumed_labels_are_the_collapse_of_the_emitted_ones(seed, ctc):
    """Final state and collected boost against the brute force on the collapsed label sequence."""
    V = 5 + seed % 3
    blank = 0
    toks, offs, wts = W.tiny_case(5000 + seed, vocab_size=V, blank_id=blank, max_phrases=8, max_len=4)
    unk = 0.25 if seed % 4 == 0 else 0.0
    bt = BruteTree(_phrases(toks, offs), wts, mode="uniform", c_unk=unk, blank=blank)
    ot = OracleTree(toks, offs, V, blank, weights=wts, unk_score=unk)
    T, B, alpha = 60, 6, 0.5
    logp = _sticky_rows(100 + seed, T, B, V, blank)
    mode = SELECT_TWO_STAGE_CTC if ctc else SELECT_TWO_STAGE
    tokens, states, scores = ot.fuse_frames_select(logp, np.zeros(B, np.int32), None, alpha, mode)
    n_repeat = 0
    for b in range(B):
        consumed = _collapse(tokens[:, b], blank, ctc)
        # B1: state = longest suffix of the consumed history that is a tree prefix
        assert ot.prefix(int(states[-1, b])) == bt.state_of(consumed)
        # cumulative boost of the consumed sequence, by brute force
        y, total = (), 0.0
        for v in consumed:
            sc, y = bt.query(y, v)
            total += float(sc)
        got = 0.0
        for t in range(T):
            got += (float(scores[t, b]) - float(logp[t, b, tokens[t, b]])) / alpha   # exact: dyadic grid
            if ctc and t and tokens[t, b] == tokens[t - 1, b] and tokens[t, b] != blank:
                n_repeat += 1
                assert states[t, b] == states[t - 1, b] and scores[t, b] == logp[t, b, tokens[t, b]]
            if tokens[t, b] == blank:
                assert scores[t, b] == logp[t, b, blank]
                assert states[t, b] == (states[t - 1, b] if t else 0)
        assert got == total
    if ctc:
        assert n_repeat > 0      # the generator must exercise the repeat rule


@pytest.mark.parametrize("mode", [SELECT_TWO_STAGE, SELECT_TWO_STAGE_CTC])
def test_alpha_zero_is_plain_argmax(mode):
    cfg = W.CONFIGS[1]
    toks, offs = W.make_phrases(cfg)
    ot = OracleTree(toks, offs, cfg.vocab_size, cfg.blank_id)
    logp = W.make_logp(cfg, blank_bias=6.0, blank_frac=0.4)
    T, B, V = logp.shape
    tokens, states, scores = ot.fuse_frames_select(logp, np.zeros(B, np.int32), None, 0.0, mode)
    assert np.array_equal(tokens, np.argmax(logp, axis=-1))
    assert np.array_equal(scores, np.max(logp, axis=-1))


def test_blank_free_two_stage_equals_single_stage_and_mode0_is_the_plain_step():
    cfg = W.CONFIGS[1]
    toks, offs = W.make_phrases(cfg)
    logp = W.make_logp(cfg, planting=W.Planting(toks, offs, cover=0.5))
    T, B, V = logp.shape
    free = OracleTree(toks, offs, V, -1)
    a = free.fuse_frames(logp, np.zeros(B, np.int32), 0.5)
    b = free.fuse_frames_select(logp, np.zeros(B, np.int32), None, 0.5, SELECT_TWO_STAGE)
    c = free.fuse_frames_select(logp, np.zeros(B, np.int32), None, 0.5, SELECT_FUSED)
    for x, y, z in zip(a, b, c):
        assert np.array_equal(x, y) and np.array_equal(x, z)


def test_frames_chain_the_previous_label():
    cfg = W.CONFIGS[1]
    toks, offs = W.make_phrases(cfg)
    ot = OracleTree(toks, offs, cfg.vocab_size, cfg.blank_id)
    logp = _sticky_rows(7, 30, 4, cfg.vocab_size, cfg.blank_id)
    last0 = np.array([-1, 5, int(np.argmax(logp[0, 2])), 0], np.int32)
    tokens, states, scores = ot.fuse_frames_select(logp, np.zeros(4, np.int32), last0, 0.5, SELECT_TWO_STAGE_CTC)
    s, last = np.zeros(4, np.int32), last0
    for t in range(30):
        tk, s, sc = ot.fuse_step_select(logp[t], s, last, 0.5, SELECT_TWO_STAGE_CTC)
        assert np.array_equal(tk, tokens[t]) and np.array_equal(s, states[t]) and np.array_equal(sc, scores[t])
        last = tk
    # hypothesis 2 starts on a repeat of its previous label: kept unboosted, state stays at the root
    assert tokens[0, 2] == last0[2] and states[0, 2] == 0 and scores[0, 2] == logp[0, 2, last0[2]]


def test_doubled_token_phrase_by_hand():
    """Phrase (1, 1, 2) over V = 4, blank 0, every arc 1.0, alpha = 1.

    CTC needs a blank between the two 1s; a 1 right after a 1 is a repeat and must neither move the
    state nor be boosted; and the previous label is not a candidate of the re-selection even when its
    boosted score would win.
    """
    ot = OracleTree(np.array([1, 1, 2], np.int32), np.array([0, 3], np.int64), 4, 0)
    lo = np.float32(-8.0)

    def row(**kw):
        r = np.full(4, lo, np.float32)
        for k, v in kw.items():
            r[int(k[1:])] = np.float32(v)
        return r

    frames = np.stack([
        row(t1=-1.0),              # 1       -> state (1),   boosted: -1 + 1
        row(t1=-1.0),              # 1 again -> repeat: state (1), score -1 (no boost)
        row(t0=-1.0),              # blank   -> state (1), score -1
        row(t1=-1.0),              # 1       -> state (1,1), boosted: -1 + 1
        row(t3=-1.0, t1=-1.5),     # arg-max 3; 1 would score -1.5 + 1 (stay in (1,1) via failure) but is the
                                   # previous label -> excluded; 2 scores -8 + 1; 3 scores -1 - 2 (backoff) = -3
        row(t2=-1.0),              # 2 from the root: no arc, c_unk = 0
    ])[:, None, :]
    tokens, states, scores = ot.fuse_frames_select(frames, np.zeros(1, np.int32), None, 1.0, SELECT_TWO_STAGE_CTC)
    assert tokens[:, 0].tolist() == [1, 1, 0, 1, 3, 2]
    assert [ot.prefix(int(s)) for s in states[:, 0]] == [(1,), (1,), (1,), (1, 1), (), ()]
    assert scores[:, 0].tolist() == [0.0, -1.0, -1.0, 0.0, -3.0, -1.0]
    # the transducer rule has no repeat handling: the second 1 is consumed and boosted
    tokens, states, scores = ot.fuse_frames_select(frames, np.zeros(1, np.int32), None, 1.0, SELECT_TWO_STAGE)
    assert tokens[:2, 0].tolist() == [1, 1] and ot.prefix(int(states[1, 0])) == (1, 1) and scores[1, 0] == 0.0


def test_ties_take_the_lowest_token_in_both_stages():
    ot = OracleTree(np.array([2, 3], np.int32), np.array([0, 2], np.int64), 5, 0)
    rows = np.array([
        [-1.0, -1.0, -4.0, -4.0, -4.0],    # stage 1 tie between the blank (0) and 1: lowest id -> blank, stop
        [-4.0, -2.0, -3.0, -1.0, -1.0],    # stage 1: 3 (first of 3, 4); stage 2: 2 gets +1 -> -2 ties with 1 -> 1;
                                           # ... but 3 and 4 score -1: 3 wins (first maximum)
        [-4.0, -2.0, -3.0, -2.5, -2.5],    # stage 1: 1; stage 2: 1 = -2, 2 = -3 + 1 = -2 -> tie -> 1
    ], np.float32)
    tokens, states, scores = ot.fuse_step_select(rows, np.zeros(3, np.int32), None, 1.0, SELECT_TWO_STAGE)
    assert tokens.tolist() == [0, 3, 1] and states.tolist() == [0, 0, 0]
    assert scores.tolist() == [-1.0, -1.0, -2.0]
    # CTC: a tie in stage 1 between the previous label (1) and a higher token is a repeat
    tokens, states, scores = ot.fuse_step_select(rows[2:3], np.zeros(1, np.int32), np.array([1], np.int32), 1.0,
                                                 SELECT_TWO_STAGE_CTC)
    assert tokens.tolist() == [1] and scores.tolist() == [-2.0]
    rows2 = np.array([[-4.0, -2.0, -2.0, -2.5, -2.5]], np.float32)   # stage 1 tie 1/2 -> 1 = previous label
    tokens, states, scores = ot.fuse_step_select(rows2, np.zeros(1, np.int32), np.array([1], np.int32), 1.0,
                                                 SELECT_TWO_STAGE_CTC)
    assert tokens.tolist() == [1] and states.tolist() == [0] and scores.tolist() == [-2.0]
    tokens, states, scores = ot.fuse_step_select(rows2, np.zeros(1, np.int32), np.array([2], np.int32), 1.0,
                                                 SELECT_TWO_STAGE_CTC)           # previous label 2: 1 is new
    assert tokens.tolist() == [1] and scores.tolist() == [-2.0]
