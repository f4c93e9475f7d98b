"""Pins for the oracle's end-of-sentence heuristics (Sec. II-C, attention encoder-decoder models):
the EOS score of a state is the largest score the tree gives to any other token from that state, plus
the final weight when the state is an end-of-phrase state; taking the EOS leaves the state unchanged.

  * brute force on token strings (tests/brute.py, no trie) for every state of many tiny trees;
  * the rest of the dense row must be exactly the row of the same tree without an EOS token;
  * values derived by hand for the tree of the paper's Fig. 1 (CAT, CATS, CSV, SIT; c0 = 1, beta = 2);
  * numpy argmax / lexsort on the patched dense rows for the greedy and the beam step.
"""
import math

import numpy as np
import pytest

import pb_workloads as W
from brute import BruteTree, topk_reference
from oracle import OracleError, OracleTree
from oracle.pb_oracle import SELECT_TWO_STAGE, W_LOGDEPTH, W_UNIFORM


def _phrases(tokens, offsets):
    return [tuple(int(x) for x in tokens[offsets[i]:offsets[i + 1]]) for i in range(len(offsets) - 1)]


@pytest.mark.parametrize("seed", range(60))
def test_eos_score_is_brute_force_row_max_plus_final_weight(seed):
    V0 = 5 + seed % 3
    blank = 0 if seed % 2 == 0 else -1
    mode = "logdepth" if seed % 3 == 0 else "uniform"
    unk = [0.0, 0.75, -0.5][seed % 3]
    c_eos = [0.0, 1.5, -0.25][(seed // 3) % 3]
    toks, offs, wts = W.tiny_case(6000 + seed, vocab_size=V0, blank_id=blank)
    if seed % 4 in (1, 2):
        wts = -wts                      # penalising lists: the row maximum can be negative
    V, eos = V0 + 1, V0                 # the EOS token is one past the tokens the phrases use
    bt = BruteTree(_phrases(toks, offs), wts, mode=mode, c_unk=unk, blank=blank)
    kw = dict(weights=wts, weight_mode=W_LOGDEPTH if mode == "logdepth" else W_UNIFORM, unk_score=unk)
    plain = OracleTree(toks, offs, V, blank, **kw)
    ot = OracleTree(toks, offs, V, blank, eos_id=eos, final_eos_score=c_eos, **kw)
    assert ot.num_states == plain.num_states
    states = np.arange(ot.num_states, dtype=np.int32)
    rows, nxt = ot.score(states)
    rows0, nxt0 = plain.score(states)
    keep = [v for v in range(V) if v != eos]
    assert np.array_equal(rows[:, keep], rows0[:, keep]) and np.array_equal(nxt[:, keep], nxt0[:, keep])
    for s in states:
        y = ot.prefix(int(s))
        best = max(bt.query(y, v)[0] for v in range(V) if v not in (eos, blank))
        fw = np.float32(c_eos) if y in bt.finals else np.float32(0.0)
        want = np.float32(np.float32(best) + fw)
        sc, nx = ot.query(int(s), eos)
        assert np.float32(sc) == want and nx == s
        assert rows[s, eos] == want and nxt[s, eos] == s
        others = np.delete(rows0[s], [eos] + ([blank] if blank >= 0 else []))
        assert rows[s, eos] == np.float32(others.max() + fw)


def test_fig1_tree_eos_scores_by_hand():
    """CAT, CATS, CSV, SIT with character tokens, c0 = 1, beta = 2, c_unk = 0, final weight 0.5.

    Arc scores (Sec. II-B): depth 1: 1, depth 2: 2 + ln 2, depth 3: 2 + ln 3, depth 4: 2 + ln 4.
      root  best continuation C or S: 1                                    -> EOS 1
      C     A or S at depth 2: 2 + ln 2                                    -> EOS 2.693147
      CA    T at depth 3: 2 + ln 3                                         -> EOS 3.098612
      CAT   end of phrase; S at depth 4: 2 + ln 4, plus the final weight   -> EOS 3.886294
      CATS  end of phrase; fails to S for free, then I: 2 + ln 2, + 0.5    -> EOS 3.193147
      CSV   end of phrase, no arcs; fails to the root for free: C or S: 1  -> EOS 1.5
      SI    T at depth 3                                                   -> EOS 3.098612
    """
    ids = {ch: i + 1 for i, ch in enumerate("ACISTV")}
    eos, V = 7, 8
    words = ["CAT", "CATS", "CSV", "SIT"]
    toks = np.array([ids[c] for w in words for c in w], np.int32)
    offs = np.cumsum([0] + [len(w) for w in words]).astype(np.int64)
    ot = OracleTree(toks, offs, V, 0, weight_mode=W_LOGDEPTH, beta=2.0, eos_id=eos, final_eos_score=0.5)
    sid = {"".join("ACISTV"[t - 1] for t in ot.prefix(s)): s for s in range(ot.num_states)}
    want = {"": 1.0, "C": 2 + math.log(2), "CA": 2 + math.log(3), "CAT": 2 + math.log(4) + 0.5,
            "CATS": 2 + math.log(2) + 0.5, "CSV": 1.5, "SI": 2 + math.log(3)}
    for name, val in want.items():
        sc, nx = ot.query(sid[name], eos)
        assert abs(sc - val) <= 2e-6 and nx == sid[name], name


def test_greedy_and_beam_steps_use_the_patched_row():
    cfg = W.CONFIGS[1]
    toks, offs = W.make_phrases(cfg)
    V, eos = cfg.vocab_size, cfg.vocab_size - 1
    toks = np.where(toks == eos, 1, toks).astype(np.int32)
    ot = OracleTree(toks, offs, V, -1, eos_id=eos, final_eos_score=2.0)
    rng = np.random.default_rng(3)
    B = 48
    states = rng.integers(0, ot.num_states, B).astype(np.int32)
    logp = W.log_softmax_rows(rng.standard_normal((B, V)) * 0.5)
    logp[:, eos] += np.float32(0.5)
    rows, nxt = ot.score(states)
    fused = (logp + (np.float32(0.5) * rows).astype(np.float32)).astype(np.float32)
    tk, st, sc = ot.fuse_step(logp, states, 0.5)
    assert np.array_equal(tk, np.argmax(fused, axis=-1))
    assert np.array_equal(st, nxt[np.arange(B), tk]) and np.array_equal(sc, fused[np.arange(B), tk])
    assert 0 < np.sum(tk == eos) < B and np.all(st[tk == eos] == states[tk == eos])
    tk2, st2, sc2 = ot.fuse_step_select(logp, states, None, 0.5, SELECT_TWO_STAGE)   # blank-free: same rule
    assert np.array_equal(tk2, tk) and np.array_equal(st2, st)
    U, K = 12, 4
    hyp = rng.standard_normal(B).astype(np.float32)
    bt, bp, bs, bsc = ot.fuse_step_beam(logp, hyp, states, 0.5, U, K)
    for u in range(U):
        tot = (hyp[u * K:(u + 1) * K, None] + fused[u * K:(u + 1) * K]).astype(np.float32).ravel()
        order = topk_reference(tot, K)
        assert np.array_equal(bt[u * K:(u + 1) * K], order % V) and np.array_equal(bp[u * K:(u + 1) * K], order // V)
        assert np.array_equal(bs[u * K:(u + 1) * K], nxt[u * K + order // V, order % V])


def test_eos_arguments_are_checked():
    toks, offs = np.array([1, 2, 3], np.int32), np.array([0, 3], np.int64)
    for bad in (2, 0, 9, -2):            # inside a phrase, the blank, outside the vocabulary
        with pytest.raises(OracleError):
            OracleTree(toks, offs, 6, 0, eos_id=bad)
    ot = OracleTree(toks, offs, 6, 0, eos_id=5)
    assert ot.query(0, 5) == (1.0, 0)    # root: the only continuation scores 1
    lone = OracleTree(np.zeros(0, np.int32), np.zeros(1, np.int64), 1, -1, eos_id=0, final_eos_score=3.0)
    assert lone.query(0, 0) == (0.0, 0)  # no other token: the maximum over nothing counts as 0
