"""Pins for the CPU oracle: what the paper and the mathematics fix, independent of the oracle's code.

  * brute force on token strings (no trie, no links) over hundreds of tiny random phrase lists;
  * closed forms that follow from backoff = acc(fail) - acc(node) (Sec. II-B): telescoping;
  * the hand-derived Fig. 1 trace (tests/golden/fig1_cat_trace.txt);
  * textbook special cases: a single phrase is a Knuth-Morris-Pratt automaton; zero weights give
    the plain Aho-Corasick goto/fail automaton (states only);
  * numpy argmax / lexsort for the selection steps.
"""
import math
import os

import numpy as np
import pytest

import pb_workloads as W
from brute import BruteTree, kmp_automaton, topk_reference
from oracle import OracleTree, OracleError
from oracle.pb_oracle import W_LOGDEPTH, W_UNIFORM, W_UNIFORM_FINAL

WM = {"uniform": W_UNIFORM, "logdepth": W_LOGDEPTH, "uniform_final": W_UNIFORM_FINAL}

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _phrases(tokens, offsets):
    return [tuple(int(x) for x in tokens[offsets[i]:offsets[i + 1]]) for i in range(len(offsets) - 1)]


def _state_strings(tree: OracleTree):
    return [tree.prefix(s) for s in range(tree.num_states)]


CASES = [(seed, mode, fzb, unk) for seed in range(60) for mode, fzb, unk in
         [("uniform", True, 0.0), ("logdepth", True, 0.0), ("uniform", False, 0.0), ("logdepth", True, 0.75),
          ("uniform_final", True, 0.0), ("uniform_final", False, 0.5)]]


@pytest.mark.parametrize("seed,mode,fzb,unk", CASES)
def test_oracle_matches_brute_force_all_pairs(seed, mode, fzb, unk):
    """Every (state, token) pair of a tiny tree: next state and fp32 score against the brute force."""
    V = 5 + seed % 3
    blank = 0 if seed % 2 == 0 else -1
    toks, offs, wts = W.tiny_case(1000 + seed, vocab_size=V, blank_id=blank)
    phrases = _phrases(toks, offs)
    bt = BruteTree(phrases, wts, mode=mode, beta=2.0, c_unk=unk, final_zero_backoff=fzb, blank=blank)
    ot = OracleTree(toks, offs, V, blank, weights=wts,
                    weight_mode=WM[mode], beta=2.0, unk_score=unk,
                    final_zero_backoff=fzb)
    strings = _state_strings(ot)
    # the states are exactly the distinct phrase prefixes
    assert sorted(strings) == sorted(bt.prefixes)
    sid = {x: i for i, x in enumerate(strings)}
    # canonical numbering: breadth-first, children by ascending token
    assert strings == sorted(strings, key=lambda x: (len(x), x))
    for s, y in enumerate(strings):
        nd = ot.node(s)
        assert nd["depth"] == len(y)
        assert nd["final"] == (y in bt.finals)
        assert abs(nd["acc"] - bt.acc[y]) == 0.0
        if s:
            assert strings[nd["fail"]] == bt.suffix_chain(y)[1]      # longest proper suffix in the tree
        for v in range(V):
            sc, nx = ot.query(s, v)
            bsc, bnext = bt.query(y, v)
            assert strings[nx] == bnext, (y, v)
            assert np.float32(sc) == bsc, (y, v, sc, bsc)
            if v != blank:
                # B1: the next state is the longest suffix of (history + v) that is a tree prefix
                assert strings[nx] == bt.state_of(y + (v,))


def test_canonical_numbering_is_bfs_with_children_by_token():
    toks, offs, wts = W.tiny_case(7, vocab_size=6, max_phrases=12, max_len=6)
    ot = OracleTree(toks, offs, 6, 0, weights=wts)
    strings = _state_strings(ot)
    # BFS with children sorted by token == sort by (length, then lexicographic by parent order),
    # which for a trie is simply (length, tuple)
    assert strings == sorted(strings, key=lambda x: (len(x), x))
    # children of a state are consecutive ids in token order
    for s, y in enumerate(strings):
        kids = [ot.child(s, v) for v in range(6) if ot.child(s, v) >= 0]
        assert kids == list(range(kids[0], kids[0] + len(kids))) if kids else True


@pytest.mark.parametrize("seed", range(40))
@pytest.mark.parametrize("mode", ["uniform", "logdepth", "uniform_final"])
def test_random_walk_history_state_and_telescoping(seed, mode):
    """Drive a long random token history through the oracle.

    B1: the state is always the longest suffix of the whole history that is a tree prefix.
    I1/C1 (plain telescoping, final_zero_backoff off, c_unk = 0): the cumulative boost equals
          acc(current state).
    C2 (paper mode): cumulative boost = acc(current state) + sum over end-of-phrase nodes abandoned
          on the way of (acc(f) - acc(fail(f))), + c_unk per unknown-token step.
    """
    V = 5
    toks, offs, wts = W.tiny_case(5000 + seed, vocab_size=V, blank_id=-1, max_phrases=8, max_len=6)
    phrases = _phrases(toks, offs)
    wm = WM[mode]
    c_unk = 0.25
    plain = OracleTree(toks, offs, V, -1, weights=wts, weight_mode=wm, unk_score=0.0, final_zero_backoff=False)
    paper = OracleTree(toks, offs, V, -1, weights=wts, weight_mode=wm, unk_score=c_unk, final_zero_backoff=True)
    bt = BruteTree(phrases, wts, mode=mode, c_unk=c_unk)
    strings = _state_strings(paper)
    rng = np.random.Generator(np.random.PCG64(seed))
    hist = ()
    s_plain = s_paper = 0
    cum_plain = 0.0
    cum_paper = 0.0
    kept = 0.0
    for _ in range(200):
        v = int(rng.integers(0, V))
        y = strings[s_paper]
        gone = bt.abandoned(y, v)
        sc1, s_plain = plain.query(s_plain, v)
        sc2, nx2 = paper.query(s_paper, v)
        hist = hist + (v,)
        assert strings[nx2] == bt.state_of(hist)
        assert s_plain == nx2                     # same automaton, same numbering
        cum_plain += sc1
        cum_paper += sc2
        chain = bt.suffix_chain(y)
        for g in gone:
            if g in bt.finals:
                kept += bt.acc[g] - bt.acc[chain[chain.index(g) + 1]]
        if strings[nx2] == () :
            kept += c_unk
        assert abs(cum_plain - plain.node(s_plain)["acc"]) < 1e-4
        assert abs(cum_paper - (paper.node(nx2)["acc"] + kept)) < 1e-4
        assert cum_plain >= -1e-4
        s_paper = nx2


def _char_ids(text):
    return [27 if ch in " _" else ord(ch) - ord("a") + 1 for ch in text.lower()]


def _load_fig1():
    blocks = []
    with open(os.path.join(GOLDEN, "fig1_cat_trace.txt")) as f:
        cur = None
        for line in f:
            line = line.rstrip("\n")
            if not line or line.startswith("#"):
                continue
            key, _, val = line.partition(" ")
            if key == "text":
                cur = {"text": val, "steps": [], "total": None}
                blocks.append(cur)
            elif key == "total":
                cur["total"] = float(val)
            else:
                cur["steps"].append((key, float(val)))
    return blocks


def test_fig1_worked_example():
    """CAT, CATS, CSV, SIT with c0 = 1, beta = 2, c_unk = 0 on the texts of the golden file."""
    words = ["cat", "cats", "csv", "sit"]
    toks = np.concatenate([_char_ids(w) for w in words]).astype(np.int32)
    offs = np.cumsum([0] + [len(w) for w in words]).astype(np.int64)
    ot = OracleTree(toks, offs, 28, -1, weights=np.ones(4, np.float32), weight_mode=W_LOGDEPTH, beta=2.0,
                    unk_score=0.0)
    assert ot.num_states == 10
    strings = _state_strings(ot)
    sid = {x: i for i, x in enumerate(strings)}
    name = lambda w: sid[tuple(_char_ids(w))]
    assert ot.node(name("cats"))["fail"] == name("s")
    assert ot.node(name("cs"))["fail"] == name("s")
    for w in ["c", "ca", "cat", "csv", "s", "si", "sit"]:
        assert ot.node(name(w))["fail"] == 0
    assert abs(ot.node(name("cats"))["acc"] - 10.178054) < 2e-6
    blocks = _load_fig1()
    assert [b["text"] for b in blocks] == ["the cat is sitting", "catsit", "csi"]
    for blk in blocks:
        s = 0
        total = 0.0
        assert len(blk["steps"]) == len(blk["text"])
        for (ch, want), cid in zip(blk["steps"], _char_ids(blk["text"])):
            assert _char_ids(ch)[0] == cid
            sc, s = ot.query(s, cid)
            assert abs(sc - want) < 2e-6, (blk["text"], ch, sc, want)
            total += sc
        assert abs(total - blk["total"]) < 5e-6


@pytest.mark.parametrize("seed", range(25))
def test_single_phrase_is_kmp_automaton(seed):
    rng = np.random.Generator(np.random.PCG64(300 + seed))
    V = 3
    L = int(rng.integers(1, 9))
    pat = rng.integers(0, V, size=L).astype(np.int32)
    ot = OracleTree(pat, np.array([0, L], np.int64), V, -1)
    delta = kmp_automaton([int(x) for x in pat], V)
    assert ot.num_states == L + 1
    for j in range(L + 1):          # canonical id of a single chain = matched length
        for v in range(V):
            assert ot.query(j, v)[1] == delta[j][v]


@pytest.mark.parametrize("seed", range(25))
def test_zero_weights_give_plain_aho_corasick(seed):
    """With all arc scores 0 every boost is 0 and only the goto/fail automaton remains; it must find
    exactly the phrase occurrences a direct scan of the text finds (end-of-phrase via suffix chain)."""
    V = 4
    toks, offs, _ = W.tiny_case(900 + seed, vocab_size=V, blank_id=-1, max_phrases=6, max_len=4)
    phrases = set(_phrases(toks, offs))
    ot = OracleTree(toks, offs, V, -1, weights=np.zeros(len(offs) - 1, np.float32))
    strings = _state_strings(ot)
    rng = np.random.Generator(np.random.PCG64(seed))
    text = [int(x) for x in rng.integers(0, V, size=120)]
    s = 0
    for i, v in enumerate(text):
        sc, s = ot.query(s, v)
        assert sc == 0.0
        # phrases ending at position i found through the state's suffix chain
        found = set()
        x = s
        while x:
            if ot.node(x)["final"]:
                found.add(strings[x])
            x = ot.node(x)["fail"]
        direct = {p for p in phrases if i + 1 >= len(p) and tuple(text[i + 1 - len(p):i + 1]) == p}
        assert found == direct


def test_blank_keeps_state_and_scores_zero_even_with_unk_score():
    toks, offs, wts = W.tiny_case(11, vocab_size=6, blank_id=0)
    ot = OracleTree(toks, offs, 6, 0, weights=wts, unk_score=0.5)
    for s in range(ot.num_states):
        assert ot.query(s, 0) == (0.0, s)
    sc, nx = ot.score(np.arange(ot.num_states))
    assert np.all(sc[:, 0] == 0.0) and np.all(nx[:, 0] == np.arange(ot.num_states))


def test_score_rows_are_the_single_query_repeated():
    cfg = W.CONFIGS[1]
    toks, offs = W.make_phrases(cfg)
    ot = OracleTree(toks, offs, cfg.vocab_size, cfg.blank_id)
    states = np.arange(ot.num_states, dtype=np.int32)
    sc, nx = ot.score(states)
    for s in range(0, ot.num_states, 5):
        for v in range(0, cfg.vocab_size, 7):
            assert (sc[s, v], nx[s, v]) == ot.query(s, v)


def test_structural_invariants_config2():
    cfg = W.CONFIGS[2]
    toks, offs = W.make_phrases(cfg)
    ot = OracleTree(toks, offs, cfg.vocab_size, cfg.blank_id)
    phrases = set(_phrases(toks, offs))
    n = ot.num_states
    assert n <= 1 + len(toks)
    finals = 0
    for s in range(1, n):
        nd = ot.node(s)
        assert ot.node(nd["fail"])["depth"] < nd["depth"]
        finals += nd["final"]
        # uniform weights of 1: acc = depth, backoff = depth(fail) - depth unless end of phrase
        assert nd["acc"] == nd["depth"]
        want_bw = 0.0 if nd["final"] else ot.node(nd["fail"])["depth"] - nd["depth"]
        assert nd["bw"] == want_bw
    assert finals == len(phrases)
    assert ot.max_depth == max(len(p) for p in phrases)


def test_greedy_step_is_numpy_argmax_of_eq1():
    cfg = W.CONFIGS[1]
    toks, offs = W.make_phrases(cfg)
    ot = OracleTree(toks, offs, cfg.vocab_size, cfg.blank_id)
    logp = W.make_logp(cfg, planting=W.Planting(toks, offs, cover=0.5))
    rng = np.random.Generator(np.random.PCG64(5))
    for t in range(cfg.steps):
        states = rng.integers(0, ot.num_states, size=cfg.batch).astype(np.int32)
        sc, nx = ot.score(states)
        fused = logp[t] + (np.float32(cfg.alpha) * sc).astype(np.float32)
        assert fused.dtype == np.float32
        tok, st, val = ot.fuse_step(logp[t], states, cfg.alpha)
        want = np.argmax(fused, axis=1)
        assert np.array_equal(tok, want)
        assert np.array_equal(st, nx[np.arange(cfg.batch), want])
        assert np.array_equal(val, fused[np.arange(cfg.batch), want])


def test_argmax_ties_take_lowest_token():
    toks = np.array([3, 4], np.int32)
    offs = np.array([0, 2], np.int64)
    ot = OracleTree(toks, offs, 8, 0)
    logp = np.full((1, 8), -2.0, np.float32)
    logp[0, 5] = -1.5          # unboosted best
    tok, st, val = ot.fuse_step(logp, np.array([0], np.int32), 0.5)
    # token 3 gets -2 + 0.5*1 = -1.5: ties with token 5, lower id wins
    assert tok[0] == 3 and st[0] == 1 and val[0] == np.float32(-1.5)


def test_beam_step_is_lexsort_of_all_candidates_and_k1_is_greedy():
    cfg = W.CONFIGS[1]
    toks, offs = W.make_phrases(cfg)
    ot = OracleTree(toks, offs, cfg.vocab_size, cfg.blank_id)
    V = cfg.vocab_size
    rng = np.random.Generator(np.random.PCG64(9))
    logp = W.make_logp(cfg, steps=6, batch=12)
    for t in range(6):
        U, K = 3, 4
        states = rng.integers(0, ot.num_states, size=U * K).astype(np.int32)
        hyp = rng.standard_normal(U * K).astype(np.float32)
        hyp[1] = -np.inf
        hyp[5] = hyp[4]         # tie between beams
        states[5] = states[4]
        lp = logp[t].copy()
        lp[5] = lp[4]
        sc, nx = ot.score(states)
        expansion = lp + (np.float32(cfg.alpha) * sc).astype(np.float32)
        total = (hyp[:, None] + expansion).astype(np.float32)
        tok, par, st, val = ot.fuse_step_beam(lp, hyp, states, cfg.alpha, U, K)
        for u in range(U):
            flat = total[u * K:(u + 1) * K].reshape(-1)
            best = topk_reference(flat, K)
            assert np.array_equal(tok[u * K:(u + 1) * K], best % V)
            assert np.array_equal(par[u * K:(u + 1) * K], best // V)
            assert np.array_equal(val[u * K:(u + 1) * K], flat[best])
            assert np.array_equal(st[u * K:(u + 1) * K], nx[u * K:(u + 1) * K].reshape(-1)[best])
        # K = 1 reproduces the greedy step
        tok1, par1, st1, val1 = ot.fuse_step_beam(lp, np.zeros(U * K, np.float32), states, cfg.alpha, U * K, 1)
        gt, gs, gv = ot.fuse_step(lp, states, cfg.alpha)
        assert np.array_equal(tok1, gt) and np.array_equal(st1, gs) and np.all(par1 == 0)
        assert np.array_equal(val1, (np.float32(0) + gv).astype(np.float32))


def test_beam_all_dead_but_one():
    toks, offs = W.make_phrases(W.CONFIGS[1])
    ot = OracleTree(toks, offs, 128, 0)
    lp = W.make_logp(W.CONFIGS[1], steps=1, batch=4)[0]
    hyp = np.array([0, -np.inf, -np.inf, -np.inf], np.float32)
    tok, par, st, val = ot.fuse_step_beam(lp, hyp, np.zeros(4, np.int32), 0.5, 1, 4)
    assert np.all(par == 0) and len(set(tok.tolist())) == 4 and np.all(np.diff(val) <= 0)


def test_frames_are_steps_chained():
    cfg = W.CONFIGS[1]
    toks, offs = W.make_phrases(cfg)
    ot = OracleTree(toks, offs, cfg.vocab_size, cfg.blank_id)
    logp = W.make_logp(cfg, planting=W.Planting(toks, offs, cover=0.6))
    tokens, states, scores = ot.fuse_frames(logp, np.zeros(cfg.batch, np.int32), cfg.alpha)
    cur = np.zeros(cfg.batch, np.int32)
    deep = 0
    for t in range(cfg.steps):
        tk, cur, sc = ot.fuse_step(logp[t], cur, cfg.alpha)
        assert np.array_equal(tk, tokens[t]) and np.array_equal(cur, states[t]) and np.array_equal(sc, scores[t])
        deep = max(deep, max(ot.node(int(s))["depth"] for s in cur))
    assert deep >= 3          # the planted variant really walks phrases


def test_logdepth_schedule_closed_form():
    """acc at depth d of a single phrase = c0 + sum_{k=2..d} (c0*beta + ln k) = c0 + (d-1) c0 beta + ln d!"""
    L = 9
    ot = OracleTree(np.arange(1, L + 1, dtype=np.int32), np.array([0, L], np.int64), 16, 0,
                    weights=np.array([1.5], np.float32), weight_mode=W_LOGDEPTH, beta=2.0)
    for d in range(1, L + 1):
        want = 1.5 + (d - 1) * 1.5 * 2.0 + math.lgamma(d + 1)
        assert abs(ot.node(d)["acc"] - want) < 1e-12


def test_first_phrase_sets_the_score_of_a_shared_arc():
    toks = np.array([1, 2, 1, 3], np.int32)
    offs = np.array([0, 2, 4], np.int64)
    ot = OracleTree(toks, offs, 8, 0, weights=np.array([2.0, 0.5], np.float32))
    strings = _state_strings(ot)
    sid = {x: i for i, x in enumerate(strings)}
    assert ot.node(sid[(1,)])["acc"] == 2.0          # arc created by the first phrase
    assert ot.node(sid[(1, 2)])["acc"] == 4.0
    assert ot.node(sid[(1, 3)])["acc"] == 2.5        # second phrase's own arc uses its weight


def test_duplicates_prefix_phrases_and_one_token_phrases():
    toks = np.array([1, 2, 1, 2, 1, 2, 3, 4], np.int32)
    offs = np.array([0, 2, 4, 7, 8], np.int64)
    ot = OracleTree(toks, offs, 8, 0)
    assert ot.num_states == 5                       # (), 1, 4, 12, 123
    strings = _state_strings(ot)
    sid = {x: i for i, x in enumerate(strings)}
    assert ot.node(sid[(1, 2)])["final"] and ot.node(sid[(1, 2)])["bw"] == 0.0
    assert ot.child(sid[(1, 2)], 3) == sid[(1, 2, 3)]
    # a one-token phrase keeps its score on exit
    assert ot.query(sid[(4,)], 5) == (0.0, 0)


@pytest.mark.parametrize("bad", ["empty", "range", "blank", "vocab", "neg"])
def test_build_rejects_bad_input(bad):
    toks = np.array([1, 2, 3], np.int32)
    offs = np.array([0, 2, 3], np.int64)
    V, blank = 8, 0
    if bad == "empty":
        offs = np.array([0, 2, 2, 3], np.int64)
    elif bad == "range":
        toks = np.array([1, 9, 3], np.int32)
    elif bad == "blank":
        toks = np.array([1, 0, 3], np.int32)
    elif bad == "vocab":
        V = 0
    elif bad == "neg":
        toks = np.array([1, -2, 3], np.int32)
    with pytest.raises(OracleError):
        OracleTree(toks, offs, V, blank)


def test_workload_generators_are_seeded_and_shaped():
    for idx, cfg in W.CONFIGS.items():
        n = min(cfg.n_phrases, 500)
        t1, o1 = W.make_phrases(cfg, n_phrases=n)
        t2, o2 = W.make_phrases(cfg, n_phrases=n)
        assert np.array_equal(t1, t2) and np.array_equal(o1, o2)
        lens = np.diff(o1)
        assert lens.min() >= cfg.len_lo and lens.max() <= cfg.len_hi
        assert t1.min() >= 1 and t1.max() < cfg.vocab_size
    cfg = W.CONFIGS[1]
    a = W.make_logp(cfg, chunk_frames=7)
    b = W.make_logp(cfg, chunk_frames=50)
    assert np.array_equal(a, b) and a.shape == (50, 4, 128) and a.dtype == np.float32
    assert np.allclose(np.exp(a.astype(np.float64)).sum(-1), 1.0, atol=1e-5)


def test_uniform_weights_with_final_reward_by_hand():
    """Phrases (1,2), (1,2,3) and (4,), every transition 1.0: the arc that completes a phrase also pays the
    accumulated uniform score of the phrase (Sec. II-B, the uniform distribution with a final-node reward).

      arc 1: 1          acc (1)     = 1
      arc 2: 1 + 2 = 3  acc (1,2)   = 4      (two transitions completed)
      arc 3: 1 + 3 = 4  acc (1,2,3) = 8      (three transitions completed)
      arc 4: 1 + 1 = 2  acc (4)     = 2
    """
    ot = OracleTree(np.array([1, 2, 1, 2, 3, 4], np.int32), np.array([0, 2, 5, 6], np.int64), 6, 0,
                    weight_mode=W_UNIFORM_FINAL)
    by = {ot.prefix(s): ot.node(s) for s in range(ot.num_states)}
    assert [by[k]["acc"] for k in [(1,), (1, 2), (1, 2, 3), (4,)]] == [1.0, 4.0, 8.0, 2.0]
    assert [by[k]["arcw"] for k in [(1,), (1, 2), (1, 2, 3), (4,)]] == [1.0, 3.0, 4.0, 2.0]
    s1 = [s for s in range(ot.num_states) if ot.prefix(s) == (1,)][0]
    assert ot.query(s1, 5) == (-1.0, 0)          # partial match abandoned: its score is paid back
    s12 = [s for s in range(ot.num_states) if ot.prefix(s) == (1, 2)][0]
    assert ot.query(s12, 5) == (0.0, 0)          # a completed phrase keeps its score
