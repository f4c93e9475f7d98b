"""GPU parity of the kernels for rows wider than 1024 tokens (the single step spread over a workgroup, the
multi-frame decoder with its chunk ring and boundary guesses), of the full-size decoding loops fed with the
GPU's own states, and of segment shapes the other tests do not reach (segments of 64 frames and more,
blank-heavy rows under every rule).  Every output against the CPU oracle: ids bit-exact, scores within 1e-5."""
import numpy as np
import pytest

import pb_workloads as W
from oracle import OracleTree

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import paper_2508_07014_amd as pb  # noqa: E402
from gpu_helpers import DEV, TOL, assert_scores, config_trees, dev, frames_ws, gpu_beam_step, gpu_score  # noqa: E402


def _random_tree(rng, V, blank, eos, nph, max_len, wmode, unk):
    cfg = W.Config(9, "wide", V, blank, nph, 1, max_len, "zipf" if rng.random() < 0.7 else "uniform", 1.1, 1, 1, 1, 2.0)
    toks, offs = W.make_phrases(cfg, seed=int(rng.integers(1 << 30)))
    for bad in (blank, eos):
        if bad >= 1:
            toks = np.where(toks == bad, bad - 1 if bad - 1 not in (blank, eos, 0) else bad - 2, toks).astype(np.int32)
    kw = dict(weight_mode=wmode, unk_score=unk)
    ot = OracleTree(toks, offs, V, blank, eos_id=eos, final_eos_score=0.75, **kw)
    tr = pb.pb_build(toks, offs, V, blank, device=0, eos_id=eos, final_eos_score=0.75, **kw)
    assert pb.pb_info(tr)["num_states"] == ot.num_states
    return toks, offs, ot, tr


def _rows(rng, kind, T, B, V, blank, toks, offs):
    seed = int(rng.integers(1 << 30))
    shape = W.Config(9, "wide", V, blank, 1, 1, 8, "uniform", 1.1, B, 1, T, 2.0)
    if kind == 0:
        return W.sticky_logp(seed, T, B, V, blank, grid=None, bump=float(rng.choice([3.0, 8.0])))
    if kind == 1:
        return W.make_logp(shape, seed=seed, planting=W.Planting(toks, offs, cover=float(rng.choice([0.3, 0.9])), bump=10.0))
    if kind == 2:
        return W.make_logp(shape, seed=seed, blank_bias=8.0, blank_frac=0.7)
    if kind == 3:
        return W.log_softmax_rows(rng.standard_normal((T, B, V)) * 0.2)
    x = np.round(rng.standard_normal((T, B, V)) * 2).astype(np.float32)   # many exact ties
    x[rng.random((T, B)) < 0.1] = -np.inf                                 # whole rows of -inf
    return x


@pytest.mark.parametrize("chunk", range(4))
def test_wide_step_random_cases(chunk):
    """pb_fuse_step_select on rows of 1028 .. 16384 tokens: states from all states, blank ids, an EOS token, every
    rule with previous labels, row strides above V, exact ties and rows of -inf."""
    rng = np.random.default_rng(9100 + chunk)
    for case in range(14):
        V = int(rng.choice([1028, 2048, 4096, 5004, 8192, 16384]))
        blank = int(rng.choice([0, -1, 5]))
        eos = int(rng.choice([-1, V - 1, 7]))
        wmode, unk = int(rng.integers(0, 3)), float(rng.choice([0.0, 0.5, -0.25]))
        toks, offs, ot, tr = _random_tree(rng, V, blank, eos, int(rng.integers(1, 1500)), int(rng.integers(2, 9)), wmode, unk)
        B = int(rng.choice([1, 3, 20, 70]))
        kind = int(rng.choice([0, 1, 2, 3, 4]))
        logp = _rows(rng, kind, 1, B, V, blank, toks, offs)[0]
        states = rng.integers(0, ot.num_states, B).astype(np.int32)
        if rng.random() < 0.2:
            states[0] = ot.num_states + 3
        last = rng.integers(-1, V, B).astype(np.int32)
        if blank >= 0:
            last[rng.random(B) < 0.3] = blank
        ok = [b for b in range(B) if 0 <= states[b] < ot.num_states]
        alpha = float(rng.choice([0.0, 0.5, 1.0, 2.0]))
        stride = V + int(rng.choice([0, 4, 64]))
        padded = np.full((B, stride), 9.0, np.float32)     # a value that would win if it were read
        padded[:, :V] = logp
        d_logp = dev(padded)
        for mode in (0, 1, 2):
            want = ot.fuse_step_select(np.ascontiguousarray(logp[ok]), states[ok], last[ok], alpha, mode)
            d_tok = torch.full((B,), -7, dtype=torch.int32, device=DEV)
            d_st = torch.full((B,), -7, dtype=torch.int32, device=DEV)
            d_sc = torch.zeros(B, dtype=torch.float32, device=DEV)
            pb.pb_fuse_step_select(tr, d_logp, stride, dev(states), dev(last), alpha, B, mode, d_tok, d_st, d_sc, 0)
            torch.cuda.synchronize()
            tk, st, sc = d_tok.cpu().numpy(), d_st.cpu().numpy(), d_sc.cpu().numpy()
            where = dict(chunk=chunk, case=case, V=V, blank=blank, eos=eos, B=B, kind=kind, mode=mode, alpha=alpha)
            assert np.array_equal(tk[ok], want[0]) and np.array_equal(st[ok], want[1]), where
            assert_scores(sc[ok], want[2])
            for b in range(B):
                if b not in ok:
                    assert tk[b] == -1 and st[b] == -1 and np.isnan(sc[b]), where
        pb.pb_free(tr)


@pytest.mark.parametrize("chunk", range(4))
def test_wide_frames_random_cases(chunk):
    """pb_fuse_frames_select on wide rows: several segments per hypothesis, every rule, an EOS token, blank-heavy
    and phrase-planted rows, start states and previous labels from the caller."""
    rng = np.random.default_rng(9300 + chunk)
    for case in range(8):
        V = int(rng.choice([1028, 2048, 4096, 5004, 8192, 16384]))
        blank = int(rng.choice([0, -1, 5]))
        eos = int(rng.choice([-1, V - 1]))
        wmode, unk = int(rng.integers(0, 3)), float(rng.choice([0.0, 0.5]))
        toks, offs, ot, tr = _random_tree(rng, V, blank, eos, int(rng.integers(1, 800)), int(rng.integers(2, 9)), wmode, unk)
        T = int(rng.choice([1, 9, 40, 130]))
        B = int(rng.choice([1, 3, 9]))
        kind = int(rng.choice([0, 1, 2, 3, 4]))
        logp = _rows(rng, kind, T, B, V, blank, toks, offs)
        s0 = rng.integers(0, ot.num_states, B).astype(np.int32)
        if rng.random() < 0.2:
            s0[0] = -1
        last0 = rng.integers(-1, V, B).astype(np.int32) if rng.random() < 0.5 else None
        ok = [b for b in range(B) if 0 <= s0[b] < ot.num_states]
        alpha = float(rng.choice([0.0, 0.5, 1.0]))
        d_logp = dev(logp)
        for mode in (0, 1, 2):
            want = ot.fuse_frames_select(np.ascontiguousarray(logp[:, ok]), s0[ok], None if last0 is None else last0[ok],
                                         alpha, mode)
            d_tok = torch.full((T, B), -7, dtype=torch.int32, device=DEV)
            d_st = torch.full((T, B), -7, dtype=torch.int32, device=DEV)
            d_sc = torch.zeros((T, B), dtype=torch.float32, device=DEV)
            pb.pb_fuse_frames_select(tr, d_logp, B * V, V, dev(s0), None if last0 is None else dev(last0), alpha, T, B,
                                     mode, d_tok, d_st, d_sc, 0)
            torch.cuda.synchronize()
            tk, st, sc = d_tok.cpu().numpy(), d_st.cpu().numpy(), d_sc.cpu().numpy()
            where = dict(chunk=chunk, case=case, V=V, blank=blank, eos=eos, T=T, B=B, kind=kind, mode=mode, alpha=alpha)
            assert np.array_equal(tk[:, ok], want[0]) and np.array_equal(st[:, ok], want[1]), where
            assert_scores(sc[:, ok], want[2])
            for b in range(B):
                if b not in ok:
                    assert np.all(tk[:, b] == -1) and np.all(st[:, b] == -1) and np.all(np.isnan(sc[:, b])), where
        pb.pb_free(tr)


@pytest.mark.parametrize("V,T,B", [(64, 256, 1024), (128, 400, 2048), (1024, 4096, 64), (256, 8200, 1)])
def test_frames_with_segments_of_64_frames_and_more(V, T, B):
    """Shapes whose segments are whole multiples of, or longer than, the 64 frames one group of lane-held outputs
    covers: the group hand-over and the boundary certificate in the last group."""
    rng = np.random.default_rng(V + T)
    toks, offs, ot, tr = _random_tree(rng, V, 0, -1, 300, 6, 0, 0.0)
    logp = W.make_logp(W.Config(9, "seg", V, 0, 1, 1, 8, "uniform", 1.1, B, 1, T, 2.0), seed=V * T,
                       planting=W.Planting(toks, offs, cover=0.3), blank_bias=6.0, blank_frac=0.3)
    s0 = np.zeros(B, np.int32)
    d_logp = dev(logp)
    for mode in (0, 2):
        want = ot.fuse_frames_select(logp, s0, None, 0.5, mode)
        d_tok = torch.full((T, B), -7, dtype=torch.int32, device=DEV)
        d_st = torch.full((T, B), -7, dtype=torch.int32, device=DEV)
        d_sc = torch.zeros((T, B), dtype=torch.float32, device=DEV)
        pb.pb_fuse_frames_select(tr, d_logp, B * V, V, dev(s0), None, 0.5, T, B, mode, d_tok, d_st, d_sc, 0)
        torch.cuda.synchronize()
        assert np.array_equal(d_tok.cpu().numpy(), want[0]) and np.array_equal(d_st.cpu().numpy(), want[1]), mode
        assert_scores(d_sc.cpu().numpy(), want[2])
        got = frames_ws(tr, d_logp, dev(s0), None, 0.5, mode)
        assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1]), mode
        assert_scores(got[2], want[2])
    pb.pb_free(tr)


def test_frames_with_workspace_config3_planted_and_blank_heavy():
    """The workspace form at the headline shape on rows where many boundary guesses are wrong (planted phrases:
    the hypotheses sit deep in the tree; blank-heavy rows: the state survives long stretches), every rule."""
    cfg, toks, offs, ot, tr = config_trees(3)
    B = cfg.batch
    for kw in (dict(planting=W.Planting(toks, offs)), dict(blank_bias=8.0, blank_frac=0.75), {}):
        logp = W.make_logp(cfg, steps=500, **kw)
        d_logp = dev(logp)
        for mode in (0, 1, 2):
            want = ot.fuse_frames_select(logp, np.zeros(B, np.int32), None, cfg.alpha, mode)
            got = frames_ws(tr, d_logp, dev(np.zeros(B, np.int32)), None, cfg.alpha, mode)
            assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1]), (list(kw), mode)
            assert np.array_equal(got[2], want[2]), (list(kw), mode)
    need = pb.pb_fuse_frames_workspace_bytes(tr, 500, B)
    assert need > 0
    with pytest.raises(pb.PbError):      # a workspace that is too small is refused
        ws = torch.zeros(need // 4, dtype=torch.int32, device=DEV)
        pb.pb_fuse_frames_ws(tr, d_logp, B * cfg.vocab_size, cfg.vocab_size, dev(np.zeros(B, np.int32)), None, cfg.alpha,
                             500, B, 0, ws, ws, ws, ws, need - 4, 0)


def test_workspace_reused_back_to_back_with_other_inputs():
    """One workspace, calls on different inputs queued one behind the other without a synchronisation in between:
    what an earlier call has left in the workspace (patches, the first frames of every segment) must mean nothing
    to the next one.  Planted rows first (many repairs), then other rows of the same shape, then a shorter call."""
    cfg, toks, offs, ot, tr = config_trees(3)
    B, V, T = cfg.batch, cfg.vocab_size, 400
    inputs = [W.make_logp(cfg, steps=T, seed=11, planting=W.Planting(toks, offs)),
              W.make_logp(cfg, steps=T, seed=12, planting=W.Planting(toks, offs)),
              W.make_logp(cfg, steps=T, seed=13, blank_bias=8.0, blank_frac=0.75),
              W.make_logp(cfg, steps=173, seed=14, planting=W.Planting(toks, offs))]
    need = max(pb.pb_fuse_frames_workspace_bytes(tr, x.shape[0], B) for x in inputs)
    ws = torch.full((need // 4,), -1, dtype=torch.int32, device=DEV)   # (never cleared)
    s0 = dev(np.zeros(B, np.int32))
    for mode in (0, 2):
        d_in = [dev(x) for x in inputs]
        outs = [(torch.full(x.shape[:2], -7, dtype=torch.int32, device=DEV), torch.full(x.shape[:2], -7, dtype=torch.int32, device=DEV),
                 torch.zeros(x.shape[:2], dtype=torch.float32, device=DEV)) for x in inputs]
        for rep in range(2):
            for x, d, o in zip(inputs, d_in, outs):
                pb.pb_fuse_frames_ws(tr, d, B * V, V, s0, None, cfg.alpha, x.shape[0], B, mode, o[0], o[1], o[2], ws, need, 0)
        torch.cuda.synchronize()
        for k, (x, o) in enumerate(zip(inputs, outs)):
            want = ot.fuse_frames_select(x, np.zeros(B, np.int32), None, cfg.alpha, mode)
            for g, w in zip(o, want):
                assert np.array_equal(g.cpu().numpy(), w), (mode, k)


def _chain_steps(tr, logp, alpha, mode=0):
    """T calls of the step entry point, each fed with the states (and labels) the previous call left on the GPU."""
    T, B, V = logp.shape
    d_logp = dev(logp)
    d_tok = torch.full((T, B), -7, dtype=torch.int32, device=DEV)
    d_st = torch.full((T, B), -7, dtype=torch.int32, device=DEV)
    d_sc = torch.zeros((T, B), dtype=torch.float32, device=DEV)
    prev, last = torch.zeros(B, dtype=torch.int32, device=DEV), None
    for t in range(T):
        pb.pb_fuse_step_select(tr, d_logp[t], V, prev, last, alpha, B, mode, d_tok[t], d_st[t], d_sc[t], 0)
        prev, last = d_st[t], d_tok[t]
    torch.cuda.synchronize()
    return d_tok.cpu().numpy(), d_st.cpu().numpy(), d_sc.cpu().numpy()


def test_step_loop_config3_all_frames():
    """Config 3 at full size through pb_fuse_step, all 1000 frames chained on the GPU."""
    cfg, toks, offs, ot, tr = config_trees(3)
    logp = W.make_logp(cfg, planting=W.Planting(toks, offs, cover=0.2))
    want = ot.fuse_frames(logp, np.zeros(cfg.batch, np.int32), cfg.alpha)
    got = _chain_steps(tr, logp, cfg.alpha)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1]) and np.array_equal(got[2], want[2])


def test_step_loop_and_frames_config5_all_steps():
    """Config 5 at full size (V = 8192, B = 256, 200 steps): the step loop chained on the GPU and the multi-frame
    call, planted phrases included so that deep states occur."""
    cfg, toks, offs, ot, tr = config_trees(5)
    logp = W.make_logp(cfg, planting=W.Planting(toks, offs, cover=0.2))
    B, V = cfg.batch, cfg.vocab_size
    want = ot.fuse_frames(logp, np.zeros(B, np.int32), cfg.alpha)
    got = _chain_steps(tr, logp, cfg.alpha)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1]) and np.array_equal(got[2], want[2])
    d_tok = torch.full((cfg.steps, B), -7, dtype=torch.int32, device=DEV)
    d_st = torch.full((cfg.steps, B), -7, dtype=torch.int32, device=DEV)
    d_sc = torch.zeros((cfg.steps, B), dtype=torch.float32, device=DEV)
    pb.pb_fuse_frames(tr, dev(logp), B * V, V, dev(np.zeros(B, np.int32)), cfg.alpha, cfg.steps, B, d_tok, d_st, d_sc, 0)
    torch.cuda.synchronize()
    assert np.array_equal(d_tok.cpu().numpy(), want[0]) and np.array_equal(d_st.cpu().numpy(), want[1])
    assert np.array_equal(d_sc.cpu().numpy(), want[2])
    assert max(ot.node(int(s))["depth"] for s in np.unique(want[1])) >= 4


def test_score_every_row_of_the_largest_sweep_shape():
    """pb_score at B = 1024, V = 8192 (the 64 MiB point of the sweep): every element of both outputs."""
    cfg, toks, offs, ot, tr = config_trees(5)
    states = W.sample_states(ot.num_states, 1024, 77)
    ws, wn = ot.score(states)
    gs, gn = gpu_score(tr, states, cfg.vocab_size)
    assert np.array_equal(gn, wn) and np.array_equal(gs, ws)


@pytest.mark.parametrize("V", [2048, 8192])
def test_beam_wide_rows_deep_states(V):
    """Beam step with K = 8 on wide rows, states drawn from all states of a 20K-phrase tree."""
    cfg = W.CONFIGS[5]
    shape = W.Config(9, "beam", V, -1, 20000 if V == 8192 else 3000, 2, 8, "zipf", 1.1, 1, 1, 1, 2.0)
    toks, offs = W.make_phrases(shape, seed=V)
    ot = OracleTree(toks, offs, V, -1, weight_mode=1)
    tr = pb.pb_build(toks, offs, V, -1, weight_mode=1, device=0)
    U, K = 6, 8
    rng = np.random.default_rng(V)
    states = W.sample_states(ot.num_states, U * K, V + 1)
    logp = W.log_softmax_rows(rng.standard_normal((U * K, V)) * 1.5)
    hyp = rng.standard_normal(U * K).astype(np.float32)
    hyp[3] = -np.inf
    want = ot.fuse_step_beam(logp, hyp, states, cfg.alpha, U, K)
    got = gpu_beam_step(tr, dev(logp), dev(hyp), dev(states), cfg.alpha, U, K)
    torch.cuda.synchronize()
    for g, w in zip(got[:3], want[:3]):
        assert np.array_equal(g.cpu().numpy(), w)
    assert_scores(got[3].cpu().numpy(), want[3])
    assert max(ot.node(int(s))["depth"] for s in states) >= 4
    pb.pb_free(tr)


def test_wide_rows_under_a_forest():
    """Per-hypothesis trees on wide rows: the multi-frame call and the step call, each row against its own oracle."""
    V, blank = 2048, 0
    rng = np.random.default_rng(31)
    members = [_random_tree(rng, V, blank, -1, 200 + 100 * i, 5, i % 3, 0.0) for i in range(3)]
    forest = pb.pb_forest_build([m[3] for m in members])
    T, B = 30, 7
    ids = rng.integers(0, 3, B).astype(np.int32)
    ids[2] = 5                                              # an unknown tree marks its row
    logp = W.sticky_logp(77, T, B, V, blank, grid=None, bump=6.0)
    d_logp = dev(logp)
    for mode in (0, 2):
        d_tok = torch.full((T, B), -7, dtype=torch.int32, device=DEV)
        d_st = torch.full((T, B), -7, dtype=torch.int32, device=DEV)
        d_sc = torch.zeros((T, B), dtype=torch.float32, device=DEV)
        pb.pb_fuse_frames_forest(forest, d_logp, B * V, V, dev(ids), dev(np.zeros(B, np.int32)), None, 0.5, T, B, mode,
                                 d_tok, d_st, d_sc, 0)
        s_tok = torch.full((B,), -7, dtype=torch.int32, device=DEV)
        s_st = torch.full((B,), -7, dtype=torch.int32, device=DEV)
        s_sc = torch.zeros(B, dtype=torch.float32, device=DEV)
        pb.pb_fuse_step_forest(forest, d_logp[0], V, dev(ids), dev(np.zeros(B, np.int32)), None, 0.5, B, mode, s_tok, s_st,
                               s_sc, 0)
        torch.cuda.synchronize()
        tk, st, sc = d_tok.cpu().numpy(), d_st.cpu().numpy(), d_sc.cpu().numpy()
        for b in range(B):
            if ids[b] >= 3:
                assert np.all(tk[:, b] == -1) and np.all(st[:, b] == -1) and np.all(np.isnan(sc[:, b]))
                assert s_tok[b].item() == -1 and s_st[b].item() == -1
                continue
            want = members[ids[b]][2].fuse_frames_select(np.ascontiguousarray(logp[:, b:b + 1]), np.zeros(1, np.int32),
                                                         None, 0.5, mode)
            assert np.array_equal(tk[:, b], want[0][:, 0]) and np.array_equal(st[:, b], want[1][:, 0]), (mode, b)
            assert np.max(np.abs(sc[:, b] - want[2][:, 0])) <= TOL
            assert s_tok[b].item() == want[0][0, 0] and s_st[b].item() == want[1][0, 0]
    pb.pb_forest_free(forest)
