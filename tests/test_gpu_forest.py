"""GPU parity of the forest calls (a different context list per hypothesis / utterance): every row must
equal what the CPU oracle of the row's own tree gives.  Ids bit-exact, scores within 1e-5."""
import numpy as np
import pytest

import pb_workloads as W
from oracle.pb_oracle import SELECT_FUSED, SELECT_TWO_STAGE_CTC, W_LOGDEPTH

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import paper_2508_07014_amd as pb  # noqa: E402
from gpu_helpers import DEV, assert_scores, build_both, dev, stream_ptr  # noqa: E402


def make_forest(V, n_trees=3, blank=0):
    cfg = W.CONFIGS[1]
    pairs = []
    for i in range(n_trees):
        toks, offs = W.make_phrases(cfg, seed=900 + i, n_phrases=5 + 20 * i)
        toks = (toks % (V - 1) + 1).astype(np.int32)
        pairs.append(build_both(toks, offs, V, blank, weight_mode=W_LOGDEPTH if i % 2 else 0))
    forest = pb.pb_forest_build([tr for _, tr in pairs])
    return [ot for ot, _ in pairs], forest


@pytest.mark.parametrize("V", [128, 130, 1024, 2048])
def test_forest_score_and_greedy_step(V):
    ots, forest = make_forest(V)
    rng = np.random.default_rng(V)
    B = 61
    ids = rng.integers(0, len(ots), B).astype(np.int32)
    ids[7] = len(ots)                      # unknown tree: the row is marked
    ids[11] = -1
    states = np.array([rng.integers(0, ots[i].num_states) if 0 <= i < len(ots) else 0 for i in ids], np.int32)
    logp = W.sticky_logp(V, 1, B, V, 0, grid=None, bump=5.0)[0]
    last = rng.integers(-1, 6, B).astype(np.int32)
    d_ids, d_states, d_logp = dev(ids), dev(states), dev(logp)
    d_scores = torch.zeros((B, V), dtype=torch.float32, device=DEV)
    d_next = torch.zeros((B, V), dtype=torch.int32, device=DEV)
    pb.pb_score_forest(forest, d_ids, d_states, B, d_scores, d_next, stream_ptr())
    outs = {}
    for mode in (SELECT_FUSED, SELECT_TWO_STAGE_CTC):
        o = [torch.zeros(B, dtype=torch.int32, device=DEV), torch.zeros(B, dtype=torch.int32, device=DEV),
             torch.zeros(B, dtype=torch.float32, device=DEV)]
        pb.pb_fuse_step_forest(forest, d_logp, V, d_ids, d_states, dev(last), 0.6, B, mode, o[0], o[1], o[2], stream_ptr())
        outs[mode] = o
    torch.cuda.synchronize()
    gs, gn = d_scores.cpu().numpy(), d_next.cpu().numpy()
    for i, ot in enumerate(ots):
        rows = np.flatnonzero(ids == i)
        ws, wn = ot.score(states[rows])
        assert np.array_equal(gn[rows], wn)
        assert_scores(gs[rows], ws)
        for mode, o in outs.items():
            want = ot.fuse_step_select(logp[rows], states[rows], last[rows], 0.6, mode)
            assert np.array_equal(o[0].cpu().numpy()[rows], want[0]) and np.array_equal(o[1].cpu().numpy()[rows], want[1])
            assert_scores(o[2].cpu().numpy()[rows], want[2])
    for b in (7, 11):
        assert np.all(np.isnan(gs[b])) and np.all(gn[b] == -1)
        for o in outs.values():
            assert o[0][b].item() == -1 and o[1][b].item() == -1 and np.isnan(o[2][b].item())


@pytest.mark.parametrize("V,K", [(128, 4), (130, 3)])
def test_forest_beam_step(V, K):
    ots, forest = make_forest(V)
    rng = np.random.default_rng(K)
    U = 9
    ids = rng.integers(0, len(ots), U).astype(np.int32)
    ids[4] = 17
    states = np.concatenate([rng.integers(0, ots[i].num_states if i < len(ots) else 1, K) for i in ids]).astype(np.int32)
    logp = W.log_softmax_rows(rng.standard_normal((U * K, V)) * 2)
    hyp = rng.standard_normal(U * K).astype(np.float32)
    o = [torch.zeros(U * K, dtype=torch.int32, device=DEV) for _ in range(3)] + [torch.zeros(U * K, device=DEV)]
    pb.pb_fuse_step_beam_forest(forest, dev(logp), V, dev(ids), dev(hyp), dev(states), 0.5, U, K, o[0], o[1], o[2], o[3],
                                stream_ptr())
    torch.cuda.synchronize()
    for u in range(U):
        sl = slice(u * K, (u + 1) * K)
        if ids[u] >= len(ots):
            assert np.all(o[0].cpu().numpy()[sl] == -1) and np.all(np.isnan(o[3].cpu().numpy()[sl]))
            continue
        want = ots[ids[u]].fuse_step_beam(logp[sl], hyp[sl], states[sl], 0.5, 1, K)
        for g, w in zip(o[:3], want[:3]):
            assert np.array_equal(g.cpu().numpy()[sl], w)
        assert_scores(o[3].cpu().numpy()[sl], want[3])


def test_forest_build_rejects_mismatched_trees():
    cfg = W.CONFIGS[1]
    toks, offs = W.make_phrases(cfg)
    a = pb.pb_build(toks, offs, 128, 0, device=0)
    b = pb.pb_build(toks, offs, 256, 0, device=0)
    c = pb.pb_build(toks, offs, 128, -1, device=0)
    d = pb.pb_build(np.where(toks == 127, 1, toks).astype(np.int32), offs, 128, 0, device=0, eos_id=127)
    h = pb.pb_build(toks, offs, 128, 0, device=-1)
    for bad, code in (([a, b], pb.PB_EUNSUPPORTED), ([a, c], pb.PB_EUNSUPPORTED), ([a, d], pb.PB_EUNSUPPORTED),
                      ([a, h], pb.PB_EINVAL), ([], pb.PB_EINVAL)):
        with pytest.raises(pb.PbError) as e:
            pb.pb_forest_build(bad)
        assert e.value.code == code
    pb.pb_forest_free(pb.pb_forest_build([a, a]))


@pytest.mark.parametrize("V,T,B", [(128, 50, 9), (1024, 150, 12), (2048, 20, 5), (130, 30, 7)])
def test_forest_frames(V, T, B):
    """All frames in one call, a tree per hypothesis: wave kernels (V % 4 == 0) and the workgroup kernel."""
    ots, forest = make_forest(V)
    rng = np.random.default_rng(T)
    ids = rng.integers(0, len(ots), B).astype(np.int32)
    ids[3] = 5                                # unknown tree: every frame of the hypothesis is marked
    s0 = np.array([rng.integers(0, ots[i].num_states) if i < len(ots) else 0 for i in ids], np.int32)
    logp = W.sticky_logp(V + T, T, B, V, 0, grid=None, bump=6.0)
    for mode in (SELECT_FUSED, SELECT_TWO_STAGE_CTC):
        d_tok = torch.full((T, B), -5, dtype=torch.int32, device=DEV)
        d_st = torch.full((T, B), -5, dtype=torch.int32, device=DEV)
        d_sc = torch.zeros((T, B), dtype=torch.float32, device=DEV)
        pb.pb_fuse_frames_forest(forest, dev(logp), B * V, V, dev(ids), dev(s0), None, 0.6, T, B, mode, d_tok, d_st, d_sc,
                                 stream_ptr())
        torch.cuda.synchronize()
        tok, st, sc = d_tok.cpu().numpy(), d_st.cpu().numpy(), d_sc.cpu().numpy()
        for i, ot in enumerate(ots):
            cols = np.flatnonzero(ids == i)
            if len(cols) == 0:
                continue
            want = ot.fuse_frames_select(np.ascontiguousarray(logp[:, cols]), s0[cols], None, 0.6, mode)
            assert np.array_equal(tok[:, cols], want[0]) and np.array_equal(st[:, cols], want[1])
            assert_scores(sc[:, cols], want[2])
        assert np.all(tok[:, 3] == -1) and np.all(st[:, 3] == -1) and np.all(np.isnan(sc[:, 3]))
