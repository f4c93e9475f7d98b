"""GPU parity of the end-of-sentence heuristics (Sec. II-C) in pb_score, pb_fuse_step(_select),
pb_fuse_frames and pb_fuse_step_beam against the CPU oracle.  Ids bit-exact, scores within 1e-5."""
import numpy as np
import pytest

import pb_workloads as W
from oracle import OracleTree
from oracle.pb_oracle import SELECT_FUSED, SELECT_TWO_STAGE, SELECT_TWO_STAGE_CTC, W_LOGDEPTH, W_UNIFORM

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import paper_2508_07014_amd as pb  # noqa: E402
from gpu_helpers import (DEV, assert_scores, dev, gpu_beam_step, gpu_fuse_frames, gpu_fuse_step, gpu_score,  # noqa: E402
                         stream_ptr)


def both(tokens, offsets, V, blank, eos, c_eos, **kw):
    ot = OracleTree(tokens, offsets, V, blank, weights=kw.get("weights"), weight_mode=kw.get("weight_mode", 0),
                    unk_score=kw.get("unk_score", 0.0), eos_id=eos, final_eos_score=c_eos)
    tr = pb.pb_build(tokens, offsets, V, blank, device=0, eos_id=eos, final_eos_score=c_eos, **kw)
    assert pb.pb_info(tr)["num_states"] == ot.num_states and pb.pb_info(tr)["eos_id"] == eos
    return ot, tr


@pytest.mark.parametrize("seed", range(12))
def test_score_rows_with_eos_all_states(seed):
    V = [6, 8, 9, 12, 66, 130][seed % 6]
    blank = 0 if seed % 2 else -1
    toks, offs, wts = W.tiny_case(7700 + seed, vocab_size=min(V - 1, 8), blank_id=blank, max_phrases=10, max_len=6)
    if seed % 3 == 1:
        wts = -wts
    eos = V - 1
    ot, tr = both(toks, offs, V, blank, eos, [0.0, 1.5, -0.25][seed % 3], weights=wts,
                  weight_mode=W_LOGDEPTH if seed % 2 else W_UNIFORM, unk_score=[0.0, -0.5][seed % 2])
    states = np.arange(ot.num_states, dtype=np.int32)
    ws, wn = ot.score(states)
    gs, gn = gpu_score(tr, states, V)
    assert np.array_equal(gn, wn)
    assert_scores(gs, ws)
    gs2, _ = gpu_score(tr, states, V, want_next=False)
    assert_scores(gs2, ws)


def _config5_with_eos():
    cfg = W.CONFIGS[5]
    toks, offs = W.make_phrases(cfg)
    eos = cfg.vocab_size - 1
    toks = np.where(toks == eos, 1, toks).astype(np.int32)
    return (cfg, toks, offs, eos) + both(toks, offs, cfg.vocab_size, -1, eos, 2.0)


def test_score_and_greedy_config5_with_eos():
    cfg, toks, offs, eos, ot, tr = _config5_with_eos()
    V, B = cfg.vocab_size, 96
    states = W.sample_states(ot.num_states, B, 11)
    ws, wn = ot.score(states)
    gs, gn = gpu_score(tr, states, V)
    assert np.array_equal(gn, wn) and np.array_equal(gs, ws)
    rng = np.random.default_rng(5)
    logp = W.log_softmax_rows(rng.standard_normal((B, V)) * 0.5)
    logp[:, eos] += np.float32(1.0)
    want = ot.fuse_step(logp, states, cfg.alpha)
    tk, st, sc = gpu_fuse_step(tr, dev(logp), dev(states), cfg.alpha)
    torch.cuda.synchronize()
    assert np.array_equal(tk.cpu().numpy(), want[0]) and np.array_equal(st.cpu().numpy(), want[1])
    assert_scores(sc.cpu().numpy(), want[2])
    assert 0 < np.sum(want[0] == eos) < B


@pytest.mark.parametrize("V", [128, 130])
def test_decoding_loop_with_eos_and_selection_rules(V):
    cfg = W.CONFIGS[1]
    toks, offs = W.make_phrases(cfg)
    eos = 127
    toks = np.where(toks == eos, 3, toks).astype(np.int32)
    ot, tr = both(toks, offs, V, 0, eos, 1.0, weight_mode=W_LOGDEPTH)
    T, B = 40, 6
    logp = W.sticky_logp(31, T, B, V, 0, grid=None, bump=7.0)
    logp[:, :, eos] += np.float32(4.0)
    d_logp = dev(logp)
    for mode in (SELECT_FUSED, SELECT_TWO_STAGE, SELECT_TWO_STAGE_CTC):
        want = ot.fuse_frames_select(logp, np.zeros(B, np.int32), None, 0.7, mode)
        d_tok = torch.zeros((T, B), dtype=torch.int32, device=DEV)
        d_st = torch.zeros((T, B), dtype=torch.int32, device=DEV)
        d_sc = torch.zeros((T, B), dtype=torch.float32, device=DEV)
        pb.pb_fuse_frames_select(tr, d_logp, B * V, V, dev(np.zeros(B, np.int32)), None, 0.7, T, B, mode, d_tok, d_st,
                                 d_sc, stream_ptr())
        torch.cuda.synchronize()
        assert np.array_equal(d_tok.cpu().numpy(), want[0]) and np.array_equal(d_st.cpu().numpy(), want[1])
        assert_scores(d_sc.cpu().numpy(), want[2])
        assert np.any(want[0] == eos)
    got = gpu_fuse_frames(tr, d_logp, dev(np.zeros(B, np.int32)), 0.7)
    want = ot.fuse_frames(logp, np.zeros(B, np.int32), 0.7)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])


@pytest.mark.parametrize("K,V", [(3, 128), (4, 8192), (8, 66)])
def test_beam_step_with_eos(K, V):
    if V == 8192:
        cfg, toks, offs, eos, ot, tr = _config5_with_eos()
    else:
        cfg = W.CONFIGS[1]
        toks, offs = W.make_phrases(cfg)
        toks = (toks % (V - 2) + 1).astype(np.int32)
        eos = V - 1
        ot, tr = both(toks, offs, V, 0, eos, 1.5)
    U = 5
    rng = np.random.default_rng(K)
    states = rng.integers(0, ot.num_states, U * K).astype(np.int32)
    logp = W.log_softmax_rows(rng.standard_normal((U * K, V)) * 0.5)
    logp[:, eos] += np.float32(1.5)
    hyp = rng.standard_normal(U * K).astype(np.float32)
    hyp[1] = -np.inf
    want = ot.fuse_step_beam(logp, hyp, states, 0.5, U, K)
    got = gpu_beam_step(tr, dev(logp), dev(hyp), dev(states), 0.5, U, K)
    torch.cuda.synchronize()
    for g, w in zip(got[:3], want[:3]):
        assert np.array_equal(g.cpu().numpy(), w)
    assert_scores(got[3].cpu().numpy(), want[3])
    assert np.any(want[0] == eos)
