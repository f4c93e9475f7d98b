"""Randomised GPU parity of the multi-frame decoder: vocabulary sizes on both kernel paths, blank ids
other than 0, all weight modes and selection rules, invalid start states, previous labels, and four
kinds of acoustic rows (CTC-shaped, planted phrases, blank-dominated, nearly flat), every output against
the CPU oracle.  Segment boundaries, guesses and re-runs fall differently in every case."""
import numpy as np
import pytest

import pb_workloads as W
from oracle import OracleTree

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import paper_2508_07014_amd as pb  # noqa: E402
from gpu_helpers import DEV, dev, frames_ws  # noqa: E402


@pytest.mark.parametrize("chunk", range(6))
def test_frames_random_cases(chunk):
    rng = np.random.default_rng(4242 + chunk)
    for case in range(25):
        V = int(rng.choice([8, 64, 128, 256, 1024, 130, 2048]))
        blank = int(rng.choice([0, -1, 3]))
        nph = int(rng.integers(1, 400))
        cfg = W.Config(9, "fuzz", V, blank, nph, 1, int(rng.integers(2, 9)), "zipf" if rng.random() < 0.7 else "uniform",
                       1.1, 1, 1, 1, 2.0)
        toks, offs = W.make_phrases(cfg, seed=int(rng.integers(1 << 30)))
        if blank >= 1:
            toks = np.where(toks == blank, blank + 1, toks).astype(np.int32)
        wmode, unk = int(rng.integers(0, 3)), float(rng.choice([0.0, 0.5, -0.25]))
        ot = OracleTree(toks, offs, V, blank, weight_mode=wmode, unk_score=unk)
        tr = pb.pb_build(toks, offs, V, blank, weight_mode=wmode, unk_score=unk, device=0)
        T = int(rng.choice([1, 2, 3, 7, 33, 64, 65, 100, 257, 600]))
        B = int(rng.choice([1, 2, 3, 5, 17, 40]))
        kind = int(rng.integers(0, 4))
        seed = int(rng.integers(1 << 30))
        shape = W.Config(9, "fuzz", V, blank, nph, 1, 8, "uniform", 1.1, B, 1, T, 2.0)
        if kind == 0:
            logp = W.sticky_logp(seed, T, B, V, blank, grid=None, bump=float(rng.choice([3.0, 8.0])))
        elif kind == 1:
            logp = W.make_logp(shape, seed=seed, planting=W.Planting(toks, offs, cover=float(rng.choice([0.3, 0.9])), bump=10.0))
        elif kind == 2:
            logp = W.make_logp(shape, seed=seed, blank_bias=8.0, blank_frac=0.7)
        else:
            logp = W.log_softmax_rows(rng.standard_normal((T, B, V)) * 0.2)
        s0 = rng.integers(0, ot.num_states, B).astype(np.int32)
        if rng.random() < 0.15:
            s0[0] = -1 if rng.random() < 0.5 else ot.num_states
        last0 = rng.integers(-1, V, B).astype(np.int32) if rng.random() < 0.5 else None
        alpha = float(rng.choice([0.0, 0.3, 0.5, 1.0, 2.0]))
        ok = [b for b in range(B) if 0 <= s0[b] < ot.num_states]
        bad = [b for b in range(B) if b not in ok]
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
            where = dict(chunk=chunk, case=case, V=V, blank=blank, T=T, B=B, kind=kind, mode=mode, alpha=alpha, wmode=wmode)
            assert np.array_equal(tk[:, ok], want[0]) and np.array_equal(st[:, ok], want[1]), where
            assert np.allclose(sc[:, ok], want[2], atol=1e-5, rtol=0), where
            for b in bad:
                assert np.all(tk[:, b] == -1) and np.all(st[:, b] == -1) and np.all(np.isnan(sc[:, b])), where
            # the same call with a workspace (wrong boundary guesses repaired by patches): identical outputs
            tk2, st2, sc2 = frames_ws(tr, d_logp, dev(s0), None if last0 is None else dev(last0), alpha, mode)
            assert np.array_equal(tk2, tk) and np.array_equal(st2, st) and np.array_equal(sc2, sc, equal_nan=True), where
        pb.pb_free(tr)


@pytest.mark.parametrize("chunk", range(4))
def test_beam_step_random_cases(chunk):
    """Beam widths on both kernels (K <= 8 wave-per-beam, wider ones per workgroup), K above V, exact ties,
    dead beams, blank ids other than 0."""
    rng = np.random.default_rng(777 + chunk)
    for case in range(40):
        V = int(rng.choice([4, 8, 64, 128, 1024, 130, 2048]))
        blank = int(rng.choice([0, -1, 2]))
        cfg = W.Config(9, "fuzz", V, blank, int(rng.integers(1, 300)), 1, int(rng.integers(2, 7)), "zipf", 1.1, 1, 1, 1, 2.0)
        toks, offs = W.make_phrases(cfg, seed=int(rng.integers(1 << 30)))
        if blank >= 1:
            toks = np.where(toks == blank, (blank + 1) % V or 1, toks).astype(np.int32)
        wmode = int(rng.integers(0, 3))
        ot = OracleTree(toks, offs, V, blank, weight_mode=wmode)
        tr = pb.pb_build(toks, offs, V, blank, weight_mode=wmode, device=0)
        K, U = int(rng.choice([1, 2, 3, 4, 5, 8, 9, 16])), int(rng.choice([1, 3, 10]))
        states = rng.integers(0, ot.num_states, U * K).astype(np.int32)
        kind = int(rng.integers(0, 3))
        if kind == 0:
            logp = W.log_softmax_rows(rng.standard_normal((U * K, V)) * 2)
        elif kind == 1:
            logp = np.round(rng.standard_normal((U * K, V)) * 2).astype(np.float32)      # many exact ties
        else:
            logp = np.full((U * K, V), -3.0, np.float32)
        hyp = rng.standard_normal(U * K).astype(np.float32)
        if rng.random() < 0.5:
            hyp[rng.integers(0, U * K, max(1, U * K // 3))] = -np.inf
        if kind == 1:
            hyp = np.round(hyp).astype(np.float32)
        alpha = float(rng.choice([0.0, 0.5, 1.0]))
        want = ot.fuse_step_beam(logp, hyp, states, alpha, U, K)
        o = [torch.zeros(U * K, dtype=torch.int32, device=DEV) for _ in range(3)] + [torch.zeros(U * K, device=DEV)]
        pb.pb_fuse_step_beam(tr, dev(logp), V, dev(hyp), dev(states), alpha, U, K, o[0], o[1], o[2], o[3], 0)
        torch.cuda.synchronize()
        where = dict(chunk=chunk, case=case, V=V, blank=blank, K=K, U=U, kind=kind, alpha=alpha, wmode=wmode)
        for g, w in zip(o[:3], want[:3]):
            assert np.array_equal(g.cpu().numpy(), w), where
        sc, fin = o[3].cpu().numpy(), np.isfinite(want[3])
        assert np.array_equal(sc[~fin], want[3][~fin]) and np.allclose(sc[fin], want[3][fin], atol=1e-5, rtol=0), where
        pb.pb_free(tr)
