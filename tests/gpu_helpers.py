"""Helpers for the GPU parity tests: torch is used for device memory only; every result comes from
libpb.so through the binding."""
import numpy as np
import torch

import paper_2508_07014_amd as pb
import pb_workloads as W
from oracle import OracleTree
from oracle.pb_oracle import W_UNIFORM

DEV = "cuda:0"
TOL = 1e-5


def build_both(tokens, offsets, V, blank, **kw):
    ot = OracleTree(tokens, offsets, V, blank, weights=kw.get("weights"), weight_mode=kw.get("weight_mode", 0),
                    beta=kw.get("beta", 2.0), unk_score=kw.get("unk_score", 0.0),
                    final_zero_backoff=kw.get("final_zero_backoff", True))
    tr = pb.pb_build(tokens, offsets, V, blank, device=0, **kw)
    assert pb.pb_info(tr)["num_states"] == ot.num_states
    return ot, tr


_cache = {}


def config_trees(idx, mode=W_UNIFORM):
    key = (idx, mode)
    if key not in _cache:
        cfg = W.CONFIGS[idx]
        toks, offs = W.make_phrases(cfg)
        _cache[key] = (cfg, toks, offs) + build_both(toks, offs, cfg.vocab_size, cfg.blank_id, weight_mode=mode)
    return _cache[key]


def assert_scores(got, want):
    assert got.shape == want.shape
    fin = np.isfinite(want)
    assert np.array_equal(got[~fin], want[~fin])          # -inf (dead beams) must match exactly
    err = np.abs(got[fin].astype(np.float64) - want[fin].astype(np.float64))
    assert err.size == 0 or err.max() <= TOL, float(err.max())


def stream_ptr() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def gpu_score(tree, states: np.ndarray, V: int, want_next: bool = True):
    B = len(states)
    d_states = dev(states.astype(np.int32))
    d_scores = torch.full((B, V), 7.0, dtype=torch.float32, device=DEV)
    d_next = torch.full((B, V), -7, dtype=torch.int32, device=DEV) if want_next else None
    pb.pb_score(tree, d_states, B, d_scores, d_next, stream_ptr())
    torch.cuda.synchronize()
    return d_scores.cpu().numpy(), (d_next.cpu().numpy() if want_next else None)


def gpu_fuse_step(tree, d_logp: torch.Tensor, d_states: torch.Tensor, alpha: float, row_stride=None,
                  in_place: bool = False):
    B = d_states.shape[0]
    V = d_logp.shape[-1] if row_stride is None else None
    d_tokens = torch.full((B,), -5, dtype=torch.int32, device=DEV)
    d_out = d_states if in_place else torch.full((B,), -5, dtype=torch.int32, device=DEV)
    d_scores = torch.zeros(B, dtype=torch.float32, device=DEV)
    pb.pb_fuse_step(tree, d_logp, row_stride if row_stride is not None else V, d_states, alpha, B, d_tokens, d_out,
                    d_scores, stream_ptr())
    return d_tokens, d_out, d_scores


def gpu_fuse_frames(tree, d_logp: torch.Tensor, d_states0: torch.Tensor, alpha: float):
    T, B, V = d_logp.shape
    d_tokens = torch.full((T, B), -5, dtype=torch.int32, device=DEV)
    d_states = torch.full((T, B), -5, dtype=torch.int32, device=DEV)
    d_scores = torch.zeros((T, B), dtype=torch.float32, device=DEV)
    pb.pb_fuse_frames(tree, d_logp, B * V, V, d_states0, alpha, T, B, d_tokens, d_states, d_scores, stream_ptr())
    torch.cuda.synchronize()
    return d_tokens.cpu().numpy(), d_states.cpu().numpy(), d_scores.cpu().numpy()


def gpu_beam_step(tree, d_logp, d_hyp, d_states, alpha, U, K, row_stride=None):
    n = U * K
    d_tokens = torch.full((n,), -5, dtype=torch.int32, device=DEV)
    d_parents = torch.full((n,), -5, dtype=torch.int32, device=DEV)
    d_out = torch.full((n,), -5, dtype=torch.int32, device=DEV)
    d_scores = torch.zeros(n, dtype=torch.float32, device=DEV)
    pb.pb_fuse_step_beam(tree, d_logp, d_logp.shape[-1] if row_stride is None else row_stride, d_hyp, d_states, alpha,
                         U, K, d_tokens, d_parents, d_out, d_scores, stream_ptr())
    return d_tokens, d_parents, d_out, d_scores


def frames_ws(tree, d_logp, d_states0, d_last0, alpha, mode, fill=-7):
    """pb_fuse_frames_ws with a workspace of exactly the size the library asks for, filled with junk first."""
    T, B, V = d_logp.shape
    need = pb.pb_fuse_frames_workspace_bytes(tree, T, B)
    ws = torch.full((max(need, 4) // 4,), 0x7f7f7f7f, dtype=torch.int32, device=DEV)
    d_tokens = torch.full((T, B), fill, dtype=torch.int32, device=DEV)
    d_states = torch.full((T, B), fill, dtype=torch.int32, device=DEV)
    d_scores = torch.zeros((T, B), dtype=torch.float32, device=DEV)
    pb.pb_fuse_frames_ws(tree, d_logp, B * V, V, d_states0, d_last0, alpha, T, B, mode, d_tokens, d_states, d_scores, ws,
                         need, stream_ptr())
    torch.cuda.synchronize()
    return d_tokens.cpu().numpy(), d_states.cpu().numpy(), d_scores.cpu().numpy()
