"""ctypes front end of the C oracle (pb_oracle.c) -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Argument marshalling only: every number comes from pb_oracle.c, which follows
Algorithm 1 and Sec. II-B of the paper step by step on the CPU.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pb_oracle.c")
_LIB = os.path.join(_HERE, "libpb_oracle.so")

W_UNIFORM = 0
W_LOGDEPTH = 1
W_UNIFORM_FINAL = 2
SELECT_FUSED = 0
SELECT_TWO_STAGE = 1
SELECT_TWO_STAGE_CTC = 2


class OracleError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"oracle: {where} failed with code {code}")
        self.code = code


def build_library(force: bool = False) -> str:
    """Compile pb_oracle.c with gcc (no FMA contraction, OpenMP over hypotheses)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build_library()
    lib = C.CDLL(_LIB)
    i32p, i64p, f32p, f64p = (C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_float),
                              C.POINTER(C.c_double))
    lib.orc_build.restype = C.c_void_p
    lib.orc_build.argtypes = [i32p, i64p, C.c_int64, f32p, C.c_int32, C.c_int32, C.c_int32, C.c_float,
                              C.c_float, C.c_int32, i32p]
    lib.orc_free.restype = None
    lib.orc_free.argtypes = [C.c_void_p]
    lib.orc_num_states.restype = C.c_int32
    lib.orc_num_states.argtypes = [C.c_void_p]
    lib.orc_max_depth.restype = C.c_int32
    lib.orc_max_depth.argtypes = [C.c_void_p]
    lib.orc_node.restype = C.c_int32
    lib.orc_node.argtypes = [C.c_void_p, C.c_int32, i32p, i32p, i32p, i32p, i32p, f64p, f32p, f32p]
    lib.orc_child.restype = C.c_int32
    lib.orc_child.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
    lib.orc_set_eos.restype = C.c_int32
    lib.orc_set_eos.argtypes = [C.c_void_p, C.c_int32, C.c_float]
    lib.orc_query.restype = C.c_int32
    lib.orc_query.argtypes = [C.c_void_p, C.c_int32, C.c_int32, f32p, i32p]
    lib.orc_score.restype = C.c_int32
    lib.orc_score.argtypes = [C.c_void_p, i32p, C.c_int32, f32p, i32p]
    lib.orc_fuse_step.restype = C.c_int32
    lib.orc_fuse_step.argtypes = [C.c_void_p, f32p, C.c_int64, i32p, C.c_float, C.c_int32, i32p, i32p, f32p]
    lib.orc_fuse_frames.restype = C.c_int32
    lib.orc_fuse_frames.argtypes = [C.c_void_p, f32p, C.c_int64, C.c_int64, i32p, C.c_float, C.c_int32,
                                    C.c_int32, i32p, i32p, f32p]
    lib.orc_fuse_step_select.restype = C.c_int32
    lib.orc_fuse_step_select.argtypes = [C.c_void_p, f32p, C.c_int64, i32p, i32p, C.c_float, C.c_int32, C.c_int32,
                                         i32p, i32p, f32p]
    lib.orc_fuse_frames_select.restype = C.c_int32
    lib.orc_fuse_frames_select.argtypes = [C.c_void_p, f32p, C.c_int64, C.c_int64, i32p, i32p, C.c_float, C.c_int32,
                                           C.c_int32, C.c_int32, i32p, i32p, f32p]
    lib.orc_fuse_step_beam.restype = C.c_int32
    lib.orc_fuse_step_beam.argtypes = [C.c_void_p, f32p, C.c_int64, f32p, i32p, C.c_float, C.c_int32,
                                       C.c_int32, i32p, i32p, i32p, f32p]
    lib.orc_set_threads.restype = None
    lib.orc_set_threads.argtypes = [C.c_int32]
    lib.orc_threads.restype = C.c_int32
    lib.orc_threads.argtypes = []
    _lib = lib
    return lib


def oracle_threads() -> int:
    """Threads the oracle's OpenMP loops use (one hypothesis / utterance per iteration)."""
    return int(_load().orc_threads())


def set_oracle_threads(n: int) -> None:
    """Timing aid: thread count of the oracle's OpenMP loops."""
    _load().orc_set_threads(int(n))


def _p(a: Optional[np.ndarray], ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


class OracleTree:
    """The oracle's boosting tree; state ids are canonical (root 0, BFS, children by token)."""

    def __init__(self, tokens, offsets, vocab_size: int, blank_id: int = 0, weights=None,
                 weight_mode: int = W_UNIFORM, beta: float = 2.0, unk_score: float = 0.0,
                 final_zero_backoff: bool = True, eos_id: int = -1, final_eos_score: float = 0.0):
        lib = _load()
        self._lib = lib
        tokens = _i32(tokens)
        offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        n = len(offsets) - 1
        w = None if weights is None else _f32(weights)
        err = C.c_int32(0)
        self._h = lib.orc_build(_p(tokens, C.c_int32), _p(offsets, C.c_int64), n, _p(w, C.c_float),
                                vocab_size, blank_id, weight_mode, beta, unk_score,
                                1 if final_zero_backoff else 0, C.byref(err))
        if not self._h:
            raise OracleError(err.value, "orc_build")
        if eos_id != -1:
            rc = lib.orc_set_eos(self._h, eos_id, final_eos_score)
            if rc:
                lib.orc_free(self._h)
                self._h = None
                raise OracleError(rc, "orc_set_eos")
        self.vocab_size = vocab_size
        self.blank_id = blank_id
        self.eos_id = eos_id
        self.num_states = int(lib.orc_num_states(self._h))
        self.max_depth = int(lib.orc_max_depth(self._h))

    def __del__(self):
        h = getattr(self, "_h", None)
        if h:
            self._lib.orc_free(h)
            self._h = None

    def node(self, s: int) -> dict:
        parent, token, depth, fail, fin = (C.c_int32() for _ in range(5))
        acc, arcw, bw = C.c_double(), C.c_float(), C.c_float()
        rc = self._lib.orc_node(self._h, s, C.byref(parent), C.byref(token), C.byref(depth), C.byref(fail),
                                C.byref(fin), C.byref(acc), C.byref(arcw), C.byref(bw))
        if rc:
            raise OracleError(rc, "orc_node")
        return dict(parent=parent.value, token=token.value, depth=depth.value, fail=fail.value,
                    final=bool(fin.value), acc=acc.value, arcw=arcw.value, bw=bw.value)

    def child(self, s: int, v: int) -> int:
        return int(self._lib.orc_child(self._h, s, v))

    def prefix(self, s: int) -> Tuple[int, ...]:
        """Token string spelled by the path root -> s."""
        out = []
        while s != 0:
            nd = self.node(s)
            out.append(nd["token"])
            s = nd["parent"]
        return tuple(reversed(out))

    def query(self, s: int, v: int) -> Tuple[float, int]:
        sc, nx = C.c_float(), C.c_int32()
        rc = self._lib.orc_query(self._h, s, v, C.byref(sc), C.byref(nx))
        if rc:
            raise OracleError(rc, "orc_query")
        return sc.value, nx.value

    def score(self, states, want_next: bool = True):
        states = _i32(states)
        B = states.shape[0]
        scores = np.empty((B, self.vocab_size), dtype=np.float32)
        nxt = np.empty((B, self.vocab_size), dtype=np.int32) if want_next else None
        rc = self._lib.orc_score(self._h, _p(states, C.c_int32), B, _p(scores, C.c_float), _p(nxt, C.c_int32))
        if rc:
            raise OracleError(rc, "orc_score")
        return scores, nxt

    def fuse_step(self, logp, states, alpha: float):
        logp = _f32(logp)
        states = _i32(states)
        B = states.shape[0]
        assert logp.shape == (B, self.vocab_size)
        tokens = np.empty(B, dtype=np.int32)
        states_out = np.empty(B, dtype=np.int32)
        scores = np.empty(B, dtype=np.float32)
        rc = self._lib.orc_fuse_step(self._h, _p(logp, C.c_float), self.vocab_size, _p(states, C.c_int32),
                                     alpha, B, _p(tokens, C.c_int32), _p(states_out, C.c_int32),
                                     _p(scores, C.c_float))
        if rc:
            raise OracleError(rc, "orc_fuse_step")
        return tokens, states_out, scores

    def fuse_frames(self, logp, states0, alpha: float):
        """logp float32[T,B,V]; returns per-frame tokens, states, scores, each [T,B]."""
        logp = _f32(logp)
        states0 = _i32(states0)
        T, B, V = logp.shape
        assert V == self.vocab_size and states0.shape == (B,)
        tokens = np.empty((T, B), dtype=np.int32)
        states = np.empty((T, B), dtype=np.int32)
        scores = np.empty((T, B), dtype=np.float32)
        rc = self._lib.orc_fuse_frames(self._h, _p(logp, C.c_float), B * V, V, _p(states0, C.c_int32), alpha,
                                       T, B, _p(tokens, C.c_int32), _p(states, C.c_int32),
                                       _p(scores, C.c_float))
        if rc:
            raise OracleError(rc, "orc_fuse_frames")
        return tokens, states, scores

    def fuse_step_select(self, logp, states, last_tokens, alpha: float, mode: int):
        """Two-stage greedy selection (Sec. II-C); last_tokens may be None (no previous label)."""
        logp = _f32(logp)
        states = _i32(states)
        last = None if last_tokens is None else _i32(last_tokens)
        B = states.shape[0]
        assert logp.shape == (B, self.vocab_size)
        tokens = np.empty(B, dtype=np.int32)
        states_out = np.empty(B, dtype=np.int32)
        scores = np.empty(B, dtype=np.float32)
        rc = self._lib.orc_fuse_step_select(self._h, _p(logp, C.c_float), self.vocab_size, _p(states, C.c_int32),
                                            _p(last, C.c_int32), alpha, B, mode, _p(tokens, C.c_int32),
                                            _p(states_out, C.c_int32), _p(scores, C.c_float))
        if rc:
            raise OracleError(rc, "orc_fuse_step_select")
        return tokens, states_out, scores

    def fuse_frames_select(self, logp, states0, last0, alpha: float, mode: int):
        """logp float32[T,B,V]; the previous label of frame t is the token of frame t-1 (last0 for t = 0)."""
        logp = _f32(logp)
        states0 = _i32(states0)
        last = None if last0 is None else _i32(last0)
        T, B, V = logp.shape
        assert V == self.vocab_size and states0.shape == (B,)
        tokens = np.empty((T, B), dtype=np.int32)
        states = np.empty((T, B), dtype=np.int32)
        scores = np.empty((T, B), dtype=np.float32)
        rc = self._lib.orc_fuse_frames_select(self._h, _p(logp, C.c_float), B * V, V, _p(states0, C.c_int32),
                                              _p(last, C.c_int32), alpha, T, B, mode, _p(tokens, C.c_int32),
                                              _p(states, C.c_int32), _p(scores, C.c_float))
        if rc:
            raise OracleError(rc, "orc_fuse_frames_select")
        return tokens, states, scores

    def fuse_step_beam(self, logp, hyp_scores, states, alpha: float, U: int, K: int):
        logp = _f32(logp)
        hyp_scores = _f32(hyp_scores)
        states = _i32(states)
        assert logp.shape == (U * K, self.vocab_size) and states.shape == (U * K,)
        tokens = np.empty(U * K, dtype=np.int32)
        parents = np.empty(U * K, dtype=np.int32)
        states_out = np.empty(U * K, dtype=np.int32)
        scores = np.empty(U * K, dtype=np.float32)
        rc = self._lib.orc_fuse_step_beam(self._h, _p(logp, C.c_float), self.vocab_size,
                                          _p(hyp_scores, C.c_float), _p(states, C.c_int32), alpha, U, K,
                                          _p(tokens, C.c_int32), _p(parents, C.c_int32),
                                          _p(states_out, C.c_int32), _p(scores, C.c_float))
        if rc:
            raise OracleError(rc, "orc_fuse_step_beam")
        return tokens, parents, states_out, scores
