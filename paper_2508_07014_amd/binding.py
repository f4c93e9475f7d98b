"""Thin ctypes binding of libpb.so: same names as the C ABI (include/pb.h), argument marshalling only.

Device buffers are passed as anything with a ``data_ptr()`` (torch tensors) or as raw integer
addresses; host arrays are numpy.  Every step of the method runs inside the library's HIP kernels.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

from . import build as _build

PB_OK, PB_EINVAL, PB_ERANGE, PB_ENOMEM, PB_EHIP, PB_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
PB_W_UNIFORM, PB_W_LOGDEPTH, PB_W_UNIFORM_FINAL = 0, 1, 2
PB_SELECT_FUSED, PB_SELECT_TWO_STAGE, PB_SELECT_TWO_STAGE_CTC = 0, 1, 2

EXPORTS = ["pb_build", "pb_free", "pb_info", "pb_host_arrays", "pb_state_prefix", "pb_score", "pb_fuse_step",
           "pb_fuse_frames", "pb_fuse_step_select", "pb_fuse_frames_select", "pb_fuse_frames_plan",
           "pb_fuse_frames_workspace_bytes",
           "pb_fuse_frames_ws", "pb_fuse_frames_static", "pb_fuse_step_beam", "pb_forest_build", "pb_forest_free", "pb_score_forest",
           "pb_fuse_step_forest", "pb_fuse_frames_forest", "pb_fuse_step_beam_forest", "pb_validate",
           "pb_validate_states", "pb_strerror"]


class PbError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where}: {strerror(code)} ({code})")
        self.code = code


class pb_build_opts(C.Structure):
    _fields_ = [("vocab_size", C.c_int32), ("blank_id", C.c_int32), ("weight_mode", C.c_int32),
                ("beta", C.c_float), ("unk_score", C.c_float), ("final_zero_backoff", C.c_int32),
                ("device", C.c_int32), ("eos_id", C.c_int32), ("final_eos_score", C.c_float)]


class pb_tree_info(C.Structure):
    _fields_ = [("num_states", C.c_int32), ("num_arcs", C.c_int32), ("max_depth", C.c_int32),
                ("max_fail_chain", C.c_int32), ("root_degree", C.c_int32), ("vocab_size", C.c_int32),
                ("blank_id", C.c_int32), ("eos_id", C.c_int32), ("device_bytes", C.c_int64)]


class pb_host_view(C.Structure):
    _fields_ = [("arc_begin", C.POINTER(C.c_int32)), ("arc_count", C.POINTER(C.c_int32)),
                ("fail", C.POINTER(C.c_int32)), ("backoff", C.POINTER(C.c_float)),
                ("is_final", C.POINTER(C.c_uint8)), ("depth", C.POINTER(C.c_int32)),
                ("parent", C.POINTER(C.c_int32)), ("arc_token", C.POINTER(C.c_int32)),
                ("arc_score", C.POINTER(C.c_float)), ("acc", C.POINTER(C.c_double)),
                ("root_score", C.POINTER(C.c_float)), ("root_next", C.POINTER(C.c_int32)),
                ("p_root", C.POINTER(C.c_float)), ("eos_score", C.POINTER(C.c_float))]


_lib = None


def library_path() -> str:
    return _build.LIB


def load():
    """Loads libpb.so; builds it first only if no built library is present.  Fails loudly otherwise."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build(force=True)
    try:  # PyTorch ships its own HIP runtime: let it load first so the process ends up with one copy
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(_build.LIB)
    vp, i32p, i64p, f32p = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_float)
    lib.pb_build.restype = C.c_int
    lib.pb_build.argtypes = [i32p, i64p, C.c_int64, f32p, C.POINTER(pb_build_opts), C.POINTER(vp)]
    lib.pb_free.restype = C.c_int
    lib.pb_free.argtypes = [vp]
    lib.pb_info.restype = C.c_int
    lib.pb_info.argtypes = [vp, C.POINTER(pb_tree_info)]
    lib.pb_host_arrays.restype = C.c_int
    lib.pb_host_arrays.argtypes = [vp, C.POINTER(pb_host_view)]
    lib.pb_state_prefix.restype = C.c_int
    lib.pb_state_prefix.argtypes = [vp, C.c_int32, i32p, C.c_int32, i32p]
    lib.pb_score.restype = C.c_int
    lib.pb_score.argtypes = [vp, vp, C.c_int32, vp, vp, vp]
    lib.pb_fuse_step.restype = C.c_int
    lib.pb_fuse_step.argtypes = [vp, vp, C.c_int64, vp, C.c_float, C.c_int32, vp, vp, vp, vp]
    lib.pb_fuse_frames.restype = C.c_int
    lib.pb_fuse_frames.argtypes = [vp, vp, C.c_int64, C.c_int64, vp, C.c_float, C.c_int32, C.c_int32, vp, vp, vp, vp]
    lib.pb_fuse_step_select.restype = C.c_int
    lib.pb_fuse_step_select.argtypes = [vp, vp, C.c_int64, vp, vp, C.c_float, C.c_int32, C.c_int32, vp, vp, vp, vp]
    lib.pb_fuse_frames_select.restype = C.c_int
    lib.pb_fuse_frames_select.argtypes = [vp, vp, C.c_int64, C.c_int64, vp, vp, C.c_float, C.c_int32, C.c_int32,
                                          C.c_int32, vp, vp, vp, vp]
    lib.pb_fuse_frames_plan.restype = C.c_int
    lib.pb_fuse_frames_plan.argtypes = [vp, C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.pb_fuse_frames_workspace_bytes.restype = C.c_int64
    lib.pb_fuse_frames_workspace_bytes.argtypes = [vp, C.c_int32, C.c_int32]
    lib.pb_fuse_frames_ws.restype = C.c_int
    lib.pb_fuse_frames_ws.argtypes = [vp, vp, C.c_int64, C.c_int64, vp, vp, C.c_float, C.c_int32, C.c_int32, C.c_int32,
                                      vp, vp, vp, vp, C.c_int64, vp]
    lib.pb_fuse_frames_static.restype = C.c_int
    lib.pb_fuse_frames_static.argtypes = [vp, vp, C.c_int64, C.c_int64, vp, vp, C.c_float, C.c_int32, C.c_int32,
                                          C.c_int32, vp, vp, vp, vp]
    lib.pb_fuse_step_beam.restype = C.c_int
    lib.pb_fuse_step_beam.argtypes = [vp, vp, C.c_int64, vp, vp, C.c_float, C.c_int32, C.c_int32, vp, vp, vp, vp, vp]
    lib.pb_forest_build.restype = C.c_int
    lib.pb_forest_build.argtypes = [C.POINTER(vp), C.c_int32, C.POINTER(vp)]
    lib.pb_forest_free.restype = C.c_int
    lib.pb_forest_free.argtypes = [vp]
    lib.pb_score_forest.restype = C.c_int
    lib.pb_score_forest.argtypes = [vp, vp, vp, C.c_int32, vp, vp, vp]
    lib.pb_fuse_step_forest.restype = C.c_int
    lib.pb_fuse_step_forest.argtypes = [vp, vp, C.c_int64, vp, vp, vp, C.c_float, C.c_int32, C.c_int32, vp, vp, vp, vp]
    lib.pb_fuse_frames_forest.restype = C.c_int
    lib.pb_fuse_frames_forest.argtypes = [vp, vp, C.c_int64, C.c_int64, vp, vp, vp, C.c_float, C.c_int32, C.c_int32,
                                          C.c_int32, vp, vp, vp, vp]
    lib.pb_fuse_step_beam_forest.restype = C.c_int
    lib.pb_fuse_step_beam_forest.argtypes = [vp, vp, C.c_int64, vp, vp, vp, C.c_float, C.c_int32, C.c_int32, vp, vp, vp,
                                             vp, vp]
    lib.pb_validate.restype = C.c_int
    lib.pb_validate.argtypes = [vp]
    lib.pb_validate_states.restype = C.c_int
    lib.pb_validate_states.argtypes = [vp, i32p, C.c_int64, i64p]
    lib.pb_strerror.restype = C.c_char_p
    lib.pb_strerror.argtypes = [C.c_int]
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load().pb_strerror(code).decode()


def _dptr(x) -> Optional[int]:
    """Device address of a tensor-like, an int address, or None."""
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    return int(x)


def _check(rc: int, where: str):
    if rc != PB_OK:
        raise PbError(rc, where)


class Tree:
    """Owner of a ``pb_tree*``; freed on ``close()`` / garbage collection."""

    def __init__(self, handle: int):
        self.handle = handle

    def close(self):
        if self.handle:
            load().pb_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def pb_build(tokens, offsets, vocab_size: int, blank_id: int = 0, weights=None, weight_mode: int = PB_W_UNIFORM,
             beta: float = 2.0, unk_score: float = 0.0, final_zero_backoff: bool = True, device: int = 0,
             eos_id: int = -1, final_eos_score: float = 0.0) -> Tree:
    lib = load()
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    w = None if weights is None else np.ascontiguousarray(weights, dtype=np.float32)
    opts = pb_build_opts(vocab_size, blank_id, weight_mode, beta, unk_score, 1 if final_zero_backoff else 0, device,
                         eos_id, final_eos_score)
    out = C.c_void_p()
    rc = lib.pb_build(tokens.ctypes.data_as(C.POINTER(C.c_int32)), offsets.ctypes.data_as(C.POINTER(C.c_int64)),
                      len(offsets) - 1, None if w is None else w.ctypes.data_as(C.POINTER(C.c_float)),
                      C.byref(opts), C.byref(out))
    _check(rc, "pb_build")
    return Tree(out.value)


def pb_free(tree: Tree):
    tree.close()


def pb_info(tree: Tree) -> dict:
    info = pb_tree_info()
    _check(load().pb_info(tree.handle, C.byref(info)), "pb_info")
    return {name: getattr(info, name) for name, _ in pb_tree_info._fields_}


def pb_host_arrays(tree: Tree) -> dict:
    """Copies of the compiled flat arrays as numpy arrays."""
    view = pb_host_view()
    _check(load().pb_host_arrays(tree.handle, C.byref(view)), "pb_host_arrays")
    info = pb_info(tree)
    n, a, v = info["num_states"], info["num_arcs"], info["vocab_size"]
    sizes = dict(arc_begin=n, arc_count=n, fail=n, backoff=n, is_final=n, depth=n, parent=n, arc_token=a,
                 arc_score=a, acc=n, root_score=v, root_next=v, p_root=n, eos_score=n)
    out = {}
    for name, cnt in sizes.items():
        ptr = getattr(view, name)
        if not ptr:  # a NULL member (eos_score of a tree without the rule)
            out[name] = None
            continue
        out[name] = np.ctypeslib.as_array(ptr, shape=(cnt,)).copy() if cnt else np.zeros(0)
    return out


def pb_validate(tree: Tree) -> int:
    """Status code of the structural check (PB_OK / PB_ERANGE)."""
    return int(load().pb_validate(tree.handle))


def pb_validate_states(tree: Tree, states) -> int:
    """Index of the first state id outside the tree, or -1 if all are valid (host array)."""
    st = np.ascontiguousarray(states, dtype=np.int32)
    bad = C.c_int64(-1)
    rc = load().pb_validate_states(tree.handle, st.ctypes.data_as(C.POINTER(C.c_int32)), st.size, C.byref(bad))
    if rc not in (PB_OK, PB_ERANGE):
        raise PbError(rc, "pb_validate_states")
    return int(bad.value) if rc == PB_ERANGE else -1


def pb_state_prefix(tree: Tree, state: int) -> tuple:
    ln = C.c_int32()
    _check(load().pb_state_prefix(tree.handle, state, None, 0, C.byref(ln)), "pb_state_prefix")
    buf = (C.c_int32 * max(1, ln.value))()
    _check(load().pb_state_prefix(tree.handle, state, buf, ln.value, C.byref(ln)), "pb_state_prefix")
    return tuple(buf[:ln.value])


def pb_score(tree: Tree, d_states, B: int, d_scores, d_next=None, stream: int = 0):
    _check(load().pb_score(tree.handle, _dptr(d_states), B, _dptr(d_scores), _dptr(d_next), stream or None),
           "pb_score")


def pb_fuse_step(tree: Tree, d_logp, row_stride: int, d_states_in, alpha: float, B: int, d_tokens, d_states_out,
                 d_scores, stream: int = 0):
    _check(load().pb_fuse_step(tree.handle, _dptr(d_logp), row_stride, _dptr(d_states_in), alpha, B,
                               _dptr(d_tokens), _dptr(d_states_out), _dptr(d_scores), stream or None),
           "pb_fuse_step")


def pb_fuse_frames(tree: Tree, d_logp, frame_stride: int, row_stride: int, d_states0, alpha: float, T: int, B: int,
                   d_tokens, d_states, d_scores, stream: int = 0):
    _check(load().pb_fuse_frames(tree.handle, _dptr(d_logp), frame_stride, row_stride, _dptr(d_states0), alpha, T, B,
                                 _dptr(d_tokens), _dptr(d_states), _dptr(d_scores), stream or None),
           "pb_fuse_frames")


def pb_fuse_step_select(tree: Tree, d_logp, row_stride: int, d_states_in, d_last_tokens, alpha: float, B: int,
                        mode: int, d_tokens, d_states_out, d_scores, stream: int = 0):
    _check(load().pb_fuse_step_select(tree.handle, _dptr(d_logp), row_stride, _dptr(d_states_in),
                                      _dptr(d_last_tokens), alpha, B, mode, _dptr(d_tokens), _dptr(d_states_out),
                                      _dptr(d_scores), stream or None), "pb_fuse_step_select")


def pb_fuse_frames_select(tree: Tree, d_logp, frame_stride: int, row_stride: int, d_states0, d_last0, alpha: float,
                          T: int, B: int, mode: int, d_tokens, d_states, d_scores, stream: int = 0):
    _check(load().pb_fuse_frames_select(tree.handle, _dptr(d_logp), frame_stride, row_stride, _dptr(d_states0),
                                        _dptr(d_last0), alpha, T, B, mode, _dptr(d_tokens), _dptr(d_states),
                                        _dptr(d_scores), stream or None), "pb_fuse_frames_select")


def pb_fuse_frames_plan(tree: Tree, T: int, B: int):
    """Frame indices at which pb_fuse_frames* would cut a call: a list of n_segments + 1 boundaries (empty plan: [0])."""
    n = C.c_int32(0)
    bounds = (C.c_int32 * 65)()
    _check(load().pb_fuse_frames_plan(tree.handle, T, B, C.byref(n), bounds), "pb_fuse_frames_plan")
    return [int(bounds[j]) for j in range(n.value + 1)]


def pb_fuse_frames_workspace_bytes(tree: Tree, T: int, B: int) -> int:
    n = int(load().pb_fuse_frames_workspace_bytes(tree.handle, T, B))
    if n < 0:
        raise PbError(n, "pb_fuse_frames_workspace_bytes")
    return n


def pb_fuse_frames_ws(tree: Tree, d_logp, frame_stride: int, row_stride: int, d_states0, d_last0, alpha: float,
                      T: int, B: int, mode: int, d_tokens, d_states, d_scores, d_workspace, workspace_bytes: int,
                      stream: int = 0):
    _check(load().pb_fuse_frames_ws(tree.handle, _dptr(d_logp), frame_stride, row_stride, _dptr(d_states0),
                                    _dptr(d_last0), alpha, T, B, mode, _dptr(d_tokens), _dptr(d_states),
                                    _dptr(d_scores), _dptr(d_workspace), workspace_bytes, stream or None),
           "pb_fuse_frames_ws")


def pb_fuse_frames_static(tree: Tree, d_logp, frame_stride: int, row_stride: int, d_states0, d_last0, alpha: float,
                          T: int, B: int, mode: int, d_tokens, d_states, d_scores, stream: int = 0):
    _check(load().pb_fuse_frames_static(tree.handle, _dptr(d_logp), frame_stride, row_stride, _dptr(d_states0),
                                        _dptr(d_last0), alpha, T, B, mode, _dptr(d_tokens), _dptr(d_states),
                                        _dptr(d_scores), stream or None), "pb_fuse_frames_static")


def pb_fuse_step_beam(tree: Tree, d_logp, row_stride: int, d_hyp_scores, d_states_in, alpha: float, U: int, K: int,
                      d_tokens, d_parents, d_states_out, d_scores_out, stream: int = 0):
    _check(load().pb_fuse_step_beam(tree.handle, _dptr(d_logp), row_stride, _dptr(d_hyp_scores), _dptr(d_states_in),
                                    alpha, U, K, _dptr(d_tokens), _dptr(d_parents), _dptr(d_states_out),
                                    _dptr(d_scores_out), stream or None), "pb_fuse_step_beam")


class Forest:
    """Owner of a ``pb_forest*``; keeps its member trees alive."""

    def __init__(self, handle: int, trees):
        self.handle = handle
        self.trees = list(trees)

    def close(self):
        if self.handle:
            load().pb_forest_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def pb_forest_build(trees) -> Forest:
    arr = (C.c_void_p * len(trees))(*[t.handle for t in trees])
    out = C.c_void_p()
    _check(load().pb_forest_build(arr, len(trees), C.byref(out)), "pb_forest_build")
    return Forest(out.value, trees)


def pb_forest_free(forest: Forest):
    forest.close()


def pb_score_forest(forest: Forest, d_tree_ids, d_states, B: int, d_scores, d_next=None, stream: int = 0):
    _check(load().pb_score_forest(forest.handle, _dptr(d_tree_ids), _dptr(d_states), B, _dptr(d_scores), _dptr(d_next),
                                  stream or None), "pb_score_forest")


def pb_fuse_step_forest(forest: Forest, d_logp, row_stride: int, d_tree_ids, d_states_in, d_last_tokens, alpha: float,
                        B: int, mode: int, d_tokens, d_states_out, d_scores, stream: int = 0):
    _check(load().pb_fuse_step_forest(forest.handle, _dptr(d_logp), row_stride, _dptr(d_tree_ids), _dptr(d_states_in),
                                      _dptr(d_last_tokens), alpha, B, mode, _dptr(d_tokens), _dptr(d_states_out),
                                      _dptr(d_scores), stream or None), "pb_fuse_step_forest")


def pb_fuse_frames_forest(forest: Forest, d_logp, frame_stride: int, row_stride: int, d_tree_ids, d_states0, d_last0,
                          alpha: float, T: int, B: int, mode: int, d_tokens, d_states, d_scores, stream: int = 0):
    _check(load().pb_fuse_frames_forest(forest.handle, _dptr(d_logp), frame_stride, row_stride, _dptr(d_tree_ids),
                                        _dptr(d_states0), _dptr(d_last0), alpha, T, B, mode, _dptr(d_tokens),
                                        _dptr(d_states), _dptr(d_scores), stream or None), "pb_fuse_frames_forest")


def pb_fuse_step_beam_forest(forest: Forest, d_logp, row_stride: int, d_tree_ids, d_hyp_scores, d_states_in,
                             alpha: float, U: int, K: int, d_tokens, d_parents, d_states_out, d_scores_out,
                             stream: int = 0):
    _check(load().pb_fuse_step_beam_forest(forest.handle, _dptr(d_logp), row_stride, _dptr(d_tree_ids),
                                           _dptr(d_hyp_scores), _dptr(d_states_in), alpha, U, K, _dptr(d_tokens),
                                           _dptr(d_parents), _dptr(d_states_out), _dptr(d_scores_out), stream or None),
           "pb_fuse_step_beam_forest")
