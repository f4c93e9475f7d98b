"""Host tree compiler (pb_build with device = -1) and C-ABI surface, without a GPU.

The compiled flat arrays are compared state by state with the oracle's tree (canonical numbering
makes ids comparable), and a plain numpy reading of the flat arrays reproduces the oracle's rows.
"""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2508_07014_amd as pb
import pb_workloads as W
from oracle import OracleTree
from oracle.pb_oracle import W_LOGDEPTH, W_UNIFORM

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _both(tokens, offsets, V, blank, **kw):
    ot = OracleTree(tokens, offsets, V, blank, weights=kw.get("weights"), weight_mode=kw.get("weight_mode", 0),
                    beta=kw.get("beta", 2.0), unk_score=kw.get("unk_score", 0.0),
                    final_zero_backoff=kw.get("final_zero_backoff", True))
    tr = pb.pb_build(tokens, offsets, V, blank, device=-1, **kw)
    return ot, tr


def _compare_trees(ot, tr):
    info = pb.pb_info(tr)
    h = pb.pb_host_arrays(tr)
    n = ot.num_states
    assert info["num_states"] == n and info["num_arcs"] == n - 1 and info["max_depth"] == ot.max_depth
    chain_max = 0
    for s in range(n):
        nd = ot.node(s)
        assert h["depth"][s] == nd["depth"] and h["fail"][s] == nd["fail"] and h["parent"][s] == nd["parent"]
        assert bool(h["is_final"][s]) == nd["final"]
        assert h["acc"][s] == nd["acc"]
        assert h["backoff"][s] == np.float32(nd["bw"])
        if s:
            assert h["arc_token"][s - 1] == nd["token"] and h["arc_score"][s - 1] == np.float32(nd["arcw"])
        toks = h["arc_token"][h["arc_begin"][s]:h["arc_begin"][s] + h["arc_count"][s]]
        assert np.all(np.diff(toks) > 0)                      # rows strictly sorted by token
        for j, v in enumerate(toks):
            assert ot.child(s, int(v)) == h["arc_begin"][s] + j + 1
        hops, x = 0, s
        while x:
            x = h["fail"][x]
            hops += 1
        chain_max = max(chain_max, hops)
    assert info["max_fail_chain"] == chain_max
    assert info["root_degree"] == h["arc_count"][0]


def _rows_from_flat(h, V, blank, unk, s):
    """Dense (score, next) row of state s read off the flat arrays: deepest chain state wins."""
    score = np.empty(V, np.float32)
    nxt = np.empty(V, np.int32)
    chain, p, x = [], np.float32(0), s
    while x:
        chain.append((x, p))
        p = np.float32(p + h["backoff"][x])
        x = h["fail"][x]
    score[:] = p + h["root_score"]
    nxt[:] = h["root_next"]
    for x, px in reversed(chain):
        b, c = h["arc_begin"][x], h["arc_count"][x]
        tk = h["arc_token"][b:b + c]
        score[tk] = px + h["arc_score"][b:b + c]
        nxt[tk] = np.arange(b + 1, b + c + 1)
    if blank >= 0:
        score[blank] = 0
        nxt[blank] = s
    return score, nxt


@pytest.mark.parametrize("seed", range(30))
@pytest.mark.parametrize("mode", [W_UNIFORM, W_LOGDEPTH, 2])
def test_tiny_trees_match_oracle(seed, mode):
    V = 5 + seed % 4
    blank = 0 if seed % 2 else -1
    toks, offs, wts = W.tiny_case(4000 + seed, vocab_size=V, blank_id=blank, max_phrases=9, max_len=6)
    unk = 0.5 if seed % 3 == 0 else 0.0
    fzb = seed % 5 != 0
    ot, tr = _both(toks, offs, V, blank, weights=wts, weight_mode=mode, unk_score=unk, final_zero_backoff=fzb)
    _compare_trees(ot, tr)
    h = pb.pb_host_arrays(tr)
    sc, nx = ot.score(np.arange(ot.num_states))
    for s in range(ot.num_states):
        fs, fn = _rows_from_flat(h, V, blank, unk, s)
        assert np.array_equal(fs, sc[s]) and np.array_equal(fn, nx[s])
        assert pb.pb_state_prefix(tr, s) == ot.prefix(s)


@pytest.mark.parametrize("idx", [1, 2])
def test_config_trees_match_oracle(idx):
    cfg = W.CONFIGS[idx]
    toks, offs = W.make_phrases(cfg)
    ot, tr = _both(toks, offs, cfg.vocab_size, cfg.blank_id)
    _compare_trees(ot, tr)


def test_config3_tree_rows_sampled():
    cfg = W.CONFIGS[3]
    toks, offs = W.make_phrases(cfg)
    ot, tr = _both(toks, offs, cfg.vocab_size, cfg.blank_id, weight_mode=W_LOGDEPTH)
    info = pb.pb_info(tr)
    assert info["num_states"] == ot.num_states > 100000 and info["max_fail_chain"] >= 5
    h = pb.pb_host_arrays(tr)
    states = W.sample_states(ot.num_states, 64, 3)
    sc, nx = ot.score(states)
    for i, s in enumerate(states):
        fs, fn = _rows_from_flat(h, cfg.vocab_size, cfg.blank_id, 0.0, int(s))
        assert np.array_equal(fs, sc[i]) and np.array_equal(fn, nx[i])


def test_empty_list_gives_root_only_tree():
    tr = pb.pb_build(np.zeros(0, np.int32), np.zeros(1, np.int64), 16, 0, unk_score=0.25, device=-1)
    info = pb.pb_info(tr)
    assert info["num_states"] == 1 and info["num_arcs"] == 0 and info["root_degree"] == 0
    h = pb.pb_host_arrays(tr)
    assert np.all(h["root_score"] == np.float32(0.25)) and np.all(h["root_next"] == 0)


@pytest.mark.parametrize("bad,code", [("empty", pb.PB_EINVAL), ("range", pb.PB_ERANGE), ("blank", pb.PB_EINVAL),
                                      ("vocab", pb.PB_EINVAL), ("neg", pb.PB_ERANGE), ("mode", pb.PB_EINVAL),
                                      ("blank_range", pb.PB_EINVAL), ("decreasing", pb.PB_EINVAL)])
def test_build_error_codes(bad, code):
    toks = np.array([1, 2, 3], np.int32)
    offs = np.array([0, 2, 3], np.int64)
    V, blank, mode = 8, 0, 0
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
    elif bad == "mode":
        mode = 7
    elif bad == "blank_range":
        blank = 8
    elif bad == "decreasing":
        offs = np.array([0, 2, 1], np.int64)
    with pytest.raises(pb.PbError) as e:
        pb.pb_build(toks, offs, V, blank, weight_mode=mode, device=-1)
    assert e.value.code == code


@pytest.mark.parametrize("what", ["weight_inf", "weight_nan", "unk_inf", "beta_nan", "final_eos_inf", "overflow"])
def test_build_rejects_weights_that_are_not_finite(what):
    """The kernels multiply a boost by 0 for the blank column and compare fused values: scores must be finite."""
    toks = np.array([1, 2, 3, 4], np.int32)
    offs = np.array([0, 2, 4], np.int64)
    kw = dict(weights=np.array([1.0, 2.0], np.float32), weight_mode=pb.PB_W_UNIFORM, device=-1)
    code = pb.PB_EINVAL
    if what == "weight_inf":
        kw["weights"] = np.array([1.0, np.inf], np.float32)
    elif what == "weight_nan":
        kw["weights"] = np.array([np.nan, 1.0], np.float32)
    elif what == "unk_inf":
        kw["unk_score"] = -np.inf
    elif what == "beta_nan":
        kw["beta"] = np.nan
    elif what == "final_eos_inf":
        kw.update(eos_id=7, final_eos_score=np.inf)
    elif what == "overflow":  # finite weights whose sum along a phrase is not
        toks = np.array([1, 2, 3, 4, 5, 6], np.int32)
        offs = np.array([0, 6], np.int64)
        kw["weights"] = np.array([3.0e38], np.float32)
        code = pb.PB_ERANGE
    with pytest.raises(pb.PbError) as e:
        pb.pb_build(toks, offs, 8, 0, **kw)
    assert e.value.code == code
    ok = pb.pb_build(np.array([1, 2, 3, 4], np.int32), np.array([0, 2, 4], np.int64), 8, 0,
                     weights=np.array([1.0, 2.0], np.float32), device=-1)  # the same list with finite weights builds
    assert pb.pb_info(ok)["num_states"] == 5


def test_step_calls_on_host_only_tree_are_rejected_not_crashing():
    tr = pb.pb_build(np.array([1, 2], np.int32), np.array([0, 2], np.int64), 8, 0, device=-1)
    for call in (lambda: pb.pb_score(tr, 0, 1, 0),
                 lambda: pb.pb_fuse_step(tr, 0, 8, 0, 0.5, 1, 0, 0, 0),
                 lambda: pb.pb_fuse_frames(tr, 0, 8, 8, 0, 0.5, 1, 1, 0, 0, 0),
                 lambda: pb.pb_fuse_step_beam(tr, 0, 8, 0, 0, 0.5, 1, 1, 0, 0, 0, 0)):
        with pytest.raises(pb.PbError) as e:
            call()
        assert e.value.code == pb.PB_EINVAL
    with pytest.raises(pb.PbError):
        pb.pb_state_prefix(tr, 99)
    assert pb.strerror(pb.PB_EUNSUPPORTED) == "unsupported size" and pb.strerror(0) == "ok"


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "pb.h")).read()
    declared = sorted(set(re.findall(r"\b(pb_[a-z_]+)\s*\(", header)))
    assert declared == sorted(pb.EXPORTS)
    lib = C.CDLL(pb.library_path())
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_layouts_match_header_field_order():
    header = open(os.path.join(ROOT, "include", "pb.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} pb_build_opts;", header, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(?:int32_t|float)\s+(\w+);", body)
    assert fields == [n for n, _ in pb.binding.pb_build_opts._fields_]
    body = re.search(r"typedef struct \{((?:(?!typedef struct).)*?)\} pb_tree_info;", header, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(?:int32_t|int64_t)\s+(\w+);", body)
    assert fields == [n for n, _ in pb.binding.pb_tree_info._fields_]


def test_eos_options_are_validated_and_reported():
    toks, offs = np.array([1, 2, 3], np.int32), np.array([0, 3], np.int64)
    for bad in (2, 0, 9, -2):            # inside a phrase, the blank, outside the vocabulary
        with pytest.raises(pb.PbError) as e:
            pb.pb_build(toks, offs, 6, 0, device=-1, eos_id=bad)
        assert e.value.code == pb.PB_EINVAL
    tr = pb.pb_build(toks, offs, 6, 0, device=-1, eos_id=5, final_eos_score=2.0)
    assert pb.pb_info(tr)["eos_id"] == 5
    assert pb.pb_info(pb.pb_build(toks, offs, 6, 0, device=-1))["eos_id"] == -1


@pytest.mark.parametrize("seed", range(40))
def test_eos_table_equals_the_oracles_row_maximum(seed):
    """The host compiler tabulates the EOS boost per state; the oracle finds it by looping over every other
    token of the state's row (Sec. II-C).  Tiny trees with mixed weights, c_unk != 0 and both weight modes."""
    rng = np.random.Generator(np.random.PCG64(4000 + seed))
    V = int(rng.integers(4, 9))
    blank = 0 if seed % 3 else -1
    toks, offs, w = W.tiny_case(4100 + seed, vocab_size=V - 1, blank_id=blank)   # the last id stays free for the EOS
    eos = V - 1
    kw = dict(weights=w * rng.choice([-1.0, 1.0], size=len(w)).astype(np.float32), weight_mode=seed % 3,
              unk_score=float(rng.integers(-2, 3)) * 0.5)
    fin = float(rng.integers(0, 4)) * 0.25
    tr = pb.pb_build(toks, offs, V, blank, device=-1, eos_id=eos, final_eos_score=fin, **kw)
    ot = OracleTree(toks, offs, V, blank, eos_id=eos, final_eos_score=fin, **kw)
    table = pb.pb_host_arrays(tr)["eos_score"]
    want = ot.score(np.arange(ot.num_states, dtype=np.int32))[0][:, eos]
    assert np.array_equal(table, want)
    assert pb.pb_host_arrays(pb.pb_build(toks, offs, V, blank, device=-1, **kw))["eos_score"] is None


def test_validate_accepts_compiled_trees_and_flags_planted_damage(monkeypatch):
    """pb_validate bounds-checks the compiled arrays; a mistake planted in the tree's own host arrays (through
    the view pointers) must be reported as PB_ERANGE.  PB_DEBUG=1 makes pb_build run the check itself."""
    cfg = W.CONFIGS[2]
    toks, offs = W.make_phrases(cfg)
    toks = np.where(toks == cfg.vocab_size - 1, 1, toks).astype(np.int32)   # the last id becomes the EOS
    tr = pb.pb_build(toks, offs, cfg.vocab_size, cfg.blank_id, device=-1, eos_id=cfg.vocab_size - 1)
    assert pb.pb_validate(tr) == pb.PB_OK
    view = pb.binding.pb_host_view()
    assert pb.load().pb_host_arrays(tr.handle, C.byref(view)) == 0
    n = pb.pb_info(tr)["num_states"]
    for name, idx, bad in (("fail", n // 2, n + 5), ("arc_count", 7, 10 ** 6), ("arc_token", 3, cfg.vocab_size),
                           ("root_next", 5, -3), ("arc_begin", n - 1, n + 1)):
        ptr = getattr(view, name)
        keep = ptr[idx]
        ptr[idx] = bad
        assert pb.pb_validate(tr) == pb.PB_ERANGE, name
        ptr[idx] = keep
        assert pb.pb_validate(tr) == pb.PB_OK
    assert pb.pb_validate_states(tr, [0, 5, n - 1]) == -1
    assert pb.pb_validate_states(tr, [0, 5, n, -1]) == 2
    assert pb.pb_validate_states(tr, [-1]) == 0
    monkeypatch.setenv("PB_DEBUG", "1")
    assert pb.pb_validate(pb.pb_build(toks, offs, cfg.vocab_size, cfg.blank_id, device=-1)) == pb.PB_OK


def test_host_compiler_is_clean_under_address_and_ub_sanitizers(tmp_path):
    """tests/host_compile_sanitized.cpp: the compiler alone (no HIP runtime) built with g++ -fsanitize."""
    import shutil
    import subprocess
    if shutil.which("g++") is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "host_compile_sanitized")
    csrc = os.path.join(ROOT, "paper_2508_07014_amd", "csrc")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-static-libasan", "-static-libubsan",
           "-I", os.path.join(ROOT, "include"), "-I", csrc, os.path.join(ROOT, "tests", "host_compile_sanitized.cpp"),
           os.path.join(csrc, "pb_compile.cpp"), "-o", exe]
    subprocess.run(cmd, check=True)
    run = subprocess.run([exe], capture_output=True, text=True)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "clean" in run.stdout


def test_segment_plan_covers_the_frames_evenly_with_a_mild_taper():
    """Host side of the multi-frame decoder: how a call is cut into segments (pb_fuse_frames_plan).  Whatever the
    shape, the segments must tile [0, T) without gaps, none may be empty, there are at most 64 per hypothesis, and
    they are even up to the taper (first segments longer, last shorter, by about a twentieth of the mean)."""
    narrow = pb.pb_build(np.array([1, 2, 3], np.int32), np.array([0, 3], np.int64), 64, 0, device=-1)
    wide = pb.pb_build(np.array([1, 2, 3], np.int32), np.array([0, 3], np.int64), 4096, 0, device=-1)
    try:
        for tree, target in ((narrow, 4096), (wide, 1024)):
            assert pb.pb_fuse_frames_plan(tree, 0, 5) == [0] and pb.pb_fuse_frames_plan(tree, 5, 0) == [0]
            for T in list(range(1, 140)) + [255, 256, 257, 500, 1000, 1023, 4096, 10007]:
                for B in (1, 2, 3, 7, 31, 64, 128, 256, 1000, 2048, 5000):
                    b = pb.pb_fuse_frames_plan(tree, T, B)
                    n = len(b) - 1
                    assert 1 <= n <= 64 and b[0] == 0 and b[-1] == T, (T, B, b)
                    lens = np.diff(b)
                    assert lens.min() >= 1, (T, B, b)
                    mean = T / n
                    assert lens.max() <= mean * 1.05 + 2 and lens.min() >= mean * 0.95 - 2, (T, B, lens)
                    if n >= 4 and mean >= 40:   # the taper: the first quarter is longer than the last
                        q = n // 4
                        assert lens[:q].mean() > lens[-q:].mean(), (T, B, lens)
                    # enough chains to fill the chip when the call is long enough, never more than about twice the aim
                    if T >= 8 * 64:
                        assert n * B >= min(target, 64 * B) * 0.5, (T, B, n)
        assert len(pb.pb_fuse_frames_plan(narrow, 1000, 128)) - 1 == 32
        assert len(pb.pb_fuse_frames_plan(wide, 200, 256)) - 1 == 4
    finally:
        pb.pb_free(narrow)
        pb.pb_free(wide)
