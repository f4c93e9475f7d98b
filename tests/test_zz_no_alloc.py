"""pb_fuse_frames_static (the multi-frame decoder with its workspace in a fixed device array, for callers that
cannot allocate) against pb_fuse_frames_ws through the C ABI: two calls in a row, the second on a smaller input,
every output bit for bit; the fixed array covers every workspace size the library can ask for."""
import numpy as np
import pytest

import pb_workloads as W

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import paper_2508_07014_amd as pb  # noqa: E402

DEV = "cuda:0"


def _run(lib, name, tree, d_logp, mode, alpha, ws=None):
    T, B, V = d_logp.shape
    out = [torch.full((T, B), -9, dtype=torch.int32, device=DEV), torch.full((T, B), -9, dtype=torch.int32, device=DEV),
           torch.zeros((T, B), dtype=torch.float32, device=DEV)]
    s0 = torch.zeros(B, dtype=torch.int32, device=DEV)
    args = [tree.handle, d_logp.data_ptr(), B * V, V, s0.data_ptr(), None, alpha, T, B, mode, out[0].data_ptr(),
            out[1].data_ptr(), out[2].data_ptr()]
    if name == "pb_fuse_frames_ws":
        args += [ws.data_ptr(), ws.numel() * 4]
    rc = getattr(lib, name)(*args, None)
    torch.cuda.synchronize()
    assert rc == 0, (name, rc)
    return [o.cpu().numpy() for o in out]


def test_static_scratch_matches_workspace_form_on_two_calls_in_a_row():
    lib = pb.load()
    cfg = W.CONFIGS[2]
    toks, offs = W.make_phrases(cfg)
    tree = pb.pb_build(toks, offs, cfg.vocab_size, cfg.blank_id, device=0)
    V = cfg.vocab_size
    for (T, B, mode) in ((300, 48, 2), (120, 7, 0)):           # the second call is the smaller one
        shape = W.Config(9, "na", V, cfg.blank_id, 1, 1, 8, "uniform", 1.1, B, 1, T, 2.0)
        logp = W.make_logp(shape, seed=T, planting=W.Planting(toks, offs, cover=0.5), blank_bias=6.0, blank_frac=0.3)
        d_logp = torch.from_numpy(logp).to(DEV)
        need = int(lib.pb_fuse_frames_workspace_bytes(tree.handle, T, B))
        assert need > 0
        ws = torch.full((need // 4,), 0x5a5a5a5a, dtype=torch.int32, device=DEV)
        want = _run(lib, "pb_fuse_frames_ws", tree, d_logp, mode, cfg.alpha, ws)
        got = _run(lib, "pb_fuse_frames_static", tree, d_logp, mode, cfg.alpha)
        for g, w in zip(got, want):
            assert np.array_equal(g, w), (T, B, mode)
        again = _run(lib, "pb_fuse_frames_static", tree, d_logp, mode, cfg.alpha)
        for g, w in zip(again, want):
            assert np.array_equal(g, w), (T, B, mode)
    # the fixed array (2 MiB) holds the largest workspace the library's segment plan can ask for
    worst = max(int(lib.pb_fuse_frames_workspace_bytes(tree.handle, T, B))
                for T in (9, 64, 1000, 100000) for B in (1, 63, 64, 65, 128, 1000, 2047, 2048, 4095, 4096, 100000))
    assert 0 < worst <= (2 << 20)
    pb.pb_free(tree)
