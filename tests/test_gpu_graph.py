"""The hot path under HIP graph capture: score -> select -> sparse prefill, plus the allocation-free retention call,
recorded once and replayed.  None of these calls allocates, synchronises or records a memset, so a serving loop can
keep a layer's calls in a graph; every replay must give exactly what the eager calls give on the same inputs (the
kernels are deterministic), also after the inputs changed in place and with eager work between the replays."""
import numpy as np
import pytest
import torch

from paper_2507_13681_amd import binding, inputs
from tests.gpu_util import Pipeline

pytestmark = pytest.mark.gpu


def _chain(pipe, qw, sc, sel, out, lse, keep_idx, keep_cnt, q_obs, budget, cshape, alpha):
    c, s = pipe.ctx, pipe.shape
    c.ls_score(s, qw, pipe.k, sc["vert"], sc["slash"], sc["vmax"], sc["smax"], sc["total"], None)
    c.ls_select(s, alpha, sc["vert"], sc["slash"], sc["vmax"], sc["smax"], sc["total"],
                sel["v_idx"], sel["v_cnt"], sel["s_idx"], sel["s_cnt"], sel["accounted"])
    c.ls_sparse_prefill(s, pipe.q, pipe.k, pipe.v, sel["v_idx"], sel["v_cnt"], sel["s_idx"], sel["s_cnt"], out, lse)
    binding.ls_kv_compress_static(cshape, budget, q_obs, pipe.k, None, keep_idx, keep_cnt, None, None)


def test_hot_path_replays_in_a_graph():
    cfg = inputs.scaled(inputs.CONFIGS["llama8b_8k"], n=4096, Hq=8, Hkv=2, heavy_lo=16, heavy_hi=48, span=128)
    q, k, v, _ = inputs.make_inputs(cfg)
    pipe = Pipeline(q, k, v, cfg.w, cfg.dtype)
    n_obs, budget = 16, 512
    cshape = binding.make_shape(cfg.B, cfg.Hq, cfg.Hkv, cfg.d, cfg.n, 1, n_obs, cfg.dtype)
    qw = pipe.q[:, :, -cfg.w:].contiguous()
    q_obs = pipe.q[:, :, -n_obs:].contiguous()

    def buffers():
        sc, sel = binding.alloc_score(pipe.shape), binding.alloc_select(pipe.shape)
        out = torch.empty_like(pipe.q)
        lse = torch.empty(pipe.q.shape[:3], dtype=torch.float32, device="cuda")
        keep_idx = torch.empty((cfg.B, cfg.Hkv, budget), dtype=torch.int32, device="cuda")
        keep_cnt = torch.empty((cfg.B, cfg.Hkv), dtype=torch.int32, device="cuda")
        return sc, sel, out, lse, keep_idx, keep_cnt

    def snapshot(sel, out, lse, keep_idx, keep_cnt):
        torch.cuda.synchronize()
        cnt_s, cnt_v = sel["s_cnt"].cpu().numpy(), sel["v_cnt"].cpu().numpy()
        s_idx, v_idx = sel["s_idx"].cpu().numpy(), sel["v_idx"].cpu().numpy()
        lists = [(s_idx[b, h, :cnt_s[b, h]].copy(), v_idx[b, h, :cnt_v[b, h]].copy())
                 for b in range(cfg.B) for h in range(cfg.Hq)]
        return dict(lists=lists, out=out.float().cpu().numpy(), lse=lse.cpu().numpy(),
                    keep=keep_idx.cpu().numpy().copy(), keep_cnt=keep_cnt.cpu().numpy().copy(),
                    acc=sel["accounted"].cpu().numpy().copy())

    def same(a, b):
        for (sa, va), (sb, vb) in zip(a["lists"], b["lists"]):
            np.testing.assert_array_equal(sa, sb)
            np.testing.assert_array_equal(va, vb)
        for name in ("out", "lse", "keep", "keep_cnt", "acc"):
            np.testing.assert_array_equal(a[name], b[name])

    eager_bufs = buffers()
    _chain(pipe, qw, *eager_bufs[:4], *eager_bufs[4:], q_obs, budget, cshape, cfg.alpha)       # also the first call on the device
    ref1 = snapshot(*eager_bufs[1:])

    g_bufs = buffers()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        _chain(pipe, qw, *g_bufs[:4], *g_bufs[4:], q_obs, budget, cshape, cfg.alpha)
    for rep in range(3):
        for t in (g_bufs[2], g_bufs[3]):
            t.fill_(float("nan"))                          # eager work between the replays
        print(f"graph replay {rep}", flush=True)
        graph.replay()
        same(snapshot(*g_bufs[1:]), ref1)
        assert pipe.ctx.ls_poll_status() == 0

    # new inputs in the same buffers: the replay must follow them, not repeat the recorded run's results
    pipe.q.mul_(0.75); qw.copy_(pipe.q[:, :, -cfg.w:]); q_obs.copy_(pipe.q[:, :, -n_obs:])
    pipe.k[:, :, : cfg.n // 2].mul_(-1.0)
    _chain(pipe, qw, *eager_bufs[:4], *eager_bufs[4:], q_obs, budget, cshape, cfg.alpha)
    ref2 = snapshot(*eager_bufs[1:])
    assert not np.array_equal(ref1["out"], ref2["out"])
    for rep in range(2):
        print(f"graph replay on new inputs {rep}", flush=True)
        graph.replay()
        same(snapshot(*g_bufs[1:]), ref2)
