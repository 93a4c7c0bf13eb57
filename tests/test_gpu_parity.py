"""GPU parity: every C-ABI entry point against the CPU oracle on the same seeded inputs."""
import math

import numpy as np
import pytest
import torch

from paper_2507_13681_amd import binding, inputs

pytestmark = pytest.mark.gpu

from tests.gpu_util import Pipeline, dev_lists, dev_scores, host  # noqa: E402


def _score_close(gpu, ref, w):
    for name in ("vert", "slash", "vmax", "smax"):
        np.testing.assert_allclose(gpu[name], ref[name], rtol=1e-3, atol=1e-6 * w, err_msg=name)
    np.testing.assert_allclose(gpu["total"], ref["total"], rtol=1e-5)


# --------------------------------------------------------------------------- ls_score

@pytest.mark.parametrize("B,Hq,Hkv,n,w,d,dtype", [
    (1, 4, 1, 1024, 32, 64, "f32"),       # the tiny workload's shape
    (2, 4, 2, 300, 20, 64, "bf16"),       # ragged: n not a multiple of the key block, w not of 32
    (1, 8, 2, 1000, 64, 128, "bf16"),
    (1, 2, 2, 129, 128, 128, "f32"),      # window almost the whole context
    (1, 2, 1, 40, 40, 64, "bf16"),        # first turn: every row scored, single key block
    (1, 4, 2, 600, 100, 128, "bf16"),     # window longer than the staged-query register budget, ragged rows
    (1, 2, 1, 700, 256, 128, "f32"),      # longest window: largest LDS footprint, diagonals through atomics
])
def test_score_matches_oracle(oracle, B, Hq, Hkv, n, w, d, dtype):
    q, k, v = inputs.make_plain(B, Hq, Hkv, n, w, d, dtype=dtype, seed=n + w, q_scale=2.0)
    print(f"score case B={B} Hq={Hq} Hkv={Hkv} n={n} w={w} d={d} {dtype}", flush=True)
    ref = oracle.score(q, k)
    pipe = Pipeline(q, k, v, w, dtype)
    gpu = host(pipe.score())
    _score_close(gpu, ref, w)


def test_score_is_bit_reproducible(oracle):
    cfg = inputs.scaled(inputs.CONFIGS["llama8b_8k"], n=2048, Hq=8, Hkv=2, heavy_lo=16, heavy_hi=16, span=128)
    q, k, v, _ = inputs.make_inputs(cfg)
    pipe = Pipeline(q, k, v, cfg.w, cfg.dtype)
    a, b = host(pipe.score()), host(pipe.score())
    for name in a:
        np.testing.assert_array_equal(a[name], b[name])
    _score_close(a, oracle.score(q[:, :, -cfg.w:], k), cfg.w)


def test_score_explicit_positions(oracle):
    B, Hq, Hkv, n, w, d = 1, 2, 1, 500, 24, 64
    q, k, v = inputs.make_plain(B, Hq, Hkv, n, w, d, dtype="bf16", seed=9, q_scale=2.0)
    pos = np.sort(np.random.default_rng(0).choice(n, size=w, replace=False))
    ref = oracle.score(q, k, q_pos=pos)
    pipe = Pipeline(q, k, v, w, "bf16")
    gpu = host(pipe.score(q_pos=pos))
    _score_close(gpu, ref, w)


# --------------------------------------------------------------------------- ls_select

def _sets(sel, b, h):
    nv, ns = int(sel["v_cnt"][b, h]), int(sel["s_cnt"][b, h])
    return sel["v_idx"][b, h, :nv], sel["s_idx"][b, h, :ns]


@pytest.mark.parametrize("alpha,n", [(0.0, 3000), (0.5, 3000), (0.9, 3000), (0.95, 3000), (1.0, 3000),
                                     (0.95, 2048), (1.0, 2048), (1.0, 5120)])
def test_select_bit_exact_on_oracle_scores(oracle, alpha, n):
    """Fed the oracle's line weights, the device walk must reproduce the oracle's sets and sum exactly.
    (Lengths that are multiples of 1024 end a list exactly at the end of a staged block; alpha = 1 walks both
    lists to their ends.)"""
    cfg = inputs.scaled(inputs.CONFIGS["llama8b_8k"], n=n, Hq=8, Hkv=2, heavy_lo=16, heavy_hi=48, span=128)
    q, k, v, _ = inputs.make_inputs(cfg)
    sc = oracle.score(q[:, :, -cfg.w:], k)
    ref = oracle.select(sc, cfg.n_hat, alpha)
    pipe = Pipeline(q, k, v, cfg.w, cfg.dtype)
    for with_acc in (True, False):
        print(f"select alpha={alpha} n={n} accounted={with_acc}", flush=True)
        gpu = host(pipe.select(dev_scores(sc), alpha, accounted=with_acc))
        np.testing.assert_array_equal(gpu["v_cnt"], ref["v_cnt"])
        np.testing.assert_array_equal(gpu["s_cnt"], ref["s_cnt"])
        for h in range(cfg.Hq):
            gv, gs = _sets(gpu, 0, h)
            rv, rs = _sets(ref, 0, h)
            np.testing.assert_array_equal(gv, rv)
            np.testing.assert_array_equal(gs, rs)
        if with_acc:
            np.testing.assert_array_equal(gpu["accounted"], ref["accounted"])


def test_select_ties_and_capacity(oracle):
    """Many equal weights (ties resolved by index) and truncated output lists."""
    n, n_hat = 700, 200
    rng = np.random.default_rng(3)
    sc = dict(vert=rng.integers(0, 4, (1, 2, n)).astype(np.float32) / 4,
              slash=rng.integers(0, 4, (1, 2, n)).astype(np.float32) / 8,
              vmax=np.full((1, 2, n), 1 / 64, np.float32), smax=np.full((1, 2, n), 1 / 128, np.float32))
    sc["total"] = sc["vert"].sum(-1).astype(np.float32)
    ref = oracle.select(sc, n_hat, 0.6, cap_v=50, cap_s=60)
    q, k, v = inputs.make_plain(1, 2, 1, n, n_hat, 64, dtype="bf16", seed=1)
    pipe = Pipeline(q, k, v, 8, "bf16")
    gpu = host(pipe.select(dev_scores(sc), 0.6, cap_v=50, cap_s=60))
    np.testing.assert_array_equal(gpu["v_cnt"], ref["v_cnt"])
    np.testing.assert_array_equal(gpu["s_cnt"], ref["s_cnt"])
    for h in range(2):
        nv, ns = min(50, int(ref["v_cnt"][0, h])), min(60, int(ref["s_cnt"][0, h]))
        np.testing.assert_array_equal(gpu["v_idx"][0, h, :nv], ref["v_idx"][0, h, :nv])
        np.testing.assert_array_equal(gpu["s_idx"][0, h, :ns], ref["s_idx"][0, h, :ns])
    np.testing.assert_array_equal(gpu["accounted"], ref["accounted"])


@pytest.mark.parametrize("heads", [2, 16, 24])
def test_select_ties_across_sort_segments(oracle, heads):
    """Equal weights spread over several sort segments (the last one ragged): the order of equal weights is by
    index, whichever segment they sit in.  The segment length follows n * heads (2048, 4096 and 8192 here)."""
    n, n_hat = 3 * 8192 + 517, 4000
    rng = np.random.default_rng(11)
    sc = dict(vert=rng.integers(0, 6, (1, heads, n)).astype(np.float32) / 8192,
              slash=rng.integers(0, 3, (1, heads, n)).astype(np.float32) / 4096,
              vmax=np.full((1, heads, n), 2.0 ** -20, np.float32), smax=np.full((1, heads, n), 2.0 ** -21, np.float32))
    sc["total"] = sc["vert"].sum(-1).astype(np.float32)
    ref = oracle.select(sc, n_hat, 0.7)
    q, k, v = inputs.make_plain(1, heads, 1, n, n_hat, 64, dtype="bf16", seed=1)
    pipe = Pipeline(q, k, v, 8, "bf16")
    print(f"select ties heads={heads}", flush=True)
    gpu = host(pipe.select(dev_scores(sc), 0.7))
    np.testing.assert_array_equal(gpu["v_cnt"], ref["v_cnt"])
    np.testing.assert_array_equal(gpu["s_cnt"], ref["s_cnt"])
    for h in range(heads):
        gv, gs = _sets(gpu, 0, h)
        rv, rs = _sets(ref, 0, h)
        np.testing.assert_array_equal(gv, rv)
        np.testing.assert_array_equal(gs, rs)
    np.testing.assert_array_equal(gpu["accounted"], ref["accounted"])


# --------------------------------------------------------------------------- ls_sparse_prefill

def _lists(B, Hq, n, fn):
    v_idx = np.zeros((B, Hq, n), np.int32); s_idx = np.zeros((B, Hq, n), np.int32)
    v_cnt = np.zeros((B, Hq), np.int32); s_cnt = np.zeros((B, Hq), np.int32)
    for b in range(B):
        for h in range(Hq):
            vs, ss = fn(b, h)
            vs, ss = sorted(vs), sorted(ss)
            v_idx[b, h, :len(vs)] = vs; v_cnt[b, h] = len(vs)
            s_idx[b, h, :len(ss)] = ss; s_cnt[b, h] = len(ss)
    return v_idx, v_cnt, s_idx, s_cnt


def _attn_close(out, lse, ref_out, ref_lse, dtype):
    out = out.reshape(ref_out.shape)
    if dtype == "bf16":
        err = np.abs(out - ref_out)
        assert err.max() <= 2e-2, err.max()
        assert err.mean() <= 5e-3, err.mean()
    else:
        np.testing.assert_allclose(out, ref_out, rtol=0, atol=1e-4)
    fin = np.isfinite(ref_lse)
    np.testing.assert_array_equal(np.isfinite(lse.reshape(-1)), fin)
    np.testing.assert_allclose(lse.reshape(-1)[fin], ref_lse[fin], rtol=0, atol=2e-3 if dtype == "bf16" else 1e-4)


PATTERNS = ["dense_slashes", "dense_columns", "window", "sink_window", "random_mixed", "columns_only",
            "isolated_diagonals", "empty_rows", "nothing"]


@pytest.mark.parametrize("pattern", PATTERNS)
@pytest.mark.parametrize("B,Hq,Hkv,n,n_hat,d,dtype", [
    (1, 4, 1, 1024, 256, 64, "f32"),
    (1, 4, 2, 700, 333, 128, "bf16"),      # ragged row blocks and key blocks
    (2, 2, 2, 200, 200, 64, "bf16"),       # first turn: n_hat = n
    (1, 2, 1, 450, 130, 128, "f32"),
    (1, 8, 1, 180, 180, 128, "bf16"),      # eight query heads per KV head, first turn shorter than two row blocks
    (1, 2, 2, 1500, 1, 128, "bf16"),       # a single new row
    (1, 4, 2, 2100, 900, 64, "bf16"),      # d = 64 over many tiles and several items per workgroup
])
def test_prefill_matches_oracle(oracle, pattern, B, Hq, Hkv, n, n_hat, d, dtype):
    q, k, v = inputs.make_plain(B, Hq, Hkv, n, n_hat, d, dtype=dtype, seed=n + d, q_scale=1.5)
    rng = np.random.default_rng(n)

    def fn(b, h):
        if pattern == "dense_slashes":
            return [], range(n)
        if pattern == "dense_columns":
            return range(n), []
        if pattern == "window":
            return [], range(70 + h)
        if pattern == "sink_window":
            return [0, 1, 2, 3], range(33)
        if pattern == "random_mixed":
            return rng.choice(n, size=n // 7, replace=False), rng.choice(n, size=n // 9, replace=False)
        if pattern == "columns_only":
            return rng.choice(n, size=min(n, 90 + 10 * h), replace=False), []
        if pattern == "isolated_diagonals":
            return [5], [0, 64, 65, min(200, n - 2), n - 1]
        if pattern == "empty_rows":
            return [n - 3], []
        return [], []

    v_idx, v_cnt, s_idx, s_cnt = _lists(B, Hq, n, fn)
    print(f"prefill case {pattern} B={B} Hq={Hq} Hkv={Hkv} n={n} n_hat={n_hat} d={d} {dtype}", flush=True)
    ref_out, ref_lse = oracle.attend(q, k, v, v_idx, v_cnt, s_idx, s_cnt, mode=0)
    pipe = Pipeline(q, k, v, min(8, n_hat), dtype)
    out, lse = pipe.prefill(dev_lists(v_idx, v_cnt, s_idx, s_cnt))
    _attn_close(out.float().cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, dtype)
    if pattern in ("empty_rows", "nothing"):
        o = out.float().cpu().numpy().reshape(B, Hq, n_hat, d)
        dead = ~np.isfinite(ref_lse.reshape(B, Hq, n_hat))
        assert (dead.any() or n_hat < 4) and np.all(o[dead] == 0)     # rows before column n - 3 see nothing


# --------------------------------------------------------------------------- ls_kv_compress

@pytest.mark.parametrize("B,Hq,Hkv,ln,n_obs,d,budget,dtype", [
    (2, 8, 2, 900, 16, 128, 128, "bf16"),
    (1, 4, 1, 300, 16, 64, 64, "f32"),
    (1, 4, 4, 100, 8, 64, 256, "bf16"),    # budget >= len keeps everything
    (1, 4, 2, 5000, 16, 64, 700, "bf16"),  # several selection chunks, the last one ragged
])
def test_compress_matches_oracle(oracle, B, Hq, Hkv, ln, n_obs, d, budget, dtype):
    q, k, v = inputs.make_plain(B, Hq, Hkv, ln, n_obs, d, dtype=dtype, seed=ln, q_scale=2.0)
    ref = oracle.compress(q, k, budget)
    pipe = Pipeline(q, k, v, n_obs, dtype, budget=budget)
    keep_idx = torch.full((B, Hkv, budget), -1, dtype=torch.int32, device="cuda")
    keep_cnt = torch.zeros((B, Hkv), dtype=torch.int32, device="cuda")
    k_out = torch.zeros((B, Hkv, budget, d), dtype=pipe.k.dtype, device="cuda")
    v_out = torch.zeros_like(k_out)
    pipe.ctx.ls_kv_compress(pipe.shape, budget, pipe.q, pipe.k, pipe.v, keep_idx, keep_cnt, k_out, v_out)
    score = torch.empty((B, Hkv, ln), dtype=torch.float32, device="cuda")
    pipe.ctx.debug_compress_score(pipe.shape, score)
    score = score.cpu().numpy()
    np.testing.assert_allclose(score, ref["score"], rtol=1e-3, atol=1e-6 * n_obs)
    np.testing.assert_array_equal(keep_cnt.cpu().numpy(), ref["keep_cnt"])
    ki = keep_idx.cpu().numpy()
    for b in range(B):
        for j in range(Hkv):
            cnt = int(ref["keep_cnt"][b, j])
            got, want = ki[b, j, :cnt], ref["keep_idx"][b, j, :cnt]
            assert np.all(np.diff(got) > 0)
            # the device ranks its own fp32 scores: exact against the oracle's ranking of those scores
            np.testing.assert_array_equal(got, oracle.topb(score[b, j], budget))
            # against the oracle's own scores only entries at the threshold may differ
            diff = np.setxor1d(got, want)
            if len(diff):
                thr = np.sort(ref["score"][b, j])[::-1][cnt - 1]
                assert np.all(np.abs(ref["score"][b, j][diff] - thr) <= 1e-3 * thr)
            np.testing.assert_array_equal(k_out[b, j, :cnt].float().cpu().numpy(), k[b, j][got])
            np.testing.assert_array_equal(v_out[b, j, :cnt].float().cpu().numpy(), v[b, j][got])


def test_compress_ties_across_chunks(oracle):
    """Repeated key rows give exactly equal scores all over the cache: the threshold falls among ties that span
    several selection chunks and must be resolved towards the smaller indices."""
    B, Hq, Hkv, ln, n_obs, d, budget = 1, 2, 1, 4500, 8, 64, 1000
    q, k, v = inputs.make_plain(B, Hq, Hkv, ln, n_obs, d, dtype="bf16", seed=5, q_scale=2.0)
    k = k[:, :, np.arange(ln) % 37].copy()
    pipe = Pipeline(q, k, v, n_obs, "bf16", budget=budget)
    keep_idx = torch.full((B, Hkv, budget), -1, dtype=torch.int32, device="cuda")
    keep_cnt = torch.zeros((B, Hkv), dtype=torch.int32, device="cuda")
    pipe.ctx.ls_kv_compress(pipe.shape, budget, pipe.q, pipe.k, None, keep_idx, keep_cnt)
    score = torch.empty((B, Hkv, ln), dtype=torch.float32, device="cuda")
    pipe.ctx.debug_compress_score(pipe.shape, score)
    score = score.cpu().numpy()
    assert len(np.unique(score[0, 0, : ln - n_obs])) <= 37       # the ties are really there
    assert int(keep_cnt.cpu().numpy()[0, 0]) == budget
    np.testing.assert_array_equal(keep_idx.cpu().numpy()[0, 0], oracle.topb(score[0, 0], budget))


# --------------------------------------------------------------------------- argument errors

def test_argument_errors_are_reported():
    shape = binding.make_shape(1, 4, 2, 64, 256, 64, 16, "bf16")
    ctx = binding.Context(shape)
    q = torch.zeros(1, 4, 64, 64, dtype=torch.bfloat16, device="cuda")
    k = torch.zeros(1, 2, 256, 64, dtype=torch.bfloat16, device="cuda")
    sc = binding.alloc_score(shape)
    sel = binding.alloc_select(shape)
    with pytest.raises(binding.LoopServeError, match="alpha"):
        ctx.ls_select(shape, 1.5, sc["vert"], sc["slash"], sc["vmax"], sc["smax"], sc["total"],
                      sel["v_idx"], sel["v_cnt"], sel["s_idx"], sel["s_cnt"], sel["accounted"])
    bad = binding.make_shape(1, 4, 3, 64, 256, 64, 16, "bf16")
    with pytest.raises(binding.LoopServeError, match="multiple"):
        ctx.ls_score(bad, q[:, :, -16:].contiguous(), k, sc["vert"], sc["slash"], sc["vmax"], sc["smax"], sc["total"])
    big = binding.make_shape(1, 4, 2, 64, 1 << 20, 64, 16, "bf16")
    with pytest.raises(binding.LoopServeError, match="LS_MAX_N"):
        ctx.ls_sparse_prefill(big, q, k, k, sel["v_idx"], sel["v_cnt"], sel["s_idx"], sel["s_cnt"], q)
    keep_idx = torch.zeros(1, 2, 8, dtype=torch.int32, device="cuda")
    keep_cnt = torch.zeros(1, 2, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.LoopServeError, match="LS_MAX_N"):      # longer than the top-B kernels take: refused on the host
        ctx.ls_kv_compress(big, 8, q[:, :, -16:].contiguous(), k, None, keep_idx, keep_cnt)
    small = binding.Context(workspace=1024)
    with pytest.raises(binding.LoopServeError, match="workspace"):
        small.ls_score(shape, q[:, :, -16:].contiguous(), k, sc["vert"], sc["slash"], sc["vmax"], sc["smax"], sc["total"])
    with pytest.raises(binding.LoopServeError, match="n_hat"):
        ctx.ls_select(binding.make_shape(1, 4, 2, 64, 256, 300, 16, "bf16"), 0.5, sc["vert"], sc["slash"], sc["vmax"],
                      sc["smax"], sc["total"], sel["v_idx"], sel["v_cnt"], sel["s_idx"], sel["s_cnt"], None)
