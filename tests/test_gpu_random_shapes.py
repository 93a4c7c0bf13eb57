"""A seeded sweep of random shapes and selections through ls_sparse_prefill: head counts (G = 1 .. 8, three KV heads), both
head dimensions and storage types, context and turn lengths with no relation to any tile size, and per head one of: nothing,
columns only, diagonals only (scattered or one run), a few of each, everything plus one kind.  Every output element against the
oracle's dense-masked evaluator, outputs pre-filled with NaN."""
import numpy as np
import pytest
import torch

from paper_2507_13681_amd import inputs
from tests.gpu_util import Pipeline, dev_lists

pytestmark = pytest.mark.gpu


def _selection(rng, B, Hq, n):
    v_idx = np.zeros((B, Hq, n), np.int32); s_idx = np.zeros((B, Hq, n), np.int32)
    v_cnt = np.zeros((B, Hq), np.int32); s_cnt = np.zeros((B, Hq), np.int32)
    few = min(n, 40)
    for b in range(B):
        for h in range(Hq):
            kind = int(rng.integers(0, 6))
            nv = [0, int(rng.integers(0, n + 1)), 0, int(rng.integers(0, few + 1)), n, int(rng.integers(0, n + 1))][kind]
            ns = [0, 0, int(rng.integers(0, n + 1)), int(rng.integers(0, few + 1)), int(rng.integers(0, n + 1)), n][kind]
            cv = np.sort(rng.choice(n, size=nv, replace=False))
            cs = np.sort(rng.choice(n, size=ns, replace=False))
            if kind == 2 and ns > 3 and rng.random() < 0.5:                  # one run of consecutive diagonals
                start = int(rng.integers(0, n))
                cs = np.arange(start, min(n, start + ns))
                ns = len(cs)
            v_idx[b, h, :nv] = cv; s_idx[b, h, :ns] = cs
            v_cnt[b, h] = nv; s_cnt[b, h] = ns
    return v_idx, v_cnt, s_idx, s_cnt


@pytest.mark.parametrize("seed", [1, 7])
def test_random_shapes_and_selections(oracle, seed):
    rng = np.random.default_rng(seed)
    for case in range(25):
        d = int(rng.choice([64, 128])); dtype = str(rng.choice(["bf16", "bf16", "f32"]))
        Hkv = int(rng.choice([1, 2, 3])); Hq = Hkv * int(rng.choice([1, 2, 4, 8])); B = int(rng.choice([1, 2]))
        n = int(rng.integers(1, 1400)) if rng.random() < 0.85 else int(rng.integers(1400, 5000))
        n_hat = int(rng.integers(1, n + 1))
        q, k, v = inputs.make_plain(B, Hq, Hkv, n, n_hat, d, dtype=dtype, seed=int(rng.integers(1 << 30)), q_scale=1.5)
        v_idx, v_cnt, s_idx, s_cnt = _selection(rng, B, Hq, n)
        print(f"case {case}: B={B} Hq={Hq} Hkv={Hkv} d={d} {dtype} n={n} n_hat={n_hat}", flush=True)
        ref_out, ref_lse = oracle.attend(q, k, v, v_idx, v_cnt, s_idx, s_cnt, mode=0)
        pipe = Pipeline(q, k, v, min(8, n_hat), dtype)
        out, lse = pipe.prefill(dev_lists(v_idx, v_cnt, s_idx, s_cnt), sentinel=True)
        torch.cuda.synchronize()
        assert pipe.ctx.ls_poll_status() == 0
        o = out.float().cpu().numpy().reshape(ref_out.shape)
        l = lse.cpu().numpy().reshape(ref_lse.shape)
        assert not np.isnan(o).any() and not np.isnan(l).any()
        tol_max, tol_mean, tol_lse = (2e-2, 5e-3, 2e-3) if dtype == "bf16" else (1e-4, 1e-5, 1e-4)
        err = np.abs(o - ref_out)
        assert err.max() <= tol_max and err.mean() <= tol_mean, (err.max(), err.mean())
        alive = np.isfinite(ref_lse)
        np.testing.assert_array_equal(np.isfinite(l), alive)                 # rows without an allowed cell: lse = -inf
        assert np.all(o[~alive] == 0)
        if alive.any():
            assert np.abs(l[alive] - ref_lse[alive]).max() <= tol_lse


def test_random_score_shapes(oracle):
    """ls_score over random head counts, lengths and window lengths (1 .. 256 rows), a third of the cases with
    explicit scattered row positions."""
    from tests.gpu_util import host
    rng = np.random.default_rng(9)
    for case in range(24):
        d = int(rng.choice([64, 128])); dtype = str(rng.choice(["bf16", "f32"]))
        Hkv = int(rng.choice([1, 2, 3])); Hq = Hkv * int(rng.choice([1, 2, 4, 8])); B = int(rng.choice([1, 2]))
        n = int(rng.integers(1, 3000)); w = int(rng.integers(1, min(n, 256) + 1))
        q, k, v = inputs.make_plain(B, Hq, Hkv, n, w, d, dtype=dtype, seed=int(rng.integers(1 << 30)), q_scale=2.0)
        explicit = rng.random() < 0.3
        print(f"score case {case}: B={B} Hq={Hq} Hkv={Hkv} d={d} {dtype} n={n} w={w} explicit={explicit}", flush=True)
        pipe = Pipeline(q, k, v, w, dtype)
        if explicit:
            pos = np.sort(rng.choice(n, size=w, replace=False)).astype(np.int64)
            ref, gpu = oracle.score(q, k, q_pos=pos), host(pipe.score(q_pos=pos))
        else:
            ref, gpu = oracle.score(q, k), host(pipe.score())
        for name in ("vert", "slash", "vmax", "smax", "total"):
            np.testing.assert_allclose(gpu[name], ref[name], rtol=1e-3, atol=1e-6 * w, err_msg=name)


def test_random_select_inputs(oracle):
    """ls_select on random weights (heavy-tailed, many ties, one list nearly empty, uniform) at random lengths up to
    40000 and alpha from 0 to 1: lists, counts and the accounted sum exactly as the oracle's walk gives them."""
    from tests.gpu_util import dev_scores, host
    rng = np.random.default_rng(3)
    for case in range(30):
        heads = int(rng.choice([1, 2, 5, 8, 17])); w = 8
        n = int(rng.integers(1, 3000)) if rng.random() < 0.7 else int(rng.integers(3000, 40000))
        n_hat = int(rng.integers(1, n + 1)); alpha = float(rng.choice([0.0, 0.3, 0.7, 0.9, 0.95, 0.99, 1.0]))
        style = int(rng.integers(0, 4))
        if style == 0:
            vert, slash = rng.pareto(1.2, (1, heads, n)), rng.pareto(1.5, (1, heads, n))
        elif style == 1:
            vert, slash = rng.integers(0, 5, (1, heads, n)) / 64, rng.integers(0, 3, (1, heads, n)) / 32
        elif style == 2:
            vert = np.zeros((1, heads, n)); vert[..., : max(1, n // 50)] = 1.0
            slash = rng.random((1, heads, n)) * 1e-3
        else:
            vert, slash = rng.random((1, heads, n)), rng.random((1, heads, n))
        norm = lambda x: (x * (w / np.maximum(x.sum(-1, keepdims=True), 1e-30))).astype(np.float32)
        vert, slash = norm(np.asarray(vert, np.float64)), norm(np.asarray(slash, np.float64))
        frac = rng.random()
        sc = dict(vert=vert, slash=slash, vmax=(vert * frac * rng.random(vert.shape)).astype(np.float32),
                  smax=(slash * frac * rng.random(slash.shape)).astype(np.float32))
        sc["total"] = sc["vert"].sum(-1).astype(np.float32)
        print(f"select case {case}: heads={heads} n={n} n_hat={n_hat} alpha={alpha} style={style}", flush=True)
        ref = oracle.select(sc, n_hat, alpha)
        q, k, v = inputs.make_plain(1, heads, 1, n, n_hat, 64, dtype="bf16", seed=1)
        pipe = Pipeline(q, k, v, min(8, n_hat), "bf16")
        for acc in (True, False):
            gpu = host(pipe.select(dev_scores(sc), alpha, accounted=acc))
            np.testing.assert_array_equal(gpu["v_cnt"], ref["v_cnt"])
            np.testing.assert_array_equal(gpu["s_cnt"], ref["s_cnt"])
            for h in range(heads):
                np.testing.assert_array_equal(gpu["v_idx"][0, h, :ref["v_cnt"][0, h]], ref["v_idx"][0, h, :ref["v_cnt"][0, h]])
                np.testing.assert_array_equal(gpu["s_idx"][0, h, :ref["s_cnt"][0, h]], ref["s_idx"][0, h, :ref["s_cnt"][0, h]])
            if acc:
                np.testing.assert_array_equal(gpu["accounted"], ref["accounted"])
        assert pipe.ctx.ls_poll_status() == 0


def test_random_compress_shapes(oracle):
    """ls_kv_compress over random cache lengths, observation windows and budgets (incl. budget >= length and all-equal
    scores): scores close to the oracle's, kept set exactly its ranking of the device's scores, gathered rows bit-exact."""
    rng = np.random.default_rng(5)
    for case in range(24):
        d = int(rng.choice([64, 128])); dtype = str(rng.choice(["bf16", "f32"]))
        Hkv = int(rng.choice([1, 2, 3])); Hq = Hkv * int(rng.choice([1, 2, 4, 8])); B = int(rng.choice([1, 2]))
        ln = int(rng.integers(1, 9000)); n_obs = int(rng.integers(1, min(ln, 64) + 1)); budget = int(rng.integers(1, 3000))
        q, k, v = inputs.make_plain(B, Hq, Hkv, ln, n_obs, d, dtype=dtype, seed=int(rng.integers(1 << 30)),
                                    q_scale=float(rng.choice([0.0, 1.0, 3.0])))
        print(f"compress case {case}: B={B} Hq={Hq} Hkv={Hkv} d={d} {dtype} len={ln} n_obs={n_obs} budget={budget}", flush=True)
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
        ki, ko, vo = keep_idx.cpu().numpy(), k_out.float().cpu().numpy(), v_out.float().cpu().numpy()
        kk, vv = pipe.k.float().cpu().numpy(), pipe.v.float().cpu().numpy()
        for b in range(B):
            for j in range(Hkv):
                c = int(ref["keep_cnt"][b, j])
                exp = oracle.topb(score[b, j], budget)[:c]
                np.testing.assert_array_equal(ki[b, j, :c], exp)
                np.testing.assert_array_equal(ko[b, j, :c], kk[b, j, exp])
                np.testing.assert_array_equal(vo[b, j, :c], vv[b, j, exp])
