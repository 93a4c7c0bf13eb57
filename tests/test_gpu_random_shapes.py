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
