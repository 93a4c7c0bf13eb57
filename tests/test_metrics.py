import numpy as np

from paper_2507_13681_amd import inputs, metrics


def _brute(n, n_hat, v, s):
    vs, ss = set(v), set(s)
    c = 0
    for a in range(n_hat):
        p = n - n_hat + a
        for b in range(p + 1):
            if b in vs or (p - b) in ss:
                c += 1
    return c


def test_allowed_cells_matches_bruteforce():
    rng = np.random.default_rng(0)
    for n, n_hat in [(40, 13), (33, 33), (64, 1), (50, 20)]:
        for _ in range(5):
            v = rng.choice(n, size=rng.integers(0, n // 2), replace=False)
            s = rng.choice(n, size=rng.integers(0, n // 2), replace=False)
            assert metrics.allowed_cells(n, n_hat, v, s) == _brute(n, n_hat, v, s)
        assert metrics.allowed_cells(n, n_hat, range(n), []) == metrics.causal_cells(n, n_hat)
        assert metrics.allowed_cells(n, n_hat, [], range(n)) == metrics.causal_cells(n, n_hat)
        assert metrics.allowed_cells(n, n_hat, range(n), range(n)) == metrics.causal_cells(n, n_hat)


def test_coverage_from_lse_matches_bruteforce(oracle):
    """exp(lse_selected - lse_dense) is the dense attention mass on the allowed cells (brute force in fp64)."""
    B, Hq, Hkv, n, n_hat, d = 1, 2, 1, 60, 20, 8
    q, k, v = inputs.make_plain(B, Hq, Hkv, n, n_hat, d, seed=4)
    vs, ss = [0, 3, 17, 41], [0, 1, 2, 9, 30]
    v_idx = np.zeros((B, Hq, n), np.int32); s_idx = np.zeros((B, Hq, n), np.int32)
    v_idx[:, :, :len(vs)] = vs; s_idx[:, :, :len(ss)] = ss
    v_cnt = np.full((B, Hq), len(vs), np.int32); s_cnt = np.full((B, Hq), len(ss), np.int32)
    _, lse_sel = oracle.attend(q, k, v, v_idx, v_cnt, s_idx, s_cnt, mode=0)
    all_idx = np.tile(np.arange(n, dtype=np.int32), (B, Hq, 1))
    _, lse_all = oracle.attend(q, k, v, all_idx, np.zeros((B, Hq), np.int32), all_idx, np.full((B, Hq), n, np.int32), mode=0)
    cov = metrics.coverage_from_lse(lse_sel, lse_all).reshape(B, Hq, n_hat)
    for h in range(Hq):
        for a in range(n_hat):
            p = n - n_hat + a
            s = (k[0, 0, :p + 1].astype(np.float64) @ q[0, h, a].astype(np.float64)) / np.sqrt(d)
            w = np.exp(s - s.max()); w /= w.sum()
            keep = np.array([(b in vs) or ((p - b) in ss) for b in range(p + 1)])
            np.testing.assert_allclose(cov[0, h, a], w[keep].sum(), rtol=1e-5)
    assert np.all(metrics.coverage_from_lse(np.array([-np.inf]), np.array([1.0])) == 0)


def test_visited_tiles_matches_bruteforce():
    rng = np.random.default_rng(4)
    n, n_hat = 700, 300
    for trial in range(4):
        s_sel = np.sort(rng.choice(n, size=int(rng.integers(0, 40)), replace=False))
        v_sel = np.sort(rng.choice(n, size=int(rng.integers(0, 200)), replace=False))
        pos0 = (n - n_hat) // 128 * 128
        want = 0
        sset = set(int(x) for x in s_sel)
        for bp in range(pos0, n, 128):
            posmax = min(bp + 127, n - 1)
            for kb in range(posmax // 64 + 1):
                rows = range(bp, bp + 128)
                keys = range(kb * 64, kb * 64 + 64)
                if any((r - c) in sset for r in (bp, bp + 127) for c in keys) or any((r - c) in sset for r in rows for c in (kb * 64, kb * 64 + 63)):
                    want += 1                                # a diagonal that crosses the tile crosses its border
            want += -(-int((v_sel <= posmax).sum()) // 64)
        assert metrics.visited_tiles(n, n_hat, v_sel, s_sel) == want
    every = np.arange(n)
    dense = metrics.visited_tiles(n, n_hat, np.arange(5), every)
    assert dense == sum(min(bp + 127, n - 1) // 64 + 1 for bp in range((n - n_hat) // 128 * 128, n, 128))
