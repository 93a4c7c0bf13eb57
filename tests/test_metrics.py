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
