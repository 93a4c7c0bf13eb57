import numpy as np

from paper_2507_13681_amd import metrics


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
