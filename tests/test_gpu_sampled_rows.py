"""Scoring on sampled rows of the newest turn (Alg. 2 draws the scored rows with RandomSelect) and the
coverage the resulting selection really keeps on those rows (the left side of Eq. 1), all on the device."""
import numpy as np
import pytest
import torch

from paper_2507_13681_amd import inputs, metrics

pytestmark = pytest.mark.gpu

from tests.gpu_util import Pipeline, dev_lists, host  # noqa: E402


def _dense_lists(B, Hq, n):
    idx = np.tile(np.arange(n, dtype=np.int32), (B, Hq, 1))
    return dev_lists(idx, np.zeros((B, Hq), np.int32), idx, np.full((B, Hq), n, np.int32))


@pytest.mark.parametrize("alpha", [0.6, 0.9])
def test_sampled_row_selection_covers_what_it_accounts_for(oracle, alpha):
    cfg = inputs.scaled(inputs.CONFIGS["llama8b_8k"], n=2600, Hq=8, Hkv=2, heavy_lo=16, heavy_hi=48, span=128)
    q, k, v, _ = inputs.make_inputs(cfg)
    rng = np.random.default_rng(17)
    w = cfg.w
    rows = np.sort(rng.choice(cfg.n_hat, size=w, replace=False))          # sampled rows of the newest turn
    pos = (cfg.n - cfg.n_hat + rows).astype(np.int64)
    pipe = Pipeline(q, k, v, w, cfg.dtype)
    q_win = pipe.q[:, :, torch.from_numpy(rows).cuda()].contiguous()
    print(f"sampled rows: score at {w} random positions, alpha={alpha}", flush=True)
    sc_dev = pipe.score(q_pos=pos, q_win=q_win)
    sc = host(sc_dev)
    ref = oracle.score(q[:, :, rows], k, q_pos=pos)
    for name in ("vert", "slash", "vmax", "smax"):
        np.testing.assert_allclose(sc[name], ref[name], rtol=1e-3, atol=1e-6 * w, err_msg=name)
    sel_dev = pipe.select(sc_dev, alpha, accounted=True)
    sel = host(sel_dev)
    _, lse_sel = pipe.prefill(sel_dev)
    _, lse_all = pipe.prefill(_dense_lists(cfg.B, cfg.Hq, cfg.n))
    torch.cuda.synchronize()
    cov = metrics.coverage_from_lse(lse_sel.cpu().numpy(), lse_all.cpu().numpy())       # [B,Hq,n_hat]
    # the device's coverage equals the oracle's on the same index sets
    flat = (np.arange(cfg.B * cfg.Hq)[:, None] * cfg.n_hat + rows[None, :]).reshape(-1)
    _, o_sel = oracle.attend(q, k, v, sel["v_idx"], sel["v_cnt"], sel["s_idx"], sel["s_cnt"], rows=flat, mode=1)
    idx = np.tile(np.arange(cfg.n, dtype=np.int32), (cfg.B, cfg.Hq, 1))
    _, o_all = oracle.attend(q, k, v, idx, np.zeros((cfg.B, cfg.Hq), np.int32), idx, np.full((cfg.B, cfg.Hq), cfg.n, np.int32),
                             rows=flat, mode=1)
    cov_ref = metrics.coverage_from_lse(o_sel, o_all).reshape(cfg.B, cfg.Hq, w)
    np.testing.assert_allclose(cov[:, :, rows], cov_ref, rtol=0, atol=5e-3)
    # the walk's running sum is a lower bound of the mass the selection keeps on the scored rows, and it
    # reached alpha * total unless the lists ran out
    kept = cov[:, :, rows].sum(-1)
    acc, total = sel["accounted"], sc["total"]
    exhausted = (sel["v_cnt"] >= cfg.n) & (sel["s_cnt"] >= cfg.n)
    assert np.all(kept >= acc - 1e-2 * w), (kept, acc)
    assert np.all((acc >= alpha * total * (1 - 1e-6)) | exhausted)
    print(f"sampled rows: kept mass / total per head {np.round(kept / total, 3).ravel().tolist()}", flush=True)
