"""ls_score_window / ls_select_exact (Alg. 2 with the overlap of a candidate counted cell by cell) against the
oracle: the window matrix entry by entry; the selection bit-exact when fed the oracle's matrix and weights; end to
end on device-side inputs up to lines at the threshold; the accounted sum against the true weight of the union,
measured independently through two ls_sparse_prefill calls on the scored rows."""
import numpy as np
import pytest
import torch

from paper_2507_13681_amd import binding, inputs

pytestmark = pytest.mark.gpu

from tests.gpu_util import Pipeline, dev_scores, host  # noqa: E402
from tests.test_gpu_configs import check_selection_exact  # noqa: E402


def _select_exact(pipe, a_win, sc, alpha, q_pos=None, cap_v=None, cap_s=None):
    out = binding.alloc_select(pipe.shape, cap_v, cap_s, accounted=True)
    qp = None if q_pos is None else torch.from_numpy(np.asarray(q_pos, np.int64)).cuda()
    pipe.ctx.ls_select_exact(pipe.shape, alpha, a_win, sc["vert"], sc["slash"], sc["total"],
                             out["v_idx"], out["v_cnt"], out["s_idx"], out["s_cnt"], out["accounted"], qp)
    return out


def _window(pipe, q_pos=None):
    s = pipe.shape
    a = torch.full((s.B, s.Hq, s.w, s.n), float("nan"), dtype=torch.float32, device="cuda")
    qp = None if q_pos is None else torch.from_numpy(np.asarray(q_pos, np.int64)).cuda()
    assert q_pos is None
    pipe.ctx.ls_score_window(s, pipe.q[:, :, -s.w:].contiguous(), pipe.k, a, qp)
    return a


@pytest.mark.parametrize("n,w,Hq,Hkv,d,dtype", [(1000, 64, 4, 2, 128, "bf16"), (700, 20, 2, 1, 64, "bf16"),
                                                (300, 100, 2, 2, 128, "f32"), (2500, 256, 2, 1, 128, "bf16")])
def test_window_matrix_matches_oracle(oracle, n, w, Hq, Hkv, d, dtype):
    q, k, v = inputs.make_plain(1, Hq, Hkv, n, w, d, dtype=dtype, seed=n + w, q_scale=2.0)
    print(f"window n={n} w={w} Hq={Hq} Hkv={Hkv} d={d} {dtype}", flush=True)
    pipe = Pipeline(q, k, v, w, dtype)
    a = _window(pipe).cpu().numpy()
    ref = oracle.window(q, k)
    np.testing.assert_allclose(a, ref, rtol=1e-3, atol=1e-7)
    assert np.all(a[ref == 0] == 0)                        # exact zeros beyond each row's position, nothing left unwritten


@pytest.mark.parametrize("alpha,n,w", [(0.5, 3000, 64), (0.9, 3000, 64), (0.95, 3000, 64), (1.0, 2048, 64), (0.95, 5000, 200), (0.9, 1500, 16)])
def test_select_exact_bit_exact_on_oracle_inputs(oracle, alpha, n, w):
    cfg = inputs.scaled(inputs.CONFIGS["llama8b_8k"], n=n, w=w, Hq=8, Hkv=2, heavy_lo=16, heavy_hi=48, span=128)
    q, k, v, _ = inputs.make_inputs(cfg)
    qw = q[:, :, -w:]
    sc = oracle.score(qw, k)
    a = oracle.window(qw, k)
    ref = oracle.select_exact(a, sc, cfg.n_hat, alpha)
    print(f"exact select alpha={alpha} n={n} w={w}: oracle counts v {ref['v_cnt'].ravel().tolist()} s {ref['s_cnt'].ravel().tolist()}", flush=True)
    pipe = Pipeline(q, k, v, w, cfg.dtype)
    gpu = host(_select_exact(pipe, torch.from_numpy(a).cuda(), dev_scores(sc), alpha))
    assert pipe.ctx.ls_poll_status() == 0
    check_selection_exact(gpu, ref)
    np.testing.assert_array_equal(gpu["accounted"], ref["accounted"])


def test_select_exact_explicit_positions_and_capacity(oracle):
    n, w = 2000, 48
    cfg = inputs.scaled(inputs.CONFIGS["llama8b_8k"], n=n, w=w, Hq=4, Hkv=2, heavy_lo=16, heavy_hi=32, span=128)
    q, k, v, _ = inputs.make_inputs(cfg)
    pos = np.sort(np.random.default_rng(5).choice(np.arange(n - cfg.n_hat, n), w, replace=False))
    qw = q[:, :, pos - (n - cfg.n_hat)]
    sc = oracle.score(qw, k, q_pos=pos)
    a = oracle.window(qw, k, q_pos=pos)
    ref = oracle.select_exact(a, sc, cfg.n_hat, 0.9, q_pos=pos, cap_v=40, cap_s=50)
    pipe = Pipeline(q, k, v, w, cfg.dtype)
    gpu = host(_select_exact(pipe, torch.from_numpy(a).cuda(), dev_scores(sc), 0.9, q_pos=pos, cap_v=40, cap_s=50))
    np.testing.assert_array_equal(gpu["v_cnt"], ref["v_cnt"])
    np.testing.assert_array_equal(gpu["s_cnt"], ref["s_cnt"])
    for h in range(cfg.Hq):
        nv, ns = min(40, int(ref["v_cnt"][0, h])), min(50, int(ref["s_cnt"][0, h]))
        np.testing.assert_array_equal(gpu["v_idx"][0, h, :nv], ref["v_idx"][0, h, :nv])
        np.testing.assert_array_equal(gpu["s_idx"][0, h, :ns], ref["s_idx"][0, h, :ns])
    np.testing.assert_array_equal(gpu["accounted"], ref["accounted"])


def test_exact_chain_end_to_end(oracle):
    """score -> window -> exact select -> sparse prefill on the device.  With both kinds of line competing, the loop's
    outcome depends on near-ties between the two list heads, so inputs that differ in the last bits (the device's window
    matrix against the oracle's) may lead to different, equally valid selections; what is unique is the result for given
    inputs.  The device's selection is therefore compared, exactly, with the oracle run on the device's own window
    matrix and weights; and the accounted sum with the true weight of the selected union on the scored rows, obtained
    from the device by another route: the softmax denominators of the scored rows with the selection and with every cell."""
    cfg = inputs.scaled(inputs.CONFIGS["llama8b_8k"], n=4096, Hq=8, Hkv=2, heavy_lo=16, heavy_hi=48, span=256)
    q, k, v, _ = inputs.make_inputs(cfg)
    pipe = Pipeline(q, k, v, cfg.w, cfg.dtype)
    sc_dev = pipe.score()
    a_dev = _window(pipe)
    sel_dev = _select_exact(pipe, a_dev, sc_dev, 0.95)
    sel = host(sel_dev)
    qw = q[:, :, -cfg.w:]
    np.testing.assert_allclose(a_dev.cpu().numpy(), oracle.window(qw, k), rtol=1e-3, atol=1e-7)
    ref = oracle.select_exact(a_dev.cpu().numpy(), host(sc_dev), cfg.n_hat, 0.95)
    check_selection_exact(sel, ref)
    np.testing.assert_array_equal(sel["accounted"], ref["accounted"])
    mixed = int(((sel["v_cnt"] > 0) & (sel["s_cnt"] > 0)).sum())
    print(f"[exact chain] counts v {sel['v_cnt'].ravel().tolist()} s {sel['s_cnt'].ravel().tolist()}, mixed heads {mixed}", flush=True)
    assert mixed > 0
    assert np.all(sel["accounted"] >= np.float32(0.95) * host(sc_dev)["total"])
    out, lse = pipe.prefill(sel_dev, sentinel=True)
    full = dict(sel_dev)
    full["s_idx"] = torch.arange(cfg.n, dtype=torch.int32, device="cuda").repeat(cfg.B, cfg.Hq, 1).contiguous()
    full["s_cnt"] = torch.full_like(sel_dev["s_cnt"], cfg.n); full["v_cnt"] = torch.zeros_like(sel_dev["v_cnt"])
    _, lse_all = pipe.prefill(full)
    kept = torch.exp(lse[:, :, -cfg.w:] - lse_all[:, :, -cfg.w:]).sum(-1).cpu().numpy()      # true weight of the union per head
    np.testing.assert_allclose(sel["accounted"], kept, rtol=5e-3)
    rows = np.arange(0, cfg.B * cfg.Hq * cfg.n_hat, 7, dtype=np.int64)
    want, _ = oracle.attend(q, k, v, sel["v_idx"], sel["v_cnt"], sel["s_idx"], sel["s_cnt"], rows=rows, mode=1)
    got = out.reshape(-1, cfg.d)[torch.from_numpy(rows).cuda()].float().cpu().numpy()
    err = np.abs(got - want)
    assert err.max() <= 2e-2 and err.mean() <= 5e-3
