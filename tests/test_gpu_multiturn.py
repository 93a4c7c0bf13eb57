"""Across dialogue turns: the accumulated line set of Alg. 1 (ls_merge_lines), a two-turn flow in which the second
turn is prefilled over the union of both turns' selections, and the first turn of a dialogue (every row new) at the
length of the long-context workload."""
import numpy as np
import pytest
import torch

from paper_2507_13681_amd import binding, inputs, metrics

pytestmark = pytest.mark.gpu

from tests.gpu_util import Pipeline, dev_lists, host  # noqa: E402
from tests.test_gpu_configs import block_rows, check_attention, check_scores, check_selection, sample_rows  # noqa: E402


def _random_lists(rng, B, Hq, n, cap, max_cnt, sort=True):
    v_idx = np.zeros((B, Hq, cap), np.int32); v_cnt = np.zeros((B, Hq), np.int32)
    s_idx = np.zeros((B, Hq, cap), np.int32); s_cnt = np.zeros((B, Hq), np.int32)
    for b in range(B):
        for h in range(Hq):
            for idx, cnt in ((v_idx, v_cnt), (s_idx, s_cnt)):
                c = int(rng.integers(0, max_cnt + 1))
                x = rng.choice(n, size=c, replace=False)
                idx[b, h, :c] = np.sort(x) if sort else x
                cnt[b, h] = c
    return dict(v_idx=v_idx, v_cnt=v_cnt, s_idx=s_idx, s_cnt=s_cnt)


def _union(a, b, n):
    out = {}
    B, Hq = a["v_cnt"].shape
    for kind in ("v", "s"):
        out[kind] = [[np.union1d(a[kind + "_idx"][bb, h, :a[kind + "_cnt"][bb, h]], b[kind + "_idx"][bb, h, :b[kind + "_cnt"][bb, h]])
                      for h in range(Hq)] for bb in range(B)]
        out[kind] = [[u[(u >= 0) & (u < n)] for u in row] for row in out[kind]]
    return out


def test_merge_lines_is_the_set_union():
    rng = np.random.default_rng(8)
    B, Hq, n, cap = 2, 3, 5000, 600
    shape = binding.make_shape(B, Hq, Hq, 64, n, 100, 16, "bf16")
    ctx = binding.Context(shape)
    a = _random_lists(rng, B, Hq, n, cap, 500)
    b = _random_lists(rng, B, Hq, n, cap, 500, sort=False)          # inputs need not be sorted
    b["v_idx"][0, 0, :3] = a["v_idx"][0, 0, :3]                      # shared entries appear once
    want = _union(a, b, n)
    out = binding.alloc_select(shape, cap_v=1200, cap_s=1200, accounted=False)
    ctx.ls_merge_lines(shape, dev_lists(**a), dev_lists(**b), out)
    assert ctx.ls_poll_status() == 0
    got = host(out)
    for bb in range(B):
        for h in range(Hq):
            for kind in ("v", "s"):
                c = int(got[kind + "_cnt"][bb, h])
                np.testing.assert_array_equal(got[kind + "_idx"][bb, h, :c], want[kind][bb][h])
    # too small an output and entries beyond the context: counts say what was needed, the status word says why
    small = binding.alloc_select(shape, cap_v=50, cap_s=1200, accounted=False)
    b2 = {k: v.copy() for k, v in b.items()}
    b2["s_idx"][1, 2, 0] = n + 7
    ctx.ls_merge_lines(shape, dev_lists(**a), dev_lists(**b2), small)
    word = ctx.ls_poll_status()
    assert word == (binding.LS_STAT_V_TRUNCATED | binding.LS_STAT_MERGE_RANGE)
    got = host(small)
    want2 = _union(a, b2, n)
    for bb in range(B):
        for h in range(Hq):
            assert int(got["v_cnt"][bb, h]) == len(want2["v"][bb][h])
            np.testing.assert_array_equal(got["v_idx"][bb, h, :min(50, len(want2["v"][bb][h]))], want2["v"][bb][h][:50])
            np.testing.assert_array_equal(got["s_idx"][bb, h, :int(got["s_cnt"][bb, h])], want2["s"][bb][h])


def test_two_turn_flow_reuses_the_first_turns_lines(oracle):
    """Turn 1 (the first half of the context, every row new) and turn 2 are each scored and selected on the device; turn 2
    is then prefilled over the union of both selections.  Checked: the union against numpy, the attention output against
    the oracle on the union, and that carrying the earlier lines can only add to the attention mass each row keeps."""
    cfg = inputs.scaled(inputs.CONFIGS["llama8b_8k"], n=4096, Hq=8, Hkv=2, heavy_lo=16, heavy_hi=48, span=256)
    q, k, v, _ = inputs.make_inputs(cfg)                              # q holds the rows of turn 2
    n1 = cfg.n - cfg.n_hat
    cfg1 = inputs.scaled(cfg, n=n1, turns=1, name="turn1")            # turn 1 seen on its own: same keys, its own queries
    q1, _, _, _ = inputs.make_inputs(cfg1, seed=99)
    k1, v1 = np.ascontiguousarray(k[:, :, :n1]), np.ascontiguousarray(v[:, :, :n1])
    pipe1 = Pipeline(q1, k1, v1, cfg.w, cfg.dtype)
    sel1 = pipe1.select(pipe1.score(), cfg.alpha, accounted=False)
    pipe2 = Pipeline(q, k, v, cfg.w, cfg.dtype)
    sel2 = pipe2.select(pipe2.score(), cfg.alpha, accounted=False)
    both = binding.alloc_select(pipe2.shape, accounted=False)
    pipe2.ctx.ls_merge_lines(pipe2.shape, sel1, sel2, both)
    assert pipe2.ctx.ls_poll_status() == 0
    h1, h2, hb = host(sel1), host(sel2), host(both)
    want = _union(h1, h2, cfg.n)
    for h in range(cfg.Hq):
        for kind in ("v", "s"):
            np.testing.assert_array_equal(hb[kind + "_idx"][0, h, :int(hb[kind + "_cnt"][0, h])], want[kind][0][h])
    out_b, lse_b = pipe2.prefill(both, sentinel=True)
    out_2, lse_2 = pipe2.prefill(sel2)
    assert not bool(torch.isnan(out_b).any())
    rows = np.arange(0, cfg.B * cfg.Hq * cfg.n_hat, 5, dtype=np.int64)
    check_attention(oracle, cfg, q, k, v, hb, out_b, lse_b, rows, mode=1)
    assert bool((lse_b >= lse_2 - 1e-3).all())                         # more allowed cells, never less mass
    c2 = metrics.selection_cells(cfg.n, cfg.n_hat, h2).sum(); cb = metrics.selection_cells(cfg.n, cfg.n_hat, hb).sum()
    print(f"[two turns] cells turn-2 selection {c2}, with turn 1's lines carried {cb}", flush=True)
    assert cb >= c2


def test_first_turn_at_long_context_scale(oracle):
    """The first turn of a dialogue at the length of the long-context workload: n_hat = n = 131072, one KV group.  Every
    row block starts at the main diagonal, 1024 row blocks per head; line weights and selection against the oracle, the
    attention output on whole row blocks and scattered rows."""
    cfg = inputs.scaled(inputs.CONFIGS["stress_131k"], Hq=4, Hkv=1, turns=1, name="first_turn_131k")
    assert cfg.n_hat == cfg.n == 131072
    print("[first_turn_131k] generating inputs", flush=True)
    q, k, v, _ = inputs.make_inputs(cfg)
    pipe = Pipeline(q, k, v, cfg.w, cfg.dtype)
    sc_ref = oracle.score(q[:, :, -cfg.w:], k)
    sc_dev = pipe.score()
    check_scores(host(sc_dev), sc_ref, cfg.w)
    sel_ref = oracle.select(sc_ref, cfg.n_hat, cfg.alpha)
    sel_dev = pipe.select(sc_dev, cfg.alpha, accounted=False)
    sel = host(sel_dev)
    tol = check_selection(sel, sel_ref, sc_ref, cfg.alpha)
    print(f"[first_turn_131k] counts v {sel['v_cnt'].ravel().tolist()} s {sel['s_cnt'].ravel().tolist()}, tolerated {tol}", flush=True)
    out, lse = pipe.prefill(sel_dev, sentinel=True)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(out).any()) and not bool(torch.isnan(lse).any())
    rng = np.random.default_rng(3)
    rows = np.union1d(sample_rows(cfg, 16, rng), block_rows(cfg, sel, rng, random_blocks=4))
    print(f"[first_turn_131k] oracle attention on {len(rows)} rows", flush=True)
    check_attention(oracle, cfg, q, k, v, sel, out, lse, rows, mode=1)
