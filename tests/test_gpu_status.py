"""The device status word (ls_poll_status): one test per bit, each condition forced from the host.
Every kernel still runs to its normal end; nothing here hangs or faults on purpose."""
import numpy as np
import pytest
import torch

from paper_2507_13681_amd import binding, inputs

pytestmark = pytest.mark.gpu

from tests.gpu_util import Pipeline, dev_lists, dev_scores, host  # noqa: E402


def _small(oracle, n=3000, Hq=4, Hkv=2):
    cfg = inputs.scaled(inputs.CONFIGS["llama8b_8k"], n=n, Hq=Hq, Hkv=Hkv, heavy_lo=16, heavy_hi=48, span=128)
    q, k, v, _ = inputs.make_inputs(cfg)
    sc = oracle.score(q[:, :, -cfg.w:], k)
    return cfg, q, k, v, sc


def test_status_is_clear_after_a_clean_chain(oracle):
    cfg, q, k, v, sc = _small(oracle)
    pipe = Pipeline(q, k, v, cfg.w, cfg.dtype)
    sel = pipe.select(pipe.score(), cfg.alpha)
    pipe.prefill(sel)
    assert pipe.ctx.ls_poll_status() == 0


def test_truncated_lists_set_their_bits(oracle):
    cfg, q, k, v, sc = _small(oracle)
    ref = oracle.select(sc, cfg.n_hat, 0.95)
    pipe = Pipeline(q, k, v, cfg.w, cfg.dtype)
    # capacities below the longest list of each kind (whichever kinds the walk produced)
    need_v, need_s = int(ref["v_cnt"].max()), int(ref["s_cnt"].max())
    cap_v, cap_s = max(need_v // 2, 1), max(need_s // 2, 1)
    gpu = host(pipe.select(dev_scores(sc), 0.95, cap_v=cap_v, cap_s=cap_s))
    word = pipe.ctx.ls_poll_status()
    assert bool(word & binding.LS_STAT_V_TRUNCATED) == (need_v > cap_v)
    assert bool(word & binding.LS_STAT_S_TRUNCATED) == (need_s > cap_s)
    assert word & (binding.LS_STAT_V_TRUNCATED | binding.LS_STAT_S_TRUNCATED)
    np.testing.assert_array_equal(gpu["v_cnt"], ref["v_cnt"])          # counts still say what was needed
    np.testing.assert_array_equal(gpu["s_cnt"], ref["s_cnt"])
    assert pipe.ctx.ls_poll_status() == 0                              # polling clears the word
    pipe.select(dev_scores(sc), 0.95)                                  # full capacity: no bit
    assert pipe.ctx.ls_poll_status() == 0


def test_walk_wait_bound_reports_dense_and_sets_bit(oracle):
    """With the wait bound of the greedy-loop kernel set to zero a wave that has to wait gives up at once.
    Every wave still leaves the kernel; a head whose walk gave up reports every line selected (which keeps
    the coverage guarantee of Alg. 2), and the status word says so."""
    cfg, q, k, v, sc = _small(oracle, n=20000)
    ref = oracle.select(sc, cfg.n_hat, 0.95)
    pipe = Pipeline(q, k, v, cfg.w, cfg.dtype)
    pipe.ctx.debug_set_walk_spin_limit(0)
    gpu = host(pipe.select(dev_scores(sc), 0.95))
    word = pipe.ctx.ls_poll_status()
    gave_up = 0
    for h in range(cfg.Hq):
        cnts = (int(gpu["v_cnt"][0, h]), int(gpu["s_cnt"][0, h]))
        if cnts == (cfg.n, cfg.n) and (int(ref["v_cnt"][0, h]), int(ref["s_cnt"][0, h])) != cnts:
            gave_up += 1
            np.testing.assert_array_equal(gpu["v_idx"][0, h], np.arange(cfg.n))
            np.testing.assert_array_equal(gpu["s_idx"][0, h], np.arange(cfg.n))
        else:                                                          # a head that never had to wait
            assert cnts == (int(ref["v_cnt"][0, h]), int(ref["s_cnt"][0, h]))
    assert bool(word & binding.LS_STAT_WALK_TIMEOUT) == (gave_up > 0)
    assert gave_up > 0, "the walk of a 20000-line head stages several blocks and must wait at least once"
    pipe.ctx.debug_set_walk_spin_limit(-1)                             # default bound: the exact result, no bit
    gpu = host(pipe.select(dev_scores(sc), 0.95))
    assert pipe.ctx.ls_poll_status() == 0
    np.testing.assert_array_equal(gpu["v_cnt"], ref["v_cnt"])
    np.testing.assert_array_equal(gpu["s_cnt"], ref["s_cnt"])


def test_invalid_column_list_is_ignored_and_reported(oracle):
    """A caller's v_idx that is not strictly ascending (or leaves [0, n)): that head is computed from its
    diagonals alone and LS_STAT_V_INVALID is set; the other heads are untouched."""
    B, Hq, Hkv, n, n_hat, d = 1, 4, 2, 700, 300, 64
    q, k, v = inputs.make_plain(B, Hq, Hkv, n, n_hat, d, dtype="bf16", seed=5)
    rng = np.random.default_rng(2)
    cap = 64
    v_idx = np.zeros((B, Hq, cap), np.int32); v_cnt = np.zeros((B, Hq), np.int32)
    s_idx = np.zeros((B, Hq, cap), np.int32); s_cnt = np.zeros((B, Hq), np.int32)
    for h in range(Hq):
        cols = np.sort(rng.choice(n, 40, replace=False)); v_idx[0, h, :40] = cols; v_cnt[0, h] = 40
        dg = np.sort(rng.choice(n, 20, replace=False)); dg[0] = 0; s_idx[0, h, :20] = dg; s_cnt[0, h] = 20
    bad = v_idx.copy()
    bad[0, 1, [3, 4]] = bad[0, 1, [4, 3]]                              # head 1: two entries swapped
    bad[0, 2, 39] = n + 5                                              # head 2: a column beyond the context
    bad[0, 3, 7] = bad[0, 3, 6]                                        # head 3: a duplicate
    pipe = Pipeline(q, k, v, 16, "bf16")
    out, lse = pipe.prefill(dev_lists(bad, v_cnt, s_idx, s_cnt))
    word = pipe.ctx.ls_poll_status()
    assert word == binding.LS_STAT_V_INVALID
    none = np.zeros_like(v_cnt); none[0, 0] = v_cnt[0, 0]              # what the call must have computed
    want, want_lse = oracle.attend(q, k, v, v_idx, none, s_idx, s_cnt, mode=0)
    got = out.float().cpu().numpy().reshape(-1, d)
    assert np.abs(got - want).max() <= 2e-2
    out2, _ = pipe.prefill(dev_lists(v_idx, v_cnt, s_idx, s_cnt))       # the valid lists: no bit
    assert pipe.ctx.ls_poll_status() == 0
    want2, _ = oracle.attend(q, k, v, v_idx, v_cnt, s_idx, s_cnt, mode=0)
    assert np.abs(out2.float().cpu().numpy().reshape(-1, d) - want2).max() <= 2e-2


def test_out_of_range_diagonals_are_skipped_and_reported(oracle):
    B, Hq, Hkv, n, n_hat, d = 1, 2, 1, 500, 200, 64
    q, k, v = inputs.make_plain(B, Hq, Hkv, n, n_hat, d, dtype="bf16", seed=6)
    cap = 16
    v_idx = np.zeros((B, Hq, cap), np.int32); v_cnt = np.zeros((B, Hq), np.int32)
    s_idx = np.zeros((B, Hq, cap), np.int32); s_cnt = np.full((B, Hq), 5, np.int32)
    s_idx[0, :, :5] = [0, 1, 2, 40, 77]
    bad = s_idx.copy(); bad_cnt = s_cnt.copy()
    bad[0, 1, 5] = n + 3; bad[0, 1, 6] = -2; bad_cnt[0, 1] = 7          # head 1 carries two entries outside [0, n)
    pipe = Pipeline(q, k, v, 16, "bf16")
    out, _ = pipe.prefill(dev_lists(v_idx, v_cnt, bad, bad_cnt))
    assert pipe.ctx.ls_poll_status() == binding.LS_STAT_S_RANGE
    want, _ = oracle.attend(q, k, v, v_idx, v_cnt, s_idx, s_cnt, mode=0)
    assert np.abs(out.float().cpu().numpy().reshape(-1, d) - want).max() <= 2e-2
