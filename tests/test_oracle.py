"""Pins for the CPU oracle: each part is checked against something other than itself
(brute force in numpy float64 on tiny inputs, closed forms, invariants, library
routines, and the hand-worked walk examples under tests/golden/)."""
import math
import os

import numpy as np
import pytest
import torch

from paper_2507_13681_amd import inputs

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- O1

def _dense_window_probs(qw, k, q_pos, scale):
    """numpy float64 softmax of the window rows, causal; [w, n] (library routines only)."""
    s = (qw.astype(np.float64) @ k.astype(np.float64).T) * scale
    n = k.shape[0]
    mask = np.arange(n)[None, :] <= np.asarray(q_pos)[:, None]
    s = np.where(mask, s, -np.inf)
    return torch.softmax(torch.from_numpy(s), dim=-1).numpy()


def _line_sums_bruteforce(P, q_pos):
    w, n = P.shape
    vert = np.zeros(n); slash = np.zeros(n); vmax = np.zeros(n); smax = np.zeros(n)
    for t in range(w):
        for b in range(n):
            if b > q_pos[t]:
                continue
            o = q_pos[t] - b
            vert[b] += P[t, b]; vmax[b] = max(vmax[b], P[t, b])
            slash[o] += P[t, b]; smax[o] = max(smax[o], P[t, b])
    return vert, slash, vmax, smax


@pytest.mark.parametrize("B,Hq,Hkv,n,w,d,seed", [(1, 2, 1, 40, 5, 8, 0), (2, 4, 2, 33, 7, 16, 1), (1, 3, 3, 17, 17, 4, 2)])
def test_score_matches_bruteforce(oracle, B, Hq, Hkv, n, w, d, seed):
    q, k, _ = inputs.make_plain(B, Hq, Hkv, n, w, d, seed=seed, q_scale=2.0)
    sc = oracle.score(q, k)
    G = Hq // Hkv
    pos = np.arange(n - w, n)
    for b in range(B):
        for h in range(Hq):
            P = _dense_window_probs(q[b, h], k[b, h // G], pos, 1.0 / math.sqrt(d))
            v, s, vm, sm = _line_sums_bruteforce(P, pos)
            np.testing.assert_allclose(sc["vert"][b, h], v, rtol=1e-6, atol=1e-9)
            np.testing.assert_allclose(sc["slash"][b, h], s, rtol=1e-6, atol=1e-9)
            np.testing.assert_allclose(sc["vmax"][b, h], vm, rtol=1e-6, atol=1e-9)
            np.testing.assert_allclose(sc["smax"][b, h], sm, rtol=1e-6, atol=1e-9)
            assert abs(sc["total"][b, h] - w) < 1e-4


def test_score_explicit_positions(oracle):
    """Scattered scoring rows (the RandomSelect variant of Alg. 2): q_pos need not be the tail."""
    n, w, d = 50, 6, 8
    q, k, _ = inputs.make_plain(1, 1, 1, n, w, d, seed=3)
    pos = np.array([3, 10, 11, 30, 42, 49])
    sc = oracle.score(q, k, q_pos=pos)
    P = _dense_window_probs(q[0, 0], k[0, 0], pos, 1.0 / math.sqrt(d))
    v, s, vm, sm = _line_sums_bruteforce(P, pos)
    np.testing.assert_allclose(sc["vert"][0, 0], v, rtol=1e-6, atol=1e-9)
    np.testing.assert_allclose(sc["slash"][0, 0], s, rtol=1e-6, atol=1e-9)
    np.testing.assert_allclose(sc["smax"][0, 0], sm, rtol=1e-6, atol=1e-9)


def test_score_closed_form_equal_keys(oracle):
    """All keys equal => A[t][b] = 1/(p_t+1): line sums are differences of harmonic numbers."""
    n, w, d = 64, 8, 4
    q, _, _ = inputs.make_plain(1, 1, 1, n, w, d, seed=4)
    k = np.ones((1, 1, n, d), np.float32) * 0.37
    sc = oracle.score(q, k)
    pos = np.arange(n - w, n)
    for x in range(n):
        expect = sum(1.0 / (p + 1) for p in pos if p >= x)
        assert abs(sc["vert"][0, 0, x] - expect) < 1e-6
        assert abs(sc["slash"][0, 0, x] - expect) < 1e-6      # diagonal x also needs p_t >= x
        emax = max([1.0 / (p + 1) for p in pos if p >= x], default=0.0)
        assert abs(sc["vmax"][0, 0, x] - emax) < 1e-7
        assert abs(sc["smax"][0, 0, x] - emax) < 1e-7


def test_score_one_hot_counts(oracle):
    """Each row has one key with an overwhelming logit => line sums count rows (catches a
    transposed operand or a wrong diagonal index)."""
    n, w, d = 32, 6, 8
    rng = np.random.default_rng(5)
    k = np.zeros((1, 1, n, d), np.float32)
    k[0, 0, :, :] = np.eye(n, d, dtype=np.float32)[:, :]      # only keys 0..d-1 are non-zero
    pos = np.arange(n - w, n)
    tgt = np.array([0, 3, 3, 7, 1, 3])                        # key each row locks on
    q = np.zeros((1, 1, w, d), np.float32)
    for t in range(w):
        q[0, 0, t, tgt[t]] = 400.0                            # logit 400/sqrt(8) = 141
    sc = oracle.score(q, k)
    ev = np.zeros(n); es = np.zeros(n)
    for t in range(w):
        ev[tgt[t]] += 1; es[pos[t] - tgt[t]] += 1
    np.testing.assert_allclose(sc["vert"][0, 0], ev, atol=1e-6)
    np.testing.assert_allclose(sc["slash"][0, 0], es, atol=1e-6)
    np.testing.assert_allclose(sc["vmax"][0, 0], (ev > 0).astype(float), atol=1e-6)
    np.testing.assert_allclose(sc["smax"][0, 0], (es > 0).astype(float), atol=1e-6)


def test_score_invariants_on_workload(oracle):
    cfg = inputs.scaled(inputs.CONFIGS["tiny"], n=512, turns=4)
    q, k, _, _ = inputs.make_inputs(cfg)
    sc = oracle.score(q[:, :, -cfg.w:], k)
    for h in range(cfg.Hq):
        assert abs(sc["vert"][0, h].astype(np.float64).sum() - cfg.w) < 1e-3
        assert abs(sc["slash"][0, h].astype(np.float64).sum() - cfg.w) < 1e-3
        assert abs(sc["total"][0, h] - cfg.w) < 1e-3
        assert np.all(sc["vmax"][0, h] <= sc["vert"][0, h] + 1e-7)
        assert np.all(sc["smax"][0, h] <= sc["slash"][0, h] + 1e-7)
        assert np.all(sc["vert"][0, h] >= 0) and np.all(sc["slash"][0, h] >= 0)


def test_gqa_head_mapping(oracle):
    """Query head h must read KV head h // G."""
    q, k, _ = inputs.make_plain(1, 4, 2, 24, 4, 8, seed=6)
    sc = oracle.score(q, k)
    for h in range(4):
        one = oracle.score(q[:, h:h + 1], k[:, h // 2:h // 2 + 1])
        np.testing.assert_array_equal(sc["vert"][0, h], one["vert"][0, 0])


# ----------------------------------------------------------------------------- O2

def _read_examples():
    out = []
    with open(os.path.join(GOLD, "walk_examples.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            p = [x.strip() for x in line.split("|")]
            arr = lambda s: np.array([float(x) for x in s.split()], np.float32)
            out.append(dict(name=p[0], alpha=float(p[1]), total=float(p[2]), ws=arr(p[3]), ms=arr(p[4]),
                            wv=arr(p[5]), mv=arr(p[6]), ts=int(p[7]), tv=int(p[8]), acc=float(p[9])))
    return out


@pytest.mark.parametrize("ex", _read_examples(), ids=lambda e: e["name"])
def test_walk_worked_examples(oracle, ex):
    ls = np.full(len(ex["ws"]), 10, np.float32); lv = np.full(len(ex["wv"]), 10, np.float32)
    ts, tv, acc, _ = oracle.walk(ex["ws"], ex["ms"], ls, ex["wv"], ex["mv"], lv, ex["alpha"], ex["total"])
    assert (ts, tv) == (ex["ts"], ex["tv"])
    assert abs(acc - ex["acc"]) < 1e-6


def test_walk_cost_uses_line_length(oracle):
    """A short line wins against a heavier long one: 1/2 >= 3/10."""
    ts, tv, acc, _ = oracle.walk([1.0], [0.5], [2.0], [3.0], [1.0], [10.0], 0.2, 4.0)
    assert (ts, tv) == (1, 0) and acc == 1.0
    ts, tv, acc, _ = oracle.walk([1.0], [0.5], [4.0], [3.0], [1.0], [10.0], 0.2, 4.0)   # 1/4 < 3/10
    assert (ts, tv) == (0, 1) and acc == 3.0


def test_walk_cost_clamped_at_one(oracle):
    """l - #other can reach zero or below; the cost is then 1 (no division by <= 0)."""
    # after v0,v1 are taken the slash of length 2 has cost max(1, 2-2) = 1
    ts, tv, acc, _ = oracle.walk([0.5], [0.0], [2.0], [9.0, 8.0, 0.1], [0.0, 0.0, 0.0], [3.0, 3.0, 3.0], 0.99, 17.6)
    # picks: v0 (9/3 vs .5/2), v1 (8/3 vs .5/1... slash cost 2-1=1: .5 < 2.67), then slash .5/1 >= .1/(3-0) -> s0
    assert (ts, tv) == (1, 2) and abs(acc - 17.5) < 1e-6


def _true_window_coverage(P, pos, s_sel, v_sel):
    w, n = P.shape
    cov = 0.0
    sset, vset = set(int(x) for x in s_sel), set(int(x) for x in v_sel)
    for t in range(w):
        for b in range(pos[t] + 1):
            if b in vset or (pos[t] - b) in sset:
                cov += P[t, b]
    return cov


@pytest.mark.parametrize("alpha", [0.0, 0.3, 0.6, 0.9])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_select_invariants(oracle, alpha, seed):
    n, n_hat, w, d = 48, 20, 6, 8
    q, k, _ = inputs.make_plain(1, 1, 1, n, n_hat, d, seed=seed, q_scale=3.0)
    sc = oracle.score(q[:, :, -w:], k)
    sel = oracle.select(sc, n_hat, alpha)
    nv, ns = int(sel["v_cnt"][0, 0]), int(sel["s_cnt"][0, 0])
    v_sel, s_sel = sel["v_idx"][0, 0, :nv], sel["s_idx"][0, 0, :ns]
    assert np.all(np.diff(v_sel) > 0) and np.all(np.diff(s_sel) > 0)      # ascending, no repeats
    if alpha == 0.0:
        assert nv == 0 and ns == 0
        return
    # the selection is a prefix of each list in (weight desc, index asc) order
    for arr, picked in ((sc["vert"][0, 0], v_sel), (sc["slash"][0, 0], s_sel)):
        order = sorted(range(n), key=lambda i: (-arr[i], i))
        assert sorted(order[:len(picked)]) == list(picked)
    target = np.float32(alpha) * sc["total"][0, 0]
    exhausted = (nv == n and ns == n)
    if not exhausted:
        assert sel["accounted"][0, 0] >= target            # the loop's exit condition
        assert sel["before_last"][0, 0] < target            # ...and it was not met one pick earlier
    # the accounted sum is a lower bound of the mass the selection really covers on the scored rows
    pos = np.arange(n - w, n)
    P = _dense_window_probs(q[0, 0, -w:], k[0, 0], pos, 1.0 / math.sqrt(d))
    cov = _true_window_coverage(P, pos, s_sel, v_sel)
    assert cov >= sel["accounted"][0, 0] - 1e-4
    if not exhausted:
        assert cov >= alpha * w - 1e-3                       # Eq. 1's constraint on the scored rows


def test_select_matches_python_walk(oracle):
    """Independent re-implementation of Alg. 2 in numpy float32 scalars, whole pipeline."""
    n, n_hat, w, d = 64, 24, 8, 8
    q, k, _ = inputs.make_plain(1, 2, 1, n, n_hat, d, seed=11, q_scale=4.0)
    sc = oracle.score(q[:, :, -w:], k)
    for alpha in (0.5, 0.8, 0.95, 1.0):
        sel = oracle.select(sc, n_hat, alpha)
        for h in range(2):
            vert, slash = sc["vert"][0, h], sc["slash"][0, h]
            vm, sm = sc["vmax"][0, h], sc["smax"][0, h]
            S = sorted(range(n), key=lambda i: (-slash[i], i)); V = sorted(range(n), key=lambda i: (-vert[i], i))
            f = np.float32
            ol_s = ol_v = acc = f(0)
            tgt = f(alpha) * sc["total"][0, h]
            Ss, Vs = [], []
            while acc < tgt and (S or V):
                if not V:
                    pick = "s"
                elif not S:
                    pick = "v"
                else:
                    ds, dv = slash[S[0]] - ol_v, vert[V[0]] - ol_s
                    cs = max(f(1), f(min(n_hat, n - S[0])) - f(len(Vs)))
                    cv = max(f(1), f(min(n_hat, n - V[0])) - f(len(Ss)))
                    pick = "s" if f(ds * cv) >= f(dv * cs) else "v"
                if pick == "s":
                    s = S.pop(0); acc = f(acc + f(slash[s] - ol_v)); ol_s = f(ol_s + sm[s]); Ss.append(s)
                else:
                    v = V.pop(0); acc = f(acc + f(vert[v] - ol_s)); ol_v = f(ol_v + vm[v]); Vs.append(v)
            assert sorted(Ss) == list(sel["s_idx"][0, h, :sel["s_cnt"][0, h]])
            assert sorted(Vs) == list(sel["v_idx"][0, h, :sel["v_cnt"][0, h]])
            assert acc == sel["accounted"][0, h]


def test_select_alpha_one_small_covers_everything_reachable(oracle):
    """alpha = 1: the accounted bound reaches the total only through lines of one kind (no
    overlap penalty) or by exhausting both lists; either way the scored rows are covered up
    to binary32 rounding of the running sum."""
    n, n_hat, w, d = 32, 12, 4, 8
    q, k, _ = inputs.make_plain(1, 1, 1, n, n_hat, d, seed=12)
    sc = oracle.score(q[:, :, -w:], k)
    sel = oracle.select(sc, n_hat, 1.0)
    nv, ns = int(sel["v_cnt"][0, 0]), int(sel["s_cnt"][0, 0])
    pos = np.arange(n - w, n)
    P = _dense_window_probs(q[0, 0, -w:], k[0, 0], pos, 1.0 / math.sqrt(d))
    cov = _true_window_coverage(P, pos, sel["s_idx"][0, 0, :ns], sel["v_idx"][0, 0, :nv])
    assert cov >= w * (1 - 1e-6)


def test_select_capacity_clamp(oracle):
    n, n_hat, w, d = 32, 12, 4, 8
    q, k, _ = inputs.make_plain(1, 1, 1, n, n_hat, d, seed=12)
    sc = oracle.score(q[:, :, -w:], k)
    full = oracle.select(sc, n_hat, 1.0)
    assert full["s_cnt"][0, 0] > 7
    small = oracle.select(sc, n_hat, 1.0, cap_v=5, cap_s=7)
    assert small["v_cnt"][0, 0] == full["v_cnt"][0, 0]                   # needed counts are reported
    assert small["s_cnt"][0, 0] == full["s_cnt"][0, 0]
    np.testing.assert_array_equal(small["s_idx"][0, 0], full["s_idx"][0, 0, :7])


# ----------------------------------------------------------------------------- O3

def _sdpa(q, k, v, mask):
    """torch CPU scaled_dot_product_attention in float64 with a boolean mask [n_hat, n]."""
    tq = torch.from_numpy(q.astype(np.float64))[None, None]
    tk = torch.from_numpy(k.astype(np.float64))[None, None]
    tv = torch.from_numpy(v.astype(np.float64))[None, None]
    return torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=torch.from_numpy(mask))[0, 0].numpy()


def _lists(B, Hq, n, v_sets, s_sets):
    v_idx = np.full((B, Hq, n), -1, np.int32); s_idx = np.full((B, Hq, n), -1, np.int32)
    v_cnt = np.zeros((B, Hq), np.int32); s_cnt = np.zeros((B, Hq), np.int32)
    for b in range(B):
        for h in range(Hq):
            vs, ss = sorted(v_sets[b][h]), sorted(s_sets[b][h])
            v_idx[b, h, :len(vs)] = vs; v_cnt[b, h] = len(vs)
            s_idx[b, h, :len(ss)] = ss; s_cnt[b, h] = len(ss)
    return v_idx, v_cnt, s_idx, s_cnt


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("pattern", ["all_slashes", "all_columns", "window", "sink_window", "mixed"])
def test_attend_matches_sdpa(oracle, mode, pattern):
    B, Hq, Hkv, n, n_hat, d = 1, 2, 1, 40, 13, 8
    q, k, v = inputs.make_plain(B, Hq, Hkv, n, n_hat, d, seed=20)
    pos = np.arange(n - n_hat, n)
    causal = np.arange(n)[None, :] <= pos[:, None]
    off = pos[:, None] - np.arange(n)[None, :]
    if pattern == "all_slashes":          # every diagonal => dense causal attention
        vs, ss, mask = [], list(range(n)), causal
    elif pattern == "all_columns":        # every column => dense causal attention
        vs, ss, mask = list(range(n)), [], causal
    elif pattern == "window":             # diagonals 0..W-1 => sliding-window attention
        W = 5; vs, ss = [], list(range(W)); mask = causal & (off < W)
    elif pattern == "sink_window":        # + columns 0..3 => sink + window
        W = 5; vs, ss = [0, 1, 2, 3], list(range(W))
        mask = causal & ((off < W) | (np.arange(n)[None, :] < 4))
    else:                                 # crossing lines: each crossing cell counted once
        vs, ss = [2, 9, 30, 35], [0, 3, 4, 17, 31]
        mask = causal & (np.isin(off, ss) | np.isin(np.arange(n), vs)[None, :])
    v_idx, v_cnt, s_idx, s_cnt = _lists(B, Hq, n, [[vs] * Hq], [[ss] * Hq])
    out, lse = oracle.attend(q, k, v, v_idx, v_cnt, s_idx, s_cnt, mode=mode)
    out = out.reshape(B, Hq, n_hat, d)
    for h in range(Hq):
        ref = _sdpa(q[0, h], k[0, 0], v[0, 0], mask)
        np.testing.assert_allclose(out[0, h], ref, rtol=1e-5, atol=1e-6)
        s = (q[0, h].astype(np.float64) @ k[0, 0].astype(np.float64).T) / math.sqrt(d)
        ref_lse = torch.logsumexp(torch.from_numpy(np.where(mask, s, -np.inf)), dim=-1).numpy()
        np.testing.assert_allclose(lse.reshape(B, Hq, n_hat)[0, h], ref_lse, rtol=1e-5, atol=1e-6)


def test_attend_modes_agree_and_rows_subset(oracle):
    cfg = inputs.scaled(inputs.CONFIGS["tiny"], n=256, turns=4)
    q, k, v, _ = inputs.make_inputs(cfg)
    sc = oracle.score(q[:, :, -cfg.w:], k)
    sel = oracle.select(sc, cfg.n_hat, 0.9)
    a0, l0 = oracle.attend(q, k, v, sel["v_idx"], sel["v_cnt"], sel["s_idx"], sel["s_cnt"], mode=0)
    a1, l1 = oracle.attend(q, k, v, sel["v_idx"], sel["v_cnt"], sel["s_idx"], sel["s_cnt"], mode=1)
    np.testing.assert_allclose(a0, a1, rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(l0, l1, rtol=1e-5, atol=1e-6)
    rows = np.array([0, 5, cfg.n_hat + 3, 3 * cfg.n_hat + cfg.n_hat - 1])
    sub, _ = oracle.attend(q, k, v, sel["v_idx"], sel["v_cnt"], sel["s_idx"], sel["s_cnt"], rows=rows, mode=1)
    np.testing.assert_array_equal(sub, a1[rows])


def test_attend_empty_row_is_zero(oracle):
    """A row with no allowed cell gives zeros and lse = -inf (column 30 is invisible to early rows)."""
    B, Hq, n, n_hat, d = 1, 1, 40, 13, 8
    q, k, v = inputs.make_plain(B, Hq, 1, n, n_hat, d, seed=21)
    v_idx, v_cnt, s_idx, s_cnt = _lists(B, Hq, n, [[[30]]], [[[]]])
    for mode in (0, 1):
        out, lse = oracle.attend(q, k, v, v_idx, v_cnt, s_idx, s_cnt, mode=mode)
        assert np.all(out[:3] == 0) and np.all(np.isneginf(lse[:3]))      # rows at positions 27..29
        np.testing.assert_allclose(out[3:], np.broadcast_to(v[0, 0, 30], (n_hat - 3, d)), rtol=1e-6)


def test_alpha_one_reproduces_dense_causal(oracle):
    """Coverage 1.0 end to end (score -> select -> attend) equals dense causal attention."""
    B, Hq, Hkv, n, n_hat, d, w = 1, 2, 1, 48, 16, 8, 4
    q, k, v = inputs.make_plain(B, Hq, Hkv, n, n_hat, d, seed=22)
    sel = oracle.select(oracle.score(q[:, :, -w:], k), n_hat, 1.0)
    out, _ = oracle.attend(q, k, v, sel["v_idx"], sel["v_cnt"], sel["s_idx"], sel["s_cnt"], mode=0)
    pos = np.arange(n - n_hat, n)
    causal = np.arange(n)[None, :] <= pos[:, None]
    for h in range(Hq):
        np.testing.assert_allclose(out.reshape(B, Hq, n_hat, d)[0, h], _sdpa(q[0, h], k[0, 0], v[0, 0], causal),
                                   rtol=1e-5, atol=1e-6)


# ----------------------------------------------------------------------------- O4

def test_compress_matches_topk(oracle):
    B, Hq, Hkv, ln, n_obs, d, budget = 2, 4, 2, 60, 5, 8, 12
    q, k, _ = inputs.make_plain(B, Hq, Hkv, ln, n_obs, d, seed=30, q_scale=2.0)
    res = oracle.compress(q, k, budget)
    pos = np.arange(ln - n_obs, ln)
    for b in range(B):
        for j in range(Hkv):
            s = np.zeros(ln)
            for g in range(2):
                s += _dense_window_probs(q[b, 2 * j + g], k[b, j], pos, 1.0 / math.sqrt(d)).sum(0)
            np.testing.assert_allclose(res["score"][b, j], s, rtol=1e-6, atol=1e-9)
            top = torch.topk(torch.from_numpy(res["score"][b, j]), budget).indices.numpy()
            assert sorted(top) == list(res["keep_idx"][b, j])
            assert res["keep_cnt"][b, j] == budget


def test_compress_budget_ge_len_keeps_all(oracle):
    q, k, _ = inputs.make_plain(1, 2, 1, 20, 4, 8, seed=31)
    res = oracle.compress(q, k, 32)
    assert res["keep_cnt"][0, 0] == 20
    np.testing.assert_array_equal(res["keep_idx"][0, 0, :20], np.arange(20))


def test_topb_ties_prefer_small_index(oracle):
    s = np.array([1, 5, 5, 5, 0, 5], np.float32)
    np.testing.assert_array_equal(oracle.topb(s, 3), [1, 2, 3])
    np.testing.assert_array_equal(oracle.topb(s, 5), [0, 1, 2, 3, 5])


# ----------------------------------------------------------------------------- O5 decode step

def _decode_case(B=2, Hq=4, Hkv=2, cap=37, T=5, d=16, seed=5):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, Hq, d)).astype(np.float32)
    kc = rng.standard_normal((B, Hkv, cap, d)).astype(np.float32); vc = rng.standard_normal((B, Hkv, cap, d)).astype(np.float32)
    kt = rng.standard_normal((B, Hkv, T, d)).astype(np.float32); vt = rng.standard_normal((B, Hkv, T, d)).astype(np.float32)
    cnt = rng.integers(1, cap + 1, (B, Hkv)).astype(np.int32)
    return q, kc, vc, cnt, kt, vt


def test_decode_matches_sdpa(oracle):
    """Library routine: SDPA over the valid retained rows followed by the tail rows, per query head."""
    q, kc, vc, cnt, kt, vt = _decode_case()
    B, Hq, d = q.shape; Hkv = kc.shape[1]; G = Hq // Hkv
    # rows beyond cnt must never be read
    kc2, vc2 = kc.copy(), vc.copy()
    for b in range(B):
        for g in range(Hkv):
            kc2[b, g, cnt[b, g]:] = np.nan; vc2[b, g, cnt[b, g]:] = np.nan
    out, lse = oracle.decode(q, kc2, vc2, cnt, kt, vt)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            K = np.concatenate([kc[b, g, :cnt[b, g]], kt[b, g]]); V = np.concatenate([vc[b, g, :cnt[b, g]], vt[b, g]])
            ref = _sdpa(q[b, h][None], K, V, np.ones((1, len(K)), bool))[0]
            np.testing.assert_allclose(out[b, h], ref, rtol=1e-5, atol=1e-6)
            s = (K.astype(np.float64) @ q[b, h].astype(np.float64)) / math.sqrt(d)
            np.testing.assert_allclose(lse[b, h], torch.logsumexp(torch.from_numpy(s), 0).item(), rtol=1e-5, atol=1e-6)


def test_decode_equals_last_row_of_dense_prefill(oracle):
    """Cross-pin with lso_attend: with the whole cache retained, the step is the last row of dense causal attention."""
    B, Hq, Hkv, n, d = 1, 4, 2, 50, 8
    q, k, v = inputs.make_plain(B, Hq, Hkv, n, 1, d, seed=9)
    all_idx = np.tile(np.arange(n, dtype=np.int32), (B, Hq, 1)); full = np.full((B, Hq), n, np.int32); none = np.zeros((B, Hq), np.int32)
    ref, ref_lse = oracle.attend(q, k, v, all_idx, none, all_idx, full, mode=0)
    out, lse = oracle.decode(q[:, :, 0], k, v)
    np.testing.assert_allclose(out.reshape(-1, d), ref, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(lse.reshape(-1), ref_lse, rtol=1e-6, atol=1e-7)


def test_decode_closed_forms(oracle):
    B, Hq, Hkv, cap, T, d = 1, 2, 1, 9, 3, 4
    rng = np.random.default_rng(0)
    q = rng.standard_normal((B, Hq, d)).astype(np.float32)
    vc = rng.standard_normal((B, Hkv, cap, d)).astype(np.float32); vt = rng.standard_normal((B, Hkv, T, d)).astype(np.float32)
    # equal keys: uniform weights, out = mean of all values, lse = logit + log(L)
    key = rng.standard_normal(d).astype(np.float32)
    kc = np.tile(key, (B, Hkv, cap, 1)); kt = np.tile(key, (B, Hkv, T, 1))
    out, lse = oracle.decode(q, kc, vc, None, kt, vt)
    mean = np.concatenate([vc[0, 0], vt[0, 0]]).astype(np.float64).mean(0)
    for h in range(Hq):
        np.testing.assert_allclose(out[0, h], mean, rtol=1e-6, atol=1e-7)
        logit = float(q[0, h].astype(np.float64) @ key.astype(np.float64)) / math.sqrt(d)
        np.testing.assert_allclose(lse[0, h], logit + math.log(cap + T), rtol=1e-6)
    # one tail key far ahead of the rest: the output is its value row
    kc = np.zeros((B, Hkv, cap, d), np.float32); kt = np.zeros((B, Hkv, T, d), np.float32)
    qq = np.ones((B, Hq, d), np.float32); kt[0, 0, 1] = 50.0
    out, _ = oracle.decode(qq, kc, vc, None, kt, vt)
    np.testing.assert_allclose(out[0, 0], vt[0, 0, 1], rtol=1e-6, atol=1e-6)
    # a custom scale is applied to the logits
    out_s, lse_s = oracle.decode(q, kc, vc, None, kt, vt, scale=0.0001)
    np.testing.assert_allclose(out_s[0, 0], np.concatenate([vc[0, 0], vt[0, 0]]).mean(0), rtol=0, atol=2e-3)


def test_decode_split_between_retained_and_tail_is_irrelevant(oracle):
    """Only the order of the rows matters, not which buffer holds them."""
    q, kc, vc, _, kt, vt = _decode_case(cap=20, T=6)
    B, Hkv = kc.shape[:2]
    full_k = np.concatenate([kc, kt], 2); full_v = np.concatenate([vc, vt], 2)
    ref, ref_lse = oracle.decode(q, full_k, full_v)
    out, lse = oracle.decode(q, kc, vc, None, kt, vt)
    np.testing.assert_array_equal(out, ref); np.testing.assert_array_equal(lse, ref_lse)
    cnt = np.full((B, Hkv), 11, np.int32)
    out2, lse2 = oracle.decode(q, full_k, full_v, cnt, full_k[:, :, 11:], full_v[:, :, 11:])
    np.testing.assert_array_equal(out2, ref); np.testing.assert_array_equal(lse2, ref_lse)


def test_decode_no_key_is_zero(oracle):
    q, kc, vc, _, _, _ = _decode_case(T=0)
    cnt = np.zeros(kc.shape[:2], np.int32)
    out, lse = oracle.decode(q, kc, vc, cnt)
    assert np.all(out == 0) and np.all(np.isneginf(lse))


# ----------------------------------------------------------------------------- inputs

def test_inputs_are_seeded_and_storage_exact():
    cfg = inputs.scaled(inputs.CONFIGS["llama8b_8k"], n=512, Hq=4, Hkv=2, heavy_lo=8, heavy_hi=8, span=32)
    a = inputs.make_inputs(cfg)
    b = inputs.make_inputs(cfg)
    for x, y in zip(a[:3], b[:3]):
        np.testing.assert_array_equal(x, y)
        assert np.all((x.view(np.uint32) & 0xFFFF) == 0)        # exactly representable in bf16
    assert a[0].shape == (1, 4, cfg.n_hat, 128) and a[1].shape == (1, 2, 512, 128)
    t = torch.from_numpy(a[1]).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(t, a[1])


def test_config_shapes_match_benchmark_definition():
    c = inputs.CONFIGS
    assert (c["tiny"].n, c["tiny"].n_hat, c["tiny"].w) == (1024, 256, 32)
    assert (c["llama8b_8k"].n, c["llama8b_8k"].n_hat) == (8192, 4096)
    assert (c["multiturn_32k"].n, c["multiturn_32k"].n_hat) == (32768, 10923)
    assert (c["stress_131k"].n, c["stress_131k"].n_hat, c["stress_131k"].w) == (131072, 16384, 128)
    assert (c["llama70b_16k_b4"].B, c["llama70b_16k_b4"].n_hat, c["llama70b_16k_b4"].Hq) == (4, 5462, 64)
    assert c["multiturn_32k"].causal_cells_per_head() == 298274361


# ------------------------------------------------------------------ exact-overlap variant of Alg. 2

def _line_sums_of(a_win, pos):
    """vert / slash / total of window matrices a_win [B,Hq,w,n] (float64 sums -> float32)."""
    B, Hq, w, n = a_win.shape
    vert = a_win.astype(np.float64).sum(2)
    slash = np.zeros((B, Hq, n))
    for t in range(w):
        for j in range(int(pos[t]) + 1):
            slash[:, :, int(pos[t]) - j] += a_win[:, :, t, j]
    return dict(vert=vert.astype(np.float32), slash=slash.astype(np.float32),
                total=vert.sum(-1).astype(np.float32))


def test_window_matrix_matches_bruteforce_and_line_sums(oracle):
    B, Hq, Hkv, n, w, d = 1, 4, 2, 50, 7, 8
    q, k, _ = inputs.make_plain(B, Hq, Hkv, n, w, d, seed=3, q_scale=3.0)
    for pos in (None, np.array([3, 10, 11, 20, 33, 48, 49])):
        a = oracle.window(q, k, q_pos=pos)
        p = np.arange(n - w, n) if pos is None else pos
        for h in range(Hq):
            P = _dense_window_probs(q[0, h], k[0, h // (Hq // Hkv)], p, 1.0 / np.sqrt(d))
            np.testing.assert_allclose(a[0, h], P, rtol=2e-6, atol=1e-12)
        np.testing.assert_allclose(a.sum(-1), 1.0, rtol=1e-6)
        sc = oracle.score(q, k, q_pos=pos)                      # the two oracle functions describe one matrix
        ls = _line_sums_of(a, p)
        np.testing.assert_allclose(ls["vert"], sc["vert"], rtol=1e-5, atol=1e-7)
        np.testing.assert_allclose(ls["slash"], sc["slash"], rtol=1e-5, atol=1e-7)


def test_exact_walk_worked_example(oracle):
    rows, kv = [], {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "walk_exact_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        if key == "row":
            rows.append([float(x) for x in vals])
        else:
            kv[key] = [float(x) for x in vals]
    n, w, n_hat = int(kv["n"][0]), int(kv["w"][0]), int(kv["n_hat"][0])
    a = np.array(rows, np.float32).reshape(1, 1, w, n)
    sc = _line_sums_of(a, np.arange(n - w, n))
    sel = oracle.select_exact(a, sc, n_hat, kv["alpha"][0])
    assert list(sel["s_idx"][0, 0, :sel["s_cnt"][0, 0]]) == [int(x) for x in kv["expect_s"]]
    assert list(sel["v_idx"][0, 0, :sel["v_cnt"][0, 0]]) == [int(x) for x in kv["expect_v"]]
    assert sel["accounted"][0, 0] == np.float32(kv["expect_accounted"][0])
    assert sel["before_last"][0, 0] == np.float32(kv["expect_before_last"][0])


def _exact_walk_bruteforce(a, pos, vert, slash, total, n_hat, alpha):
    """Alg. 2's loop where the gain of a line is, by definition, the weight of its cells that no selected line covers yet:
    a boolean `covered` matrix is kept and re-read for every candidate (no overlap bookkeeping at all)."""
    w, n = a.shape
    f = np.float32
    S = sorted(range(n), key=lambda i: (-slash[i], i)); V = sorted(range(n), key=lambda i: (-vert[i], i))
    covered = np.zeros((w, n), bool)
    cells_s = lambda o: [(t, int(pos[t]) - o) for t in range(w) if int(pos[t]) - o >= 0]
    cells_v = lambda b: [(t, b) for t in range(w) if b <= int(pos[t])]
    gain = lambda cells, wt: f(wt - f(sum(float(a[t, c]) for t, c in cells if covered[t, c])))
    acc = f(0); tgt = f(alpha) * total
    Ss, Vs = [], []
    while acc < tgt and (S or V):
        if not V:
            pick = "s"
        elif not S:
            pick = "v"
        else:
            ds, dv = gain(cells_s(S[0]), slash[S[0]]), gain(cells_v(V[0]), vert[V[0]])
            cs = max(f(1), f(min(n_hat, n - S[0])) - f(len(Vs))); cv = max(f(1), f(min(n_hat, n - V[0])) - f(len(Ss)))
            pick = "s" if f(ds * cv) >= f(dv * cs) else "v"
        if pick == "s":
            s = S.pop(0); acc = f(acc + gain(cells_s(s), slash[s])); Ss.append(s)
            for t, c in cells_s(s): covered[t, c] = True
        else:
            v = V.pop(0); acc = f(acc + gain(cells_v(v), vert[v])); Vs.append(v)
            for t, c in cells_v(v): covered[t, c] = True
    return sorted(Ss), sorted(Vs), acc, float(a.astype(np.float64)[covered].sum())


@pytest.mark.parametrize("seed,pos_kind", [(1, "last"), (2, "last"), (3, "random")])
def test_exact_walk_matches_bruteforce_union_coverage(oracle, seed, pos_kind):
    """Sets and sum against the covered-matrix loop; the sum is the true weight of the union (up to binary32 rounding of the
    running sum), gains are never negative, the walk stops at the first pick that reaches the target."""
    n, n_hat, w, d = 72, 30, 9, 8
    q, k, _ = inputs.make_plain(1, 2, 1, n, w, d, seed=seed, q_scale=4.0)
    pos = np.arange(n - w, n) if pos_kind == "last" else np.sort(np.random.default_rng(seed).choice(np.arange(n - n_hat, n), w, replace=False))
    qp = None if pos_kind == "last" else pos
    a = oracle.window(q, k, q_pos=qp)
    sc = oracle.score(q, k, q_pos=qp)
    for alpha in (0.3, 0.8, 0.95, 1.0):
        sel = oracle.select_exact(a, sc, n_hat, alpha, q_pos=qp)
        for h in range(2):
            Ss, Vs, acc, cov = _exact_walk_bruteforce(a[0, h], pos, sc["vert"][0, h], sc["slash"][0, h], sc["total"][0, h], n_hat, alpha)
            assert Ss == list(sel["s_idx"][0, h, :sel["s_cnt"][0, h]])
            assert Vs == list(sel["v_idx"][0, h, :sel["v_cnt"][0, h]])
            assert acc == sel["accounted"][0, h]
            np.testing.assert_allclose(sel["accounted"][0, h], cov, rtol=2e-5)
            tgt = np.float32(alpha) * sc["total"][0, h]
            exhausted = sel["s_cnt"][0, h] == n and sel["v_cnt"][0, h] == n
            assert sel["before_last"][0, h] < tgt
            assert exhausted or sel["accounted"][0, h] >= tgt
            assert sel["before_last"][0, h] <= sel["accounted"][0, h]          # no pick ever lowers the sum


def test_exact_walk_keeps_mixed_selections_where_the_bound_gives_up(oracle):
    """On a structured workload the listing's bound drives some heads to take every line; with exact overlaps the same heads
    stop at a mixed selection whose accounted weight reaches the target."""
    cfg = inputs.scaled(inputs.CONFIGS["llama8b_8k"], n=1536, Hq=8, Hkv=2, heavy_lo=16, heavy_hi=48, span=128)
    q, k, _, _ = inputs.make_inputs(cfg)
    qw = q[:, :, -cfg.w:]
    sc = oracle.score(qw, k)
    a = oracle.window(qw, k)
    bound = oracle.select(sc, cfg.n_hat, 0.95)
    exact = oracle.select_exact(a, sc, cfg.n_hat, 0.95)
    tgt = np.float32(0.95) * sc["total"]
    assert np.all(exact["accounted"] >= tgt)
    assert np.all((exact["s_cnt"] < cfg.n) | (exact["v_cnt"] < cfg.n))          # nobody takes everything
    both = (exact["s_cnt"] > 0) & (exact["v_cnt"] > 0)
    print("exact: mixed heads", int(both.sum()), "bound: exhausted heads", int(((bound["s_cnt"] == cfg.n) & (bound["v_cnt"] == cfg.n)).sum()))
    assert both.any()
