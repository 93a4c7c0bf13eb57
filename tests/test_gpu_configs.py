"""End-to-end parity on the five benchmark workloads, at their full sizes and in the launch
configuration bench.py times: score -> select -> sparse prefill (-> KV retention for the decode
workload) through the C ABI, against the CPU oracle.

  * line weights: every entry compared (rel 1e-3, abs 1e-6 * w);
  * ls_select fed the ORACLE's weights: sets and counts must equal the oracle's exactly, at full n;
  * ls_select on the device's own weights: sets must equal the oracle's, except
      (order) lines whose weight lies within 1e-3 (relative) of the lightest weight the oracle
              selected from that list, or
      (stop)  a walk that ends one pick earlier or up to two picks later than the oracle's because
              the running sum sits at the target: the differing lines must be exactly the oracle's
              last pick, or the next lines of that list in the oracle's order, and the oracle's
              running sum at the device's stopping point must be within 1e-3 (relative) of
              alpha * total;
  * attention outputs: `out` and `lse` are pre-filled with NaN and every row must have been written;
    compared against the oracle evaluated on the device's own index sets -- every row for the tiny,
    8k and 32k workloads, whole 128-row blocks (first, last and eight random ones of heads of each
    kind) plus scattered rows of every head for the 131k and batch-4 workloads: max-abs <= 2e-2,
    mean-abs <= 5e-3 for bf16, 1e-4 for fp32.
"""
import numpy as np
import pytest
import torch

from paper_2507_13681_amd import inputs, metrics

pytestmark = pytest.mark.gpu

from tests.gpu_util import Pipeline, dev_scores, host  # noqa: E402


def check_scores(gpu, ref, w):
    for name in ("vert", "slash", "vmax", "smax"):
        np.testing.assert_allclose(gpu[name], ref[name], rtol=1e-3, atol=1e-6 * w, err_msg=name)
    np.testing.assert_allclose(gpu["total"], ref["total"], rtol=1e-5)


def check_selection_exact(gpu, ref):
    np.testing.assert_array_equal(gpu["v_cnt"], ref["v_cnt"])
    np.testing.assert_array_equal(gpu["s_cnt"], ref["s_cnt"])
    B, Hq = ref["v_cnt"].shape
    for b in range(B):
        for h in range(Hq):
            for idx, cnt in (("v_idx", "v_cnt"), ("s_idx", "s_cnt")):
                c = int(ref[cnt][b, h])
                np.testing.assert_array_equal(gpu[idx][b, h, :c], ref[idx][b, h, :c], err_msg=f"{idx} b={b} h={h}")


def check_selection(gpu, ref, sc_ref, alpha, tol=1e-3):
    """Sets equal up to lines at the selection threshold (see the module docstring).
    Returns (lines tolerated by the order rule, lines tolerated by the stop rule)."""
    B, Hq = ref["v_cnt"].shape
    tol_order = tol_stop = 0
    for b in range(B):
        for h in range(Hq):
            diffs = {}
            for idx, cnt, wname in (("v_idx", "v_cnt", "vert"), ("s_idx", "s_cnt", "slash")):
                g = gpu[idx][b, h, :int(gpu[cnt][b, h])]
                r = ref[idx][b, h, :int(ref[cnt][b, h])]
                if len(g) == len(r) and np.array_equal(g, r):
                    continue
                diffs[wname] = (g, r, np.setxor1d(g, r))
            if not diffs:
                continue
            # (order) every differing line weighs within tol of the lightest line the oracle took from its list
            order_ok = True
            for wname, (g, r, diff) in diffs.items():
                wts = sc_ref[wname][b, h]
                thr = wts[r].min() if len(r) else wts.max()
                order_ok = order_ok and bool(np.all(np.abs(wts[diff] - thr) <= tol * max(thr, 1e-30)))
            if order_ok:
                tol_order += sum(len(d[2]) for d in diffs.values())
                continue
            # (stop) one pick fewer or up to two picks more than the oracle, with the sum at the target
            target = float(np.float32(alpha) * sc_ref["total"][b, h])
            n_diff = sum(len(d[2]) for d in diffs.values())
            msg = f"b={b} h={h}: " + ", ".join(f"{w}: gpu {len(g)} / oracle {len(r)} lines, {len(d)} differ" for w, (g, r, d) in diffs.items())
            assert n_diff <= 2, msg + " (not at the threshold, and more than two lines)"
            earlier = all(len(g) < len(r) for g, r, _ in diffs.values())
            later = all(len(g) > len(r) for g, r, _ in diffs.values())
            assert earlier or later, msg
            for wname, (g, r, diff) in diffs.items():
                wts = sc_ref[wname][b, h]
                order = np.lexsort((np.arange(len(wts)), -wts.astype(np.float64)))     # descending weight, then index
                if earlier:                                  # the oracle's last pick(s) of this list are missing
                    np.testing.assert_array_equal(np.sort(order[len(g):len(r)]), diff, err_msg=msg)
                else:                                        # the next lines of this list were taken as well
                    np.testing.assert_array_equal(np.sort(order[len(r):len(g)]), diff, err_msg=msg)
                np.testing.assert_array_equal(np.sort(order[:min(len(g), len(r))]), np.sort(np.intersect1d(g, r)), err_msg=msg)
            if earlier:
                assert n_diff == 1, msg + " (only the sum before the oracle's last pick is known)"
                at_stop = float(ref["before_last"][b, h])    # the oracle's running sum where the device stopped
            else:
                at_stop = float(ref["accounted"][b, h])      # the oracle stopped here; the device went on
            assert abs(at_stop - target) <= tol * target, msg + f" (sum {at_stop!r} vs target {target!r})"
            tol_stop += n_diff
    return tol_order, tol_stop


def sample_rows(cfg, per_head, rng):
    """Flat row ids: the first, last and block-boundary rows of each head plus random ones."""
    rows = []
    nh = cfg.n_hat
    first_block = 128 - (cfg.n - nh) % 128            # rows up to the first 128-aligned position
    fixed = [0, 1, nh - 1, nh - 2, min(first_block, nh - 1), min(first_block + 1, nh - 1), nh // 2]
    for bh in range(cfg.B * cfg.Hq):
        pick = set(x for x in fixed if 0 <= x < nh)
        pick.update(int(x) for x in rng.integers(0, nh, size=per_head))
        rows.extend(bh * nh + a for a in sorted(pick))
    return np.array(rows, np.int64)


def check_attention(oracle, cfg, q, k, v, sel_gpu, out_gpu, lse_gpu, rows, mode=1):
    ref_out, ref_lse = oracle.attend(q, k, v, sel_gpu["v_idx"], sel_gpu["v_cnt"], sel_gpu["s_idx"], sel_gpu["s_cnt"],
                                     rows=rows, mode=mode)
    got = out_gpu.reshape(-1, cfg.d)[torch.from_numpy(rows).to(out_gpu.device)].float().cpu().numpy()
    err = np.abs(got - ref_out)
    if cfg.dtype == "bf16":
        assert err.max() <= 2e-2, err.max()
        assert err.mean() <= 5e-3, err.mean()
    else:
        assert err.max() <= 1e-4, err.max()
    lse = lse_gpu.reshape(-1)[torch.from_numpy(rows).to(lse_gpu.device)].cpu().numpy()
    fin = np.isfinite(ref_lse)
    np.testing.assert_array_equal(np.isfinite(lse), fin)
    np.testing.assert_allclose(lse[fin], ref_lse[fin], rtol=0, atol=2e-3 if cfg.dtype == "bf16" else 1e-4)
    return float(err.max()), float(err.mean())


def block_rows(cfg, sel, rng, heads_per_kind=2, random_blocks=8):
    """Flat row ids of whole 128-row blocks (aligned to absolute positions that are multiples of 128, the
    attention kernel's work items): the first, the last and `random_blocks` random ones, for up to
    `heads_per_kind` heads of each kind of selection (everything / diagonals only / columns only / mixed)."""
    nh, hist = cfg.n_hat, cfg.n - cfg.n_hat
    pos0 = hist // 128 * 128
    nqb = (cfg.n - pos0 + 127) // 128
    nv, ns = sel["v_cnt"].reshape(-1), sel["s_cnt"].reshape(-1)
    kinds = {"all": (nv >= cfg.n) & (ns >= cfg.n), "slash": (nv == 0) & (ns > 0), "vert": (ns == 0) & (nv > 0)}
    kinds["mixed"] = (nv > 0) & (ns > 0) & ~kinds["all"]
    rows = []
    for kind, m in kinds.items():
        heads = np.flatnonzero(m)
        if len(heads) == 0:
            continue
        heavy = heads[np.argmax((nv + ns)[heads])]
        pick = {int(heavy)} | set(int(x) for x in rng.choice(heads, size=min(heads_per_kind - 1, len(heads)), replace=False))
        for bh in sorted(pick):
            qbs = {0, nqb - 1} | set(int(x) for x in rng.integers(0, nqb, size=random_blocks))
            for qb in sorted(qbs):
                a0, a1 = max(pos0 + 128 * qb - hist, 0), min(pos0 + 128 * qb + 128 - hist, nh)
                rows.extend(bh * nh + a for a in range(a0, a1))
    return np.array(sorted(set(rows)), np.int64)


def check_queues(pipe):
    """The work queues of the attention kernel hold every (head, 128-row block) item exactly once."""
    queues, nqb = pipe.ctx.debug_prefill_queues(pipe.shape)
    items = np.concatenate(queues).astype(np.int64)
    BH = pipe.shape.B * pipe.shape.Hq
    expect = (np.arange(BH, dtype=np.int64)[:, None] << 16 | np.arange(nqb, dtype=np.int64)[None, :]).ravel()
    np.testing.assert_array_equal(np.sort(items), np.sort(expect))


def run_prefill_config(oracle, name, alphas=None, per_head=6, all_rows=False, dense_mode=False):
    cfg = inputs.CONFIGS[name]
    print(f"[{name}] generating inputs", flush=True)
    q, k, v, _ = inputs.make_inputs(cfg)
    pipe = Pipeline(q, k, v, cfg.w, cfg.dtype)
    print(f"[{name}] oracle score", flush=True)
    sc_ref = oracle.score(q[:, :, -cfg.w:], k)
    sc_gpu_dev = pipe.score()
    sc_gpu = host(sc_gpu_dev)
    check_scores(sc_gpu, sc_ref, cfg.w)
    sc_ref_dev = dev_scores(sc_ref)
    rng = np.random.default_rng(cfg.seed)
    for alpha in (alphas or [cfg.alpha]):
        print(f"[{name}] alpha={alpha}: select", flush=True)
        sel_ref = oracle.select(sc_ref, cfg.n_hat, alpha)
        # the oracle's weights in, the oracle's sets out: exact (the full-length sort, merge and walk)
        check_selection_exact(host(pipe.select(sc_ref_dev, alpha, accounted=False)), sel_ref)
        sel_dev = pipe.select(sc_gpu_dev, alpha, accounted=False)
        sel_gpu = host(sel_dev)
        tol_order, tol_stop = check_selection(sel_gpu, sel_ref, sc_ref, alpha)
        cells = metrics.selection_cells(cfg.n, cfg.n_hat, sel_gpu)
        dens = cells.sum() / (cfg.B * cfg.Hq * metrics.causal_cells(cfg.n, cfg.n_hat))
        print(f"[{name}] alpha={alpha}: density {dens:.4f}, lines tolerated at the threshold: {tol_order} by weight, "
              f"{tol_stop} by the stop rule", flush=True)
        out, lse = pipe.prefill(sel_dev, sentinel=True)
        check_queues(pipe)
        torch.cuda.synchronize()
        assert pipe.ctx.ls_poll_status() == 0
        # every row written by some work item: no sentinel left (an empty row is zeros / -inf, never NaN)
        assert not bool(torch.isnan(out).any()), "rows of `out` were never written"
        assert not bool(torch.isnan(lse).any()), "rows of `lse` were never written"
        if all_rows:
            rr = np.arange(cfg.B * cfg.Hq * cfg.n_hat, dtype=np.int64)
        else:
            rr = np.union1d(sample_rows(cfg, per_head, rng), block_rows(cfg, sel_gpu, rng))
        print(f"[{name}] alpha={alpha}: oracle attention on {len(rr)} rows", flush=True)
        mx, mean = check_attention(oracle, cfg, q, k, v, sel_gpu, out, lse, rr, mode=0 if dense_mode else 1)
        print(f"[{name}] alpha={alpha}: attention max-abs {mx:.2e} mean-abs {mean:.2e} on {len(rr)} rows", flush=True)
    return cfg, q, k, v, pipe


def test_config1_tiny(oracle):
    run_prefill_config(oracle, "tiny", all_rows=True, dense_mode=True)


def test_config2_llama8b_8k(oracle):
    run_prefill_config(oracle, "llama8b_8k", all_rows=True)


def test_config3_multiturn_32k(oracle):
    """Every row of every head against the oracle: more than 1024 (head, row block) items, so the persistent
    workgroups take several items each, steal across queues and walk key-block lists longer than 256 entries."""
    run_prefill_config(oracle, "multiturn_32k", all_rows=True)


def test_config4_stress_131k(oracle):
    run_prefill_config(oracle, "stress_131k", alphas=[0.90, 0.95, 0.98], per_head=2)


def test_config5_llama70b_decode_compress(oracle):
    """Batch-4 prefill, then 256 decode steps with the cache re-scored every 16 generated tokens
    from the last 16 query vectors (first re-selection after 16 tokens, Sec. 5.2), 2048 kept per KV head."""
    cfg, q, k, v, pipe = run_prefill_config(oracle, "llama70b_16k_b4", per_head=1)
    steps, n_d, budget = 256, 16, 2048
    dq, dk, dv = inputs.make_decode_step(cfg, steps)
    from tests.gpu_util import to_dev
    from paper_2507_13681_amd import binding
    cap = cfg.n + steps
    Kc = torch.empty((cfg.B, cfg.Hkv, cap, cfg.d), dtype=torch.bfloat16, device="cuda")
    Vc = torch.empty_like(Kc)
    Kc[:, :, :cfg.n] = pipe.k; Vc[:, :, :cfg.n] = pipe.v
    Kc[:, :, cfg.n:] = to_dev(dk, "bf16"); Vc[:, :, cfg.n:] = to_dev(dv, "bf16")
    dqd = to_dev(dq, "bf16")
    kfull = np.concatenate([k, dk], axis=2)
    del pipe
    ctx = binding.Context(binding.make_shape(cfg.B, cfg.Hq, cfg.Hkv, cfg.d, cap, 1, n_d, "bf16"), budget)
    keep_idx = torch.empty((cfg.B, cfg.Hkv, budget), dtype=torch.int32, device="cuda")
    keep_cnt = torch.empty((cfg.B, cfg.Hkv), dtype=torch.int32, device="cuda")
    checked = 0
    for call in range(1, steps // n_d + 1):
        ln = cfg.n + n_d * call                      # cache length after 16*call generated tokens
        shape = binding.make_shape(cfg.B, cfg.Hq, cfg.Hkv, cfg.d, ln, 1, n_d, "bf16")
        k_now = Kc[:, :, :ln].contiguous()
        q_obs = dqd[:, :, n_d * (call - 1):n_d * call].contiguous()
        ctx.ls_kv_compress(shape, budget, q_obs, k_now, None, keep_idx, keep_cnt)
        if True:                                     # the oracle is run on every one of the 16 calls
            print(f"[llama70b_16k_b4] compress call {call}, cache length {ln}", flush=True)
            score = torch.empty((cfg.B, cfg.Hkv, ln), dtype=torch.float32, device="cuda")
            ctx.debug_compress_score(shape, score)
            score = score.cpu().numpy()
            ref = oracle.compress(dq[:, :, n_d * (call - 1):n_d * call], kfull[:, :, :ln], budget)
            np.testing.assert_allclose(score, ref["score"], rtol=1e-3, atol=1e-6 * n_d)
            ki = keep_idx.cpu().numpy()
            assert np.all(keep_cnt.cpu().numpy() == budget)
            for b in range(cfg.B):
                for j in range(cfg.Hkv):
                    got = ki[b, j]
                    np.testing.assert_array_equal(got, oracle.topb(score[b, j], budget))
                    diff = np.setxor1d(got, ref["keep_idx"][b, j])
                    if len(diff):
                        thr = np.sort(ref["score"][b, j])[::-1][budget - 1]
                        assert np.all(np.abs(ref["score"][b, j][diff] - thr) <= 1e-3 * thr)
            checked += 1
    assert checked == steps // n_d


def test_maximum_context_length(oracle):
    """n = LS_MAX_N (262144): 32 sort segments, the largest diagonal bitmap and activity table, a short newest turn
    so that the oracle stays quick.  Structured inputs (sinks, heavy columns, a local band) as in the workloads."""
    cfg = inputs.scaled(inputs.CONFIGS["llama8b_8k"], n=262144, Hq=2, Hkv=1, turns=256, name="max_n")
    assert cfg.n_hat == 1024
    print(f"[max_n] generating inputs n={cfg.n} n_hat={cfg.n_hat}", flush=True)
    q, k, v, _ = inputs.make_inputs(cfg)
    pipe = Pipeline(q, k, v, cfg.w, cfg.dtype)
    sc_ref = oracle.score(q[:, :, -cfg.w:], k)
    sc_dev = pipe.score()
    check_scores(host(sc_dev), sc_ref, cfg.w)
    for alpha in (0.9, 0.999):
        sel_ref = oracle.select(sc_ref, cfg.n_hat, alpha)
        sel_dev = pipe.select(sc_dev, alpha, accounted=False)
        sel_gpu = host(sel_dev)
        check_selection_exact(host(pipe.select(dev_scores(sc_ref), alpha, accounted=False)), sel_ref)
        tolerated = check_selection(sel_gpu, sel_ref, sc_ref, alpha)
        print(f"[max_n] alpha={alpha}: counts v {sel_gpu['v_cnt'].ravel().tolist()} s {sel_gpu['s_cnt'].ravel().tolist()}, tolerated {tolerated}", flush=True)
        out, lse = pipe.prefill(sel_dev, sentinel=True)
        check_queues(pipe)
        torch.cuda.synchronize()
        assert not bool(torch.isnan(out).any()) and not bool(torch.isnan(lse).any())
        rng = np.random.default_rng(1)
        rows = np.union1d(sample_rows(cfg, 12, rng), block_rows(cfg, sel_gpu, rng, random_blocks=2))
        check_attention(oracle, cfg, q, k, v, sel_gpu, out, lse, rows, mode=1)


def test_first_turn_prefill(oracle):
    """The first turn of a dialogue: every row is new (n_hat = n), so the causal triangle starts at row 0."""
    cfg = inputs.scaled(inputs.CONFIGS["llama8b_8k"], n=1800, Hq=4, Hkv=2, turns=1, heavy_lo=8, heavy_hi=24, span=128, name="first_turn")
    assert cfg.n_hat == cfg.n
    q, k, v, _ = inputs.make_inputs(cfg)
    pipe = Pipeline(q, k, v, cfg.w, cfg.dtype)
    sc_ref = oracle.score(q[:, :, -cfg.w:], k)
    sc_dev = pipe.score()
    check_scores(host(sc_dev), sc_ref, cfg.w)
    sel_ref = oracle.select(sc_ref, cfg.n_hat, 0.9)
    sel_dev = pipe.select(sc_dev, 0.9, accounted=False)
    sel_gpu = host(sel_dev)
    check_selection(sel_gpu, sel_ref, sc_ref, 0.9)
    print("[first_turn] prefill of all rows", flush=True)
    out, lse = pipe.prefill(sel_dev, sentinel=True)
    check_queues(pipe)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(out).any()) and not bool(torch.isnan(lse).any())
    rows = np.arange(cfg.B * cfg.Hq * cfg.n_hat, dtype=np.int64)
    check_attention(oracle, cfg, q, k, v, sel_gpu, out, lse, rows, mode=1)
