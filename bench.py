"""Benchmark of the LoopServe hot path on one MI355X.

One step = one pass of the whole path for one attention layer on one synthetic batch:
    ls_score -> ls_select -> ls_sparse_prefill   (online-sparsified prefill of the newest turn)
    + one ls_kv_compress call                    (decode-time re-scoring of the same cache; second stream)
with every input already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload multiturn_32k] [--no-cpu]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_FP32_MFMA_TFLOPS = 157.3


def per_row_cells(n, n_hat, rows_a, v_sel, s_sel):
    """Allowed cells of each sampled row a (position p = n - n_hat + a) for one head."""
    col = np.zeros(n, bool); col[v_sel] = True
    vs = np.sort(v_sel); ss = np.sort(s_sel)
    out = []
    for a in rows_a:
        p = n - n_hat + a
        nv = np.searchsorted(vs, p, side="right")
        s_ok = ss[:np.searchsorted(ss, p, side="right")]
        out.append(int(nv + len(s_ok) - col[p - s_ok].sum()))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="multiturn_32k")
    ap.add_argument("--alpha", type=float, default=None)
    ap.add_argument("--budget", type=int, default=2048)
    ap.add_argument("--n-obs", type=int, default=16)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--compress-gather", action="store_true",
                    help="ls_kv_compress also writes the compacted K / V copies of the kept rows (adds its row-gather kernel to the step)")
    ap.add_argument("--exact-overlap", action="store_true",
                    help="select with ls_score_window + ls_select_exact (overlaps counted cell by cell) instead of ls_select; "
                         "not the headline configuration")
    ap.add_argument("--first-turn", action="store_true",
                    help="every position of the context is a new row (n_hat = n): the first turn of a dialogue; not the "
                         "headline configuration")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per launch of the dominant kernel, measured by rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of "
                         "this same command (see profiles/); counters cannot be read inside a timed run, so roofline.traffic is "
                         "null unless this is given")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MIB",
                    help="only run a plain device copy of MIB MiB (10 launches): calibrates the rocprofv3 FETCH_SIZE / "
                         "WRITE_SIZE counters against a kernel of known traffic")
    ap.add_argument("--decode-probe", action="store_true",
                    help="only time ls_decode_attend (the decode step over a compressed cache) and print its own JSON line")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the path shards by KV-head group with no "
              "exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2507_13681_amd import binding, inputs, metrics

    if args.copy_probe:
        x = torch.empty(args.copy_probe << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        y = torch.empty_like(x)
        for _ in range(10):
            y.copy_(x)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": x.numel(), "copy_probe_bytes_written": x.numel(), "launches": 10}))
        return

    if args.decode_probe:
        # the decode step of Alg. 3 over a compressed cache (ls_decode_attend), at the decode shape of the
        # llama70b_16k_b4 workload: budget retained rows + 16 tokens since the retention.  HBM-bound.
        c5 = inputs.CONFIGS["llama70b_16k_b4"]
        B, Hq, Hkv, d, cap, T = c5.B, c5.Hq, c5.Hkv, c5.d, args.budget, 16
        g = torch.Generator(device="cuda").manual_seed(1234)
        mk = lambda *sh: torch.randn(*sh, device="cuda", generator=g).to(torch.bfloat16)
        q, kc, vc, kt, vt = mk(B, Hq, d), mk(B, Hkv, cap, d), mk(B, Hkv, cap, d), mk(B, Hkv, T, d), mk(B, Hkv, T, d)
        cnt = torch.full((B, Hkv), cap, dtype=torch.int32, device="cuda")
        dshape = binding.make_shape(B, Hq, Hkv, d, cap + T, 1, 1, "bf16")
        dctx = binding.Context(workspace=binding.decode_workspace_bytes(dshape, cap, T))
        out = torch.empty_like(q)
        f = lambda: dctx.ls_decode_attend(dshape, q, kc, vc, cnt, kt, vt, out, None)
        for _ in range(args.warmup):
            f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            f()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        nbytes = 2 * B * Hkv * (cap + T) * d * 2 + 2 * B * Hq * d * 2
        print(json.dumps({"metric": "decode step over the compressed cache, algorithmic bytes per second", "value": round(nbytes / (ms * 1e-3) / 1e9, 2),
                          "unit": "GB/s", "ms_per_call": round(ms, 5), "steps": args.steps, "warmup": args.warmup, "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": "llama70b_16k_b4 decode", "B": B, "Hq": Hq, "Hkv": Hkv, "d": d, "retained": cap, "since": T},
                          "roofline": {"kernel": "decode_partial_kernel", "bound": "hbm", "achieved": round(nbytes / (ms * 1e-3) / 1e9, 2), "peak": 8000.0,
                                       "unit": "GB/s", "frac": round(nbytes / (ms * 1e-3) / 8e12, 4), "bytes": nbytes,
                                       "note": "per call (two kernels), launch gaps included"}}))
        return

    cfg = inputs.CONFIGS[args.workload]
    if args.first_turn:
        cfg = inputs.scaled(cfg, n_hat=cfg.n)
    alpha = cfg.alpha if args.alpha is None else args.alpha
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    q, k, v, _ = inputs.make_inputs(cfg)
    dev = lambda x: torch.from_numpy(x).cuda().to(tdt)
    qd, kd, vd = dev(q), dev(k), dev(v)
    qwin = qd[:, :, -cfg.w:].contiguous()
    qobs = qd[:, :, -args.n_obs:].contiguous()
    shape = binding.make_shape(cfg.B, cfg.Hq, cfg.Hkv, cfg.d, cfg.n, cfg.n_hat, cfg.w, cfg.dtype)
    cshape = binding.make_shape(cfg.B, cfg.Hq, cfg.Hkv, cfg.d, cfg.n, 1, args.n_obs, cfg.dtype)
    ctx = binding.Context(workspace=binding.workspace_bytes(shape))
    # ls_kv_compress does not depend on the prefill chain (it re-scores the same cache for the decode phase), so it
    # runs beside it on a second stream with a context (workspace) of its own: it fills the CUs that the
    # selection kernels, a few workgroups wide, leave idle.
    cctx = binding.Context(workspace=binding.workspace_bytes(cshape, args.budget))
    side = torch.cuda.Stream()
    sc = binding.alloc_score(shape)
    sel = binding.alloc_select(shape, accounted=False)
    out = torch.empty_like(qd)
    lse = torch.empty(qd.shape[:3], dtype=torch.float32, device="cuda")
    keep_idx = torch.empty((cfg.B, cfg.Hkv, args.budget), dtype=torch.int32, device="cuda")
    keep_cnt = torch.empty((cfg.B, cfg.Hkv), dtype=torch.int32, device="cuda")

    def f_score():
        ctx.ls_score(shape, qwin, kd, sc["vert"], sc["slash"], sc["vmax"], sc["smax"], sc["total"])

    a_win = torch.empty((cfg.B, cfg.Hq, cfg.w, cfg.n), dtype=torch.float32, device="cuda") if args.exact_overlap else None

    def f_select():
        if args.exact_overlap:
            ctx.ls_score_window(shape, qwin, kd, a_win)
            ctx.ls_select_exact(shape, alpha, a_win, sc["vert"], sc["slash"], sc["total"],
                                sel["v_idx"], sel["v_cnt"], sel["s_idx"], sel["s_cnt"], None)
            return
        ctx.ls_select(shape, alpha, sc["vert"], sc["slash"], sc["vmax"], sc["smax"], sc["total"],
                      sel["v_idx"], sel["v_cnt"], sel["s_idx"], sel["s_cnt"], None)

    def f_prefill():
        ctx.ls_sparse_prefill(shape, qd, kd, vd, sel["v_idx"], sel["v_cnt"], sel["s_idx"], sel["s_cnt"], out, lse)

    k_keep = v_keep = None
    if args.compress_gather:
        k_keep = torch.empty((cfg.B, cfg.Hkv, args.budget, cfg.d), dtype=tdt, device="cuda")
        v_keep = torch.empty_like(k_keep)

    def f_compress():
        cctx.ls_kv_compress(cshape, args.budget, qobs, kd, vd if args.compress_gather else None, keep_idx, keep_cnt, k_keep, v_keep)

    def step():
        # compress is issued once the scoring kernels (which fill the chip themselves) are queued, so that it runs
        # beside the selection kernels; measured: beside score + select 2.80 ms per step, after everything 2.86,
        # beside select only 2.73, beside the attention kernel 3.40
        main = torch.cuda.current_stream()
        f_score()
        side.wait_stream(main)
        with torch.cuda.stream(side):
            f_compress()
        f_select(); f_prefill()
        main.wait_stream(side)

    def timed(fn, reps):
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.profile_enable(True)
    t0 = time.perf_counter()
    ms_step = timed(step, args.steps)
    wall = time.perf_counter() - t0
    kern_ms, launches = ctx.profile_prefill_kernel_ms()
    ctx.profile_enable(False)
    assert launches == args.steps

    # per-call breakdown (outside the timed region)
    br = {name: timed(fn, max(3, args.steps // 2)) for name, fn in
          (("ls_score", f_score), ("ls_select", f_select), ("ls_sparse_prefill", f_prefill), ("ls_kv_compress", f_compress))}

    sel_h = {a: b.cpu().numpy() for a, b in sel.items() if b is not None}
    cells = metrics.selection_cells(cfg.n, cfg.n_hat, sel_h)

    # What each kind of head costs the attention kernel.  The kernel's time per visited tile hardly depends on the tile
    # (its four waves move from barrier to barrier together), so the measured kernel time is split between the kinds in proportion to the 128 x 64 tiles
    # their heads make the kernel visit (counted on the host from the index sets, as the kernel's own plan does).
    nvh, nsh = sel_h["v_cnt"], sel_h["s_cnt"]
    kind_masks = {"exhausted": (nvh >= cfg.n) & (nsh >= cfg.n), "slash_only": (nvh == 0) & (nsh > 0),
                  "vertical_only": (nsh == 0) & (nvh > 0)}
    kind_masks["mixed"] = (nvh > 0) & (nsh > 0) & ~kind_masks["exhausted"]
    tiles = np.zeros_like(cells)
    for b_ in range(cfg.B):
        for h_ in range(cfg.Hq):
            tiles[b_, h_] = metrics.visited_tiles(cfg.n, cfg.n_hat, sel_h["v_idx"][b_, h_, :min(int(nvh[b_, h_]), sel_h["v_idx"].shape[-1])],
                                                  sel_h["s_idx"][b_, h_, :min(int(nsh[b_, h_]), sel_h["s_idx"].shape[-1])])
    by_kind = {}
    for kname, m in kind_masks.items():
        if int(m.sum()) == 0:
            continue
        kc, kt = int(cells[m].sum()), int(tiles[m].sum())
        ms_k = kern_ms * kt / max(int(tiles.sum()), 1)
        by_kind[kname] = {"heads": int(m.sum()), "selected_cells": kc, "visited_tiles": kt,
                          "cells_per_tile_cell": round(kc / max(kt * 128 * 64, 1), 4), "kernel_ms_share": round(ms_k, 4),
                          "effective_tflops": round(4.0 * cfg.d * kc / max(ms_k * 1e-3, 1e-12) / 1e12, 1)}
    total_cells = int(cells.sum())
    dense_cells = cfg.B * cfg.Hq * metrics.causal_cells(cfg.n, cfg.n_hat)
    flops = 4.0 * cfg.d * total_cells                     # 2 d for q.k and 2 d for p.v per allowed cell
    value = flops / (ms_step * 1e-3) / 1e12
    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_FP32_MFMA_TFLOPS
    achieved = flops / (kern_ms * 1e-3) / 1e12
    nv, ns = sel_h["v_cnt"].ravel(), sel_h["s_cnt"].ravel()

    result = {
        "metric": "sparse prefill effective TFLOP/s over selected entries (whole hot path per layer)",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "selection": "exact overlap" if args.exact_overlap else "Alg. 2 bound", "B": cfg.B, "n": cfg.n, "n_hat": cfg.n_hat, "Hq": cfg.Hq, "Hkv": cfg.Hkv,
                   "d": cfg.d, "w": cfg.w, "alpha": alpha, "kv_budget": args.budget, "n_obs": args.n_obs,
                   "parallelism": "single GPU"},
        "pct_of_peak": round(100.0 * value / peak, 2),
        "selected_cells": total_cells, "density": round(total_cells / dense_cells, 5),
        "heads": {"dense": int(((nv >= cfg.n) & (ns >= cfg.n)).sum()), "slash_only": int(((nv == 0) & (ns > 0)).sum()),
                  "vertical_only": int(((ns == 0) & (nv > 0)).sum()),
                  "mixed": int(((ns > 0) & (nv > 0) & ~((nv >= cfg.n) & (ns >= cfg.n))).sum())},
        "by_head_kind": by_kind,
        "ms_per_call": {a: round(b, 4) for a, b in br.items()},
        "wall_s": round(wall, 3),
        "roofline": {"kernel": "prefill_bf16_kernel" if cfg.dtype == "bf16" else "prefill_kernel", "bound": "mfma", "achieved": round(achieved, 3), "peak": peak,
                     "unit": "TFLOP/s", "frac": round(achieved / peak, 4), "traffic": args.traffic_bytes,
                     "kernel_ms": round(kern_ms, 4), "launches": launches},
        "paper_context": "no speed-up printed in the paper's text; its machine: 1x H100 80GB + 8-core Xeon Gold 6542Y",
    }

    if not args.no_cpu:
        from oracle import ref
        t = time.perf_counter(); sc_ref = ref.score(q[:, :, -cfg.w:], k); t_score = time.perf_counter() - t
        t = time.perf_counter(); sel_ref = ref.select(sc_ref, cfg.n_hat, alpha); t_sel = time.perf_counter() - t
        rng = np.random.default_rng(0)
        BH = cfg.B * cfg.Hq
        rows, row_cells = [], 0
        t_att, budget_s, per = 0.0, 12.0, 2
        while t_att < budget_s and len(rows) < BH * cfg.n_hat // 4:
            batch = []
            for bh in range(BH):
                a = np.sort(rng.integers(0, cfg.n_hat, size=per))
                b_, h_ = divmod(bh, cfg.Hq)
                row_cells += sum(per_row_cells(cfg.n, cfg.n_hat, a,
                                               sel_ref["v_idx"][b_, h_, :sel_ref["v_cnt"][b_, h_]],
                                               sel_ref["s_idx"][b_, h_, :sel_ref["s_cnt"][b_, h_]]))
                batch.extend(bh * cfg.n_hat + a)
            t = time.perf_counter()
            ref.attend(q, k, v, sel_ref["v_idx"], sel_ref["v_cnt"], sel_ref["s_idx"], sel_ref["s_cnt"],
                       rows=np.array(batch, np.int64), mode=1, want_lse=False)
            t_att += time.perf_counter() - t
            rows.extend(batch)
            per = min(per * 2, 64)
        ref_cells = int(metrics.selection_cells(cfg.n, cfg.n_hat, sel_ref).sum())
        est_att = t_att * ref_cells / max(row_cells, 1)
        est_step = t_score + t_sel + est_att
        result["cpu_baseline"] = {
            "value": round(4.0 * cfg.d * ref_cells / est_step / 1e12, 6), "unit": "TFLOP/s", "cores": ref.threads(),
            "kind": "oracle",
            "sample": (f"score + select on all {BH} heads ({t_score:.2f} s + {t_sel:.2f} s), sparse attention on "
                       f"{len(rows)} random new-turn rows ({row_cells} cells, {t_att:.2f} s) extrapolated by cell count "
                       f"to all {ref_cells} selected cells; fp64 oracle, OpenMP"),
            "est_ms_per_step": round(est_step * 1e3, 1)}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
