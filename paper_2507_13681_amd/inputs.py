"""Seeded synthetic inputs shaped like multi-turn long-context attention.

This module holds no arithmetic of the method itself (no softmax, no line sums,
no selection): it only draws Q, K, V with planted structure, so that both the
device path and the CPU oracle can be fed identical numbers.

The planted structure stands in for the attention patterns of the paper's
multi-turn benchmark (Sec. 4, Appendix dataset table: 2-3 turns, 2k-30k tokens,
query at the start / middle / end of a turn) and for Observation 1 of Sec. 3.1
(a small fraction of key columns and diagonals carries most attention mass):

  * attention sinks:   the first `sinks` keys get +3 units along a direction u
                       that every query of the KV group leans towards;
  * heavy columns:     each query head h has its own direction u_h and its own
                       set of history keys boosted by +2 units along u_h;
  * local band:        a slowly varying positional vector r_p (AR(1) process over
                       positions, correlation length `band`) shared by q_p and k_p,
                       so logits decay with distance |p - p'|;
  * relevant span:     a contiguous key span in some turn gets +2 units along
                       u_span; a 64-row query block placed at the start, middle or
                       end of the newest turn (by head index mod 3) leans on u_span;
  * background:        everything else is N(0,1), with the planted directions
                       projected out of K so they add no background noise.

One "unit" is `tau` in logit space (after the 1/sqrt(d) scale).  All values are
produced in float32, rounded once to the workload's storage type (bf16 or fp32)
and returned as float32 arrays holding exactly those rounded values.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    n: int            # keys in context
    n_hat: int        # rows of the newest turn (the last n_hat positions)
    Hq: int
    Hkv: int
    d: int
    dtype: str        # "bf16" | "f32"
    w: int            # scoring window rows
    alpha: float      # coverage target
    turns: int
    sinks: int
    heavy_lo: int     # heavy columns per query head ~ Uniform[heavy_lo, heavy_hi]
    heavy_hi: int
    band: int         # correlation length of the positional component
    span: int         # relevant-span length (0: none)
    tau: float        # logit unit of the planted boosts
    beta: float       # peak logit of the local band
    rho: float        # std of background logits
    seed: int

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    def causal_cells_per_head(self) -> int:
        return self.n_hat * (self.n - self.n_hat) + self.n_hat * (self.n_hat + 1) // 2


def turn_bounds(n: int, turns: int):
    """Turn i covers [floor(i*n/turns), floor((i+1)*n/turns))."""
    return [(i * n) // turns for i in range(turns + 1)]


def _mk(name, B, n, turns, Hq, Hkv, d, dtype, w, alpha, sinks, hlo, hhi, band, span, tau, beta, rho, idx):
    n_hat = n - turn_bounds(n, turns)[turns - 1]
    return Workload(name, B, n, n_hat, Hq, Hkv, d, dtype, w, alpha, turns, sinks, hlo, hhi, band, span,
                    tau, beta, rho, 1234 + idx)


# The five workloads of the benchmark definition.  n_hat = length of the last turn.
CONFIGS = {
    "tiny": _mk("tiny", 1, 1024, 4, 4, 1, 64, "f32", 32, 0.90, 4, 8, 8, 32, 0, 3.0, 5.0, 0.5, 0),
    "llama8b_8k": _mk("llama8b_8k", 1, 8192, 2, 32, 8, 128, "bf16", 64, 0.95, 4, 64, 64, 256, 512,
                      3.4, 6.0, 0.5, 1),
    "multiturn_32k": _mk("multiturn_32k", 1, 32768, 3, 32, 8, 128, "bf16", 64, 0.95, 4, 16, 256, 256, 1024,
                         3.8, 6.0, 0.5, 2),
    "stress_131k": _mk("stress_131k", 1, 131072, 8, 32, 8, 128, "bf16", 128, 0.95, 4, 16, 256, 256, 1024,
                       4.2, 6.0, 0.5, 3),
    "llama70b_16k_b4": _mk("llama70b_16k_b4", 4, 16384, 3, 64, 8, 128, "bf16", 64, 0.95, 4, 16, 256, 256, 1024,
                           3.6, 6.0, 0.5, 4),
}


def scaled(cfg: Workload, **kw) -> Workload:
    """A copy with some fields replaced (n_hat is recomputed if n or turns change)."""
    c = replace(cfg, **kw)
    if ("n" in kw or "turns" in kw) and "n_hat" not in kw:
        c = replace(c, n_hat=c.n - turn_bounds(c.n, c.turns)[c.turns - 1])
    return c


def round_to(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values to the storage type and return them as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype != "bf16":
        raise ValueError(dtype)
    u = x.view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)   # round to nearest even
    return ((u + r) & np.uint32(0xFFFF0000)).view(np.float32)


def _ar1(rng, n, m, corr_len):
    """n x m array, each column a stationary unit-variance AR(1) path over positions."""
    a = np.float32(np.exp(-1.0 / max(corr_len, 1)))
    e = rng.standard_normal((n, m), dtype=np.float32)
    e[1:] *= np.float32(np.sqrt(1.0 - float(a) ** 2))
    from scipy.signal import lfilter
    return lfilter([1.0], [1.0, -float(a)], e, axis=0).astype(np.float32)


def make_inputs(cfg: Workload, seed: int | None = None):
    """Draw q [B,Hq,n_hat,d], k, v [B,Hkv,n,d] (float32 arrays holding dtype-rounded values).

    Also returns `meta`: the planted positions per (batch, head), for reporting only.
    """
    rng = np.random.Generator(np.random.PCG64(cfg.seed if seed is None else seed))
    B, n, nh, Hq, Hkv, d, G = cfg.B, cfg.n, cfg.n_hat, cfg.Hq, cfg.Hkv, cfg.d, cfg.G
    m = max(d // 4, 8)                       # dimension of the positional subspace
    sq = np.float32(np.sqrt(d))
    bounds = turn_bounds(n, cfg.turns)
    hist = n - nh                            # keys before the newest turn
    q = np.empty((B, Hq, nh, d), np.float32)
    k = np.empty((B, Hkv, n, d), np.float32)
    v = rng.standard_normal((B, Hkv, n, d), dtype=np.float32)
    gk = np.float32(np.sqrt(cfg.beta / m))   # positional amplitude on each side
    meta = []
    for b in range(B):
        for j in range(Hkv):
            E, _ = np.linalg.qr(rng.standard_normal((d, 2 + G + m)).astype(np.float64))
            E = E.astype(np.float32)
            u, u_span, Uh, Ep = E[:, 0], E[:, 1], E[:, 2:2 + G], E[:, 2 + G:]
            r = _ar1(rng, n, m, cfg.band)                       # positional path, [n, m]
            Kj = rng.standard_normal((n, d), dtype=np.float32)
            Kj -= (Kj @ E) @ E.T                                # planted directions carry no noise
            Kj += gk * (r @ Ep.T)
            Kj[:cfg.sinks] += np.float32(3.0) * u
            span_lo = -1
            if cfg.span > 0:
                t = int(rng.integers(0, cfg.turns))
                lo, hi = bounds[t], max(bounds[t + 1] - cfg.span, bounds[t] + 1)
                span_lo = int(rng.integers(lo, hi))
                Kj[span_lo:span_lo + cfg.span] += np.float32(2.0) * u_span
            for g in range(G):
                h = j * G + g
                cnt = int(rng.integers(cfg.heavy_lo, cfg.heavy_hi + 1))
                cols = np.sort(rng.choice(np.arange(cfg.sinks, max(hist, cfg.sinks + cnt)), size=cnt,
                                          replace=False))
                Kj[cols] += np.float32(2.0) * Uh[:, g]
                Qh = np.float32(cfg.rho) * rng.standard_normal((nh, d), dtype=np.float32)
                Qh += sq * np.float32(cfg.tau) * (u + Uh[:, g])
                Qh += sq * gk * (r[hist:] @ Ep.T)
                blk = -1
                if cfg.span > 0:
                    qb = min(64, nh)
                    blk = [0, (nh - qb) // 2, nh - qb][h % 3]   # start / middle / end of the turn
                    Qh[blk:blk + qb] += sq * np.float32(cfg.tau) * u_span
                q[b, h] = Qh
                meta.append(dict(b=b, h=h, heavy=cols, span_lo=span_lo, query_block=blk))
            k[b, j] = Kj
    return round_to(q, cfg.dtype), round_to(k, cfg.dtype), round_to(v, cfg.dtype), meta


def make_decode_step(cfg: Workload, steps: int, seed: int | None = None):
    """Fresh q [B,Hq,steps,d], k, v [B,Hkv,steps,d] ~ N(0,1) for the decode phase."""
    rng = np.random.Generator(np.random.PCG64((cfg.seed if seed is None else seed) + 7919))
    q = rng.standard_normal((cfg.B, cfg.Hq, steps, cfg.d), dtype=np.float32)
    k = rng.standard_normal((cfg.B, cfg.Hkv, steps, cfg.d), dtype=np.float32)
    v = rng.standard_normal((cfg.B, cfg.Hkv, steps, cfg.d), dtype=np.float32)
    return round_to(q, cfg.dtype), round_to(k, cfg.dtype), round_to(v, cfg.dtype)


def make_plain(B, Hq, Hkv, n, n_hat, d, dtype="f32", seed=0, q_scale=1.0):
    """Unstructured N(0,1) tensors for small tests: q [B,Hq,n_hat,d], k, v [B,Hkv,n,d]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    q = np.float32(q_scale) * rng.standard_normal((B, Hq, n_hat, d), dtype=np.float32)
    k = rng.standard_normal((B, Hkv, n, d), dtype=np.float32)
    v = rng.standard_normal((B, Hkv, n, d), dtype=np.float32)
    return round_to(q, dtype), round_to(k, dtype), round_to(v, dtype)
