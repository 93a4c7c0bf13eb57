"""ctypes front end of the CPU oracle (oracle/ls_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
the cpu_baseline leg of bench.py.  The product package never imports it.

All arrays are numpy, float32 / int32 / int64, C-contiguous.  Inputs that the
device path holds in bf16 are passed here as the same bf16-rounded values
widened to float32, so both sides start from identical numbers.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "ls_oracle.c")
_LIB = os.path.join(_DIR, "libls_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (contraction off so binary32 steps round once)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.lso_walk.restype = None
    return _lib


def _f(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(C.POINTER(C.c_float))


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


def _i64(a):
    a = np.ascontiguousarray(a, dtype=np.int64)
    return a, a.ctypes.data_as(C.POINTER(C.c_int64))


def threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    return int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))


def score(q_win, k, scale=None, q_pos=None):
    """Alg. 2 window softmax + line sums.  q_win [B,Hq,w,d], k [B,Hkv,n,d].
    Returns dict(vert, slash, vmax, smax [B,Hq,n], total [B,Hq])."""
    q_win, qp = _f(q_win)
    k, kp = _f(k)
    B, Hq, w, d = q_win.shape
    _, Hkv, n, _ = k.shape
    scale = float(scale) if scale else 1.0 / np.sqrt(d)
    out = {name: np.empty((B, Hq, n), np.float32) for name in ("vert", "slash", "vmax", "smax")}
    out["total"] = np.empty((B, Hq), np.float32)
    if q_pos is not None:
        q_pos, pp = _i64(q_pos)
        assert q_pos.shape == (w,)
    else:
        pp = None
    rc = lib().lso_score(B, Hq, Hkv, d, C.c_int64(n), w, C.c_double(scale), qp, pp, kp,
                         *[_f(out[x])[1] for x in ("vert", "slash", "vmax", "smax", "total")])
    if rc:
        raise RuntimeError(f"lso_score rc={rc}")
    return out


def walk(ws, ms, ls, wv, mv, lv, alpha, total):
    """The while-loop of Alg. 2 on two pre-sorted lists (see lso_walk).
    Returns (taken_s, taken_v, accounted, before_last)."""
    ws, a1 = _f(ws); ms, a2 = _f(ms); ls, a3 = _f(ls)
    wv, b1 = _f(wv); mv, b2 = _f(mv); lv, b3 = _f(lv)
    ts, tv = C.c_int64(), C.c_int64()
    acc, prev = C.c_float(), C.c_float()
    lib().lso_walk(C.c_int64(len(ws)), a1, a2, a3, C.c_int64(len(wv)), b1, b2, b3,
                   C.c_float(alpha), C.c_float(total),
                   C.byref(ts), C.byref(tv), C.byref(acc), C.byref(prev))
    return ts.value, tv.value, acc.value, prev.value


def select(sc, n_hat, alpha, cap_v=None, cap_s=None):
    """Alg. 2 sort + walk for every head.  sc = dict from score().
    Returns dict(v_idx [B,Hq,cap_v], v_cnt [B,Hq], s_idx, s_cnt, accounted, before_last)."""
    vert, vp = _f(sc["vert"]); slash, sp = _f(sc["slash"])
    vmax, vmp = _f(sc["vmax"]); smax, smp = _f(sc["smax"]); total, tp = _f(sc["total"])
    B, Hq, n = vert.shape
    cap_v = int(cap_v or n)
    cap_s = int(cap_s or n)
    v_idx = np.full((B, Hq, cap_v), -1, np.int32); s_idx = np.full((B, Hq, cap_s), -1, np.int32)
    v_cnt = np.zeros((B, Hq), np.int32); s_cnt = np.zeros((B, Hq), np.int32)
    acc = np.zeros((B, Hq), np.float32); prev = np.zeros((B, Hq), np.float32)
    rc = lib().lso_select_all(C.c_int64(B * Hq), C.c_int64(n), C.c_int64(n_hat), C.c_float(alpha),
                              vp, sp, vmp, smp, tp,
                              _i32(v_idx)[1], _i32(v_cnt)[1], C.c_int64(cap_v),
                              _i32(s_idx)[1], _i32(s_cnt)[1], C.c_int64(cap_s),
                              _f(acc)[1], _f(prev)[1])
    if rc:
        raise RuntimeError(f"lso_select_all rc={rc}")
    return dict(v_idx=v_idx, v_cnt=v_cnt, s_idx=s_idx, s_cnt=s_cnt, accounted=acc, before_last=prev)


def window(q_win, k, scale=None, q_pos=None):
    """The window attention matrix of Alg. 2 (softmax step): a_win [B,Hq,w,n] float32, zero beyond each row's position."""
    q_win, qp = _f(q_win); k, kp = _f(k)
    B, Hq, w, d = q_win.shape
    _, Hkv, n, _ = k.shape
    scale = (1.0 / np.sqrt(d)) if scale is None else scale
    a = np.zeros((B, Hq, w, n), np.float32)
    pp = None
    if q_pos is not None:
        q_pos, pp = _i64(q_pos)
    rc = lib().lso_window(B, Hq, Hkv, d, C.c_int64(n), w, C.c_double(scale), qp, pp, kp, _f(a)[1])
    if rc:
        raise RuntimeError(f"lso_window rc={rc}")
    return a


def select_exact(a_win, sc, n_hat, alpha, q_pos=None, cap_v=None, cap_s=None):
    """Alg. 2 with the overlap of a candidate line counted cell by cell (lso_select_exact), every head.
    a_win from window(), sc = dict from score() (vert, slash, total are used).  Same result dict as select()."""
    a_win, ap = _f(a_win)
    vert, vp = _f(sc["vert"]); slash, sp = _f(sc["slash"]); total, tp = _f(sc["total"])
    B, Hq, w, n = a_win.shape
    cap_v = int(cap_v or n); cap_s = int(cap_s or n)
    v_idx = np.full((B, Hq, cap_v), -1, np.int32); s_idx = np.full((B, Hq, cap_s), -1, np.int32)
    v_cnt = np.zeros((B, Hq), np.int32); s_cnt = np.zeros((B, Hq), np.int32)
    acc = np.zeros((B, Hq), np.float32); prev = np.zeros((B, Hq), np.float32)
    pp = None
    if q_pos is not None:
        q_pos, pp = _i64(q_pos)
    rc = lib().lso_select_exact_all(C.c_int64(B * Hq), C.c_int64(n), C.c_int64(n_hat), w, C.c_float(alpha), ap, pp,
                                    vp, sp, tp, _i32(v_idx)[1], _i32(v_cnt)[1], C.c_int64(cap_v),
                                    _i32(s_idx)[1], _i32(s_cnt)[1], C.c_int64(cap_s), _f(acc)[1], _f(prev)[1])
    if rc:
        raise RuntimeError(f"lso_select_exact_all rc={rc}")
    return dict(v_idx=v_idx, v_cnt=v_cnt, s_idx=s_idx, s_cnt=s_cnt, accounted=acc, before_last=prev)


def attend(q, k, v, v_idx, v_cnt, s_idx, s_cnt, scale=None, rows=None, mode=1, want_lse=True):
    """Masked attention over selected lines for the rows of the newest turn.
    q [B,Hq,n_hat,d]; k, v [B,Hkv,n,d].  rows: flat ids ((b*Hq+h)*n_hat+a) or None = all.
    mode 0 = dense-masked (literal), 1 = row-sparse.  Returns (out [R,d], lse [R])."""
    q, qp = _f(q); k, kp = _f(k); v, vp = _f(v)
    B, Hq, n_hat, d = q.shape
    _, Hkv, n, _ = k.shape
    v_idx, vip = _i32(v_idx); s_idx, sip = _i32(s_idx)
    v_cnt, vcp = _i32(v_cnt); s_cnt, scp = _i32(s_cnt)
    cap_v, cap_s = v_idx.shape[-1], s_idx.shape[-1]
    scale = float(scale) if scale else 1.0 / np.sqrt(d)
    if rows is not None:
        rows, rp = _i64(rows)
        R = len(rows)
    else:
        rp, R = None, B * Hq * n_hat
    out = np.empty((R, d), np.float32)
    lse = np.empty((R,), np.float32)
    rc = lib().lso_attend(B, Hq, Hkv, d, C.c_int64(n), C.c_int64(n_hat), C.c_double(scale), qp, kp, vp,
                          vip, vcp, C.c_int64(cap_v), sip, scp, C.c_int64(cap_s),
                          C.c_int64(R), rp, int(mode), _f(out)[1], _f(lse)[1] if want_lse else None)
    if rc:
        raise RuntimeError(f"lso_attend rc={rc}")
    return out, lse


def compress(q_obs, k, budget, scale=None):
    """Alg. 3 retention: top-`budget` cache entries per KV head.
    q_obs [B,Hq,n_obs,d], k [B,Hkv,len,d].  Returns dict(keep_idx [B,Hkv,budget], keep_cnt, score)."""
    q_obs, qp = _f(q_obs); k, kp = _f(k)
    B, Hq, n_obs, d = q_obs.shape
    _, Hkv, ln, _ = k.shape
    scale = float(scale) if scale else 1.0 / np.sqrt(d)
    keep_idx = np.full((B, Hkv, budget), -1, np.int32)
    keep_cnt = np.zeros((B, Hkv), np.int32)
    sc = np.empty((B, Hkv, ln), np.float32)
    rc = lib().lso_compress(B, Hq, Hkv, d, C.c_int64(ln), n_obs, C.c_double(scale), C.c_int64(budget),
                            qp, kp, _i32(keep_idx)[1], _i32(keep_cnt)[1], _f(sc)[1])
    if rc:
        raise RuntimeError(f"lso_compress rc={rc}")
    return dict(keep_idx=keep_idx, keep_cnt=keep_cnt, score=sc)


def topb(score_vec, budget):
    """Top-`budget` indices of one score vector, ascending (ties: smaller index)."""
    s, sp = _f(score_vec)
    keep = np.full((budget,), -1, np.int32)
    cnt = C.c_int32()
    rc = lib().lso_topb(C.c_int64(len(s)), C.c_int64(budget), sp, _i32(keep)[1], C.byref(cnt))
    if rc:
        raise RuntimeError(f"lso_topb rc={rc}")
    return keep[:cnt.value]


def decode(q, kc, vc, cnt=None, kt=None, vt=None, scale=None, want_lse=True):
    """Alg. 3 Decoding step of one layer: the newest token attends over the retained entries and the tokens since.
    q [B,Hq,d]; kc, vc [B,Hkv,cap,d] (first cnt[b,kvh] rows valid; None: all); kt, vt [B,Hkv,T,d] or None.
    Returns (out [B,Hq,d] float32, lse [B,Hq] float32 or None)."""
    q, qp = _f(q); kc, kcp = _f(kc); vc, vcp = _f(vc)
    B, Hq, d = q.shape
    _, Hkv, cap, _ = kc.shape
    T = 0 if kt is None else kt.shape[2]
    if T:
        kt, ktp = _f(kt); vt, vtp = _f(vt)
    else:
        ktp = vtp = None
    cp = None if cnt is None else _i32(cnt)[1]
    scale = float(scale) if scale else 1.0 / np.sqrt(d)
    out = np.empty((B, Hq, d), np.float32)
    lse = np.empty((B, Hq), np.float32) if want_lse else None
    rc = lib().lso_decode(B, Hq, Hkv, d, C.c_int64(cap), C.c_int64(T), C.c_double(scale), qp, kcp, vcp, cp, ktp, vtp,
                          _f(out)[1], None if lse is None else _f(lse)[1])
    if rc:
        raise RuntimeError(f"lso_decode rc={rc}")
    return out, lse
