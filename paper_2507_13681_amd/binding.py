"""Thin ctypes binding of libloopserve (see include/loopserve.h, include/loopserve_test_hooks.h).

Argument marshalling only: every step of the path runs in the HIP kernels of the library.
PyTorch supplies device memory and the current stream.  The library must have been built
(`python -m paper_2507_13681_amd.build` or `__graft_entry__.build()`); loading fails loudly
otherwise -- there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import math
import os

import torch

_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_DIR, "libloopserve.so")
LS_BF16, LS_F32 = 0, 1
LS_MAX_N, LS_MAX_W = 262144, 256
_lib = None

ENTRY_POINTS = ("ls_workspace_bytes", "ls_create", "ls_destroy", "ls_last_error",
                "ls_score", "ls_select", "ls_sparse_prefill", "ls_kv_compress", "ls_poll_status")
# bits of the device status word (ls_poll_status)
LS_STAT_WALK_TIMEOUT, LS_STAT_S_TRUNCATED, LS_STAT_V_TRUNCATED, LS_STAT_S_RANGE, LS_STAT_V_INVALID = 1, 2, 4, 8, 16
LS_STAT_MERGE_RANGE = 32


class LsShape(C.Structure):
    _fields_ = [("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("d", C.c_int32),
                ("n", C.c_int64), ("n_hat", C.c_int64), ("w", C.c_int32), ("dtype", C.c_int32),
                ("scale", C.c_float)]


class LoopServeError(RuntimeError):
    pass


def load_library():
    """dlopen the HIP library and declare the signatures of include/loopserve.h."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise LoopServeError(f"{LIB_PATH} is missing: build it with `python -m paper_2507_13681_amd.build`")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    sp = C.POINTER(LsShape)
    lib.ls_workspace_bytes.restype = C.c_size_t
    lib.ls_workspace_bytes.argtypes = [sp, i32]
    lib.ls_create.restype = C.c_int
    lib.ls_create.argtypes = [C.POINTER(vp), C.c_int, C.c_size_t]
    lib.ls_destroy.restype = None
    lib.ls_destroy.argtypes = [vp]
    lib.ls_last_error.restype = C.c_char_p
    lib.ls_last_error.argtypes = [vp]
    lib.ls_score.restype = C.c_int
    lib.ls_score.argtypes = [vp, sp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.ls_select.restype = C.c_int
    lib.ls_select.argtypes = [vp, sp, f32, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, i32, vp, vp]
    lib.ls_score_window.restype = C.c_int
    lib.ls_score_window.argtypes = [vp, sp, vp, vp, vp, vp, vp]
    lib.ls_select_exact.restype = C.c_int
    lib.ls_select_exact.argtypes = [vp, sp, f32, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, i32, vp, vp]
    lib.ls_merge_lines.restype = C.c_int
    lib.ls_merge_lines.argtypes = [vp, sp] + [vp, vp, i32] * 6 + [vp]
    lib.ls_sparse_prefill.restype = C.c_int
    lib.ls_sparse_prefill.argtypes = [vp, sp, vp, vp, vp, vp, vp, i32, vp, vp, i32, vp, vp, vp]
    lib.ls_kv_compress.restype = C.c_int
    lib.ls_kv_compress.argtypes = [vp, sp, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.ls_kv_compress_static.restype = C.c_int
    lib.ls_kv_compress_static.argtypes = [C.c_int, sp, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.ls_static_scratch_bytes.restype = C.c_size_t
    lib.ls_static_scratch_bytes.argtypes = []
    lib.ls_decode_attend.restype = C.c_int
    lib.ls_decode_attend.argtypes = [vp, sp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.ls_decode_workspace_bytes.restype = C.c_size_t
    lib.ls_decode_workspace_bytes.argtypes = [sp, i32, i32]
    lib.ls_debug_copy_compress_score.restype = C.c_int
    lib.ls_debug_copy_compress_score.argtypes = [vp, sp, vp, vp]
    lib.ls_poll_status.restype = C.c_int
    lib.ls_poll_status.argtypes = [vp, C.POINTER(i32), vp]
    lib.ls_debug_set_walk_spin_limit.restype = C.c_int
    lib.ls_debug_set_walk_spin_limit.argtypes = [vp, i32]
    lib.ls_debug_copy_prefill_queues.restype = C.c_int
    lib.ls_debug_copy_prefill_queues.argtypes = [vp, sp, vp, vp, C.POINTER(i32), vp]
    lib.ls_profile_enable.restype = C.c_int
    lib.ls_profile_enable.argtypes = [vp, C.c_int]
    lib.ls_profile_prefill_kernel_ms.restype = C.c_int
    lib.ls_profile_prefill_kernel_ms.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i32)]
    _lib = lib
    return lib


def make_shape(B, Hq, Hkv, d, n, n_hat, w, dtype, scale=0.0) -> LsShape:
    code = {torch.bfloat16: LS_BF16, torch.float32: LS_F32, "bf16": LS_BF16, "f32": LS_F32}[dtype]
    return LsShape(B, Hq, Hkv, d, n, n_hat, w, code, float(scale))


def workspace_bytes(shape: LsShape, budget: int = 0) -> int:
    return int(load_library().ls_workspace_bytes(C.byref(shape), budget))


def decode_workspace_bytes(shape: LsShape, cap: int, T: int) -> int:
    return int(load_library().ls_decode_workspace_bytes(C.byref(shape), cap, T))


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "tensors must be contiguous device tensors"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Context:
    """An ls_ctx: a device workspace that the four calls carve their scratch from."""

    def __init__(self, shape: LsShape | None = None, budget: int = 0, device: int = 0, workspace: int | None = None):
        self.lib = load_library()
        if workspace is None:
            workspace = workspace_bytes(shape, budget)
            if workspace == 0:
                raise LoopServeError("invalid shape")
        self.workspace = int(workspace)
        self.device = device
        h = C.c_void_p()
        rc = self.lib.ls_create(C.byref(h), device, self.workspace)
        if rc != 0:
            raise LoopServeError(f"ls_create failed with {rc}")
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.ls_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc != 0:
            raise LoopServeError(f"{self.lib.ls_last_error(self.h).decode()} (status {rc})")

    # -- the four entry points, same names as the C ABI -------------------------------------
    def ls_score(self, shape, q_win, k, vert, slash, vmax, smax, total, q_pos=None):
        self._check(self.lib.ls_score(self.h, C.byref(shape), _ptr(q_win), _ptr(q_pos), _ptr(k), _ptr(vert),
                                      _ptr(slash), _ptr(vmax), _ptr(smax), _ptr(total), _stream()))

    def ls_select(self, shape, alpha, vert, slash, vmax, smax, total, v_idx, v_cnt, s_idx, s_cnt, accounted=None):
        self._check(self.lib.ls_select(self.h, C.byref(shape), alpha, _ptr(vert), _ptr(slash), _ptr(vmax), _ptr(smax),
                                       _ptr(total), _ptr(v_idx), _ptr(v_cnt), v_idx.shape[-1], _ptr(s_idx),
                                       _ptr(s_cnt), s_idx.shape[-1], _ptr(accounted), _stream()))

    def ls_score_window(self, shape, q_win, k, a_win, q_pos=None):
        self._check(self.lib.ls_score_window(self.h, C.byref(shape), _ptr(q_win), _ptr(q_pos), _ptr(k), _ptr(a_win), _stream()))

    def ls_select_exact(self, shape, alpha, a_win, vert, slash, total, v_idx, v_cnt, s_idx, s_cnt, accounted=None, q_pos=None):
        self._check(self.lib.ls_select_exact(self.h, C.byref(shape), alpha, _ptr(a_win), _ptr(q_pos), _ptr(vert), _ptr(slash),
                                             _ptr(total), _ptr(v_idx), _ptr(v_cnt), v_idx.shape[-1], _ptr(s_idx),
                                             _ptr(s_cnt), s_idx.shape[-1], _ptr(accounted), _stream()))

    def ls_merge_lines(self, shape, a, b, out):
        """a, b, out: dicts with v_idx, v_cnt, s_idx, s_cnt (as alloc_select returns them)."""
        args = []
        for d in (a, b, out):
            args += [_ptr(d["v_idx"]), _ptr(d["v_cnt"]), d["v_idx"].shape[-1], _ptr(d["s_idx"]), _ptr(d["s_cnt"]), d["s_idx"].shape[-1]]
        self._check(self.lib.ls_merge_lines(self.h, C.byref(shape), *args, _stream()))

    def ls_sparse_prefill(self, shape, q, k, v, v_idx, v_cnt, s_idx, s_cnt, out, lse=None):
        self._check(self.lib.ls_sparse_prefill(self.h, C.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(v_idx),
                                               _ptr(v_cnt), v_idx.shape[-1], _ptr(s_idx), _ptr(s_cnt),
                                               s_idx.shape[-1], _ptr(out), _ptr(lse), _stream()))

    def ls_kv_compress(self, shape, budget, q_obs, k, v, keep_idx, keep_cnt, k_out=None, v_out=None):
        self._check(self.lib.ls_kv_compress(self.h, C.byref(shape), budget, _ptr(q_obs), _ptr(k), _ptr(v),
                                            _ptr(keep_idx), _ptr(keep_cnt), _ptr(k_out), _ptr(v_out), _stream()))

    def ls_decode_attend(self, shape, q, k_c, v_c, cnt, k_t, v_t, out, lse=None):
        T = 0 if k_t is None else k_t.shape[2]
        self._check(self.lib.ls_decode_attend(self.h, C.byref(shape), k_c.shape[2], T, _ptr(q), _ptr(k_c), _ptr(v_c),
                                              _ptr(cnt), _ptr(k_t), _ptr(v_t), _ptr(out), _ptr(lse), _stream()))

    def ls_poll_status(self) -> int:
        """Waits for the current stream, returns the context's device status word and clears it."""
        word = C.c_int32()
        self._check(self.lib.ls_poll_status(self.h, C.byref(word), _stream()))
        return word.value

    def debug_set_walk_spin_limit(self, limit: int):
        self._check(self.lib.ls_debug_set_walk_spin_limit(self.h, limit))

    def debug_prefill_queues(self, shape):
        """Work queues of the last ls_sparse_prefill call: list of eight int arrays of item words."""
        import numpy as np
        items = shape.B * shape.Hq * ((int(shape.n) + 127) // 128 + 1)        # at least B * Hq * nqb
        qlen = np.zeros(8, dtype=np.int32)
        nqb = C.c_int32()
        # the library packs the queues at the true stride B * Hq * nqb: read flat, then cut
        flat = np.zeros(8 * items, dtype=np.uint32)
        self._check(self.lib.ls_debug_copy_prefill_queues(self.h, C.byref(shape), flat.ctypes.data_as(C.c_void_p),
                                                          qlen.ctypes.data_as(C.c_void_p), C.byref(nqb), _stream()))
        stride = shape.B * shape.Hq * nqb.value
        return [flat[x * stride: x * stride + int(qlen[x])].copy() for x in range(8)], nqb.value

    def profile_enable(self, on=True):
        self._check(self.lib.ls_profile_enable(self.h, 1 if on else 0))

    def profile_prefill_kernel_ms(self):
        ms, cnt = C.c_double(), C.c_int32()
        self._check(self.lib.ls_profile_prefill_kernel_ms(self.h, C.byref(ms), C.byref(cnt)))
        return ms.value, cnt.value

    def debug_compress_score(self, shape, dst):
        self._check(self.lib.ls_debug_copy_compress_score(self.h, C.byref(shape), _ptr(dst), _stream()))


def ls_kv_compress_static(shape, budget, q_obs, k, v, keep_idx, keep_cnt, k_out=None, v_out=None, device=0):
    """ls_kv_compress without a context, on the library's static scratch (allocates nothing)."""
    lib = load_library()
    rc = lib.ls_kv_compress_static(device, C.byref(shape), budget, _ptr(q_obs), _ptr(k), _ptr(v), _ptr(keep_idx),
                                   _ptr(keep_cnt), _ptr(k_out), _ptr(v_out), _stream())
    if rc != 0:
        raise LoopServeError(f"{lib.ls_last_error(None).decode()} (status {rc})")


def static_scratch_bytes() -> int:
    return int(load_library().ls_static_scratch_bytes())


# -- convenience: allocate outputs with torch and run one call ----------------------------------

def alloc_score(shape: LsShape, device="cuda"):
    B, Hq, n = shape.B, shape.Hq, shape.n
    f = dict(dtype=torch.float32, device=device)
    return dict(vert=torch.empty(B, Hq, n, **f), slash=torch.empty(B, Hq, n, **f), vmax=torch.empty(B, Hq, n, **f),
                smax=torch.empty(B, Hq, n, **f), total=torch.empty(B, Hq, **f))


def alloc_select(shape: LsShape, cap_v=None, cap_s=None, device="cuda", accounted=True):
    B, Hq, n = shape.B, shape.Hq, shape.n
    i = dict(dtype=torch.int32, device=device)
    return dict(v_idx=torch.empty(B, Hq, cap_v or n, **i), v_cnt=torch.empty(B, Hq, **i),
                s_idx=torch.empty(B, Hq, cap_s or n, **i), s_cnt=torch.empty(B, Hq, **i),
                accounted=torch.empty(B, Hq, dtype=torch.float32, device=device) if accounted else None)


def default_scale(d):
    return 1.0 / math.sqrt(d)
