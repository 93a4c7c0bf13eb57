"""Helpers for the GPU parity tests: move numpy inputs to the device in the workload's storage
type and run the C-ABI calls through the binding."""
import numpy as np
import torch

from paper_2507_13681_amd import binding


def to_dev(x, dtype):
    t = torch.from_numpy(np.ascontiguousarray(x)).to("cuda")
    return t.to(torch.bfloat16) if dtype == "bf16" else t


class Pipeline:
    """Holds device copies of q, k, v and a context sized for the shape."""

    def __init__(self, q, k, v, w, dtype, scale=0.0, budget=0):
        B, Hq, n_hat, d = q.shape
        _, Hkv, n, _ = k.shape
        self.dtype = dtype
        self.shape = binding.make_shape(B, Hq, Hkv, d, n, n_hat, w, dtype, scale)
        self.ctx = binding.Context(self.shape, budget)
        self.q, self.k, self.v = to_dev(q, dtype), to_dev(k, dtype), to_dev(v, dtype)
        self.w = w

    def score(self, q_pos=None, q_win=None):
        out = binding.alloc_score(self.shape)
        qw = self.q[:, :, -self.w:].contiguous() if q_win is None else q_win
        qp = None if q_pos is None else torch.from_numpy(np.asarray(q_pos, np.int64)).cuda()
        self.ctx.ls_score(self.shape, qw, self.k, out["vert"], out["slash"], out["vmax"], out["smax"], out["total"], qp)
        return out

    def select(self, sc, alpha, cap_v=None, cap_s=None, accounted=True):
        out = binding.alloc_select(self.shape, cap_v, cap_s, accounted=accounted)
        self.ctx.ls_select(self.shape, alpha, sc["vert"], sc["slash"], sc["vmax"], sc["smax"], sc["total"],
                           out["v_idx"], out["v_cnt"], out["s_idx"], out["s_cnt"], out["accounted"])
        return out

    def prefill(self, sel, want_lse=True, sentinel=False):
        """sentinel: pre-fill the outputs with NaN, so that a row no work item wrote stays recognisable."""
        out = torch.empty_like(self.q)
        lse = torch.empty(self.q.shape[:3], dtype=torch.float32, device="cuda") if want_lse else None
        if sentinel:
            out.fill_(float("nan"))
            if lse is not None:
                lse.fill_(float("nan"))
        self.ctx.ls_sparse_prefill(self.shape, self.q, self.k, self.v, sel["v_idx"], sel["v_cnt"], sel["s_idx"],
                                   sel["s_cnt"], out, lse)
        return out, lse


def dev_scores(sc_np):
    return {k: torch.from_numpy(np.ascontiguousarray(v)).cuda() for k, v in sc_np.items()}


def dev_lists(v_idx, v_cnt, s_idx, s_cnt):
    f = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    return dict(v_idx=f(v_idx), v_cnt=f(v_cnt), s_idx=f(s_idx), s_cnt=f(s_cnt))


def host(d):
    return {k: (v.float().cpu().numpy() if v.dtype == torch.bfloat16 else v.cpu().numpy())
            for k, v in d.items() if v is not None}
