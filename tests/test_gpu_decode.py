"""Parity of ls_decode_attend (HIP, through the C ABI) with the oracle's decode step."""
import numpy as np
import pytest
import torch

from paper_2507_13681_amd import binding, inputs

pytestmark = pytest.mark.gpu


def _bf16(x):
    return torch.from_numpy(x).to(torch.bfloat16)


def _case(B, Hq, Hkv, cap, T, d, seed, q_scale=1.5, ragged=True):
    rng = np.random.default_rng(seed)
    mk = lambda *s: _bf16(rng.standard_normal(s).astype(np.float32))
    q = _bf16((rng.standard_normal((B, Hq, d)) * q_scale).astype(np.float32))
    kc, vc = mk(B, Hkv, cap, d), mk(B, Hkv, cap, d)
    kt, vt = (mk(B, Hkv, T, d), mk(B, Hkv, T, d)) if T else (None, None)
    cnt = rng.integers(max(1, cap // 3), cap + 1, (B, Hkv)).astype(np.int32) if ragged else None
    return q, kc, vc, cnt, kt, vt


def _run(q, kc, vc, cnt, kt, vt, want_lse=True):
    B, Hq, d = q.shape
    Hkv, cap = kc.shape[1], kc.shape[2]
    T = 0 if kt is None else kt.shape[2]
    shape = binding.make_shape(B, Hq, Hkv, d, cap + T, 1, 1, "bf16")
    ctx = binding.Context(workspace=binding.decode_workspace_bytes(shape, cap, T))
    dev = lambda t: None if t is None else t.cuda().contiguous()
    out = torch.full((B, Hq, d), 7.0, dtype=torch.bfloat16, device="cuda")
    lse = torch.full((B, Hq), 7.0, dtype=torch.float32, device="cuda") if want_lse else None
    dcnt = None if cnt is None else torch.from_numpy(cnt).cuda()
    ctx.ls_decode_attend(shape, dev(q), dev(kc), dev(vc), dcnt, dev(kt), dev(vt), out, lse)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), None if lse is None else lse.cpu().numpy()


def _f32(t):
    return None if t is None else t.float().numpy()


def _check(oracle, case, want_lse=True):
    q, kc, vc, cnt, kt, vt = case
    ref, ref_lse = oracle.decode(_f32(q), _f32(kc), _f32(vc), cnt, _f32(kt), _f32(vt))
    out, lse = _run(q, kc, vc, cnt, kt, vt, want_lse)
    err = np.abs(out - ref)
    assert err.max() <= 2e-2, err.max()
    assert err.mean() <= 5e-3, err.mean()
    if want_lse:
        fin = np.isfinite(ref_lse)
        np.testing.assert_array_equal(np.isfinite(lse), fin)
        np.testing.assert_allclose(lse[fin], ref_lse[fin], rtol=0, atol=2e-3)
    return out, lse


@pytest.mark.parametrize("B,Hq,Hkv,cap,T,d", [
    (2, 8, 2, 300, 7, 128),      # several 128-key rounds, ragged counts, a short tail
    (1, 4, 4, 45, 0, 64),        # one partial tile, no tail, one query head per KV head
    (4, 64, 8, 2048, 16, 128),   # the 70B decode shape: budget 2048 + 16 tokens since the retention
    (1, 32, 1, 1000, 130, 64),   # 32 query heads on one KV head; the tail spans tiles
    (3, 6, 3, 1, 1, 128),        # a single retained row
])
def test_decode_matches_oracle(oracle, B, Hq, Hkv, cap, T, d):
    print(f"decode case B={B} Hq={Hq} Hkv={Hkv} cap={cap} T={T} d={d}", flush=True)
    _check(oracle, _case(B, Hq, Hkv, cap, T, d, seed=cap + T))


def test_decode_full_count_and_no_lse(oracle):
    print("decode case cnt=NULL, lse=NULL", flush=True)
    _check(oracle, _case(2, 8, 4, 500, 3, 128, seed=3, ragged=False), want_lse=False)


def test_decode_rows_beyond_count_are_not_read(oracle):
    """Poison (NaN) in the rows past cnt must not reach the output."""
    q, kc, vc, cnt, kt, vt = _case(2, 8, 2, 200, 5, 128, seed=8)
    kc2, vc2 = kc.clone(), vc.clone()
    for b in range(2):
        for g in range(2):
            kc2[b, g, cnt[b, g]:] = float("nan"); vc2[b, g, cnt[b, g]:] = float("nan")
    print("decode case poisoned rows", flush=True)
    out, _ = _run(q, kc2, vc2, cnt, kt, vt)
    ref, _ = oracle.decode(_f32(q), _f32(kc), _f32(vc), cnt, _f32(kt), _f32(vt))
    assert np.isfinite(out).all()
    assert np.abs(out - ref).max() <= 2e-2


def test_decode_no_key_gives_zeros(oracle):
    q, kc, vc, _, _, _ = _case(1, 4, 2, 64, 0, 128, seed=1)
    cnt = np.array([[0, 64]], np.int32)          # the first KV head has nothing, the second everything
    print("decode case empty KV head", flush=True)
    out, lse = _check(oracle, (q, kc, vc, cnt, None, None))
    assert np.all(out[0, :2] == 0) and np.all(np.isneginf(lse[0, :2]))


def test_decode_large_logits(oracle):
    """Keys far apart in logit: the running reference must follow without overflow."""
    q, kc, vc, cnt, kt, vt = _case(1, 8, 2, 700, 9, 128, seed=21, q_scale=6.0)
    print("decode case large logits", flush=True)
    _check(oracle, (q, kc, vc, cnt, kt, vt))


def test_decode_follows_compress(oracle):
    """End to end as in Alg. 3: ls_kv_compress writes the compacted rows and their count, ls_decode_attend reads them."""
    B, Hq, Hkv, ln, n_obs, d, budget, T = 2, 8, 2, 1200, 16, 128, 256, 5
    q_obs, k, v = inputs.make_plain(B, Hq, Hkv, ln, n_obs, d, dtype="bf16", seed=5, q_scale=2.0)
    shape = binding.make_shape(B, Hq, Hkv, d, ln, 1, n_obs, "bf16")
    ctx = binding.Context(workspace=max(binding.workspace_bytes(shape, budget), binding.decode_workspace_bytes(shape, budget, T)))
    dq, dk, dv = (_bf16(x).cuda() for x in (q_obs, k, v))
    keep_idx = torch.empty((B, Hkv, budget), dtype=torch.int32, device="cuda")
    keep_cnt = torch.empty((B, Hkv), dtype=torch.int32, device="cuda")
    k_out = torch.zeros((B, Hkv, budget, d), dtype=torch.bfloat16, device="cuda"); v_out = torch.zeros_like(k_out)
    print("decode case after compress", flush=True)
    ctx.ls_kv_compress(shape, budget, dq, dk, dv, keep_idx, keep_cnt, k_out, v_out)
    rng = np.random.default_rng(2)
    qn = _bf16(rng.standard_normal((B, Hq, d)).astype(np.float32))
    kt = _bf16(rng.standard_normal((B, Hkv, T, d)).astype(np.float32)); vt = _bf16(rng.standard_normal((B, Hkv, T, d)).astype(np.float32))
    out = torch.empty((B, Hq, d), dtype=torch.bfloat16, device="cuda"); lse = torch.empty((B, Hq), dtype=torch.float32, device="cuda")
    ctx.ls_decode_attend(shape, qn.cuda(), k_out, v_out, keep_cnt, kt.cuda(), vt.cuda(), out, lse)
    torch.cuda.synchronize()
    ki = keep_idx.cpu().numpy(); kc_n = keep_cnt.cpu().numpy()
    kc_ref = np.zeros((B, Hkv, budget, d), np.float32); vc_ref = np.zeros_like(kc_ref)
    for b in range(B):
        for g in range(Hkv):
            kc_ref[b, g, :kc_n[b, g]] = k[b, g][ki[b, g, :kc_n[b, g]]]; vc_ref[b, g, :kc_n[b, g]] = v[b, g][ki[b, g, :kc_n[b, g]]]
    ref, ref_lse = oracle.decode(_f32(qn), kc_ref, vc_ref, kc_n, _f32(kt), _f32(vt))
    assert np.abs(out.float().cpu().numpy() - ref).max() <= 2e-2
    np.testing.assert_allclose(lse.cpu().numpy(), ref_lse, rtol=0, atol=2e-3)


def test_decode_argument_errors():
    shape = binding.make_shape(1, 4, 2, 128, 64, 1, 1, "bf16")
    ctx = binding.Context(workspace=1 << 20)
    q = torch.zeros((1, 4, 128), dtype=torch.bfloat16, device="cuda")
    kc = torch.zeros((1, 2, 64, 128), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros_like(q)
    with pytest.raises(binding.LoopServeError):           # fp32 is not supported by this entry point
        ctx.ls_decode_attend(binding.make_shape(1, 4, 2, 128, 64, 1, 1, "f32"), q, kc, kc, None, None, None, out)
    with pytest.raises(binding.LoopServeError):           # more than 32 query heads per KV head
        ctx.ls_decode_attend(binding.make_shape(1, 66, 2, 128, 64, 1, 1, "bf16"), q, kc, kc, None, None, None, out)
    with pytest.raises(binding.LoopServeError):           # workspace too small
        small = binding.Context(workspace=256)
        small.ls_decode_attend(shape, q, kc, kc, None, None, None, out)
