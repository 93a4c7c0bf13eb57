"""ls_kv_compress_static, the entry point that allocates nothing (its scratch is a fixed block inside the
library image), against ls_kv_compress through the C ABI: same kept indices, counts and compacted rows,
bit for bit, on two calls in a row, the second with a smaller input (the scratch keeps the first call's
contents)."""
import numpy as np
import pytest
import torch

from paper_2507_13681_amd import binding, inputs

pytestmark = pytest.mark.gpu

from tests.gpu_util import to_dev  # noqa: E402


def _case(B, Hq, Hkv, ln, n_obs, d, budget, seed):
    q, k, v = inputs.make_plain(B, Hq, Hkv, ln, n_obs, d, dtype="bf16", seed=seed, q_scale=2.0)
    shape = binding.make_shape(B, Hq, Hkv, d, ln, 1, n_obs, "bf16")
    return shape, to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16"), budget


def _outputs(shape, budget, poison):
    B, Hkv, d = shape.B, shape.Hkv, shape.d
    keep_idx = torch.full((B, Hkv, budget), poison, dtype=torch.int32, device="cuda")
    keep_cnt = torch.full((B, Hkv), poison, dtype=torch.int32, device="cuda")
    k_out = torch.zeros((B, Hkv, budget, d), dtype=torch.bfloat16, device="cuda")
    v_out = torch.zeros_like(k_out)
    return keep_idx, keep_cnt, k_out, v_out


def test_static_scratch_variant_matches_ls_kv_compress():
    assert binding.static_scratch_bytes() == 16 << 20
    # second call smaller in every respect: fewer heads, a shorter cache (fewer top-B chunks), a smaller budget
    cases = [_case(2, 8, 2, 9000, 16, 128, 512, seed=21), _case(1, 4, 2, 1500, 16, 128, 200, seed=22)]
    for i, (shape, q, k, v, budget) in enumerate(cases):
        print(f"call {i}: B={shape.B} Hq={shape.Hq} Hkv={shape.Hkv} len={shape.n} budget={budget}", flush=True)
        assert binding.workspace_bytes(shape, budget) <= binding.static_scratch_bytes()
        got = _outputs(shape, budget, -7)
        binding.ls_kv_compress_static(shape, budget, q, k, v, *got)
        torch.cuda.synchronize()
        ctx = binding.Context(shape, budget)
        want = _outputs(shape, budget, -9)
        ctx.ls_kv_compress(shape, budget, q, k, v, *want)
        torch.cuda.synchronize()
        assert int(want[1].min()) == min(budget, shape.n)
        for g, w, name in zip(got, want, ("keep_idx", "keep_cnt", "k_out", "v_out")):
            assert torch.equal(g, w), name
        # the kept rows really are rows of the cache
        idx = got[0].long()
        torch.testing.assert_close(got[2], torch.gather(k, 2, idx[..., None].expand(-1, -1, -1, shape.d)), rtol=0, atol=0)


def test_static_scratch_variant_refuses_oversized_shapes():
    """A shape whose intermediate results do not fit the fixed block is refused on the host, before any launch."""
    shape = binding.make_shape(4, 64, 8, 128, 131072, 1, 64, "bf16")
    assert binding.workspace_bytes(shape, 2048) > binding.static_scratch_bytes()
    z = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    i = torch.zeros(16, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.LoopServeError, match="scratch"):
        binding.ls_kv_compress_static(shape, 2048, z, z, None, i, i)
