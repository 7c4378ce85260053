"""The whole-path entry point that takes no workspace (its scratch is a fixed device array
inside the library) against the one that does: same kernels, so every output must be equal bit
for bit.  Two calls in a row on one context, the second on a smaller input, so that stale
contents of the shared scratch from the first call are in place when the second one runs."""
import numpy as np
import pytest
import torch

from paper_2512_07090_amd import binding as B
from paper_2512_07090_amd import synth

pytestmark = pytest.mark.gpu

NAMES = ("keep", "kept_idx", "fused", "tau", "O")


def _both(ctx, shape, ratio, seed):
    dt, Bn, Hq, Hkv, n = shape
    print("[case] no-alloc entry point %s ratio %g" % (shape, ratio), flush=True)
    q, k, v, _ = synth.make_random_qkv(Bn, Hq, Hkv, n, 128, dtype=dt, seed=seed)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    p = B.make_params(tuple(q.shape), tuple(k.shape), q.dtype, ratio)
    assert B.tf_workspace_bytes(p) <= B.TF_STATIC_SCRATCH_BYTES
    ref = B.Buffers(p, "cuda:0")
    ref.O.fill_(float("nan"))
    ctx.tf_filtered_attention(p, qd, kd, vd, ref.keep, ref.kept_idx, ref.fused, ref.tau, ref.O, ref.ws)
    got = B.Buffers(p, "cuda:0")
    got.O.fill_(float("nan"))
    got.fused.fill_(float("nan"))
    got.keep.fill_(9)
    got.kept_idx.fill_(-7)
    ctx.tf_filtered_attention_static(p, qd, kd, vd, got.keep, got.kept_idx, got.fused, got.tau, got.O)
    torch.cuda.synchronize()
    assert not torch.isnan(got.O.float()).any()
    for name in NAMES:
        assert torch.equal(getattr(got, name), getattr(ref, name)), name
    return got


def test_static_scratch_entry_point_matches_the_workspace_one_twice_in_a_row():
    assert torch.cuda.is_available(), "this test needs the MI355X"
    ctx = B.Context(0)
    try:
        # few chains: the scan is cut into segments and the segment totals go through the scratch
        _both(ctx, ("bf16", 2, 8, 2, 4133), 0.5, seed=11)
        # then a smaller input of another shape, on the scratch the first call left behind
        _both(ctx, ("bf16", 1, 4, 4, 700), 0.25, seed=12)
        _both(ctx, ("f32", 1, 4, 2, 300), 0.5, seed=13)
        # a shape beyond the fixed scratch is refused before anything is enqueued
        big = B.make_params((8, 128, 8192, 128), (8, 128, 8192, 128), torch.bfloat16, 0.5)
        assert B.tf_workspace_bytes(big) > B.TF_STATIC_SCRATCH_BYTES
        with pytest.raises(B.TokfiltError) as e:
            ctx.tf_filtered_attention_static(big, None, None, None, None, None, None, None, None)
        assert e.value.status == B.TF_ERR_UNSUPPORTED and "scratch" in ctx.tf_last_error()
    finally:
        ctx.close()
