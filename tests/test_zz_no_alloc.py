"""The entry point that allocates nothing (tw_reduce_add_rmsnorm_unfused_static) against the entry
point it is a variant of (tw_reduce_add_rmsnorm_unfused, caller's workspace): same bits, on two calls
in a row that share the library's built-in buffer, the second with a smaller input."""
import numpy as np
import pytest

import tw_workloads as W
from helpers import to_bits, to_gpu

pytestmark = pytest.mark.gpu


def _case(tw, torch, N, H, P, seed):
    cfg = dict(N=N, H=H, P=P, partial_std=0.5, residual_std=1.0, outlier_frac=0.0, outlier_scale=1.0,
               eps=1e-5, seed=seed)
    d = W.make_fused_inputs(cfg)
    parts = [to_gpu(p) for p in d["partials"]]
    resid, w = to_gpu(d["residual"]), to_gpu(d["weight"])
    return d, parts, resid, w


def test_static_scratch_entry_point_matches_the_workspace_one(tw):
    import torch
    assert torch.cuda.is_available()
    # first call: a batch that fills the buffer to the last byte (2048 x 8192 bf16 = 32 MiB);
    # second call: a smaller one, whose rows land on the first call's leftovers
    for (N, H, P, seed) in [(tw.STATIC_SCRATCH_BYTES // (8192 * 2), 8192, 8, 11), (77, 4096, 2, 12),
                            (3, 24, 3, 13)]:
        print("no-alloc case N=%d H=%d P=%d" % (N, H, P), flush=True)
        d, parts, resid, w = _case(tw, torch, N, H, P, seed)
        want_out, want_res = tw.reduce_add_rmsnorm_unfused(parts, resid, w, d["eps"])
        out = torch.full_like(resid, float("nan"))
        res = torch.full_like(resid, float("nan"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated(), torch.cuda.memory_reserved()
        tw.reduce_add_rmsnorm_unfused_static(parts, resid, w, d["eps"], out, res)
        torch.cuda.synchronize()
        assert (torch.cuda.memory_allocated(), torch.cuda.memory_reserved()) == before
        assert np.array_equal(to_bits(out), to_bits(want_out)), "out differs at N=%d H=%d P=%d" % (N, H, P)
        assert np.array_equal(to_bits(res), to_bits(want_res)), "residual_out differs at N=%d H=%d P=%d" % (N, H, P)


def test_static_scratch_entry_point_refuses_what_does_not_fit(tw):
    import torch
    N = tw.STATIC_SCRATCH_BYTES // (8192 * 2) + 1
    z = torch.zeros((N, 8192), dtype=torch.bfloat16, device="cuda:0")
    w = torch.ones(8192, dtype=torch.bfloat16, device="cuda:0")
    out, res = torch.empty_like(z), torch.empty_like(z)
    with pytest.raises(tw.TwError) as e:
        tw.reduce_add_rmsnorm_unfused_static([z], z, w, 1e-5, out, res)
    assert e.value.status == 2      # TW_ERR_SHAPE
