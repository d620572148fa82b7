"""GPU parity of tw_reduce_add_rmsnorm / tw_split_launch against the fp64 oracle,
element by element, through the C ABI (TokenWeave, arXiv 2505.11329, Appendix A
Listing 1). Tolerance: |gpu - ref| <= 1e-2 |ref| + 1e-3 for both outputs; GPU vs
GPU comparisons (CU budgets, token split) are bit-exact."""
import numpy as np
import pytest

import oracle
import tw_workloads as W
from helpers import assert_parity, to_bits, to_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def upload(d):
    return dict(partials=[to_gpu(p) for p in d["partials"]], residual=to_gpu(d["residual"]),
                weight=to_gpu(d["weight"]), eps=d["eps"])


def run(tw, torch, g, cu_budget=0, **kw):
    out, res = tw.reduce_add_rmsnorm(g["partials"], g["residual"], g["weight"], g["eps"],
                                     cu_budget=cu_budget, **kw)
    torch.cuda.synchronize()
    return to_bits(out), to_bits(res)


def check_against_oracle(d, out_bits, res_bits, what, rows=None):
    parts, resid = d["partials"], d["residual"]
    if rows is not None:
        parts = [np.ascontiguousarray(p[rows]) for p in parts]
        resid = np.ascontiguousarray(resid[rows])
        out_bits, res_bits = out_bits[rows], res_bits[rows]
    ref_out, ref_res = oracle.fused(parts, resid, d["weight"], d["eps"])
    assert_parity(oracle.bf16_to_f64(res_bits), ref_res, what + " residual_out")
    assert_parity(oracle.bf16_to_f64(out_bits), ref_out, what + " out")


def small(N, H, P, seed=0, eps=1e-5):
    cfg = dict(N=N, H=H, P=P, partial_std=0.5, residual_std=1.0, outlier_frac=0.0, outlier_scale=1.0,
               eps=eps, seed=seed)
    return W.make_fused_inputs(cfg)


# ---- the five workload configurations at full size --------------------------

@pytest.mark.parametrize("name", ["c1_tiny", "c2_8b_tp2", "c3_70b_shard_tp8"])
def test_config_full_size(tw, torch_cuda, name):
    d = W.make_fused_inputs(name)
    budgets = W.CONFIGS[name].get("cu_budgets", (32, 0))
    g = upload(d)
    first = None
    for b in budgets:
        out, res = run(tw, torch_cuda, g, cu_budget=b)
        if first is None:
            check_against_oracle(d, out, res, "%s budget %d" % (name, b))
            first = (out, res)
        else:   # other budgets: same bits, so the same verdict
            assert np.array_equal(out, first[0]) and np.array_equal(res, first[1]), (name, b)


@pytest.mark.parametrize("N", [256, 1024, 4096, 16384])
def test_config4_split_sweep(tw, torch_cuda, N):
    torch = torch_cuda
    cfg = W.CONFIGS["c4_split_sweep_tp4"]
    d = W.make_fused_inputs(cfg, N=N)
    g = upload(d)
    k = tw.split_point(N, cfg["split_multiple"])
    assert k == N // 2
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    ref_bits = None
    for b in cfg["cu_budgets"]:
        out, res = run(tw, torch, g, cu_budget=b)
        o2, r2 = tw.split_launch(g["partials"], g["residual"], g["weight"], g["eps"], k, sa, sb, cu_budget=b)
        torch.cuda.synchronize()
        assert np.array_equal(to_bits(o2), out) and np.array_equal(to_bits(r2), res), (N, b)
        if ref_bits is None:
            ref_bits = (out, res)
        else:
            assert np.array_equal(out, ref_bits[0]) and np.array_equal(res, ref_bits[1])
    out, res = ref_bits
    if N <= 4096:
        check_against_oracle(d, out, res, "c4 N=%d" % N)
    else:   # the oracle takes sampled rows: both ends, the cut, and random ones
        rng = np.random.default_rng(0)
        rows = np.unique(np.concatenate([[0, 1, k - 1, k, k + 1, N - 2, N - 1], rng.integers(0, N, 200)]))
        check_against_oracle(d, out, res, "c4 N=%d sampled" % N, rows=rows)


def test_config5_fused_half(tw, torch_cuda):
    cfg = W.CONFIGS["c5_overlap_tp8"]
    d = W.make_fused_inputs(cfg)
    half = cfg["N"] // 2
    dA = dict(d, partials=[p[:half] for p in d["partials"]], residual=d["residual"][:half])
    g = upload(dA)
    out, res = run(tw, torch_cuda, g, cu_budget=32)
    check_against_oracle(dA, out, res, "c5 half A")


# ---- shapes that exercise every kernel geometry and ragged tails ---------------

SHAPES = [
    (1, 8, 1), (3, 24, 3), (5, 64, 2), (130, 512, 16), (1000, 64, 7), (17, 520, 5), (33, 1024, 4),
    (19, 4096, 8), (7, 8008, 2), (65, 8192, 1), (9, 8200, 2), (33, 16384, 4), (6, 24000, 8),
    (9, 32768, 2), (5, 40000, 3), (3, 65536, 1), (4, 65536, 8), (2049, 256, 2), (1025, 8192, 8),
    # rows of a whole number of waves that is not a power of two (5, 7, 10, 12, 14 waves; 10 and 12 x 2)
    (50, 2560, 8), (14, 3584, 2), (37, 5120, 8), (21, 6144, 2), (9, 7168, 4), (5, 10240, 8), (7, 12288, 2),
    (3, 20480, 4), (40, 1536, 3), (11, 4104, 8),
]


@pytest.mark.parametrize("N,H,P", SHAPES)
def test_shapes_and_tails(tw, torch_cuda, N, H, P):
    d = small(N, H, P, seed=N + H + P)
    g = upload(d)
    out, res = run(tw, torch_cuda, g, cu_budget=0)
    check_against_oracle(d, out, res, "N=%d H=%d P=%d" % (N, H, P))
    out2, res2 = run(tw, torch_cuda, g, cu_budget=3)
    assert np.array_equal(out, out2) and np.array_equal(res, res2)


@pytest.mark.parametrize("H,P", [(8192, 8), (8192, 4), (4096, 2), (2048, 8), (6144, 1), (520, 2)])
def test_decode_sized_whole_device_launches_on_both_sides_of_the_all_at_once_limit(tw, torch_cuda, H, P):
    """A whole-device launch of a few rows requests a row and the weights at once (inputs of at most
    6 MiB, at most one workgroup per compute unit); one row more than that, or the shared mode, takes
    the two-chunks-at-a-time form. Same bits either way, and the oracle's values."""
    limit = (6 << 20) // (H * 2 * (P + 1))
    for N in sorted({1, 2, 7, min(limit, 256), min(limit, 256) + 1}):
        d = small(N, H, P, seed=31 * N + H + P)
        g = upload(d)
        out, res = run(tw, torch_cuda, g, cu_budget=0)
        check_against_oracle(d, out, res, "decode-sized N=%d H=%d P=%d" % (N, H, P))
        for budget in (tw.CU_SHARED, 5):
            out2, res2 = run(tw, torch_cuda, g, cu_budget=budget)
            assert np.array_equal(out, out2) and np.array_equal(res, res2), (N, budget)


def test_every_p_from_1_to_16(tw, torch_cuda):
    for P in range(1, 17):
        d = small(40, 2048, P, seed=P)
        out, res = run(tw, torch_cuda, upload(d), cu_budget=5)
        check_against_oracle(d, out, res, "P=%d" % P)


# ---- determinism: budgets, split points, repeated runs -------------------------

def test_bits_do_not_depend_on_budget_or_split(tw, torch_cuda):
    torch = torch_cuda
    d = W.make_fused_inputs("c2_8b_tp2", N=777)
    g = upload(d)
    base = run(tw, torch, g, cu_budget=0)
    for b in (1, 2, 7, 8, 16, 32, 64, 255, 256, 1000):
        got = run(tw, torch, g, cu_budget=b)
        assert np.array_equal(got[0], base[0]) and np.array_equal(got[1], base[1]), b
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    for k in (0, 1, 2, 128, 389, 776, 777):
        o, r = tw.split_launch(g["partials"], g["residual"], g["weight"], g["eps"], k, sa, sb, cu_budget=16)
        torch.cuda.synchronize()
        assert np.array_equal(to_bits(o), base[0]) and np.array_equal(to_bits(r), base[1]), k
    # a row's bits do not depend on its position in the batch either
    sub = dict(partials=[p[100:300].contiguous() for p in g["partials"]],
               residual=g["residual"][100:300].contiguous(), weight=g["weight"], eps=g["eps"])
    got = run(tw, torch, sub, cu_budget=4)
    assert np.array_equal(got[0], base[0][100:300]) and np.array_equal(got[1], base[1][100:300])


def test_split_waits_for_parent_and_joins(tw, torch_cuda):
    """The inputs are produced on the parent stream right before the split launch
    and the outputs consumed on it right after: ordering comes from the fork/join."""
    torch = torch_cuda
    d = W.make_fused_inputs("c4_split_sweep_tp4", N=2048)
    g = upload(d)
    want = run(tw, torch, g, cu_budget=16)
    sa, sb, parent = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    stage = [torch.zeros_like(p) for p in g["partials"]]
    torch.cuda.synchronize()
    for _ in range(3):
        with torch.cuda.stream(parent):
            for s, p in zip(stage, g["partials"]):
                s.zero_()
                s.copy_(p)
            o, r = tw.split_launch(stage, g["residual"], g["weight"], g["eps"], 1024, sa, sb,
                                   cu_budget=16, parent=parent, use_parent=True, join=True)
            o_copy, r_copy = o.clone(), r.clone()
        parent.synchronize()
        assert np.array_equal(to_bits(o_copy), want[0]) and np.array_equal(to_bits(r_copy), want[1])


# ---- aliasing, special values, empty input ------------------------------------

@pytest.mark.parametrize("N,H,P", [(300, 4096, 4), (700, 8192, 8), (50, 6144, 3), (1000, 1024, 2), (2100, 8192, 1)])
def test_in_place_residual_and_out_over_a_partial(tw, torch_cuda, N, H, P):
    """The paper's in-place form in every launch mode: the residual stream updated in place and the output
    written over one of the partials. Both kernels store a row's outputs only after all of its inputs have
    been loaded by the very threads that store them, with loads of later rows already in flight."""
    torch = torch_cuda
    d = small(N, H, P, seed=3)
    want = run(tw, torch, upload(d), cu_budget=8)
    check_against_oracle(d, want[0], want[1], "in-place reference N=%d H=%d P=%d" % (N, H, P))
    for budget in (8, 0, tw.CU_SHARED):
        g2 = upload(d)
        over = g2["partials"][P - 1]
        out, res = tw.reduce_add_rmsnorm(g2["partials"], g2["residual"], g2["weight"], g2["eps"], cu_budget=budget,
                                         out=over, residual_out=g2["residual"])
        torch.cuda.synchronize()
        assert out.data_ptr() == over.data_ptr() and res.data_ptr() == g2["residual"].data_ptr()
        assert np.array_equal(to_bits(out), want[0]) and np.array_equal(to_bits(res), want[1]), budget


def test_non_finite_values_stay_in_their_row(tw, torch_cuda):
    d = small(6, 1024, 2, seed=5)
    d["partials"][0][1, 3] = 0x7F80      # +Inf
    d["partials"][1][2, 700] = 0x7FC0    # NaN
    d["residual"][4, 9] = 0xFF80         # -Inf
    out, res = run(tw, torch_cuda, upload(d), cu_budget=2)
    check_against_oracle(d, out, res, "non-finite")
    ref_out, _ = oracle.fused(d["partials"], d["residual"], d["weight"], d["eps"])
    assert np.isfinite(ref_out[[0, 3, 5]]).all()
    assert np.isfinite(oracle.bf16_to_f64(out)[[0, 3, 5]]).all()


def test_zero_rows_and_zero_eps(tw, torch_cuda):
    d = small(4, 512, 2, seed=6, eps=0.0)
    for p in d["partials"]:
        p[2, :] = 0
    d["residual"][2, :] = 0
    out, res = run(tw, torch_cuda, upload(d), cu_budget=1)
    check_against_oracle(d, out, res, "eps=0 with a zero row")      # NaN row in both
    assert np.isnan(oracle.bf16_to_f64(out)[2]).all()
    d["eps"] = 1e-6
    out, res = run(tw, torch_cuda, upload(d), cu_budget=1)
    assert (oracle.bf16_to_f64(out)[2] == 0).all()
    check_against_oracle(d, out, res, "eps>0 with a zero row")


def test_empty_batch(tw, torch_cuda):
    torch = torch_cuda
    z = torch.empty((0, 512), dtype=torch.bfloat16, device="cuda:0")
    w = torch.ones(512, dtype=torch.bfloat16, device="cuda:0")
    out, res = tw.reduce_add_rmsnorm([z, z], z, w, 1e-5)
    torch.cuda.synchronize()
    assert out.shape == (0, 512) and res.shape == (0, 512)


def test_large_values_and_outliers(tw, torch_cuda):
    """Residual stream with x50 outliers and partials near the top of bf16 range
    scaled down so that the sum of squares stays finite in fp32."""
    cfg = dict(W.CONFIGS["c3_70b_shard_tp8"], N=64)
    d = W.make_fused_inputs(cfg)
    big = W.f32_to_bf16_bits(W.bf16_bits_to_f32(d["residual"]) * np.float32(2.0 ** 40))
    d["residual"] = big
    out, res = run(tw, torch_cuda, upload(d), cu_budget=8)
    check_against_oracle(d, out, res, "large magnitudes")


def test_batch_longer_than_one_launch_can_address(tw, torch_cuda):
    """More than 2 GiB per tensor goes out as several launches; rows around the
    seam and at both ends are checked against the oracle. Inputs are drawn on the
    GPU (seeded) because the host generator would take minutes at this size."""
    torch = torch_cuda
    H, P = 8192, 1
    N = (1 << 31) // (H * 2) + 300
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(1234)
    part = torch.empty((N, H), device="cuda:0", dtype=torch.bfloat16).normal_(0.0, 0.5, generator=gen)
    resid = torch.empty((N, H), device="cuda:0", dtype=torch.bfloat16).normal_(0.0, 1.0, generator=gen)
    w = to_gpu(W.uniform_bf16((H,), 0.5, 1.5, 0, W.STREAM_WEIGHT))
    out, res = tw.reduce_add_rmsnorm([part], resid, w, 1e-5, cu_budget=0)
    torch.cuda.synchronize()
    seam = (1 << 31) // (H * 2)
    rows = np.array([0, 1, seam - 2, seam - 1, seam, seam + 1, N - 2, N - 1, 777, 99999])
    idx = torch.from_numpy(rows).to("cuda:0")
    d = dict(partials=[to_bits(part[idx])], residual=to_bits(resid[idx]), weight=to_bits(w), eps=1e-5)
    check_against_oracle(d, to_bits(out[idx]), to_bits(res[idx]), "multi-launch batch")
    # the same batch through the unfused pipeline (also cut into several launches) and through the
    # shared mode, on the same sampled rows
    o3, r3 = tw.reduce_add_rmsnorm([part], resid, w, 1e-5, cu_budget=tw.CU_SHARED)
    torch.cuda.synchronize()
    assert torch.equal(o3[idx], out[idx]) and torch.equal(r3[idx], res[idx])
    del o3, r3
    o2, r2 = tw.reduce_add_rmsnorm_unfused([part], resid, w, 1e-5)
    torch.cuda.synchronize()
    ref_out, ref_res = oracle.unfused(d["partials"], d["residual"], d["weight"], d["eps"])
    assert_parity(oracle.bf16_to_f64(to_bits(o2[idx])), ref_out, "multi-launch unfused out")
    assert np.array_equal(to_bits(r2[idx]), oracle.f64_to_bf16(ref_res))


@pytest.mark.parametrize("N,H,P", [(8200, 8192, 8), (8195, 8192, 2), (16500, 4096, 4), (5500, 12288, 3)])
def test_outputs_larger_than_the_last_level_cache(tw, torch_cuda, N, H, P):
    """Calls whose two outputs exceed 256 MiB take the kernels that store with the streaming policy when
    they run on the whole device or in shared mode, and the ordinary ones under a CU budget: the same
    bits from all three (every element), and the oracle's on sampled rows. Inputs drawn on the GPU."""
    torch = torch_cuda
    assert 2 * N * H * 2 >= 256 << 20
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(N + P)
    parts = [torch.empty((N, H), device="cuda:0", dtype=torch.bfloat16).normal_(0.0, 0.5, generator=gen)
             for _ in range(P)]
    resid = torch.empty((N, H), device="cuda:0", dtype=torch.bfloat16).normal_(0.0, 1.0, generator=gen)
    w = to_gpu(W.uniform_bf16((H,), 0.5, 1.5, 0, W.STREAM_WEIGHT))
    want = tw.reduce_add_rmsnorm(parts, resid, w, 1e-5, cu_budget=16)
    torch.cuda.synchronize()
    for budget in (0, tw.CU_SHARED):
        out, res = tw.reduce_add_rmsnorm(parts, resid, w, 1e-5, cu_budget=budget)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), want[0].view(torch.int16)), budget
        assert torch.equal(res.view(torch.int16), want[1].view(torch.int16)), budget
        del out, res
    rng = np.random.default_rng(N)
    rows = np.unique(np.concatenate([[0, 1, N - 2, N - 1], rng.integers(0, N, 60)]))
    idx = torch.from_numpy(rows).to("cuda:0")
    d = dict(partials=[to_bits(p[idx]) for p in parts], residual=to_bits(resid[idx]), weight=to_bits(w), eps=1e-5)
    check_against_oracle(d, to_bits(want[0][idx]), to_bits(want[1][idx]), "large outputs N=%d H=%d P=%d" % (N, H, P))


def test_traced_launch_reports_distinct_compute_units(tw, torch_cuda):
    """Each workgroup of a budgeted launch sits on its own compute unit: the
    (XCC, SE, CU) triples decoded from the hardware id registers are distinct and
    as many as the budget."""
    torch = torch_cuda
    d = W.make_fused_inputs("c3_70b_shard_tp8", N=512)
    g = upload(d)
    want = run(tw, torch, g, cu_budget=32)
    for budget in (8, 32, 64):
        out, res, hw = tw.reduce_add_rmsnorm_traced(g["partials"], g["residual"], g["weight"], g["eps"],
                                                    cu_budget=budget)
        torch.cuda.synchronize()
        assert np.array_equal(to_bits(out), want[0]) and np.array_equal(to_bits(res), want[1])
        hw = hw.cpu().numpy().astype(np.int64) & 0xFFFFFFFF
        assert hw.shape[0] == budget
        cu = (hw[:, 0] >> 8) & 0xF
        se = (hw[:, 0] >> 13) & 0x7
        sh = (hw[:, 0] >> 12) & 0x1
        xcc = hw[:, 1] & 0xF
        places = set(zip(xcc.tolist(), se.tolist(), sh.tolist(), cu.tolist()))
        assert len(places) == budget, "workgroups shared a compute unit: %d places for %d workgroups" % (
            len(places), budget)


# ---- shared (co-resident) launch mode: same bits as the budgeted kernel --------

SHARED_SHAPES = [(1, 8, 1), (3, 24, 3), (1000, 64, 7), (130, 512, 16), (17, 520, 5), (33, 1024, 4),
                 (300, 2048, 2), (19, 4096, 8), (77, 4096, 2), (7, 8008, 2), (65, 8192, 1), (1025, 8192, 8),
                 (9, 8200, 2), (5, 16384, 4), (50, 2560, 8), (14, 3584, 2), (37, 5120, 8), (21, 6144, 2),
                 (9, 7168, 4), (300, 6144, 8), (11, 4104, 8), (40, 1536, 3)]


@pytest.mark.parametrize("N,H,P", SHARED_SHAPES)
def test_shared_mode_same_bits_as_budgeted(tw, torch_cuda, N, H, P):
    d = small(N, H, P, seed=7 * N + H + P)
    g = upload(d)
    want = run(tw, torch_cuda, g, cu_budget=16)
    got = run(tw, torch_cuda, g, cu_budget=tw.CU_SHARED)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
    if N * H <= 1 << 20:
        check_against_oracle(d, got[0], got[1], "shared N=%d H=%d P=%d" % (N, H, P))


@pytest.mark.parametrize("name,N", [("c2_8b_tp2", None), ("c3_70b_shard_tp8", None), ("c4_split_sweep_tp4", 4096)])
def test_shared_mode_on_configs_and_split(tw, torch_cuda, name, N):
    torch = torch_cuda
    d = W.make_fused_inputs(name, N=N)
    g = upload(d)
    want = run(tw, torch, g, cu_budget=32)
    got = run(tw, torch, g, cu_budget=tw.CU_SHARED)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    k = tw.split_point(d["N"], 128)
    o, r = tw.split_launch(g["partials"], g["residual"], g["weight"], g["eps"], k, sa, sb, cu_budget=tw.CU_SHARED)
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(o), want[0]) and np.array_equal(to_bits(r), want[1])
    # in place, as the paper's kernel updates the residual stream
    g2 = upload(d)
    o, r = tw.reduce_add_rmsnorm(g2["partials"], g2["residual"], g2["weight"], g2["eps"], cu_budget=tw.CU_SHARED,
                                 out=g2["partials"][0], residual_out=g2["residual"])
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(o), want[0]) and np.array_equal(to_bits(r), want[1])


# ---- the unfused three-pass pipeline (ablation) against its own oracle ----------

def assert_stream_is_one_of_the_two_readings(d, res_bits, ref_res):
    """The all-reduce stage's rounding decides a bf16 value. The paper does not say in which precision
    that sum is accumulated, so the oracle has two readings of it (exact sum, or binary32 in rank order,
    each rounded once); they part only where a rounding boundary lies between the two sums. Every stored
    element must carry the bits of one of them, and almost all those of the exact reading."""
    exact = oracle.f64_to_bf16(ref_res)
    _, alt_res = oracle.unfused_f32sum(d["partials"], d["residual"], d["weight"], d["eps"])
    alt = oracle.f64_to_bf16(alt_res)
    is_exact, is_alt = res_bits == exact, res_bits == alt
    assert np.all(is_exact | is_alt), "%d elements match neither reading" % int((~(is_exact | is_alt)).sum())
    assert (~is_exact).mean() <= 1e-3


UNFUSED_SHAPES = [(1, 8, 1), (3, 24, 3), (64, 512, 2), (130, 520, 5), (33, 2048, 4), (77, 4096, 2),
                  (19, 6152, 7), (65, 8192, 8), (300, 8192, 16)]


@pytest.mark.parametrize("N,H,P", UNFUSED_SHAPES)
def test_unfused_pipeline_matches_its_oracle(tw, torch_cuda, N, H, P):
    d = small(N, H, P, seed=N + H + P)
    g = upload(d)
    scratch = torch_cuda.full((N, H), float("nan"), dtype=torch_cuda.bfloat16, device="cuda:0")
    out, res = tw.reduce_add_rmsnorm_unfused(g["partials"], g["residual"], g["weight"], g["eps"],
                                             sum_scratch=scratch)
    torch_cuda.cuda.synchronize()
    ref_out, ref_res = oracle.unfused(d["partials"], d["residual"], d["weight"], d["eps"])
    assert_parity(oracle.bf16_to_f64(to_bits(out)), ref_out, "unfused out N=%d H=%d P=%d" % (N, H, P))
    assert_parity(oracle.bf16_to_f64(to_bits(res)), ref_res, "unfused residual N=%d H=%d P=%d" % (N, H, P))
    assert_stream_is_one_of_the_two_readings(d, to_bits(res), ref_res)


def test_unfused_pipeline_on_the_headline_config_and_in_place(tw, torch_cuda):
    torch = torch_cuda
    d = W.make_fused_inputs("c3_70b_shard_tp8")
    g = upload(d)
    ref_out, ref_res = oracle.unfused(d["partials"], d["residual"], d["weight"], d["eps"])
    out, res = tw.reduce_add_rmsnorm_unfused(g["partials"], g["residual"], g["weight"], g["eps"])
    torch.cuda.synchronize()
    assert_parity(oracle.bf16_to_f64(to_bits(out)), ref_out, "unfused c3 out")
    assert_parity(oracle.bf16_to_f64(to_bits(res)), ref_res, "unfused c3 residual")
    assert_stream_is_one_of_the_two_readings(d, to_bits(res), ref_res)
    # paper's in-place form: residual updated in place, result written over a partial
    want_out, want_res = to_bits(out), to_bits(res)
    out2, res2 = tw.reduce_add_rmsnorm_unfused(g["partials"], g["residual"], g["weight"], g["eps"],
                                               out=g["partials"][0], residual_out=g["residual"])
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(out2), want_out) and np.array_equal(to_bits(res2), want_res)


# ---- randomized shapes: every launch mode against the oracle and each other ------

def test_random_shapes_all_modes_agree(tw, torch_cuda):
    """Seeded random (N, H, P): whole device, a small budget, the shared mode and a
    two-stream split must give the same bits, and those bits must match the oracle."""
    torch = torch_cuda
    rng = np.random.default_rng(20250511)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    for case in range(40):
        H = 8 * int(rng.integers(1, 1200)) if case % 4 else 8 * int(rng.integers(1, 64))
        N = int(rng.integers(1, 400)) if H <= 4096 else int(rng.integers(1, 60))
        P = int(rng.integers(1, 17))
        d = small(N, H, P, seed=1000 + case, eps=float(rng.choice([0.0, 1e-6, 1e-5, 1e-2])))
        g = upload(d)
        what = "case %d: N=%d H=%d P=%d" % (case, N, H, P)
        want = run(tw, torch, g, cu_budget=0)
        check_against_oracle(d, want[0], want[1], what)
        for budget in (int(rng.integers(1, 9)), tw.CU_SHARED):
            got = run(tw, torch, g, cu_budget=budget)
            assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1]), (what, budget)
        k = int(rng.integers(0, N + 1))
        o2, r2 = tw.split_launch(g["partials"], g["residual"], g["weight"], g["eps"], k, sa, sb,
                                 cu_budget=int(rng.integers(1, 9)))
        torch.cuda.synchronize()
        assert np.array_equal(to_bits(o2), want[0]) and np.array_equal(to_bits(r2), want[1]), (what, "split", k)


# ---- several host threads at once -------------------------------------------------

def test_split_launch_from_four_host_threads(tw, torch_cuda):
    """Calls may come from several host threads: four threads, each with its own parent and split
    streams and its own tensors, each making 200 split launches whose halves must wait for work
    enqueued on the parent just before (the inputs are rewritten there every time) and whose outputs
    the parent reads just after. A wait that ordered against another thread's stream would let a half
    run on stale inputs or let the parent read an unfinished output."""
    import threading
    torch = torch_cuda
    n_threads, n_calls = 4, 200
    failures = []

    def worker(t):
        try:
            N, H, P = 96 + 32 * t, 2048, 2
            d = small(N, H, P, seed=500 + t)
            g = upload(d)
            want_out, want_res = tw.reduce_add_rmsnorm(g["partials"], g["residual"], g["weight"], g["eps"])
            master = g["partials"][0].clone()
            parent, sa, sb = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
            out, res = torch.empty_like(want_out), torch.empty_like(want_res)
            bad = torch.zeros((), dtype=torch.int32, device="cuda:0")
            torch.cuda.synchronize()
            k = tw.split_point(N, 32)
            for i in range(n_calls):
                with torch.cuda.stream(parent):
                    g["partials"][0].zero_()
                    out.zero_()
                    g["partials"][0].copy_(master)
                tw.split_launch(g["partials"], g["residual"], g["weight"], g["eps"], k, sa, sb, cu_budget=4 + t,
                                out=out, residual_out=res, parent=parent, join=True)
                with torch.cuda.stream(parent):
                    bad += (out.view(torch.int16) != want_out.view(torch.int16)).any().to(torch.int32)
                    bad += (res.view(torch.int16) != want_res.view(torch.int16)).any().to(torch.int32)
                if i % 25 == 24 or i == n_calls - 1:
                    parent.synchronize()
                    if int(bad.item()) != 0:
                        failures.append("thread %d: outputs differ by call %d" % (t, i))
                        return
        except Exception as e:  # noqa: BLE001 - reported to the main thread
            failures.append("thread %d: %r" % (t, e))

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(n_threads)]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=100)
    assert not any(th.is_alive() for th in threads), "a worker thread did not finish"
    torch.cuda.synchronize()
    assert not failures, failures
