"""tw_weave_layer: the chain G1 -> fused -> G2 over two token splits on two
streams (TokenWeave Fig. 7b). Each stage is checked against the fp64 oracle fed
with the bits the previous GPU stage produced, and every split row must give the
same bits as the unsplit chain."""
import numpy as np
import pytest

import oracle
import tw_workloads as W
from helpers import assert_parity, to_bits, to_gpu

pytestmark = pytest.mark.gpu

T, K1, H, P, N2 = 640, 512, 1024, 4, 768
STD = 0.15


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available()
    return torch


def gemm_tol_check(got, ref, K, sa, sb, what):
    tol = 1e-2 * np.abs(ref) + 1e-3 * np.sqrt(K) * sa * sb
    bad = np.abs(got - ref) > tol
    assert not bad.any(), "%s: %d of %d out of tolerance" % (what, bad.sum(), bad.size)


def make_inputs():
    g1 = W.make_gemm_inputs(T, K1, H, STD, seed=3, b_layout="nk")
    cfg = dict(N=T, H=H, P=P, partial_std=0.5, residual_std=1.0, outlier_frac=0.01, outlier_scale=20.0,
               eps=1e-5, seed=5)
    f = W.make_fused_inputs(cfg)
    W2 = W.normal_bf16((N2, H), 0.05, 9, W.STREAM_GEMM_B)
    return g1, f, W2


def run_layer(tw, torch, g1, f, W2, split_row, streams, parent=None, budgets=(32, 224), schedule=1):
    X1, W1 = to_gpu(g1["A"]), to_gpu(g1["B"])
    parts = [torch.zeros((T, H), dtype=torch.bfloat16, device="cuda:0")] + [to_gpu(p) for p in f["partials"][1:]]
    out, res, Y = tw.weave_layer(X1, W1, parts, to_gpu(f["residual"]), to_gpu(f["weight"]), f["eps"], to_gpu(W2),
                                 split_row, streams[0], streams[1], fused_cu_budget=budgets[0],
                                 gemm_cu_budget=budgets[1], parent=parent, use_parent=True, join=True,
                                 schedule=schedule)
    torch.cuda.synchronize()
    return to_bits(parts[0]), to_bits(out), to_bits(res), to_bits(Y)


def test_weave_layer_stagewise_parity_and_split_invariance(tw, torch_cuda):
    torch = torch_cuda
    g1, f, W2 = make_inputs()
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    C0, out0, res0, Y0 = run_layer(tw, torch, g1, f, W2, 0, streams)

    # G1 against the textbook product
    gemm_tol_check(oracle.bf16_to_f64(C0), oracle.gemm(g1["A"], g1["B"], "nk"), K1, STD, STD, "G1")
    # F against the fused oracle on the bits G1 produced
    ref_out, ref_res = oracle.fused([C0] + f["partials"][1:], f["residual"], f["weight"], f["eps"])
    assert_parity(oracle.bf16_to_f64(res0), ref_res, "weave residual_out")
    assert_parity(oracle.bf16_to_f64(out0), ref_out, "weave out")
    # G2 against the textbook product on the bits F produced (|out| ~ 1)
    gemm_tol_check(oracle.bf16_to_f64(Y0), oracle.gemm(out0, W2, "nk"), H, 1.5, 0.05, "G2")

    for k in (T, 256, 512, 384, 1, T - 1, 320):
        C, out, res, Y = run_layer(tw, torch, g1, f, W2, k, streams)
        assert np.array_equal(C, C0) and np.array_equal(out, out0), k
        assert np.array_equal(res, res0) and np.array_equal(Y, Y0), k
    # the other schedule (one chain per split) and the library's own choice, with the fused kernel
    # confined to a budget, co-resident, and on the whole device
    for schedule in (tw.WEAVE_CHAINS, tw.WEAVE_AUTO):
        for budgets in ((32, 224), (tw.CU_SHARED, 0), (0, 0)):
            for k in (256, 100, T - 1):
                C, out, res, Y = run_layer(tw, torch, g1, f, W2, k, streams, budgets=budgets, schedule=schedule)
                assert np.array_equal(C, C0) and np.array_equal(out, out0), (schedule, budgets, k)
                assert np.array_equal(res, res0) and np.array_equal(Y, Y0), (schedule, budgets, k)


def test_weave_layer_cuts_any_number_of_splits_gives_the_unsplit_bits(tw, torch_cuda):
    """tw_weave_layer_cuts: two, three (an odd split at the end), five and sixteen splits, ragged and
    one-row pieces, in both schedules and the three launch modes of the fused step, launched behind a
    parent stream that still holds the writing of an input; every output carries the bits of the
    unsplit chain (which the stagewise test checks against the oracle on these very inputs)."""
    torch = torch_cuda
    g1, f, W2 = make_inputs()
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    want = run_layer(tw, torch, g1, f, W2, 0, streams)
    X1_src, W1 = to_gpu(g1["A"]), to_gpu(g1["B"])
    resid, weight, W2g = to_gpu(f["residual"]), to_gpu(f["weight"]), to_gpu(W2)
    parent = torch.cuda.Stream()
    cut_sets = ([], [320], [256, 512], [1, 2, 639], [128, 256, 384, 512], [100, 228, 229, 600],
                list(range(40, 640, 40)))
    assert len(cut_sets[-1]) == 15
    for schedule in (tw.WEAVE_ORDERED, tw.WEAVE_CHAINS, tw.WEAVE_AUTO):
        for budgets in ((32, 224), (tw.CU_SHARED, 0), (0, 0)):
            for cuts in cut_sets:
                X1 = torch.zeros_like(X1_src)
                parts = [torch.full((T, H), float("nan"), dtype=torch.bfloat16, device="cuda:0")] + \
                        [to_gpu(p) for p in f["partials"][1:]]
                torch.cuda.synchronize()
                with torch.cuda.stream(parent):
                    X1.copy_(X1_src)            # the call must wait for this
                out, res, Y = tw.weave_layer_cuts(X1, W1, parts, resid, weight, f["eps"], W2g, cuts, streams[0],
                                                  streams[1], fused_cu_budget=budgets[0], gemm_cu_budget=budgets[1],
                                                  parent=parent, use_parent=True, join=True, schedule=schedule)
                parent.synchronize()            # joined: everything is done once the parent is
                got = (to_bits(parts[0]), to_bits(out), to_bits(res), to_bits(Y))
                for name, g_, w_ in zip(("G1", "out", "residual_out", "Y"), got, want):
                    assert np.array_equal(g_, w_), (schedule, budgets, cuts, name)


@pytest.mark.parametrize("schedule", [1, 2])   # TW_WEAVE_ORDERED, TW_WEAVE_CHAINS
def test_weave_layer_orders_itself_after_the_parent_stream(tw, torch_cuda, schedule):
    torch = torch_cuda
    g1, f, W2 = make_inputs()
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    want = run_layer(tw, torch, g1, f, W2, 0, streams)
    parent = torch.cuda.Stream()
    X1_src, W1 = to_gpu(g1["A"]), to_gpu(g1["B"])
    X1 = torch.zeros_like(X1_src)
    parts = [torch.zeros((T, H), dtype=torch.bfloat16, device="cuda:0")] + [to_gpu(p) for p in f["partials"][1:]]
    resid, weight, W2g = to_gpu(f["residual"]), to_gpu(f["weight"]), to_gpu(W2)
    torch.cuda.synchronize()
    for _ in range(3):
        with torch.cuda.stream(parent):
            X1.zero_()
            X1.copy_(X1_src)             # the input is produced on the parent right before the launch
            out, res, Y = tw.weave_layer(X1, W1, parts, resid, weight, f["eps"], W2g, 384, streams[0], streams[1],
                                         fused_cu_budget=32, gemm_cu_budget=224, parent=parent, schedule=schedule)
            yc, oc = Y.clone(), out.clone()   # and consumed on it right after
        parent.synchronize()
        assert np.array_equal(to_bits(yc), want[3]) and np.array_equal(to_bits(oc), want[1])


@pytest.mark.parametrize("K1,N2", [(1024, 3584), (3584, 1280)])
def test_weave_layer_at_full_size_gives_the_unsplit_bits_every_time(tw, torch_cuda, K1, N2):
    """The two block boundaries of the 70B-class layer at T = 4096 (H = 8192, P = 8),
    co-resident mode, both schedules, several cuts, a dozen launches each: every
    output must carry the unsplit chain's bits. At this size the kernels really
    overlap for tens of microseconds, which is when a missing wait or a misplaced
    event shows; the outputs start as NaNs so that nothing stale can pass. Inputs
    are drawn on the GPU (seeded); the unsplit chain is the reference, and it is
    itself checked against the oracle on sampled outputs first."""
    torch = torch_cuda
    T_, H_, P_ = 4096, 8192, 8
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(K1 + N2)

    def rnd(shape, std):
        return torch.empty(shape, dtype=torch.bfloat16, device="cuda:0").normal_(0.0, std, generator=gen)
    X1, W1, W2g = rnd((T_, K1), 0.02), rnd((H_, K1), 0.02), rnd((N2, H_), 0.02)
    parts, resid = [rnd((T_, H_), 0.25) for _ in range(P_)], rnd((T_, H_), 1.0)
    weight = to_gpu(W.uniform_bf16((H_,), 0.5, 1.5, 0, W.STREAM_WEIGHT))
    out, res = torch.empty_like(resid), torch.empty_like(resid)
    Y = torch.empty((T_, N2), dtype=torch.bfloat16, device="cuda:0")
    sx, sc = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()

    def run(split_row, schedule):
        with torch.cuda.stream(sx):
            for t in (parts[0], out, res, Y):
                t.fill_(float("nan"))
            tw.weave_layer(X1, W1, parts, resid, weight, 1e-5, W2g, split_row, sx, sc, fused_cu_budget=tw.CU_SHARED,
                           gemm_cu_budget=0, out=out, residual_out=res, Y=Y, parent=sx, use_parent=True, join=True,
                           schedule=schedule)
        torch.cuda.synchronize()
        return [to_bits(t).copy() for t in (parts[0], out, res, Y)]
    want = run(0, tw.WEAVE_ORDERED)
    assert not np.isnan(oracle.bf16_to_f64(want[3])).any()

    # The reference itself against the oracle at this size, stage by stage on sampled outputs, each
    # stage fed with the bits the previous GPU stage produced: 2048 cells of G1, 192 whole rows of the
    # fused step, 2048 cells of G2 (the rows straddle every 256-row GEMM tile and both halves).
    rng = np.random.default_rng(K1 * 7 + N2)
    rows = np.unique(np.concatenate([rng.integers(0, T_, 180), [0, 1, 255, 256, 2047, 2048, T_ - 2, T_ - 1]]))[:192]
    ridx = torch.from_numpy(rows).to("cuda:0")
    ms = rng.integers(0, len(rows), 2048)
    G1_rows, out_rows, res_rows, Y_rows = (w_[rows] for w_ in want)
    ns = rng.integers(0, H_, 2048)
    ref = oracle.gemm_samples(to_bits(X1[ridx]), to_bits(W1), "nk", ms, ns)
    gemm_tol_check(oracle.bf16_to_f64(G1_rows[ms, ns]), ref, K1, 0.02, 0.02, "G1 at T=4096 (sampled)")
    ref_out, ref_res = oracle.fused([G1_rows] + [to_bits(p[ridx]) for p in parts[1:]], to_bits(resid[ridx]),
                                    to_bits(weight), 1e-5)
    assert_parity(oracle.bf16_to_f64(res_rows), ref_res, "weave residual_out at T=4096 (sampled rows)")
    assert_parity(oracle.bf16_to_f64(out_rows), ref_out, "weave out at T=4096 (sampled rows)")
    ns = rng.integers(0, N2, 2048)
    ref = oracle.gemm_samples(out_rows, to_bits(W2g), "nk", ms, ns)
    gemm_tol_check(oracle.bf16_to_f64(Y_rows[ms, ns]), ref, H_, 1.1, 0.02, "G2 at T=4096 (sampled)")

    k_smart = tw.smart_split_point(T_, 64, [H_, N2], tw.device_cu_count(), gemm_k=[K1, H_])[0]
    for it in range(12):
        schedule = (tw.WEAVE_ORDERED, tw.WEAVE_CHAINS)[it % 2]
        k = (k_smart, 2048 + 64 * (it % 5), 128 * (1 + it % 7))[it % 3]
        got = run(k, schedule)
        for name, g_, w_ in zip(("G1", "out", "residual_out", "Y"), got, want):
            assert np.array_equal(g_, w_), (it, schedule, k, name, int((g_ != w_).sum()))


# ---- the per-iteration policy as one call (Fig. 3) ---------------------------------

def test_weave_layer_auto_applies_threshold_and_smart_split(tw, torch_cuda):
    """Below the threshold the chain runs unsplit, at or above it the batch is cut where
    tw_smart_split_point says; either way the bits are the unsplit chain's (which the stagewise test
    above checks against the oracle on these very inputs)."""
    torch = torch_cuda
    g1, f, W2 = make_inputs()
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    want = run_layer(tw, torch, g1, f, W2, 0, streams)
    cus = tw.device_cu_count()
    for threshold, multiple, budgets in ((T + 1, 64, (tw.CU_SHARED, 0)), (T, 64, (tw.CU_SHARED, 0)), (512, 32, (32, 224)),
                                         (1, 0, (0, 0))):
        X1, W1 = to_gpu(g1["A"]), to_gpu(g1["B"])
        parts = [torch.zeros((T, H), dtype=torch.bfloat16, device="cuda:0")] + [to_gpu(p) for p in f["partials"][1:]]
        out, res, Y, taken = tw.weave_layer_auto(X1, W1, parts, to_gpu(f["residual"]), to_gpu(f["weight"]), f["eps"],
                                                 to_gpu(W2), streams[0], streams[1], threshold=threshold,
                                                 multiple=multiple, fused_cu_budget=budgets[0],
                                                 gemm_cu_budget=budgets[1])
        torch.cuda.synchronize()
        if T < threshold:
            assert taken == T
        else:
            gemm_cus = budgets[1] if 0 < budgets[1] < cus else cus
            assert taken == tw.smart_split_point(T, multiple or 64, [H, N2], gemm_cus, gemm_k=[K1, H])[0]
            assert 0 < taken < T
        got = (to_bits(parts[0]), to_bits(out), to_bits(res), to_bits(Y))
        for name, g_, w_ in zip(("G1", "out", "residual_out", "Y"), got, want):
            assert np.array_equal(g_, w_), (threshold, name)


@pytest.mark.parametrize("K1,N2", [(1024, 3584), (3584, 1280)])
def test_weave_layer_auto_at_full_size_on_both_sides_of_the_built_in_threshold(tw, torch_cuda, K1, N2):
    """The two 70B-class boundaries (H = 8192, P = 8) with the library's own rule: a batch below half the
    threshold, two between half of it and it (one whose cut costs no GEMM waves and is split, one whose
    cut does and is not), one at the threshold, one above (the MLP-side boundary, which the built-in rule
    never splits, is run at the same sizes); the policy's outputs carry the bits of the plain unsplit
    chain."""
    torch = torch_cuda
    H_, P_ = 8192, 8
    never = 2 ** 63 - 1
    thr = tw.split_threshold(K1, H_, P_, N2, tw.device_cu_count())
    assert thr == (8192 if K1 == 1024 else never)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(K1 * 3 + N2)

    def rnd(shape, std):
        return torch.empty(shape, dtype=torch.bfloat16, device="cuda:0").normal_(0.0, std, generator=gen)
    T_max = 8192 + 640
    X1, W1, W2g = rnd((T_max, K1), 0.02), rnd((H_, K1), 0.02), rnd((N2, H_), 0.02)
    parts, resid = [rnd((T_max, H_), 0.25) for _ in range(P_)], rnd((T_max, H_), 1.0)
    weight = to_gpu(W.uniform_bf16((H_,), 0.5, 1.5, 0, W.STREAM_WEIGHT))
    sx, sc = torch.cuda.Stream(), torch.cuda.Stream()
    cus = tw.device_cu_count()
    for T_ in (2048, 6144, 8192 - 256, 8192, T_max):
        args = (X1[:T_], W1, [p[:T_] for p in parts], resid[:T_], weight, 1e-5, W2g)
        with torch.cuda.stream(sx):
            want = tw.weave_layer(*args, 0, sx, sc, fused_cu_budget=tw.CU_SHARED, parent=sx)
            want = [t.clone() for t in (parts[0][:T_],) + want]
            parts[0][:T_].fill_(float("nan"))
            out, res, Y, taken = tw.weave_layer_auto(*args, sx, sc, fused_cu_budget=tw.CU_SHARED, parent=sx)
        torch.cuda.synchronize()
        assert taken == tw.policy_split_row(T_, K1, H_, P_, N2, cus), (T_, taken)
        if thr == never:
            assert taken == T_
        elif cus == 256:
            assert (taken < T_) == (T_ in (8192 - 256, 8192, T_max)), (T_, taken)
        for name, g_, w_ in zip(("G1", "out", "residual_out", "Y"), (parts[0][:T_], out, res, Y), want):
            assert torch.equal(g_.view(torch.int16), w_.view(torch.int16)), (T_, taken, name)


def test_weave_tune_times_the_candidates_and_leaves_the_layers_outputs(tw, torch_cuda):
    """The offline search (Algorithm 1, timed): every candidate that lies inside the batch gets a time,
    the others a negative one; the row reported is the fastest candidate's; and the buffers hold what any
    call leaves there, the unsplit chain's bits."""
    torch = torch_cuda
    g1, f, W2 = make_inputs()
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    want = run_layer(tw, torch, g1, f, W2, 0, streams, budgets=(tw.CU_SHARED, 0))
    X1, W1 = to_gpu(g1["A"]), to_gpu(g1["B"])
    parts = [torch.zeros((T, H), dtype=torch.bfloat16, device="cuda:0")] + [to_gpu(p) for p in f["partials"][1:]]
    resid, weight, W2g = to_gpu(f["residual"]), to_gpu(f["weight"]), to_gpu(W2)
    out, res = torch.empty_like(resid), torch.empty_like(resid)
    Y = torch.empty((T, N2), dtype=torch.bfloat16, device="cuda:0")
    offsets = (0, 64, -64, 4096, 0)          # one far outside the batch, one repeated
    best, us = tw.weave_tune(X1, W1, parts, resid, weight, f["eps"], W2g, streams[0], streams[1], offsets=offsets,
                             reps=3, multiple=64, out=out, residual_out=res, Y=Y)
    torch.cuda.synchronize()
    base = tw.split_point(T, 64)
    smart = tw.smart_split_point(T, 64, [H, N2], tw.device_cu_count(), gemm_k=[K1, H])[0]
    rows = [T, smart] + [base + o for o in offsets]
    assert len(us) == 2 + len(offsets) and us[0] > 0 and us[1] > 0
    seen = set()
    for i, (row, t) in enumerate(zip(rows, us)):
        ran = i == 0 or (0 < row < T and row not in seen)
        assert (t > 0) == ran, (row, t)
        seen.add(row)
    timed = [(t, row) for row, t in zip(rows, us) if t > 0]
    assert best == min(timed)[1]
    got = (to_bits(parts[0]), to_bits(out), to_bits(res), to_bits(Y))
    for name, g_, w_ in zip(("G1", "out", "residual_out", "Y"), got, want):
        assert np.array_equal(g_, w_), name


@pytest.mark.parametrize("schedule", [1, 2])   # TW_WEAVE_ORDERED, TW_WEAVE_CHAINS
def test_two_boundaries_woven_through_without_a_join_in_between(tw, torch_cuda, schedule):
    """Consecutive boundaries as an engine runs them: the second boundary's input is the first one's
    output, only the first call forks from the parent, none joins, and one event joins the second
    stream at the end. With the same cut in both, every row of a split depends only on rows of that
    split, so stream order alone carries the dependency; the bits are those of the unsplit pair."""
    torch = torch_cuda
    g1, f, W2 = make_inputs()
    sx, sc, parent = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    X1, W1, W2g = to_gpu(g1["A"]), to_gpu(g1["B"]), to_gpu(W2)
    resid, weight = to_gpu(f["residual"]), to_gpu(f["weight"])
    W1b = to_gpu(W.normal_bf16((H, N2), 0.05, 21, W.STREAM_GEMM_B))        # second boundary: [T x N2] x [N2 x H]
    W2b = to_gpu(W.normal_bf16((K1, H), 0.05, 22, W.STREAM_GEMM_B))

    def run_pair(cut, first_has_parent):
        parts_a = [torch.full((T, H), float("nan"), dtype=torch.bfloat16, device="cuda:0")] + \
                  [to_gpu(p) for p in f["partials"][1:]]
        parts_b = [torch.full((T, H), float("nan"), dtype=torch.bfloat16, device="cuda:0")] + \
                  [to_gpu(p) for p in f["partials"][1:]]
        src = torch.zeros_like(X1)
        torch.cuda.synchronize()
        with torch.cuda.stream(parent):
            src.copy_(X1)                                  # the first call must wait for this
        kw = dict(fused_cu_budget=tw.CU_SHARED, gemm_cu_budget=0, schedule=schedule)
        out1, res1, Y1 = tw.weave_layer(src, W1, parts_a, resid, weight, f["eps"], W2g, cut, sx, sc, parent=parent,
                                        use_parent=first_has_parent, join=False, **kw)
        out2, res2, Y2 = tw.weave_layer(Y1, W1b, parts_b, res1, weight, f["eps"], W2b, cut, sx, sc, parent=None,
                                        use_parent=False, join=False, **kw)
        ev = torch.cuda.Event()
        ev.record(sc)
        sx.wait_event(ev)
        sx.synchronize()
        return [to_bits(t) for t in (Y1, res1, out2, res2, Y2)]
    want = run_pair(0, True)
    for cut in (320, 256, 1, T - 1):
        got = run_pair(cut, True)
        for name, g_, w_ in zip(("Y1", "res1", "out2", "res2", "Y2"), got, want):
            assert np.array_equal(g_, w_), (schedule, cut, name)


@pytest.mark.parametrize("schedule", [1, 2])   # TW_WEAVE_ORDERED, TW_WEAVE_CHAINS
def test_weave_train_of_four_boundaries_gives_the_unsplit_bits(tw, torch_cuda, schedule):
    """tw_weave_train: four boundaries, each fed by the one before (X1 = previous Y, residual = previous
    residual_out), forked from a parent that still holds the writing of the first input and joined
    into it; the woven train's outputs carry the bits of the same train unsplit."""
    torch = torch_cuda
    g1, f, W2 = make_inputs()
    sx, sc, parent = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    X1_src, resid = to_gpu(g1["A"]), to_gpu(f["residual"])
    weight = to_gpu(f["weight"])
    dims = [(K1, N2), (N2, K1), (K1, N2), (N2, 64)]             # (depth of G1, width of G2) per boundary
    Ws = [(to_gpu(W.normal_bf16((H, k), 0.05, 40 + i, W.STREAM_GEMM_B)),
           to_gpu(W.normal_bf16((n, H), 0.05, 50 + i, W.STREAM_GEMM_B))) for i, (k, n) in enumerate(dims)]

    def run_train(cut):
        src = torch.zeros_like(X1_src)
        bs, x, r = [], src, resid
        for i, (k, n) in enumerate(dims):
            parts = [torch.full((T, H), float("nan"), dtype=torch.bfloat16, device="cuda:0")] + \
                    [to_gpu(p) for p in f["partials"][1:]]
            b = dict(X1=x, W1=Ws[i][0], partials=parts, residual=r, weight=weight, eps=f["eps"], W2=Ws[i][1],
                     out=torch.empty((T, H), dtype=torch.bfloat16, device="cuda:0"),
                     residual_out=torch.empty((T, H), dtype=torch.bfloat16, device="cuda:0"),
                     Y=torch.full((T, n), float("nan"), dtype=torch.bfloat16, device="cuda:0"))
            bs.append(b)
            x, r = b["Y"], b["residual_out"]
        torch.cuda.synchronize()
        with torch.cuda.stream(parent):
            src.copy_(X1_src)
        tw.weave_train(bs, cut, sx, sc, parent=parent, use_parent=True, join=True, schedule=schedule)
        parent.synchronize()
        return [to_bits(b[k]) for b in bs for k in ("Y", "residual_out", "out")]
    want = run_train(0)
    assert not np.isnan(oracle.bf16_to_f64(want[-3])).any()
    for cut in (320, 256, 1, T - 1, T):
        got = run_train(cut)
        for i, (g_, w_) in enumerate(zip(got, want)):
            assert np.array_equal(g_, w_), (schedule, cut, i)


def test_weave_layer_random_shapes_cuts_and_schedules(tw, torch_cuda):
    """Ragged layer boundaries (hidden sizes that are no power of two, odd token counts, P from 1 to 5,
    GEMM widths and depths that are no multiple of a tile) through tw_weave_layer_cuts with random cuts,
    schedules and launch modes: every stage of the unsplit chain against the oracle fed with the bits
    of the stage before, and every woven run bit-equal to the unsplit one."""
    torch = torch_cuda
    rng = np.random.default_rng(2505)
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    cus = tw.device_cu_count()
    for case in range(14):
        T_ = int(rng.integers(1, 700))
        H_ = int(rng.choice([64, 264, 520, 1024, 1536, 2048, 4104]))
        P_ = int(rng.integers(1, 6))
        K1_ = 8 * int(rng.integers(1, 80))
        N2_ = 8 * int(rng.integers(1, 70))
        g1 = W.make_gemm_inputs(T_, K1_, H_, STD, seed=100 + case, b_layout="nk")
        f = W.make_fused_inputs(dict(N=T_, H=H_, P=P_, partial_std=0.5, residual_std=1.0, outlier_frac=0.01,
                                     outlier_scale=20.0, eps=1e-5, seed=200 + case))
        W2 = W.normal_bf16((N2_, H_), 0.05, 300 + case, W.STREAM_GEMM_B)
        X1, W1, W2g = to_gpu(g1["A"]), to_gpu(g1["B"]), to_gpu(W2)
        resid, weight = to_gpu(f["residual"]), to_gpu(f["weight"])

        def run_cuts(cuts, schedule, budgets):
            parts = [torch.full((T_, H_), float("nan"), dtype=torch.bfloat16, device="cuda:0")] + \
                    [to_gpu(p) for p in f["partials"][1:]]
            out, res, Y = tw.weave_layer_cuts(X1, W1, parts, resid, weight, f["eps"], W2g, cuts, streams[0], streams[1],
                                              fused_cu_budget=budgets[0], gemm_cu_budget=budgets[1], schedule=schedule)
            torch.cuda.synchronize()
            return to_bits(parts[0]), to_bits(out), to_bits(res), to_bits(Y)
        what = "case %d: T=%d H=%d P=%d K1=%d N2=%d" % (case, T_, H_, P_, K1_, N2_)
        C0, out0, res0, Y0 = run_cuts([], tw.WEAVE_AUTO, (0, 0))
        gemm_tol_check(oracle.bf16_to_f64(C0), oracle.gemm(g1["A"], g1["B"], "nk"), K1_, STD, STD, what + " G1")
        ref_out, ref_res = oracle.fused([C0] + f["partials"][1:], f["residual"], f["weight"], f["eps"])
        assert_parity(oracle.bf16_to_f64(res0), ref_res, what + " residual_out")
        assert_parity(oracle.bf16_to_f64(out0), ref_out, what + " out")
        # |out| is at most ~sqrt(H) * max|w| on a row that one outlier dominates; its typical size is ~1
        gemm_tol_check(oracle.bf16_to_f64(Y0), oracle.gemm(out0, W2, "nk"), H_, 1.5, 0.05, what + " G2")
        for trial in range(3):
            n_cuts = int(rng.integers(1, min(T_ - 1, 6) + 1)) if T_ > 1 else 0
            cuts = sorted(int(c) for c in rng.choice(np.arange(1, T_), size=n_cuts, replace=False)) if n_cuts else []
            schedule = int(rng.choice([tw.WEAVE_AUTO, tw.WEAVE_ORDERED, tw.WEAVE_CHAINS]))
            budgets = [(32, cus - 32), (tw.CU_SHARED, 0), (0, 0), (8, 16)][int(rng.integers(0, 4))]
            got = run_cuts(cuts, schedule, budgets)
            for name, g_, w_ in zip(("G1", "out", "residual_out", "Y"), got, (C0, out0, res0, Y0)):
                assert np.array_equal(g_, w_), (what, cuts, schedule, budgets, name)

