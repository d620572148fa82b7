"""GPU parity of tw_gemm_bf16 (the compute stand-in of the other token split,
TokenWeave Fig. 7b) against the fp64 textbook product, and of tw_overlap_launch
against the two calls made one after the other.

Tolerance for C (bf16, fp32 accumulation over K): the rounding to bf16 costs up
to 2^-8 relative; fp32 accumulation of K products of magnitude ~sa*sb adds an
absolute error of about K * 2^-24 * sa * sb in the worst case, far below
1e-3 * sqrt(K) * sa * sb. So: |gpu - ref| <= 1e-2 |ref| + 1e-3 * sqrt(K) * sa * sb."""
import numpy as np
import pytest

import oracle
import tw_workloads as W
from helpers import to_bits, to_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available()
    return torch


def gemm_check(got_f64, ref_f64, K, std, what):
    tol = 1e-2 * np.abs(ref_f64) + 1e-3 * np.sqrt(max(K, 1)) * std * std
    bad = np.abs(got_f64 - ref_f64) > tol
    assert not bad.any(), "%s: %d of %d out of tolerance, first %s" % (
        what, bad.sum(), bad.size, np.argwhere(bad)[:1])


SHAPES = [(256, 128, 64), (64, 64, 64), (300, 200, 136), (1, 8, 8), (257, 136, 72), (512, 384, 1024),
          (33, 1000, 264), (700, 24, 4096)]


@pytest.mark.parametrize("layout", ["nk", "kn"])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_small_shapes_full_compare(tw, torch_cuda, M, N, K, layout):
    g = W.make_gemm_inputs(M, K, N, 0.5, seed=M + N + K, b_layout=layout)
    code = tw.B_NK if layout == "nk" else tw.B_KN
    C = tw.gemm_bf16(to_gpu(g["A"]), to_gpu(g["B"]), b_layout=code)
    torch_cuda.cuda.synchronize()
    ref = oracle.gemm(g["A"], g["B"], layout)
    gemm_check(oracle.bf16_to_f64(to_bits(C)), ref, K, 0.5, "gemm %s %dx%dx%d" % (layout, M, N, K))
    # a budgeted (persistent) launch walks the same tiles: same bits
    C2 = tw.gemm_bf16(to_gpu(g["A"]), to_gpu(g["B"]), b_layout=code, cu_budget=3)
    torch_cuda.cuda.synchronize()
    assert np.array_equal(to_bits(C), to_bits(C2))


def test_gemm_both_layouts_give_the_same_bits(tw, torch_cuda):
    """B(k, n) is the same matrix whichever way it is stored, and both kernels
    multiply and add in the same order."""
    a = W.make_gemm_inputs(520, 1000, 392, 0.3, seed=11, b_layout="nk")
    b = W.make_gemm_inputs(520, 1000, 392, 0.3, seed=11, b_layout="kn")
    C1 = tw.gemm_bf16(to_gpu(a["A"]), to_gpu(a["B"]), b_layout=tw.B_NK)
    C2 = tw.gemm_bf16(to_gpu(b["A"]), to_gpu(b["B"]), b_layout=tw.B_KN)
    torch_cuda.cuda.synchronize()
    assert np.array_equal(to_bits(C1), to_bits(C2))


@pytest.mark.parametrize("M,N,K,budget", [(4096, 4096, 2048, 0), (1000, 1096, 520, 10), (2304, 2048, 4104, 72),
                                          (513, 520, 96, 9), (512, 512, 40, 4), (768, 1024, 64, 6), (520, 264, 200, 3)])
def test_gemm_large_product_tiles_give_the_same_bits(tw, torch_cuda, M, N, K, budget):
    """A large product launched on its own takes 256 x 256 tiles (four waves of 128 x 128, K steps of 64
    through a ring of five LDS slots) where those fill the compute units of the launch; stored [K x N] the same
    product always takes the 256 x 128 ones. Same bits (ragged edges and a K that is no multiple of the
    K step included), checked against the oracle on sampled outputs."""
    a = W.make_gemm_inputs(M, K, N, 0.05, seed=M + K, b_layout="nk")
    b = W.make_gemm_inputs(M, K, N, 0.05, seed=M + K, b_layout="kn")
    cus = tw.device_cu_count()
    use = budget if 0 < budget < cus else cus
    fill = lambda tiles: tiles / (-(-tiles // use) * use)
    tm = -(-M // 256)
    assert 2 * tm * -(-N // 128) > use and fill(tm * -(-N // 256)) >= fill(tm * -(-N // 128)) - 0.05, \
        "the case is meant to take the 256 x 256 tiles"
    C = torch_cuda.full((M, N), float("nan"), dtype=torch_cuda.bfloat16, device="cuda:0")
    tw.gemm_bf16(to_gpu(a["A"]), to_gpu(a["B"]), C=C, b_layout=tw.B_NK, cu_budget=budget)
    C2 = tw.gemm_bf16(to_gpu(b["A"]), to_gpu(b["B"]), b_layout=tw.B_KN, cu_budget=budget)
    torch_cuda.cuda.synchronize()
    Cb = to_bits(C)
    assert np.array_equal(Cb, to_bits(C2))
    rng = np.random.default_rng(M)
    ms = np.concatenate([rng.integers(0, M, 2040), [0, 0, M - 1, M - 1, min(255, M - 1), min(256, M - 1), M // 2, 1]])
    ns = np.concatenate([rng.integers(0, N, 2040), [0, N - 1, 0, N - 1, min(255, N - 1), min(256, N - 1), N // 2, 1]])
    ref = oracle.gemm_samples(a["A"], a["B"], "nk", ms, ns)
    gemm_check(oracle.bf16_to_f64(Cb[ms, ns]), ref, K, 0.05, "large-tile gemm %dx%dx%d" % (M, N, K))


def test_gemm_k_zero_gives_zeros(tw, torch_cuda):
    torch = torch_cuda
    for (M, N, budget) in ((40, 24, 0), (512, 512, 4)):      # the second takes the 256 x 256 tiles
        A = torch.empty((M, 0), dtype=torch.bfloat16, device="cuda:0")
        B = torch.empty((N, 0), dtype=torch.bfloat16, device="cuda:0")
        C = torch.full((M, N), 7.0, dtype=torch.bfloat16, device="cuda:0")
        tw.gemm_bf16(A, B, C=C, cu_budget=budget)
        torch.cuda.synchronize()
        assert (to_bits(C) == 0).all()


def test_gemm_at_the_largest_k(tw, torch_cuda):
    """K = 2^22, the deepest product the entry point accepts: rows of 8 MiB, a full 256-row tile of A is
    2 GiB, and every byte offset inside it still has to fit the 32 bits a buffer instruction adds up.
    Inputs drawn on the GPU; rows 0, 63, 64, 191 and 255 of the tile (the first and last rows of the
    first, second and last load instruction) and two rows of a ragged second tile against the fp64
    product of those rows."""
    torch = torch_cuda
    M, N, K, std = 256 + 3, 16, 1 << 22, 0.02
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(22)
    A = torch.empty((M, K), dtype=torch.bfloat16, device="cuda:0").normal_(0.0, std, generator=gen)
    B = torch.empty((N, K), dtype=torch.bfloat16, device="cuda:0").normal_(0.0, std, generator=gen)
    C = tw.gemm_bf16(A, B)
    torch.cuda.synchronize()
    rows = [0, 63, 64, 191, 255, 256, M - 1]
    ref = oracle.gemm(to_bits(A[rows]), to_bits(B), "nk")
    gemm_check(oracle.bf16_to_f64(to_bits(C[rows])), ref, K, std, "gemm at K = 2^22")
    assert np.count_nonzero(to_bits(C)) > 0.99 * M * N
    del A, B, C
    torch.cuda.empty_cache()


@pytest.mark.parametrize("layout", ["nk", "kn"])
def test_gemm_taller_than_four_gib(tw, torch_cuda, layout):
    """M = 1.1 M rows: C is 4.5 GB, so tile base addresses run past 2^32 bytes (row 1048576 of C starts
    there, row 524288 at 2^31; A passes 2^30 at row 1048576). Rows around those seams, the first, the
    last (a ragged tile) and random ones against the fp64 product of those rows; [N x K] operands take
    the 256 x 256 tiles, [K x N] the 256 x 128 ones."""
    torch = torch_cuda
    M, N, K, std = 1100000 + 37, 2048, 512, 0.05
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(5)
    A = torch.empty((M, K), dtype=torch.bfloat16, device="cuda:0").normal_(0.0, std, generator=gen)
    Bnk = torch.empty((N, K), dtype=torch.bfloat16, device="cuda:0").normal_(0.0, std, generator=gen)
    B = Bnk if layout == "nk" else Bnk.t().contiguous()
    C = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    tw.gemm_bf16(A, B, C=C, b_layout=tw.B_NK if layout == "nk" else tw.B_KN)
    torch.cuda.synchronize()
    rng = np.random.default_rng(9)
    rows = sorted(set([0, 255, 256, 524287, 524288, 1048575, 1048576, 1048577, M - 38, M - 37, M - 1]
                      + [int(r) for r in rng.integers(0, M, 40)]))
    idx = torch.tensor(rows, device="cuda:0")
    ref = oracle.gemm(to_bits(A[idx]), to_bits(Bnk), "nk")
    gemm_check(oracle.bf16_to_f64(to_bits(C[idx])), ref, K, std, "tall gemm " + layout)
    # every element was written: no NaN is left anywhere
    assert not torch.isnan(C).any().item()
    del A, B, Bnk, C
    torch.cuda.empty_cache()


@pytest.mark.parametrize("layout", ["nk", "kn"])
def test_gemm_demo_shape_sampled(tw, torch_cuda, layout):
    """[2048 x 8192] x [8192 x 3584], N(0, 0.02^2): 4096 sampled outputs, one by one."""
    gc = W.CONFIGS["c5_overlap_tp8"]["gemm"]
    g = W.make_gemm_inputs(gc["M"], gc["K"], gc["N"], gc["std"], seed=0, b_layout=layout)
    C = tw.gemm_bf16(to_gpu(g["A"]), to_gpu(g["B"]), b_layout=tw.B_NK if layout == "nk" else tw.B_KN)
    torch_cuda.cuda.synchronize()
    Cb = to_bits(C)
    rng = np.random.default_rng(0)
    ms = np.concatenate([rng.integers(0, gc["M"], 4088), [0, 0, gc["M"] - 1, gc["M"] - 1, 255, 256, 1023, 1024]])
    ns = np.concatenate([rng.integers(0, gc["N"], 4088), [0, gc["N"] - 1, 0, gc["N"] - 1, 127, 128, 3583, 1792]])
    ref = oracle.gemm_samples(g["A"], g["B"], layout, ms, ns)
    gemm_check(oracle.bf16_to_f64(Cb[ms, ns]), ref, gc["K"], gc["std"], "demo gemm " + layout)
    assert np.count_nonzero(Cb) > 0.99 * Cb.size


def test_overlap_launch_equals_the_two_calls(tw, torch_cuda):
    """Fused kernel on half A next to the GEMM on half B (two streams, fork and
    join on a parent stream): same bits as the plain calls, every replay."""
    torch = torch_cuda
    cfg = W.CONFIGS["c5_overlap_tp8"]
    d = W.make_fused_inputs(cfg, N=512)
    g = dict(partials=[to_gpu(p) for p in d["partials"]], residual=to_gpu(d["residual"]),
             weight=to_gpu(d["weight"]), eps=d["eps"])
    gm = W.make_gemm_inputs(512, 1024, 640, 0.02, seed=0, b_layout="nk")
    A, B = to_gpu(gm["A"]), to_gpu(gm["B"])
    out0, res0 = tw.reduce_add_rmsnorm(g["partials"], g["residual"], g["weight"], g["eps"], cu_budget=32)
    C0 = tw.gemm_bf16(A, B)
    torch.cuda.synchronize()
    comm, comp, parent = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    for _ in range(3):
        with torch.cuda.stream(parent):
            out, res, C = tw.overlap_launch(dict(g, cu_budget=32), dict(A=A, B=B, cu_budget=0), comm, comp,
                                            parent=parent, use_parent=True, join=True)
            oc, rc, cc = out.clone(), res.clone(), C.clone()
        parent.synchronize()
        assert np.array_equal(to_bits(oc), to_bits(out0))
        assert np.array_equal(to_bits(rc), to_bits(res0))
        assert np.array_equal(to_bits(cc), to_bits(C0))


@pytest.mark.parametrize("layout", ["nk", "kn"])
@pytest.mark.parametrize("M,K,N", [(1024, 2048, 1536), (512, 1024, 4096), (2048, 8192, 1280), (2048, 2048, 4096)])
def test_overlap_launch_shared_mode_equals_the_two_calls(tw, torch_cuda, M, K, N, layout):
    """The co-resident mode: small fused workgroups on every compute unit next to
    the GEMM's. Same bits as the plain calls, on every one of many launches: next
    to the fused kernel the GEMM's LDS reads and loads take longer, which is when
    a missing wait shows (C starts as NaNs, so a store that went astray is seen).
    The shapes cover the narrow tiles (at most half of the compute units filled by
    wide ones) and the wide tiles, for both storage orders of B (the [K x N] one
    reads its fragments with the transposing LDS read and has waits of its own)."""
    torch = torch_cuda
    cfg = W.CONFIGS["c5_overlap_tp8"]
    d = W.make_fused_inputs(cfg, N=1024)
    g = dict(partials=[to_gpu(p) for p in d["partials"]], residual=to_gpu(d["residual"]),
             weight=to_gpu(d["weight"]), eps=d["eps"])
    gm = W.make_gemm_inputs(M, K, N, 0.02, seed=0, b_layout=layout)
    bl = tw.B_NK if layout == "nk" else tw.B_KN
    A, B = to_gpu(gm["A"]), to_gpu(gm["B"])
    out0, res0 = tw.reduce_add_rmsnorm(g["partials"], g["residual"], g["weight"], g["eps"], cu_budget=32)
    C0 = tw.gemm_bf16(A, B, b_layout=bl, cu_budget=16)      # alone, wide tiles
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(tw.gemm_bf16(A, B, b_layout=bl)), to_bits(C0))
    if layout == "kn":      # and the same bits as the other storage order of the same matrix
        nk = W.make_gemm_inputs(M, K, N, 0.02, seed=0, b_layout="nk")
        assert np.array_equal(to_bits(tw.gemm_bf16(A, to_gpu(nk["B"]), cu_budget=16)), to_bits(C0))
    comm, comp, parent = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    C = torch.empty((M, N), dtype=torch.bfloat16, device="cuda:0")
    out = torch.empty_like(g["residual"])
    res = torch.empty_like(g["residual"])
    for it in range(30):
        with torch.cuda.stream(parent):
            C.fill_(float("nan"))
            if it % 2 == 0:
                tw.overlap_launch(dict(g, cu_budget=tw.CU_SHARED, out=out, residual_out=res),
                                  dict(A=A, B=B, C=C, b_layout=bl, cu_budget=0), comm, comp, parent=parent,
                                  use_parent=True, join=True)
            else:
                # the two calls made by hand on two streams: tw_gemm_bf16 picks its tiles as for a
                # launch on its own (the narrow ones where few wide tiles would fill the device)
                comp.wait_stream(parent)
                comm.wait_stream(parent)
                tw.gemm_bf16(A, B, C=C, b_layout=bl, cu_budget=0, stream=comp)
                tw.reduce_add_rmsnorm(g["partials"], g["residual"], g["weight"], g["eps"], cu_budget=tw.CU_SHARED,
                                      out=out, residual_out=res, stream=comm)
                parent.wait_stream(comp)
                parent.wait_stream(comm)
            oc, rc, cc = out.clone(), res.clone(), C.clone()
        parent.synchronize()
        assert np.array_equal(to_bits(oc), to_bits(out0)), it
        assert np.array_equal(to_bits(rc), to_bits(res0)), it
        assert np.array_equal(to_bits(cc), to_bits(C0)), (it, int((to_bits(cc) != to_bits(C0)).sum()))


def test_gemm_random_shapes_both_layouts(tw, torch_cuda):
    """Seeded random M, N, K (N and K multiples of 8): both operand layouts and a
    budgeted launch give the same bits, and those match the oracle."""
    rng = np.random.default_rng(7)
    for case in range(16):
        M = int(rng.integers(1, 600))
        N = 8 * int(rng.integers(1, 60))
        K = 8 * int(rng.integers(1, 90))
        a = W.make_gemm_inputs(M, K, N, 0.3, seed=100 + case, b_layout="nk")
        b = W.make_gemm_inputs(M, K, N, 0.3, seed=100 + case, b_layout="kn")
        C1 = tw.gemm_bf16(to_gpu(a["A"]), to_gpu(a["B"]), b_layout=tw.B_NK)
        C2 = tw.gemm_bf16(to_gpu(b["A"]), to_gpu(b["B"]), b_layout=tw.B_KN)
        C3 = tw.gemm_bf16(to_gpu(a["A"]), to_gpu(a["B"]), b_layout=tw.B_NK, cu_budget=int(rng.integers(1, 9)))
        torch_cuda.cuda.synchronize()
        what = "case %d: %dx%dx%d" % (case, M, N, K)
        assert np.array_equal(to_bits(C1), to_bits(C2)), what
        assert np.array_equal(to_bits(C1), to_bits(C3)), what
        gemm_check(oracle.bf16_to_f64(to_bits(C1)), oracle.gemm(a["A"], a["B"], "nk"), K, 0.3, what)


def test_traced_gemm_counts_phases_and_gives_the_same_product(tw, torch_cuda):
    """The tracing variant of the 256 x 256 kernel: same bits as the plain call; every wave reports the
    tiles it worked on (all of them together: the tile count), phases that add up to no more than its
    total, and at least the matrix work's clocks in the two sub-steps (64 MFMAs of 16 clocks per sub-step
    and K step). Products that would not take those tiles are refused."""
    torch = torch_cuda
    M, N, K = 4096, 4096, 1024
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(7)
    A = torch.empty((M, K), dtype=torch.bfloat16, device="cuda:0").normal_(0.0, 0.05, generator=gen)
    B = torch.empty((N, K), dtype=torch.bfloat16, device="cuda:0").normal_(0.0, 0.05, generator=gen)
    want = tw.gemm_bf16(A, B, b_layout=tw.B_NK)
    C, cycles = tw.gemm_bf16_traced(A, B)
    torch.cuda.synchronize()
    assert torch.equal(C.view(torch.int16), want.view(torch.int16))
    c = cycles.cpu().numpy()
    names = tw.GEMM_PHASE_NAMES
    tiles = (M // 256) * (N // 256)
    ran = c[:, names.index("tiles")] > 0
    assert ran.sum() == min(tiles, tw.device_cu_count()) * 4
    assert c[ran, names.index("tiles")].sum() == 4 * tiles
    parts = c[:, :6].sum(axis=1)
    assert (parts[ran] <= c[ran, names.index("kernel")]).all() and (c[ran, names.index("kernel")] < 10 ** 8).all()
    steps = c[ran, names.index("tiles")] * (K // 64)
    assert (c[ran, names.index("sub_step_0")] >= 1024 * steps).all()
    assert (c[ran, names.index("sub_step_1")] >= 1024 * steps).all()
    with pytest.raises(tw.TwError):
        tw.gemm_bf16_traced(A[:256], B[:128])
