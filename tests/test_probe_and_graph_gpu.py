"""GPU checks of the measurement probes (they are exported, so they must do what
the header says) and of HIP-graph capture of the library's multi-stream calls."""
import numpy as np
import pytest

import tw_workloads as W
from helpers import to_bits, to_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available()
    return torch


def test_copy_and_write_probes_move_the_bytes_they_claim(tw, torch_cuda):
    torch = torch_cuda
    n = (3 << 20) + 4096 + 16          # not a multiple of the grid stride: exercises the tail loop
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda:0")
    for budget in (1, 8, 0):
        dst = torch.zeros(n + 64, dtype=torch.uint8, device="cuda:0")
        tw.hbm_probe(src, dst, n, tw.PROBE_COPY, cu_budget=budget)
        torch.cuda.synchronize()
        assert torch.equal(dst[:n], src) and int(dst[n:].sum()) == 0
    dst = torch.zeros(n + 64, dtype=torch.uint8, device="cuda:0")
    tw.hbm_probe(None, dst, n, tw.PROBE_WRITE, cu_budget=8)
    torch.cuda.synchronize()
    pat = dst[:n].view(torch.int32)
    assert bool((pat == 0x3F803F80).all()) and int(dst[n:].sum()) == 0
    sink = torch.zeros(256 * tw.device_cu_count(), dtype=torch.uint8, device="cuda:0")
    tw.hbm_probe(src, sink, n, tw.PROBE_READ, cu_budget=8)
    torch.cuda.synchronize()


def test_mixed_probe_writes_only_its_write_streams(tw, torch_cuda):
    torch = torch_cuda
    sb = 1 << 20
    src = torch.randint(0, 256, (9 * sb,), dtype=torch.uint8, device="cuda:0")
    dst = torch.zeros(2 * sb + 4096, dtype=torch.uint8, device="cuda:0")
    for n_read in (0, 1, 5, 9, 17):
        if n_read > 9:
            src17 = torch.randint(0, 256, (17 * sb,), dtype=torch.uint8, device="cuda:0")
            tw.hbm_probe_mixed(src17, dst, sb, n_read, 2, cu_budget=4)
        else:
            tw.hbm_probe_mixed(src, dst, sb, n_read, 2, cu_budget=4)
        torch.cuda.synchronize()
        assert int(dst[2 * sb:].sum()) == 0          # nothing past the two streams
    before = src.clone()
    tw.hbm_probe_mixed(src, dst, sb, 9, 0, cu_budget=4)
    torch.cuda.synchronize()
    assert torch.equal(src, before)


@pytest.mark.parametrize("schedule", [1, 2])   # TW_WEAVE_ORDERED, TW_WEAVE_CHAINS
def test_weave_layer_can_be_captured_in_a_hip_graph(tw, torch_cuda, schedule):
    """tw_weave_layer forks and joins a second stream with events; captured on the
    caller's stream it becomes one graph. Every replay (with eager work and
    synchronisations in between) must reproduce the eager result bit for bit."""
    torch = torch_cuda
    T, K1, H, P, N2 = 512, 256, 2048, 4, 640
    g1 = W.make_gemm_inputs(T, K1, H, 0.1, seed=3, b_layout="nk")
    cfg = dict(N=T, H=H, P=P, partial_std=0.5, residual_std=1.0, outlier_frac=0.0, outlier_scale=1.0,
               eps=1e-5, seed=5)
    f = W.make_fused_inputs(cfg)
    X1, W1 = to_gpu(g1["A"]), to_gpu(g1["B"])
    W2 = to_gpu(W.normal_bf16((N2, H), 0.05, 9, W.STREAM_GEMM_B))
    parts = [torch.zeros((T, H), dtype=torch.bfloat16, device="cuda:0")] + [to_gpu(p) for p in f["partials"][1:]]
    resid, weight = to_gpu(f["residual"]), to_gpu(f["weight"])
    out, res, Y = (torch.empty_like(resid), torch.empty_like(resid),
                   torch.empty((T, N2), dtype=torch.bfloat16, device="cuda:0"))
    main, comm = torch.cuda.Stream(), torch.cuda.Stream()

    def layer():
        tw.weave_layer(X1, W1, parts, resid, weight, f["eps"], W2, 256, main, comm,
                       fused_cu_budget=tw.CU_SHARED, gemm_cu_budget=0, out=out, residual_out=res, Y=Y,
                       parent=main, use_parent=True, join=True, schedule=schedule)
    with torch.cuda.stream(main):
        layer()                                   # eager: also the warm-up that capture needs
    torch.cuda.synchronize()
    want = (to_bits(out).copy(), to_bits(res).copy(), to_bits(Y).copy())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=main):
        layer()
    for rep in range(4):
        with torch.cuda.stream(main):
            out.zero_()
            res.zero_()
            Y.zero_()
            parts[0].zero_()
            graph.replay()
        main.synchronize()
        assert np.array_equal(to_bits(out), want[0]) and np.array_equal(to_bits(res), want[1])
        assert np.array_equal(to_bits(Y), want[2])
        with torch.cuda.stream(main):            # eager work between replays
            tw.reduce_add_rmsnorm(parts, resid, weight, f["eps"], cu_budget=8)
        torch.cuda.synchronize()


@pytest.mark.parametrize("schedule", [1, 2])   # TW_WEAVE_ORDERED, TW_WEAVE_CHAINS
def test_weave_train_can_be_captured_in_a_hip_graph(tw, torch_cuda, schedule):
    """A woven train of boundaries is what an engine would capture once per batch shape: one fork from the
    caller's stream, the two chains running through three boundaries (each fed by the one before), one
    join. Every replay must reproduce the eager result bit for bit."""
    torch = torch_cuda
    T, K1, H, P, N2 = 512, 256, 2048, 4, 256
    g1 = W.make_gemm_inputs(T, K1, H, 0.1, seed=3, b_layout="nk")
    f = W.make_fused_inputs(dict(N=T, H=H, P=P, partial_std=0.5, residual_std=1.0, outlier_frac=0.0,
                                 outlier_scale=1.0, eps=1e-5, seed=5))
    X1, weight = to_gpu(g1["A"]), to_gpu(f["weight"])
    main, comm = torch.cuda.Stream(), torch.cuda.Stream()
    bs, x, r = [], X1, to_gpu(f["residual"])
    for i in range(3):
        b = dict(X1=x, W1=to_gpu(W.normal_bf16((H, K1), 0.1, 60 + i, W.STREAM_GEMM_B)),
                 partials=[torch.zeros((T, H), dtype=torch.bfloat16, device="cuda:0")] + [to_gpu(p) for p in f["partials"][1:]],
                 residual=r, weight=weight, eps=f["eps"], W2=to_gpu(W.normal_bf16((N2, H), 0.05, 70 + i, W.STREAM_GEMM_B)),
                 out=torch.empty((T, H), dtype=torch.bfloat16, device="cuda:0"),
                 residual_out=torch.empty((T, H), dtype=torch.bfloat16, device="cuda:0"),
                 Y=torch.empty((T, N2), dtype=torch.bfloat16, device="cuda:0"))
        bs.append(b)
        x, r = b["Y"], b["residual_out"]

    def train():
        tw.weave_train(bs, 256, main, comm, parent=main, use_parent=True, join=True, schedule=schedule)
    with torch.cuda.stream(main):
        train()                                   # eager: also the warm-up that capture needs
    torch.cuda.synchronize()
    want = [to_bits(b[k]).copy() for b in bs for k in ("Y", "residual_out", "out")]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=main):
        train()
    for rep in range(3):
        with torch.cuda.stream(main):
            for b in bs:
                b["Y"].zero_()
                b["out"].zero_()
                b["residual_out"].zero_()
                b["partials"][0].zero_()
            graph.replay()
        main.synchronize()
        got = [to_bits(b[k]) for b in bs for k in ("Y", "residual_out", "out")]
        for i, (g_, w_) in enumerate(zip(got, want)):
            assert np.array_equal(g_, w_), (rep, i)
        with torch.cuda.stream(main):            # eager work between replays
            tw.reduce_add_rmsnorm(bs[0]["partials"], bs[0]["residual"], weight, f["eps"], cu_budget=8)
        torch.cuda.synchronize()


def test_shaped_probes_move_the_same_bytes_in_every_shape(tw, torch_cuda):
    """Workgroup size and accesses in flight change the launch, not what is copied."""
    torch = torch_cuda
    n = (2 << 20) + 4096 + 48
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda:0")
    sink = torch.zeros(256 * tw.device_cu_count(), dtype=torch.uint8, device="cuda:0")
    for threads in (64, 192, 256, 512, 1024):
        for depth in (1, 2, 4, 8, 16):
            dst = torch.zeros(n + 64, dtype=torch.uint8, device="cuda:0")
            tw.hbm_probe_shaped(src, dst, n, tw.PROBE_COPY, cu_budget=3, threads=threads, in_flight=depth)
            tw.hbm_probe_shaped(src, sink, n, tw.PROBE_READ, cu_budget=3, threads=threads, in_flight=depth)
            torch.cuda.synchronize()
            assert torch.equal(dst[:n], src) and int(dst[n:].sum()) == 0, (threads, depth)
    sb = 1 << 20
    srcs = torch.randint(0, 256, (9 * sb,), dtype=torch.uint8, device="cuda:0")
    for threads in (64, 256, 512, 1024):
        dst = torch.zeros(2 * sb + 4096, dtype=torch.uint8, device="cuda:0")
        tw.hbm_probe_mixed_shaped(srcs, dst, sb, 9, 2, cu_budget=4, threads=threads)
        torch.cuda.synchronize()
        # every word of the two write streams was written (the stored words are xors of loaded data:
        # a zero among them is a 2^-32 event per word)
        assert int(dst[2 * sb:].sum()) == 0 and int(dst[:2 * sb].view(torch.int32).ne(0).sum()) >= 2 * sb // 4 - 8


@pytest.mark.parametrize("N", [1, 16, 256])
def test_decode_sized_train_of_fused_steps_replays_from_a_graph(tw, torch_cuda, N):
    """A decode iteration is a train of many small fused steps (two per layer). Captured once into a HIP
    graph (nothing in the library allocates or clears memory per call, so there is no memset node), every
    replay must give the eager train's bits; eager work and synchronisations sit between the replays."""
    torch = torch_cuda
    H, P, layers = 8192, 8, 12
    cfg = dict(N=N, H=H, P=P, partial_std=0.25, residual_std=1.0, outlier_frac=0.01, outlier_scale=50.0,
               eps=1e-5, seed=N)
    d = W.make_fused_inputs(cfg)
    parts = [to_gpu(p) for p in d["partials"]]
    resid0, weight = to_gpu(d["residual"]), to_gpu(d["weight"])
    resid = torch.empty_like(resid0)
    outs = [torch.empty_like(resid0) for _ in range(layers)]
    main = torch.cuda.Stream()

    def train():
        # the residual stream is carried in place from step to step, as in the paper's kernel
        for i in range(layers):
            tw.reduce_add_rmsnorm(parts, resid, weight, d["eps"], cu_budget=(0, tw.CU_SHARED)[i % 2], out=outs[i],
                                  residual_out=resid, stream=main)

    def reset():
        with torch.cuda.stream(main):
            resid.copy_(resid0)
            for o in outs:
                o.fill_(float("nan"))
    reset()
    train()
    main.synchronize()
    want = [to_bits(o).copy() for o in outs] + [to_bits(resid).copy()]
    assert not np.array_equal(want[0], want[-2])           # the steps do differ
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=main):
        train()
    for rep in range(4):
        reset()
        with torch.cuda.stream(main):
            graph.replay()
        main.synchronize()
        got = [to_bits(o) for o in outs] + [to_bits(resid)]
        for i, (g_, w_) in enumerate(zip(got, want)):
            assert np.array_equal(g_, w_), (rep, i)
        tw.reduce_add_rmsnorm(parts, resid0, weight, d["eps"], cu_budget=8)   # eager work between replays
        torch.cuda.synchronize()


def test_streams_overlap_finds_a_partner_stream(tw, torch_cuda):
    """A stream never overlaps with itself; among a handful of new streams at least one sits on another
    hardware queue than the first and is reported as running side by side with it, repeatably."""
    torch = torch_cuda
    a = torch.cuda.Stream()
    assert tw.streams_overlap(a, a) is False
    verdicts = []
    for _ in range(6):
        b = torch.cuda.Stream()
        v = tw.streams_overlap(a, b)
        assert tw.streams_overlap(a, b) == v and tw.streams_overlap(b, a) == v
        verdicts.append(v)
    assert any(verdicts), verdicts
    torch.cuda.synchronize()


def test_cu_masked_streams_confine_kernels_to_disjoint_compute_units(tw, torch_cuda):
    """tw_stream_create_cu_masked: every workgroup of a launch on the masked stream, whatever its grid,
    reports a compute unit from a set of exactly n_cus, spread evenly over the XCDs; the sets of two
    disjoint ranges are disjoint; the two streams run side by side; and the bits are those of an
    ordinary launch."""
    torch = torch_cuda
    cus = tw.device_cu_count()
    d = W.make_fused_inputs("c3_70b_shard_tp8", N=1024)
    g = {k: ([to_gpu(p) for p in v] if k == "partials" else to_gpu(v) if k in ("residual", "weight") else v)
         for k, v in d.items()}
    want = tw.reduce_add_rmsnorm(g["partials"], g["residual"], g["weight"], g["eps"], cu_budget=32)
    torch.cuda.synchronize()

    def places_of(stream, budget):
        out, res, hw = tw.reduce_add_rmsnorm_traced(g["partials"], g["residual"], g["weight"], g["eps"],
                                                    cu_budget=budget, stream=stream)
        stream.synchronize()
        assert torch.equal(out.view(torch.int16), want[0].view(torch.int16))
        assert torch.equal(res.view(torch.int16), want[1].view(torch.int16))
        hw = hw.cpu().numpy().astype(np.int64) & 0xFFFFFFFF
        cu, se, sh, xcc = (hw[:, 0] >> 8) & 0xF, (hw[:, 0] >> 13) & 0x7, (hw[:, 0] >> 12) & 0x1, hw[:, 1] & 0xF
        return set(zip(xcc.tolist(), se.tolist(), sh.tolist(), cu.tolist()))
    few, rest = tw.CuMaskedStream(0, 32), tw.CuMaskedStream(32, cus - 32)
    try:
        a = places_of(few.stream, tw.CU_SHARED)            # 1024 small workgroups on 32 compute units
        assert len(a) == 32
        per_xcd = np.bincount([p[0] for p in a], minlength=8)
        assert (per_xcd == 4).all(), per_xcd
        assert places_of(few.stream, 64) <= a              # a persistent grid of 64: two per masked unit, in turn
        b = places_of(rest.stream, tw.CU_SHARED)
        assert len(b) == cus - 32 and not (a & b)
        # (both streams have run kernels by now: the first dispatch on a new queue starts late)
        assert any(tw.streams_overlap(few.stream, rest.stream) for _ in range(3))
    finally:
        few.close()
        rest.close()
    for bad in ((0, cus + 1), (cus - 7, 8), (cus, 1)):
        with pytest.raises(tw.TwError) as e:
            tw.CuMaskedStream(*bad)
        assert e.value.status == 2                          # TW_ERR_SHAPE

