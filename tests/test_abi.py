"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function include/tw.h declares, and rejects bad arguments before touching
the device. No call here passes a complete valid argument set with made-up
pointers unless the machine has no GPU, so nothing can be launched on them."""
import ctypes
import os
import re

import pytest

import paper_2505_11329_amd as tw
from paper_2505_11329_amd.binding import FusedArgs, GemmArgs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
VP = ctypes.c_void_p

OK, E_NULL, E_SHAPE, E_ALIGN, E_ALIAS, E_UNSUP, E_SPLIT, E_HIP = range(8)


def declared_functions(headers=("tw.h", "tw_measure.h")):
    names = set()
    for h in headers:
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(tw_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_documented_entry_points():
    names = declared_functions(("tw.h",))
    for must in ("tw_reduce_add_rmsnorm", "tw_split_launch", "tw_split_point", "tw_gemm_bf16",
                 "tw_overlap_launch", "tw_weave_layer", "tw_weave_layer_cuts", "tw_weave_train", "tw_weave_layer_auto", "tw_weave_tune", "tw_smart_split_point",
                 "tw_should_split", "tw_split_threshold", "tw_policy_split_row", "tw_device_cu_count", "tw_status_str",
                 "tw_version", "tw_last_hip_error"):
        assert must in names
    # measurement and introspection aids are declared apart from the method's interface
    aids = declared_functions(("tw_measure.h",))
    for must in ("tw_hbm_probe", "tw_hbm_probe_mixed", "tw_hbm_probe_shaped", "tw_hbm_probe_mixed_shaped",
                 "tw_fused_grid", "tw_fused_layout", "tw_weave_schedule", "tw_gemm_tile_shape",
                 "tw_reduce_add_rmsnorm_traced", "tw_streams_overlap", "tw_gemm_bf16_traced",
                 "tw_stream_create_cu_masked", "tw_stream_destroy"):
        assert must in aids and must not in names


def test_library_exports_every_declared_symbol():
    L = ctypes.CDLL(tw.library_path())
    for name in declared_functions():
        assert hasattr(L, name), "libtw.so does not export %s" % name


def test_cu_masked_stream_argument_checks():
    L = tw.lib()
    h = VP()
    assert L.tw_stream_create_cu_masked(0, 32, None) == E_NULL
    assert L.tw_stream_create_cu_masked(-1, 32, ctypes.byref(h)) == E_SHAPE
    assert L.tw_stream_create_cu_masked(0, 0, ctypes.byref(h)) == E_SHAPE
    assert h.value is None
    assert L.tw_stream_destroy(None) == E_NULL


def test_status_strings_and_version():
    for s in range(8):
        assert tw.status_str(s) and tw.status_str(s) != "unknown status"
    assert tw.status_str(99) == "unknown status"
    assert "gfx950" in tw.version()


# fake but well-formed device addresses: never dereferenced, because every call
# below fails validation (or the machine has no GPU)
BASE = 0x7000_0000_0000
N, H, P = 4, 64, 2
TENSOR = N * H * 2


def addr(i):
    return BASE + i * 0x10000


def fused_call(partials=None, residual=addr(4), weight=addr(5), eps=1e-5, n=N, h=H, p=P, budget=8,
               out=addr(6), res_out=addr(7)):
    if partials is None:
        partials = [addr(0), addr(1), addr(2), addr(3)][:max(p, 0)] or [addr(0)]
    arr = (VP * len(partials))(*partials)
    return tw.lib().tw_reduce_add_rmsnorm(arr, VP(residual), VP(weight), eps, n, h, p, budget,
                                         VP(out), VP(res_out), VP(None))


def test_fused_rejects_null_pointers():
    assert fused_call(residual=None) == E_NULL
    assert fused_call(weight=None) == E_NULL
    assert fused_call(out=None) == E_NULL
    assert fused_call(res_out=None) == E_NULL
    assert fused_call(partials=[addr(0), None]) == E_NULL
    assert tw.lib().tw_reduce_add_rmsnorm(None, VP(addr(4)), VP(addr(5)), 1e-5, N, H, P, 8,
                                         VP(addr(6)), VP(addr(7)), VP(None)) == E_NULL


def test_fused_rejects_bad_sizes():
    assert fused_call(n=-1) == E_SHAPE
    assert fused_call(h=0) == E_SHAPE
    assert fused_call(h=-8) == E_SHAPE
    assert fused_call(p=0) == E_SHAPE
    assert fused_call(partials=[addr(0)] * 17, p=17) == E_SHAPE
    assert fused_call(eps=-1.0) == E_SHAPE
    assert fused_call(eps=float("nan")) == E_SHAPE
    assert fused_call(eps=float("inf")) == E_SHAPE
    assert fused_call(h=60) == E_UNSUP        # not a multiple of 8
    assert fused_call(h=65544) == E_UNSUP     # above TW_MAX_H
    assert fused_call(n=2 ** 62, h=64) == E_SHAPE


def test_fused_rejects_misaligned_pointers():
    assert fused_call(residual=addr(4) + 2) == E_ALIGN
    assert fused_call(weight=addr(5) + 8) == E_ALIGN
    assert fused_call(out=addr(6) + 4) == E_ALIGN
    assert fused_call(res_out=addr(7) + 2) == E_ALIGN
    assert fused_call(partials=[addr(0), addr(1) + 2]) == E_ALIGN


def test_fused_aliasing_rules():
    # outputs overlapping each other, the weight, or an input at a different start
    assert fused_call(out=addr(7)) == E_ALIAS
    assert fused_call(out=addr(7) + 16) == E_ALIAS
    assert fused_call(out=addr(5)) == E_ALIAS
    assert fused_call(res_out=addr(4) + 16) == E_ALIAS       # shifted over the residual
    assert fused_call(out=addr(4)) == E_ALIAS                # out on the residual
    assert fused_call(res_out=addr(0)) == E_ALIAS            # residual_out on a partial
    assert fused_call(out=addr(1) + TENSOR - 16) == E_ALIAS  # straddles the end of a partial


@pytest.mark.skipif(tw.device_cu_count() > 0, reason="complete valid calls on made-up pointers only without a GPU")
def test_valid_calls_without_a_gpu_return_hip_error_and_allowed_aliasing_passes_validation():
    assert fused_call() == E_HIP
    assert tw.lib().tw_last_hip_error() != 0
    assert fused_call(res_out=addr(4)) == E_HIP   # in-place residual is allowed
    assert fused_call(out=addr(1)) == E_HIP       # out over a partial is allowed
    assert tw.fused_grid(4, 64, 2, 8) == -1


def test_empty_batch_is_ok_everywhere():
    assert fused_call(n=0) == OK
    assert fused_call(n=0, residual=None, out=None, res_out=None, partials=[None, None]) == OK
    assert fused_call(n=0, weight=None) == E_NULL
    assert fused_call(n=0, h=60) == E_UNSUP
    assert tw.fused_grid(0, 64, 2, 8) == 0
    assert tw.fused_grid(4, 60, 2, 8) == -1
    assert tw.fused_grid(4, 64, 0, 8) == -1 and tw.fused_grid(4, 64, 17, 8) == -1


def split_call(split_row, sa=1, sb=2, n=N, **kw):
    arr = (VP * P)(addr(0), addr(1))
    a = FusedArgs(ctypes.cast(arr, ctypes.POINTER(VP)), addr(4), addr(5), 1e-5, n, H, P, 8, addr(6), addr(7))
    for k, v in kw.items():
        setattr(a, k, v)
    return tw.lib().tw_split_launch(ctypes.byref(a), split_row, VP(sa), VP(sb), VP(None), 0, 0)


def test_split_launch_argument_checks():
    assert tw.lib().tw_split_launch(None, 0, VP(1), VP(2), VP(None), 0, 0) == E_NULL
    assert split_call(-1) == E_SPLIT
    assert split_call(N + 1) == E_SPLIT
    assert split_call(2, sa=3, sb=3) == E_SPLIT        # both halves on one stream
    assert split_call(2, H=60) == E_UNSUP              # fused validation comes first
    assert split_call(0, n=0) == OK                    # nothing to do


def unfused_call(scratch=addr(8), n=N, **kw):
    arr = (VP * P)(addr(0), addr(1))
    a = FusedArgs(ctypes.cast(arr, ctypes.POINTER(VP)), addr(4), addr(5), 1e-5, n, H, P, 8, addr(6), addr(7))
    for k, v in kw.items():
        setattr(a, k, v)
    return tw.lib().tw_reduce_add_rmsnorm_unfused(ctypes.byref(a), VP(scratch), VP(None))


def test_unfused_argument_checks():
    assert tw.lib().tw_reduce_add_rmsnorm_unfused(None, VP(addr(8)), VP(None)) == E_NULL
    assert unfused_call(scratch=None) == E_NULL
    assert unfused_call(scratch=addr(8) + 2) == E_ALIGN
    assert unfused_call(H=60) == E_UNSUP               # fused validation comes first
    assert unfused_call(H=8200, n=1) == E_UNSUP        # wider than its kernels cover
    assert unfused_call(n=0) == OK
    assert unfused_call(n=0, scratch=None) == OK       # nothing to do, nothing to check
    for other in (0, 1, 4, 5, 6, 7):                   # a partial, residual, weight, out, residual_out
        assert unfused_call(scratch=addr(other)) == E_ALIAS
    assert unfused_call(scratch=addr(6) + TENSOR - 16) == E_ALIAS


def static_call(n=N, **kw):
    arr = (VP * P)(addr(0), addr(1))
    a = FusedArgs(ctypes.cast(arr, ctypes.POINTER(VP)), addr(4), addr(5), 1e-5, n, H, P, 8, addr(6), addr(7))
    for k, v in kw.items():
        setattr(a, k, v)
    return tw.lib().tw_reduce_add_rmsnorm_unfused_static(ctypes.byref(a), VP(None))


def test_unfused_static_argument_checks():
    """The entry point that allocates nothing rejects what does not fit its built-in buffer on the
    host, before any HIP call."""
    assert tw.lib().tw_reduce_add_rmsnorm_unfused_static(None, VP(None)) == E_NULL
    assert static_call(H=60) == E_UNSUP
    assert static_call(H=8200, n=1) == E_UNSUP
    assert static_call(n=0) == OK
    assert static_call(P=0) == E_SHAPE
    assert static_call(out=addr(7)) == E_ALIAS          # the fused call's own rules still apply
    limit = tw.STATIC_SCRATCH_BYTES
    text = open(os.path.join(ROOT, "include", "tw.h")).read()
    assert re.search(r"#define\s+TW_STATIC_SCRATCH_BYTES\s+\(32u\s*<<\s*20\)", text) and limit == 32 << 20
    rows = limit // (8192 * 2)
    # tensors far enough apart not to overlap at this size; one row too many is refused
    far = lambda i: BASE + i * (1 << 32)
    arr = (VP * P)(far(0), far(1))
    a = FusedArgs(ctypes.cast(arr, ctypes.POINTER(VP)), far(4), far(5), 1e-5, rows + 1, 8192, P, 0, far(6), far(7))
    assert tw.lib().tw_reduce_add_rmsnorm_unfused_static(ctypes.byref(a), VP(None)) == E_SHAPE


def test_split_point_matches_its_definition():
    # independent statement: the smallest multiple of m that is >= N/2, capped at N
    for n in list(range(0, 70)) + [127, 128, 129, 255, 256, 1000, 1024, 4096, 16384, 10 ** 12 + 7]:
        for m in (1, 2, 3, 64, 128, 1000):
            want = next((k for k in range(0, n + m, m) if 2 * k >= n), n) if n < 10 ** 6 else None
            if want is None:
                q = -(-n // 2)
                want = -(-q // m) * m
            want = min(want, n)
            assert tw.split_point(n, m) == want, (n, m)
    assert tw.split_point(-5, 128) == 0
    assert tw.split_point(100, 0) == 50
    assert tw.split_point(100, -3) == 50
    assert tw.split_point(2 ** 62, 2 ** 62) == 2 ** 62
    for n in (256, 1024, 4096, 16384):                  # the sweep's sizes: exactly N/2
        assert tw.split_point(n, 128) == n // 2


def gemm_call(A=addr(0), B=addr(20), C=addr(40), M=16, Nn=16, K=16, layout=0):
    return tw.lib().tw_gemm_bf16(VP(A), VP(B), VP(C), M, Nn, K, layout, 0, VP(None))


def test_gemm_argument_checks():
    assert gemm_call(M=-1) == E_SHAPE
    assert gemm_call(layout=7) == E_SHAPE
    assert gemm_call(M=0) == OK
    assert gemm_call(Nn=0) == OK
    assert gemm_call(C=None) == E_NULL
    assert gemm_call(A=None) == E_NULL
    assert gemm_call(K=12) == E_UNSUP
    assert gemm_call(Nn=12) == E_UNSUP
    # a tile's rows are addressed with 32-bit byte offsets: K and N stop at 2^22
    assert gemm_call(K=(1 << 22) + 8) == E_UNSUP
    assert gemm_call(Nn=(1 << 22) + 8) == E_UNSUP
    assert gemm_call(A=addr(0) + 2) == E_ALIGN
    assert gemm_call(C=addr(0)) == E_ALIAS
    assert gemm_call(C=addr(20) + 16) == E_ALIAS


def test_overlap_launch_argument_checks():
    L = tw.lib()
    assert L.tw_overlap_launch(None, None, VP(1), VP(2), VP(None), 0, 0) == E_NULL
    arr = (VP * P)(addr(0), addr(1))
    f = FusedArgs(ctypes.cast(arr, ctypes.POINTER(VP)), addr(4), addr(5), 1e-5, N, H, P, 8, addr(6), addr(7))
    g = GemmArgs(addr(0), addr(20), addr(40), 16, 16, 16, 0, 0)
    assert L.tw_overlap_launch(ctypes.byref(f), ctypes.byref(g), VP(3), VP(3), VP(None), 0, 0) == E_SPLIT
    f.H = 60
    assert L.tw_overlap_launch(ctypes.byref(f), ctypes.byref(g), VP(1), VP(2), VP(None), 0, 0) == E_UNSUP
    f.H = H
    g.K = 12
    assert L.tw_overlap_launch(ctypes.byref(f), ctypes.byref(g), VP(1), VP(2), VP(None), 0, 0) == E_UNSUP


def test_probe_argument_checks():
    L = tw.lib()
    assert L.tw_hbm_probe(VP(addr(0)), VP(addr(9)), 1024, 9, 8, VP(None)) == E_SHAPE
    assert L.tw_hbm_probe(VP(None), VP(addr(9)), 1024, tw.PROBE_READ, 8, VP(None)) == E_NULL
    assert L.tw_hbm_probe(VP(addr(0)), VP(None), 1024, tw.PROBE_COPY, 8, VP(None)) == E_NULL
    assert L.tw_hbm_probe(VP(addr(0)), VP(addr(9)), 1000, tw.PROBE_COPY, 8, VP(None)) == E_SHAPE
    assert L.tw_hbm_probe(VP(addr(0)), VP(addr(9)), -16, tw.PROBE_COPY, 8, VP(None)) == E_SHAPE
    assert L.tw_hbm_probe(VP(addr(0) + 4), VP(addr(9)), 1024, tw.PROBE_COPY, 8, VP(None)) == E_ALIGN
    assert L.tw_hbm_probe(VP(addr(0)), VP(addr(0) + 512), 1024, tw.PROBE_COPY, 8, VP(None)) == E_ALIAS
    assert L.tw_hbm_probe(VP(addr(0)), VP(addr(9)), 0, tw.PROBE_COPY, 8, VP(None)) == OK


def test_shaped_probe_argument_checks():
    L = tw.lib()
    ok_args = (VP(addr(0)), VP(addr(9)), 1024, tw.PROBE_COPY, 8)
    for threads in (0, 32, 100, 1088, -64):
        assert L.tw_hbm_probe_shaped(*ok_args, threads, 8, VP(None)) == E_SHAPE
    for depth in (0, 3, 5, 32, -1):
        assert L.tw_hbm_probe_shaped(*ok_args, 256, depth, VP(None)) == E_UNSUP
    assert L.tw_hbm_probe_shaped(VP(addr(0)), VP(addr(9)), 0, tw.PROBE_COPY, 8, 192, 16, VP(None)) == OK
    sb = 16384 * 4
    for threads in (0, 96, 192, 768, 2048):       # must divide the 1024-vector granule
        assert L.tw_hbm_probe_mixed_shaped(VP(addr(0)), VP(addr(2000)), sb, 9, 2, 8, threads, VP(None)) == E_SHAPE
    assert L.tw_hbm_probe_mixed_shaped(VP(addr(0)), VP(addr(2000)), 0, 9, 2, 8, 256, VP(None)) == OK


def test_streams_overlap_argument_checks():
    L = tw.lib()
    assert L.tw_streams_overlap(VP(1), VP(2), None) == E_NULL
    yes = ctypes.c_int(7)
    assert L.tw_streams_overlap(VP(3), VP(3), ctypes.byref(yes)) == OK and yes.value == 0   # one stream: no


def test_mixed_probe_argument_checks():
    L = tw.lib()
    sb = 1 << 20
    assert L.tw_hbm_probe_mixed(VP(addr(0)), VP(addr(2000)), sb, 0, 0, 8, VP(None)) == E_SHAPE
    assert L.tw_hbm_probe_mixed(VP(addr(0)), VP(addr(2000)), sb, 18, 2, 8, VP(None)) == E_SHAPE
    assert L.tw_hbm_probe_mixed(VP(addr(0)), VP(addr(2000)), sb, 9, 5, 8, VP(None)) == E_SHAPE
    assert L.tw_hbm_probe_mixed(VP(addr(0)), VP(addr(2000)), sb + 16, 9, 2, 8, VP(None)) == E_SHAPE
    assert L.tw_hbm_probe_mixed(VP(None), VP(addr(2000)), sb, 9, 2, 8, VP(None)) == E_NULL
    assert L.tw_hbm_probe_mixed(VP(addr(0)), VP(None), sb, 9, 2, 8, VP(None)) == E_NULL
    assert L.tw_hbm_probe_mixed(VP(addr(0) + 8), VP(addr(2000)), sb, 9, 2, 8, VP(None)) == E_ALIGN
    assert L.tw_hbm_probe_mixed(VP(addr(0)), VP(addr(0) + 8 * sb), sb, 9, 2, 8, VP(None)) == E_ALIAS
    assert L.tw_hbm_probe_mixed(VP(addr(0)), VP(addr(2000)), 0, 9, 2, 8, VP(None)) == OK


def test_smart_split_point_matches_its_definition():
    """Independent statement of the criterion: among k = base + j*multiple (k < T,
    offset <= 512) take the fewest total GEMM waves, ties to the fewest 256-row tiles
    over both splits, then to the smallest k."""
    tm, tn = tw.gemm_tile_shape()
    assert (tm, tn) == (256, 128)

    def waves(rows, n, cus):
        if rows <= 0:
            return 0
        return -(-(-(-rows // tm) * -(-n // tn)) // cus)

    for T in (0, 1, 64, 100, 255, 256, 257, 1000, 1024, 2048, 3000, 4096, 8192, 16384, 20000):
        for mult in (64, 128):
            for widths in ([8192], [8192, 3584], [4096, 14336, 1024]):
                for cus in (224, 256, 132, 8):
                    k, ws, wu = tw.smart_split_point(T, mult, widths, cus)
                    base = tw.split_point(T, mult)
                    want_u = sum(waves(T, n, cus) for n in widths)
                    assert wu == want_u
                    if base >= T:
                        assert k == T and ws == wu
                        continue
                    cands = [c for c in range(base, T, mult) if c - base <= 512]
                    cost = {c: sum(waves(c, n, cus) + waves(T - c, n, cus) for n in widths) for c in cands}
                    tiles = {c: -(-c // tm) + -(-(T - c) // tm) for c in cands}
                    best = min(cands, key=lambda c: (cost[c], tiles[c], c))
                    assert (k, ws) == (best, cost[best]), (T, mult, widths, cus)
                    # with depths, a wave of GEMM i weighs depths[i]
                    depths = [1024, 8192, 512][:len(widths)]
                    k, ws, wu = tw.smart_split_point(T, mult, widths, cus, gemm_k=depths)
                    cost = {c: sum((waves(c, n, cus) + waves(T - c, n, cus)) * d for n, d in zip(widths, depths))
                            for c in cands}
                    best = min(cands, key=lambda c: (cost[c], tiles[c], c))
                    assert (k, ws) == (best, cost[best]), (T, mult, widths, cus)
                    assert wu == sum(waves(T, n, cus) * d for n, d in zip(widths, depths))
    # the situation of the paper's example (Section 4.1.1): 300 workgroups (10 row
    # tiles x 30 column tiles) on 132 units are 3 waves; the even cut (150 + 150)
    # needs 2 + 2 = 4, moving one row tile to the prefix (180 + 120) needs 2 + 1 = 3
    k, ws, wu = tw.smart_split_point(10 * 256, 256, [30 * 128], 132)
    assert (k, ws, wu) == (6 * 256, 3, 3)
    assert tw.smart_split_point(-1, 64, [8], 8)[0] == -1
    assert tw.smart_split_point(64, 64, [], 8)[0] == -1
    assert tw.smart_split_point(64, 64, [0], 8)[0] == -1
    assert tw.smart_split_point(64, 64, [8], 0)[0] == -1
    assert tw.smart_split_point(64, 64, [8], 8, gemm_k=[0])[0] == -1
    # a cut that saves one long wave at the price of one short wave is taken only
    # when the depths say so: T=5632 over widths 8192 (depth 1024) and 3584 (depth
    # 8192) on 256 units -- 2816+2816 and 3328+2304 both make 10 waves, but the
    # second has one deep wave fewer
    assert tw.smart_split_point(5632, 64, [8192, 3584], 256)[0] == 2816
    assert tw.smart_split_point(5632, 64, [8192, 3584], 256, gemm_k=[1024, 8192])[0] == 3328


def test_weave_layer_argument_checks():
    from paper_2505_11329_amd.binding import LayerArgs
    L = tw.lib()
    assert L.tw_weave_layer(None, 0, VP(1), VP(2), VP(None), 0, 0) == E_NULL
    arr = (VP * P)(addr(0), addr(1))
    f = FusedArgs(ctypes.cast(arr, ctypes.POINTER(VP)), addr(4), addr(5), 1e-5, N, H, P, 8, addr(6), addr(7))
    la = LayerArgs(addr(10), addr(11), 64, f, addr(12), 64, addr(13), 0)
    assert L.tw_weave_layer(ctypes.byref(la), -1, VP(1), VP(2), VP(None), 0, 0) == E_SPLIT
    assert L.tw_weave_layer(ctypes.byref(la), N + 1, VP(1), VP(2), VP(None), 0, 0) == E_SPLIT
    assert L.tw_weave_layer(ctypes.byref(la), 2, VP(3), VP(3), VP(None), 0, 0) == E_SPLIT
    la.K1 = 12
    assert L.tw_weave_layer(ctypes.byref(la), 2, VP(1), VP(2), VP(None), 0, 0) == E_UNSUP
    la.K1 = 64
    la.N2 = 12
    assert L.tw_weave_layer(ctypes.byref(la), 2, VP(1), VP(2), VP(None), 0, 0) == E_UNSUP
    la.N2 = 64
    la.X1 = None
    assert L.tw_weave_layer(ctypes.byref(la), 2, VP(1), VP(2), VP(None), 0, 0) == E_NULL
    la.X1 = addr(10)
    la.Y = addr(6)          # Y on top of the fused output it is computed from
    assert L.tw_weave_layer(ctypes.byref(la), 2, VP(1), VP(2), VP(None), 0, 0) == E_ALIAS
    la.Y = addr(13)
    # a fused output on top of an operand another split's GEMM is still reading
    for field, target in (("out", 10), ("out", 11), ("out", 12), ("residual_out", 10), ("residual_out", 11),
                          ("residual_out", 12)):
        keep = getattr(la.fused, field)
        setattr(la.fused, field, addr(target))
        assert L.tw_weave_layer(ctypes.byref(la), 2, VP(1), VP(2), VP(None), 0, 0) == E_ALIAS, (field, target)
        assert L.tw_weave_layer(ctypes.byref(la), 0, VP(1), VP(2), VP(None), 0, 0) == E_ALIAS, (field, target)
        setattr(la.fused, field, keep)
    la.fused.H = 60
    assert L.tw_weave_layer(ctypes.byref(la), 2, VP(1), VP(2), VP(None), 0, 0) == E_UNSUP
    la.fused.H = H
    for bad in (-1, 3, 99):
        la.schedule = bad
        assert L.tw_weave_layer(ctypes.byref(la), 2, VP(1), VP(2), VP(None), 0, 0) == E_UNSUP
    la.fused.N = 0
    for schedule in (tw.WEAVE_AUTO, tw.WEAVE_ORDERED, tw.WEAVE_CHAINS):
        la.schedule = schedule
        assert L.tw_weave_layer(ctypes.byref(la), 0, VP(1), VP(2), VP(None), 0, 0) == OK


def test_weave_layer_cuts_argument_checks():
    from paper_2505_11329_amd.binding import LayerArgs
    L = tw.lib()
    I64 = ctypes.c_int64

    def call(la, cuts, n=None, sx=1, sc=2):
        arr = (I64 * max(len(cuts), 1))(*cuts)
        return L.tw_weave_layer_cuts(ctypes.byref(la) if la is not None else None, arr, len(cuts) if n is None else n,
                                     VP(sx), VP(sc), VP(None), 0, 0)
    arr = (VP * P)(addr(0), addr(1))
    f = FusedArgs(ctypes.cast(arr, ctypes.POINTER(VP)), addr(4), addr(5), 1e-5, N, H, P, 8, addr(6), addr(7))
    la = LayerArgs(addr(10), addr(11), 64, f, addr(12), 64, addr(13), 0)
    assert call(None, [2]) == E_NULL
    assert L.tw_weave_layer_cuts(ctypes.byref(la), None, 1, VP(1), VP(2), VP(None), 0, 0) == E_NULL
    assert call(la, [2], n=-1) == E_SPLIT
    assert call(la, list(range(1, 17)), n=16) == E_SPLIT          # more than TW_MAX_CUTS
    for bad in ([0], [N], [N + 1], [-1], [2, 2], [3, 2], [1, 2, 2], [1, 3, N]):
        assert call(la, bad) == E_SPLIT, bad
    assert call(la, [2], sx=3, sc=3) == E_SPLIT
    la.Y = addr(6)
    assert call(la, [1, 2, 3]) == E_ALIAS
    assert call(la, []) == E_ALIAS
    la.Y = addr(13)
    la.schedule = 9
    assert call(la, [1, 2]) == E_UNSUP
    la.schedule = 0
    la.fused.N = 0                  # an empty batch has no row to cut at
    assert call(la, []) == OK
    assert call(la, [1]) == E_SPLIT


def test_weave_train_argument_checks():
    """Every boundary of a train is checked before anything is launched."""
    from paper_2505_11329_amd.binding import LayerArgs
    L = tw.lib()
    arr = (VP * P)(addr(0), addr(1))

    def boundary(n=N):
        f = FusedArgs(ctypes.cast(arr, ctypes.POINTER(VP)), addr(4), addr(5), 1e-5, n, H, P, 8, addr(6), addr(7))
        return LayerArgs(addr(10), addr(11), 64, f, addr(12), 64, addr(13), 0)
    las = (LayerArgs * 3)(boundary(), boundary(), boundary())

    def call(n=3, split=2, sx=1, sc=2, ptr=las):
        return L.tw_weave_train(ptr, n, split, VP(sx), VP(sc), VP(None), 0, 0)
    assert call(n=-1) == E_SHAPE
    assert call(n=4097) == E_SHAPE
    assert call(n=0, ptr=None) == OK
    assert call(ptr=None) == E_NULL
    assert call(split=-1) == E_SPLIT
    assert call(split=N + 1) == E_SPLIT
    assert call(sx=3, sc=3) == E_SPLIT
    las[2].fused.N = N + 1                     # token counts differ
    assert call() == E_SHAPE
    las[2].fused.N = N
    las[1].Y = addr(6)                         # the second boundary's Y on top of its fused output
    assert call() == E_ALIAS
    las[1].Y = addr(13)
    las[2].K1 = 12
    assert call() == E_UNSUP
    las[2].K1 = 64
    for i in range(3):
        las[i].fused.N = 0                     # an empty train: nothing to launch
    assert call(split=0) == OK
    assert call(split=1) == E_SPLIT


def test_split_threshold_matches_its_definition():
    """tw_split_threshold restated: never when the GEMM after the fused step is the shorter of the two
    (N2 < 200 (P + 3)); else the larger of 'the fused step takes 290 us at 5 TB/s' and 'half the batch
    still tiles the narrower GEMM output over half of the compute units', in whole 256-row tiles."""
    import math
    never = 2 ** 63 - 1
    for (K1, Hh, Pp, N2, cus) in [(1024, 8192, 8, 3584, 256), (3584, 8192, 8, 1280, 256), (3584, 8192, 4, 1280, 256),
                                  (512, 4096, 2, 4096, 256), (1024, 8192, 8, 3584, 64), (8, 8, 1, 8, 1),
                                  (8, 8, 1, 800, 1), (4096, 16384, 16, 128, 304), (4096, 16384, 16, 3800, 304),
                                  (1024, 8192, 8, 2200, 256), (1024, 8192, 8, 2192, 256)]:
        if N2 < 200 * (Pp + 3):
            want = never
        else:
            t_gain = math.floor(290.0 * 5.0e6 / (2.0 * Hh * (Pp + 3))) + 1
            col_tiles = -(-min(Hh, N2) // 128)
            t_fill = 2 * 256 * -(-((cus + 1) // 2) // col_tiles)
            want = -(-max(t_gain, t_fill) // 256) * 256
        assert tw.split_threshold(K1, Hh, Pp, N2, cus) == want, (K1, Hh, Pp, N2, cus)
    assert tw.split_threshold(1024, 8192, 8, 3584, 256) == 8192      # the figures tw.h quotes
    assert tw.split_threshold(3584, 8192, 8, 1280, 256) == never
    assert not tw.should_split(10 ** 9, never)
    for bad in ((0, 8192, 8, 3584, 256), (1024, 0, 8, 3584, 256), (1024, 8192, 0, 3584, 256),
                (1024, 8192, 8, 0, 256), (1024, 8192, 8, 3584, 0)):
        assert tw.split_threshold(*bad) == -1


def test_policy_split_row_follows_threshold_band_and_wave_criterion():
    """tw_policy_split_row restated from its parts (Fig. 3; Section 4.1.1): a caller's threshold is the
    whole rule; the built-in one never splits a boundary whose threshold is 'never', always from the
    threshold up, and above half of it and below it only when the cut's GEMM waves (tw_smart_split_point's
    costs) do not exceed the whole batch's."""
    K1, Hh, Pp, N2, cus = 1024, 8192, 8, 3584, 256
    thr = tw.split_threshold(K1, Hh, Pp, N2, cus)
    assert thr == 8192
    for T in list(range(0, 20000, 448)) + [4096, 4352, 4608, 6144, 7168, 8192, 8191, 4095]:
        k, cs, cu_ = tw.smart_split_point(T, 64, [Hh, N2], cus, gemm_k=[K1, Hh])
        if T <= thr // 2 or k >= T:
            want = T
        elif T >= thr:
            want = k
        else:
            want = k if cs <= cu_ else T
        assert tw.policy_split_row(T, K1, Hh, Pp, N2, cus) == want, T
        # a caller's threshold: nothing but the comparison
        for t_user in (1, 3000, 8192):
            assert tw.policy_split_row(T, K1, Hh, Pp, N2, cus, threshold=t_user) == (k if T >= t_user else T), (T, t_user)
    # the band, by hand (256 x 128 tiles on 256 compute units, waves weighted by depth): 17 row tiles
    # unsplit are 5 + 2 waves, 9 + 8 row tiles are (3 + 1) + (2 + 1): the same -> split at 2304
    assert tw.policy_split_row(4352, K1, Hh, Pp, N2, cus) == 2304
    # 18 row tiles unsplit: 5 + 2 waves; 9 + 9: (3 + 1) + (3 + 1): one shallow wave more -> unsplit
    assert tw.policy_split_row(4608, K1, Hh, Pp, N2, cus) == 4608
    assert tw.policy_split_row(6144, K1, Hh, Pp, N2, cus) == 6144
    assert tw.policy_split_row(7168, K1, Hh, Pp, N2, cus) == 4096
    # the MLP-side boundary never splits by itself, and does with a caller's threshold
    assert tw.policy_split_row(16384, 3584, 8192, 8, 1280, cus) == 16384
    assert tw.policy_split_row(16384, 3584, 8192, 8, 1280, cus, threshold=4096) == 8192
    # another multiple moves the candidates
    assert tw.policy_split_row(8192 + 128, K1, Hh, Pp, N2, cus, multiple=128) % 128 == 0
    for bad in ((-1, K1, Hh, Pp, N2, cus), (4096, 0, Hh, Pp, N2, cus), (4096, K1, 0, Pp, N2, cus),
                (4096, K1, Hh, 0, N2, cus), (4096, K1, Hh, Pp, 0, cus), (4096, K1, Hh, Pp, N2, 0)):
        assert tw.policy_split_row(*bad) == -1


def test_weave_layer_auto_argument_checks():
    from paper_2505_11329_amd.binding import LayerArgs
    L = tw.lib()
    taken = ctypes.c_int64(-7)
    assert L.tw_weave_layer_auto(None, 0, 0, VP(1), VP(2), VP(None), 0, 0, ctypes.byref(taken)) == E_NULL
    arr = (VP * P)(addr(0), addr(1))
    f = FusedArgs(ctypes.cast(arr, ctypes.POINTER(VP)), addr(4), addr(5), 1e-5, N, H, P, 8, addr(6), addr(7))
    la = LayerArgs(addr(10), addr(11), 64, f, addr(12), 64, addr(13), 0)
    la.fused.H = 60
    assert L.tw_weave_layer_auto(ctypes.byref(la), 0, 0, VP(1), VP(2), VP(None), 0, 0, None) == E_UNSUP
    la.fused.H = H
    la.K1 = -8
    assert L.tw_weave_layer_auto(ctypes.byref(la), 0, 0, VP(1), VP(2), VP(None), 0, 0, None) == E_SHAPE
    la.K1 = 64
    la.fused.N = 0              # an empty batch: nothing to decide, nothing to launch
    assert L.tw_weave_layer_auto(ctypes.byref(la), 0, 0, VP(1), VP(2), VP(None), 0, 0, ctypes.byref(taken)) == OK
    assert taken.value == 0


def test_weave_tune_argument_checks():
    """The offline search refuses bad arguments before it creates an event or launches anything."""
    from paper_2505_11329_amd.binding import LayerArgs
    L = tw.lib()
    best = ctypes.c_int64(-7)
    us = (ctypes.c_float * 18)()
    offs = (ctypes.c_int64 * 17)(*range(0, 17 * 64, 64))
    arr = (VP * P)(addr(0), addr(1))
    f = FusedArgs(ctypes.cast(arr, ctypes.POINTER(VP)), addr(4), addr(5), 1e-5, N, H, P, 8, addr(6), addr(7))
    la = LayerArgs(addr(10), addr(11), 64, f, addr(12), 64, addr(13), 0)
    ok_args = (0, offs, 2, 3, VP(1), VP(2), ctypes.byref(best), us)
    assert L.tw_weave_tune(None, *ok_args) == E_NULL
    assert L.tw_weave_tune(ctypes.byref(la), 0, offs, 2, 3, VP(1), VP(2), None, us) == E_NULL
    assert L.tw_weave_tune(ctypes.byref(la), 0, offs, 2, 3, VP(1), VP(2), ctypes.byref(best), None) == E_NULL
    assert L.tw_weave_tune(ctypes.byref(la), 0, None, 2, 3, VP(1), VP(2), ctypes.byref(best), us) == E_NULL
    for reps in (0, -1, 65):
        assert L.tw_weave_tune(ctypes.byref(la), 0, offs, 2, reps, VP(1), VP(2), ctypes.byref(best), us) == E_SHAPE
    for n_off in (-1, 17):
        assert L.tw_weave_tune(ctypes.byref(la), 0, offs, n_off, 3, VP(1), VP(2), ctypes.byref(best), us) == E_SHAPE
    la.fused.H = 60
    assert L.tw_weave_tune(ctypes.byref(la), *ok_args) == E_UNSUP
    la.fused.H = H
    la.N2 = -8
    assert L.tw_weave_tune(ctypes.byref(la), *ok_args) == E_SHAPE


def test_traced_gemm_argument_checks():
    L = tw.lib()
    L.tw_gemm_bf16_traced.argtypes = [VP, VP, VP, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, VP, ctypes.c_int64, VP]
    small = (256, 128, 64)      # operands of 32, 16 and 64 KiB at the fake addresses
    assert L.tw_gemm_bf16_traced(addr(0), addr(1), None, *small, addr(6), 1 << 20, None) == E_NULL
    assert L.tw_gemm_bf16_traced(addr(0), addr(1), addr(3), *small, None, 1 << 20, None) == E_NULL
    assert L.tw_gemm_bf16_traced(addr(0), addr(1), addr(3), 256, 128, 60, addr(6), 1 << 20, None) == E_UNSUP
    assert L.tw_gemm_bf16_traced(addr(0), addr(1), addr(3), -1, 128, 64, addr(6), 1 << 20, None) == E_SHAPE
    assert L.tw_gemm_bf16_traced(addr(0), addr(1), addr(0), *small, addr(6), 1 << 20, None) == E_ALIAS


def test_fused_layout_covers_every_row_width_without_idle_waves():
    """Host arithmetic of the budgeted kernel's launch shape, for every H it takes."""
    for H in list(range(8, 8192 + 8, 8)) + list(range(8192, 65536 + 1, 264)) + [65536]:
        H -= H % 8
        wpr, vpt, rows, block = tw.fused_layout(H)
        hv = H // 8
        assert vpt in (1, 2, 4, 8) and 64 <= block <= 1024 and block % 64 == 0, H
        if hv <= 64:
            assert wpr == 0 and vpt == 1 and block == 1024, H
            lanes = 1024 // rows                      # a power of two, the smallest that holds the row
            assert lanes * rows == 1024 and lanes >= hv and (lanes == 1 or lanes // 2 < hv), H
            continue
        assert 2 <= wpr <= 16, H
        assert wpr * 64 * vpt >= hv, H                # the row's waves cover it
        assert (wpr - 1) * 64 * vpt < hv, H           # and none of them is idle
        assert vpt == 1 or hv > 1024 * vpt // 2, H    # no more vectors per thread than the width asks for
        assert rows == 16 // wpr and block == rows * wpr * 64, H
    assert tw.fused_layout(8192) == (16, 1, 1, 1024)
    assert tw.fused_layout(5120) == (10, 1, 1, 640)
    assert tw.fused_layout(3072) == (6, 1, 2, 768)
    assert tw.fused_layout(12288) == (12, 2, 1, 768)
    L = tw.lib()
    assert L.tw_fused_layout(0, None, None, None, None) == E_SHAPE
    assert L.tw_fused_layout(12, None, None, None, None) == E_UNSUP
    assert L.tw_fused_layout(65536 + 8, None, None, None, None) == E_UNSUP
    assert L.tw_fused_layout(4096, None, None, None, None) == OK


def test_weave_schedule_is_chains_unless_the_fused_kernel_has_a_budget():
    O, C = tw.WEAVE_ORDERED, tw.WEAVE_CHAINS
    attn = dict(K1=1024, H=8192, P=8, N2=3584)
    mlp = dict(K1=3584, H=8192, P=8, N2=1280)
    assert [tw.weave_schedule(T, **attn) for T in (1024, 4096, 6144, 8192, 16384)] == [C] * 5
    assert [tw.weave_schedule(T, **mlp) for T in (1024, 4096, 6144, 8192, 16384)] == [C] * 5
    assert tw.weave_schedule(16384, K1=2048, H=4096, P=2, N2=2048) == C
    # a fused kernel confined to a CU budget keeps the ordered schedule; a budget that is the
    # whole device does not count as one
    assert tw.weave_schedule(4096, fused_cu_budget=32, **attn) == O
    assert tw.weave_schedule(4096, fused_cu_budget=0, **attn) == C
    assert tw.weave_schedule(4096, fused_cu_budget=256, **attn) == C
    # an explicit schedule is passed through
    assert tw.weave_schedule(4096, schedule=O, **attn) == O and tw.weave_schedule(16384, schedule=C, **attn) == C
    assert tw.weave_schedule(4096, schedule=7, **attn) == -1 and tw.weave_schedule(-1, **attn) == -1
    assert tw.weave_schedule(4096, cus=0, **attn) == -1


def test_should_split_threshold():
    assert not tw.should_split(0) and not tw.should_split(8191)
    assert tw.should_split(8192) and tw.should_split(10 ** 6)
    assert tw.should_split(1024, 1024) and not tw.should_split(1023, 1024)
    assert tw.should_split(8192, -5) and not tw.should_split(100, 0)
