"""ctypes binding of include/tw.h and include/tw_measure.h. Argument marshalling only.

Tensors are torch tensors on the GPU (bfloat16, contiguous); the binding passes
their data_ptr() and sizes. Streams are torch.cuda.Stream objects (or None for
the current stream). Every function raises TwError on a non-zero status.
"""
import ctypes
import os
import threading

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtw.so")
_lock = threading.Lock()
_lib = None

STATUS = {0: "TW_OK", 1: "TW_ERR_NULL", 2: "TW_ERR_SHAPE", 3: "TW_ERR_ALIGN", 4: "TW_ERR_ALIAS",
          5: "TW_ERR_UNSUPPORTED", 6: "TW_ERR_SPLIT", 7: "TW_ERR_HIP"}
PROBE_READ, PROBE_COPY, PROBE_WRITE = 0, 1, 2
B_NK, B_KN = 0, 1
CU_SHARED = -1
WEAVE_AUTO, WEAVE_ORDERED, WEAVE_CHAINS = 0, 1, 2
MAX_P = 16
STATIC_SCRATCH_BYTES = 32 << 20

_vp = ctypes.c_void_p
_i64 = ctypes.c_int64


class FusedArgs(ctypes.Structure):
    """struct tw_fused_args"""
    _fields_ = [("partials", ctypes.POINTER(_vp)), ("residual", _vp), ("weight", _vp),
                ("eps", ctypes.c_float), ("N", _i64), ("H", _i64), ("P", ctypes.c_int),
                ("cu_budget", ctypes.c_int), ("out", _vp), ("residual_out", _vp)]


class GemmArgs(ctypes.Structure):
    """struct tw_gemm_args"""
    _fields_ = [("A", _vp), ("B", _vp), ("C", _vp), ("M", _i64), ("N", _i64), ("K", _i64),
                ("b_layout", ctypes.c_int), ("cu_budget", ctypes.c_int)]


class LayerArgs(ctypes.Structure):
    """struct tw_layer_args"""
    _fields_ = [("X1", _vp), ("W1", _vp), ("K1", _i64), ("fused", FusedArgs), ("W2", _vp), ("N2", _i64),
                ("Y", _vp), ("gemm_cu_budget", ctypes.c_int), ("schedule", ctypes.c_int)]


class TwError(RuntimeError):
    def __init__(self, status, what):
        self.status = int(status)
        msg = "%s failed: %s (%s)" % (what, STATUS.get(self.status, self.status), status_str(self.status))
        if self.status == 7:
            msg += " hipError=%d at %s" % (lib().tw_last_hip_error(), lib().tw_last_hip_error_where().decode())
        super().__init__(msg)


def library_path():
    return _LIB_PATH


def lib():
    """The loaded libtw.so (built with hipcc first if it is not there)."""
    global _lib
    with _lock:
        if _lib is not None:
            return _lib
        if not os.path.exists(_LIB_PATH):
            from .build import build_libtw
            build_libtw()
        # libtw must share ONE HIP runtime with PyTorch (streams and device
        # pointers cross the boundary). PyTorch ships its own libamdhip64 with
        # the same soname as the system one: importing torch first puts that
        # copy in the process, and the loader then resolves libtw's dependency
        # to it instead of opening a second runtime.
        import torch  # noqa: F401
        L = ctypes.CDLL(_LIB_PATH)
        fused_sig = [ctypes.POINTER(_vp), _vp, _vp, ctypes.c_float, _i64, _i64, ctypes.c_int,
                     ctypes.c_int, _vp, _vp]
        L.tw_reduce_add_rmsnorm.argtypes = fused_sig + [_vp]
        L.tw_reduce_add_rmsnorm.restype = ctypes.c_int
        L.tw_reduce_add_rmsnorm_traced.argtypes = fused_sig + [_vp, _i64, _vp]
        L.tw_reduce_add_rmsnorm_traced.restype = ctypes.c_int
        L.tw_fused_grid.argtypes = [_i64, _i64, ctypes.c_int, ctypes.c_int]
        L.tw_fused_grid.restype = _i64
        L.tw_reduce_add_rmsnorm_unfused.argtypes = [ctypes.POINTER(FusedArgs), _vp, _vp]
        L.tw_reduce_add_rmsnorm_unfused.restype = ctypes.c_int
        L.tw_reduce_add_rmsnorm_unfused_static.argtypes = [ctypes.POINTER(FusedArgs), _vp]
        L.tw_reduce_add_rmsnorm_unfused_static.restype = ctypes.c_int
        L.tw_split_launch.argtypes = [ctypes.POINTER(FusedArgs), _i64, _vp, _vp, _vp, ctypes.c_int, ctypes.c_int]
        L.tw_split_launch.restype = ctypes.c_int
        L.tw_split_point.argtypes = [_i64, _i64]
        L.tw_split_point.restype = _i64
        L.tw_gemm_bf16.argtypes = [_vp, _vp, _vp, _i64, _i64, _i64, ctypes.c_int, ctypes.c_int, _vp]
        L.tw_gemm_bf16.restype = ctypes.c_int
        L.tw_overlap_launch.argtypes = [ctypes.POINTER(FusedArgs), ctypes.POINTER(GemmArgs), _vp, _vp, _vp,
                                        ctypes.c_int, ctypes.c_int]
        L.tw_overlap_launch.restype = ctypes.c_int
        L.tw_hbm_probe.argtypes = [_vp, _vp, _i64, ctypes.c_int, ctypes.c_int, _vp]
        L.tw_hbm_probe.restype = ctypes.c_int
        L.tw_weave_layer.argtypes = [ctypes.POINTER(LayerArgs), _i64, _vp, _vp, _vp, ctypes.c_int, ctypes.c_int]
        L.tw_weave_layer.restype = ctypes.c_int
        L.tw_weave_layer_cuts.argtypes = [ctypes.POINTER(LayerArgs), ctypes.POINTER(_i64), ctypes.c_int, _vp, _vp, _vp,
                                          ctypes.c_int, ctypes.c_int]
        L.tw_weave_layer_cuts.restype = ctypes.c_int
        L.tw_weave_train.argtypes = [ctypes.POINTER(LayerArgs), ctypes.c_int, _i64, _vp, _vp, _vp, ctypes.c_int,
                                     ctypes.c_int]
        L.tw_weave_train.restype = ctypes.c_int
        L.tw_weave_layer_auto.argtypes = [ctypes.POINTER(LayerArgs), _i64, _i64, _vp, _vp, _vp, ctypes.c_int, ctypes.c_int,
                                          ctypes.POINTER(_i64)]
        L.tw_weave_layer_auto.restype = ctypes.c_int
        L.tw_weave_tune.argtypes = [ctypes.POINTER(LayerArgs), _i64, ctypes.POINTER(_i64), ctypes.c_int, ctypes.c_int,
                                    _vp, _vp, ctypes.POINTER(_i64), ctypes.POINTER(ctypes.c_float)]
        L.tw_weave_tune.restype = ctypes.c_int
        L.tw_gemm_bf16_traced.argtypes = [_vp, _vp, _vp, _i64, _i64, _i64, _vp, _i64, _vp]
        L.tw_gemm_bf16_traced.restype = ctypes.c_int
        L.tw_stream_create_cu_masked.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(_vp)]
        L.tw_stream_create_cu_masked.restype = ctypes.c_int
        L.tw_stream_destroy.argtypes = [_vp]
        L.tw_stream_destroy.restype = ctypes.c_int
        L.tw_split_threshold.argtypes = [_i64, _i64, ctypes.c_int, _i64, ctypes.c_int]
        L.tw_split_threshold.restype = _i64
        L.tw_policy_split_row.argtypes = [_i64, _i64, _i64, ctypes.c_int, _i64, ctypes.c_int, _i64, _i64]
        L.tw_policy_split_row.restype = _i64
        L.tw_smart_split_point.argtypes = [_i64, _i64, ctypes.POINTER(_i64), ctypes.POINTER(_i64), ctypes.c_int,
                                           ctypes.c_int,
                                           ctypes.POINTER(_i64), ctypes.POINTER(_i64)]
        L.tw_smart_split_point.restype = _i64
        L.tw_weave_schedule.argtypes = [_i64, _i64, _i64, ctypes.c_int, _i64, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        L.tw_weave_schedule.restype = ctypes.c_int
        L.tw_fused_layout.argtypes = [_i64] + [ctypes.POINTER(ctypes.c_int)] * 4
        L.tw_fused_layout.restype = ctypes.c_int
        L.tw_should_split.argtypes = [_i64, _i64]
        L.tw_should_split.restype = ctypes.c_int
        L.tw_gemm_tile_shape.argtypes = [ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
        L.tw_gemm_tile_shape.restype = None
        L.tw_hbm_probe_mixed.argtypes = [_vp, _vp, _i64, ctypes.c_int, ctypes.c_int, ctypes.c_int, _vp]
        L.tw_hbm_probe_mixed.restype = ctypes.c_int
        L.tw_hbm_probe_shaped.argtypes = [_vp, _vp, _i64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, _vp]
        L.tw_hbm_probe_shaped.restype = ctypes.c_int
        L.tw_hbm_probe_mixed_shaped.argtypes = [_vp, _vp, _i64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                _vp]
        L.tw_hbm_probe_mixed_shaped.restype = ctypes.c_int
        L.tw_streams_overlap.argtypes = [_vp, _vp, ctypes.POINTER(ctypes.c_int)]
        L.tw_streams_overlap.restype = ctypes.c_int
        L.tw_device_cu_count.argtypes = []
        L.tw_device_cu_count.restype = ctypes.c_int
        L.tw_status_str.argtypes = [ctypes.c_int]
        L.tw_status_str.restype = ctypes.c_char_p
        L.tw_version.argtypes = []
        L.tw_version.restype = ctypes.c_char_p
        L.tw_last_hip_error.argtypes = []
        L.tw_last_hip_error.restype = ctypes.c_int
        L.tw_last_hip_error_where.argtypes = []
        L.tw_last_hip_error_where.restype = ctypes.c_char_p
        _lib = L
        return L


def _check(status, what):
    if status != 0:
        raise TwError(status, what)


def status_str(status):
    return lib().tw_status_str(int(status)).decode()


def version():
    return lib().tw_version().decode()


def device_cu_count():
    return lib().tw_device_cu_count()


def split_point(N, multiple):
    return int(lib().tw_split_point(int(N), int(multiple)))


def fused_grid(N, H, P, cu_budget=0):
    return int(lib().tw_fused_grid(int(N), int(H), int(P), int(cu_budget)))


# ---- marshalling helpers -------------------------------------------------

def _stream_handle(stream):
    """hipStream_t of a torch stream; None means torch's current stream."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return _vp(stream.cuda_stream)


def _bf16_ptr(t, name, shape=None):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a GPU tensor" % name)
    if t.dtype != torch.bfloat16:
        raise TypeError("%s must be bfloat16, got %s" % (name, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s has shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))
    return _vp(t.data_ptr())


def _fused_pack(partials, residual, weight, eps, cu_budget, out, residual_out):
    import torch
    if residual.dim() != 2:
        raise ValueError("residual must be [N, H]")
    N, H = residual.shape
    P = len(partials)
    if out is None:
        out = torch.empty_like(residual)
    if residual_out is None:
        residual_out = torch.empty_like(residual)
    arr = (_vp * max(P, 1))(*[_bf16_ptr(p, "partials[%d]" % i, (N, H)) for i, p in enumerate(partials)])
    args = FusedArgs(ctypes.cast(arr, ctypes.POINTER(_vp)), _bf16_ptr(residual, "residual"),
                     _bf16_ptr(weight, "weight", (H,)), float(eps), N, H, P, int(cu_budget),
                     _bf16_ptr(out, "out", (N, H)), _bf16_ptr(residual_out, "residual_out", (N, H)))
    return args, arr, out, residual_out


# ---- entry points ----------------------------------------------------------

def reduce_add_rmsnorm(partials, residual, weight, eps, cu_budget=0, out=None, residual_out=None,
                       stream=None):
    """tw_reduce_add_rmsnorm. Returns (out, residual_out)."""
    a, keep, out, residual_out = _fused_pack(partials, residual, weight, eps, cu_budget, out, residual_out)
    _check(lib().tw_reduce_add_rmsnorm(a.partials, a.residual, a.weight, a.eps, a.N, a.H, a.P,
                                       a.cu_budget, a.out, a.residual_out, _stream_handle(stream)),
           "tw_reduce_add_rmsnorm")
    return out, residual_out


def prepare_reduce_add_rmsnorm(partials, residual, weight, eps, cu_budget=0, out=None, residual_out=None,
                               stream=None):
    """Marshals the arguments of tw_reduce_add_rmsnorm once and returns
    (launch, out, residual_out); launch() enqueues the call again with the same
    tensors and stream (for loops that must not pay for marshalling every time).
    The tensors are kept alive by the returned closure."""
    a, keep, out, residual_out = _fused_pack(partials, residual, weight, eps, cu_budget, out, residual_out)
    fn = lib().tw_reduce_add_rmsnorm
    sh = _stream_handle(stream)
    alive = (partials, residual, weight, out, residual_out, keep)
    argv = (a.partials, a.residual, a.weight, a.eps, a.N, a.H, a.P, a.cu_budget, a.out, a.residual_out, sh)

    def launch(_alive=alive):
        st = fn(*argv)
        if st != 0:
            raise TwError(st, "tw_reduce_add_rmsnorm")

    return launch, out, residual_out


def reduce_add_rmsnorm_traced(partials, residual, weight, eps, cu_budget=0, out=None,
                              residual_out=None, stream=None):
    """tw_reduce_add_rmsnorm_traced. Returns (out, residual_out, hw_ids int32 [grid, 2])."""
    import torch
    a, keep, out, residual_out = _fused_pack(partials, residual, weight, eps, cu_budget, out, residual_out)
    grid = max(fused_grid(a.N, a.H, a.P, cu_budget), 1)
    hw = torch.zeros((grid, 2), dtype=torch.int32, device=residual.device)
    _check(lib().tw_reduce_add_rmsnorm_traced(a.partials, a.residual, a.weight, a.eps, a.N, a.H, a.P,
                                              a.cu_budget, a.out, a.residual_out, _vp(hw.data_ptr()),
                                              grid, _stream_handle(stream)),
           "tw_reduce_add_rmsnorm_traced")
    return out, residual_out, hw


def reduce_add_rmsnorm_unfused(partials, residual, weight, eps, out=None, residual_out=None, sum_scratch=None,
                               stream=None):
    """tw_reduce_add_rmsnorm_unfused (the three-pass ablation). Returns (out, residual_out)."""
    import torch
    a, keep, out, residual_out = _fused_pack(partials, residual, weight, eps, 0, out, residual_out)
    if sum_scratch is None:
        sum_scratch = torch.empty_like(residual)
    T, H = residual.shape
    _check(lib().tw_reduce_add_rmsnorm_unfused(ctypes.byref(a), _bf16_ptr(sum_scratch, "sum_scratch", (T, H)),
                                               _stream_handle(stream)), "tw_reduce_add_rmsnorm_unfused")
    return out, residual_out


def reduce_add_rmsnorm_unfused_static(partials, residual, weight, eps, out, residual_out, stream=None):
    """tw_reduce_add_rmsnorm_unfused_static: the three-pass ablation with the library's own scratch.
    `out` and `residual_out` must be given: this call allocates nothing. Returns (out, residual_out)."""
    a, keep, out, residual_out = _fused_pack(partials, residual, weight, eps, 0, out, residual_out)
    _check(lib().tw_reduce_add_rmsnorm_unfused_static(ctypes.byref(a), _stream_handle(stream)),
           "tw_reduce_add_rmsnorm_unfused_static")
    return out, residual_out


def split_launch(partials, residual, weight, eps, split_row, stream_a, stream_b, cu_budget=0,
                 out=None, residual_out=None, parent=None, use_parent=True, join=True):
    """tw_split_launch. parent=None with use_parent=True means torch's current stream."""
    a, keep, out, residual_out = _fused_pack(partials, residual, weight, eps, cu_budget, out, residual_out)
    _check(lib().tw_split_launch(ctypes.byref(a), int(split_row), _stream_handle(stream_a),
                                 _stream_handle(stream_b),
                                 _stream_handle(parent) if use_parent else _vp(None),
                                 1 if use_parent else 0, 1 if join else 0),
           "tw_split_launch")
    return out, residual_out


def _gemm_pack(A, B, C, b_layout, cu_budget):
    import torch
    if A.dim() != 2 or B.dim() != 2:
        raise ValueError("A and B must be matrices")
    M, K = A.shape
    if b_layout == B_NK:
        N = B.shape[0]
        _bf16_ptr(B, "B", (N, K))
    elif b_layout == B_KN:
        N = B.shape[1]
        _bf16_ptr(B, "B", (K, N))
    else:
        raise ValueError("b_layout must be B_NK or B_KN")
    if C is None:
        C = torch.empty((M, N), dtype=torch.bfloat16, device=A.device)
    g = GemmArgs(_bf16_ptr(A, "A"), _bf16_ptr(B, "B"), _bf16_ptr(C, "C", (M, N)), M, N, K,
                 int(b_layout), int(cu_budget))
    return g, C


def gemm_bf16(A, B, C=None, b_layout=B_NK, cu_budget=0, stream=None):
    """tw_gemm_bf16. Returns C."""
    g, C = _gemm_pack(A, B, C, b_layout, cu_budget)
    _check(lib().tw_gemm_bf16(g.A, g.B, g.C, g.M, g.N, g.K, g.b_layout, g.cu_budget,
                              _stream_handle(stream)), "tw_gemm_bf16")
    return C


def overlap_launch(fused, gemm, stream_comm, stream_compute, parent=None, use_parent=True, join=True):
    """tw_overlap_launch. `fused` is a dict(partials, residual, weight, eps, cu_budget, out,
    residual_out) or None; `gemm` a dict(A, B, C, b_layout, cu_budget) or None.
    Returns (out, residual_out, C) with None for the side left out."""
    fa = ga = None
    out = residual_out = C = None
    keep = None
    if fused is not None:
        fa, keep, out, residual_out = _fused_pack(fused["partials"], fused["residual"], fused["weight"],
                                                  fused["eps"], fused.get("cu_budget", 0),
                                                  fused.get("out"), fused.get("residual_out"))
    if gemm is not None:
        ga, C = _gemm_pack(gemm["A"], gemm["B"], gemm.get("C"), gemm.get("b_layout", B_NK),
                           gemm.get("cu_budget", 0))
    _check(lib().tw_overlap_launch(ctypes.byref(fa) if fa is not None else None,
                                   ctypes.byref(ga) if ga is not None else None,
                                   _stream_handle(stream_comm), _stream_handle(stream_compute),
                                   _stream_handle(parent) if use_parent else _vp(None),
                                   1 if use_parent else 0, 1 if join else 0),
           "tw_overlap_launch")
    return out, residual_out, C


def hbm_probe(src, dst, nbytes, mode, cu_budget=0, stream=None):
    """tw_hbm_probe on two GPU tensors of any dtype (byte counts are explicit)."""
    _check(lib().tw_hbm_probe(_vp(src.data_ptr()) if src is not None else _vp(None), _vp(dst.data_ptr()),
                              int(nbytes), int(mode), int(cu_budget), _stream_handle(stream)),
           "tw_hbm_probe")


def hbm_probe_mixed(src, dst, stream_bytes, n_read, n_write, cu_budget=0, stream=None):
    """tw_hbm_probe_mixed: n_read streams read from src, n_write written to dst."""
    _check(lib().tw_hbm_probe_mixed(_vp(src.data_ptr()) if src is not None else _vp(None), _vp(dst.data_ptr()),
                                    int(stream_bytes), int(n_read), int(n_write), int(cu_budget),
                                    _stream_handle(stream)), "tw_hbm_probe_mixed")


def hbm_probe_shaped(src, dst, nbytes, mode, cu_budget=0, threads=1024, in_flight=8, stream=None):
    """tw_hbm_probe_shaped: tw_hbm_probe with the workgroup size and the accesses in flight per thread given."""
    _check(lib().tw_hbm_probe_shaped(_vp(src.data_ptr()) if src is not None else _vp(None), _vp(dst.data_ptr()),
                                     int(nbytes), int(mode), int(cu_budget), int(threads), int(in_flight),
                                     _stream_handle(stream)), "tw_hbm_probe_shaped")


def hbm_probe_mixed_shaped(src, dst, stream_bytes, n_read, n_write, cu_budget=0, threads=1024, stream=None):
    """tw_hbm_probe_mixed_shaped: tw_hbm_probe_mixed with the workgroup size given."""
    _check(lib().tw_hbm_probe_mixed_shaped(_vp(src.data_ptr()) if src is not None else _vp(None),
                                           _vp(dst.data_ptr()), int(stream_bytes), int(n_read), int(n_write),
                                           int(cu_budget), int(threads), _stream_handle(stream)),
           "tw_hbm_probe_mixed_shaped")


def streams_overlap(stream_a, stream_b):
    """tw_streams_overlap: True if kernels on the two torch streams run side by side (blocks ~0.5 ms)."""
    yes = ctypes.c_int(0)
    _check(lib().tw_streams_overlap(_stream_handle(stream_a), _stream_handle(stream_b), ctypes.byref(yes)),
           "tw_streams_overlap")
    return bool(yes.value)


def smart_split_point(T, multiple, gemm_n_out, cus, gemm_k=None):
    """tw_smart_split_point. Returns (split_row, cost_split, cost_unsplit); without gemm_k the costs are
    wave counts."""
    arr = (_i64 * max(len(gemm_n_out), 1))(*[int(x) for x in gemm_n_out])
    karr = None
    if gemm_k is not None:
        if len(gemm_k) != len(gemm_n_out):
            raise ValueError("gemm_k needs one depth per GEMM")
        karr = (_i64 * max(len(gemm_k), 1))(*[int(x) for x in gemm_k])
    ws, wu = _i64(0), _i64(0)
    k = int(lib().tw_smart_split_point(int(T), int(multiple), arr, karr, len(gemm_n_out), int(cus),
                                       ctypes.byref(ws), ctypes.byref(wu)))
    return k, int(ws.value), int(wu.value)


def gemm_tile_shape():
    m, n = ctypes.c_int(0), ctypes.c_int(0)
    lib().tw_gemm_tile_shape(ctypes.byref(m), ctypes.byref(n))
    return m.value, n.value


def weave_layer(X1, W1, partials, residual, weight, eps, W2, split_row, stream_compute, stream_comm,
                fused_cu_budget=32, gemm_cu_budget=0, out=None, residual_out=None, Y=None, parent=None,
                use_parent=True, join=True, schedule=WEAVE_AUTO):
    """tw_weave_layer. partials[0] is overwritten with X1 @ W1.T. Returns (out, residual_out, Y)."""
    import torch
    a, keep, out, residual_out = _fused_pack(partials, residual, weight, eps, fused_cu_budget, out, residual_out)
    T, H = residual.shape
    K1 = X1.shape[1]
    N2 = W2.shape[0]
    if Y is None:
        Y = torch.empty((T, N2), dtype=torch.bfloat16, device=residual.device)
    la = LayerArgs(_bf16_ptr(X1, "X1", (T, K1)), _bf16_ptr(W1, "W1", (H, K1)), K1, a,
                   _bf16_ptr(W2, "W2", (N2, H)), N2, _bf16_ptr(Y, "Y", (T, N2)), int(gemm_cu_budget), int(schedule))
    _check(lib().tw_weave_layer(ctypes.byref(la), int(split_row), _stream_handle(stream_compute),
                                _stream_handle(stream_comm),
                                _stream_handle(parent) if use_parent else _vp(None),
                                1 if use_parent else 0, 1 if join else 0), "tw_weave_layer")
    return out, residual_out, Y


def weave_layer_cuts(X1, W1, partials, residual, weight, eps, W2, cuts, stream_compute, stream_comm,
                     fused_cu_budget=CU_SHARED, gemm_cu_budget=0, out=None, residual_out=None, Y=None, parent=None,
                     use_parent=True, join=True, schedule=WEAVE_AUTO):
    """tw_weave_layer_cuts: the boundary over len(cuts) + 1 splits. Returns (out, residual_out, Y)."""
    import torch
    a, keep, out, residual_out = _fused_pack(partials, residual, weight, eps, fused_cu_budget, out, residual_out)
    T, H = residual.shape
    K1 = X1.shape[1]
    N2 = W2.shape[0]
    if Y is None:
        Y = torch.empty((T, N2), dtype=torch.bfloat16, device=residual.device)
    la = LayerArgs(_bf16_ptr(X1, "X1", (T, K1)), _bf16_ptr(W1, "W1", (H, K1)), K1, a,
                   _bf16_ptr(W2, "W2", (N2, H)), N2, _bf16_ptr(Y, "Y", (T, N2)), int(gemm_cu_budget), int(schedule))
    cuts = [int(c) for c in cuts]
    arr = (_i64 * max(len(cuts), 1))(*cuts)
    _check(lib().tw_weave_layer_cuts(ctypes.byref(la), arr, len(cuts), _stream_handle(stream_compute),
                                     _stream_handle(stream_comm),
                                     _stream_handle(parent) if use_parent else _vp(None),
                                     1 if use_parent else 0, 1 if join else 0), "tw_weave_layer_cuts")
    return out, residual_out, Y


def weave_train(boundaries, split_row, stream_compute, stream_comm, parent=None, use_parent=True, join=True,
                fused_cu_budget=CU_SHARED, gemm_cu_budget=0, schedule=WEAVE_AUTO):
    """tw_weave_train. `boundaries` is a list of dicts(X1, W1, partials, residual, weight, eps, W2, out,
    residual_out, Y), all with the same number of rows; every tensor must be given. Returns None."""
    n = len(boundaries)
    arr = (LayerArgs * max(n, 1))()
    keep = []
    for i, b in enumerate(boundaries):
        a, k, out, residual_out = _fused_pack(b["partials"], b["residual"], b["weight"], b["eps"], fused_cu_budget,
                                              b["out"], b["residual_out"])
        T, H = b["residual"].shape
        K1, N2 = b["X1"].shape[1], b["W2"].shape[0]
        arr[i] = LayerArgs(_bf16_ptr(b["X1"], "X1", (T, K1)), _bf16_ptr(b["W1"], "W1", (H, K1)), K1, a,
                           _bf16_ptr(b["W2"], "W2", (N2, H)), N2, _bf16_ptr(b["Y"], "Y", (T, N2)), int(gemm_cu_budget),
                           int(schedule))
        keep.append(k)
    _check(lib().tw_weave_train(arr, n, int(split_row), _stream_handle(stream_compute), _stream_handle(stream_comm),
                                _stream_handle(parent) if use_parent else _vp(None),
                                1 if use_parent else 0, 1 if join else 0), "tw_weave_train")


def weave_layer_auto(X1, W1, partials, residual, weight, eps, W2, stream_compute, stream_comm, threshold=0,
                     multiple=0, fused_cu_budget=CU_SHARED, gemm_cu_budget=0, out=None, residual_out=None, Y=None,
                     parent=None, use_parent=True, join=True, schedule=WEAVE_AUTO):
    """tw_weave_layer_auto. Returns (out, residual_out, Y, split_row_taken)."""
    import torch
    a, keep, out, residual_out = _fused_pack(partials, residual, weight, eps, fused_cu_budget, out, residual_out)
    T, H = residual.shape
    K1 = X1.shape[1]
    N2 = W2.shape[0]
    if Y is None:
        Y = torch.empty((T, N2), dtype=torch.bfloat16, device=residual.device)
    la = LayerArgs(_bf16_ptr(X1, "X1", (T, K1)), _bf16_ptr(W1, "W1", (H, K1)), K1, a,
                   _bf16_ptr(W2, "W2", (N2, H)), N2, _bf16_ptr(Y, "Y", (T, N2)), int(gemm_cu_budget), int(schedule))
    taken = _i64(-1)
    _check(lib().tw_weave_layer_auto(ctypes.byref(la), int(threshold), int(multiple), _stream_handle(stream_compute),
                                     _stream_handle(stream_comm),
                                     _stream_handle(parent) if use_parent else _vp(None),
                                     1 if use_parent else 0, 1 if join else 0, ctypes.byref(taken)),
           "tw_weave_layer_auto")
    return out, residual_out, Y, int(taken.value)


GEMM_PHASES = 8
GEMM_PHASE_NAMES = ("sub_step_0", "wait_landed", "barrier", "sub_step_1", "tile_fill", "tile_stores", "tiles", "kernel")


def gemm_bf16_traced(A, B, C=None, stream=None):
    """tw_gemm_bf16_traced: C = A [M x K] * B [N x K]^T on 256 x 256 tiles with per-wave phase clocks.
    Returns (C, cycles) with cycles an int64 tensor [waves, GEMM_PHASES] (device)."""
    import torch
    M, K = A.shape
    N = B.shape[0]
    if C is None:
        C = torch.empty((M, N), dtype=torch.bfloat16, device=A.device)
    waves = device_cu_count() * 4
    if stream is None:
        stream = torch.cuda.current_stream()
    with torch.cuda.stream(stream):      # the zero fill must precede the kernel on the kernel's stream
        cycles = torch.zeros((waves, GEMM_PHASES), dtype=torch.int64, device=A.device)
    _check(lib().tw_gemm_bf16_traced(_bf16_ptr(A, "A", (M, K)), _bf16_ptr(B, "B", (N, K)), _bf16_ptr(C, "C", (M, N)),
                                     M, N, K, _vp(cycles.data_ptr()), cycles.numel(), _stream_handle(stream)),
           "tw_gemm_bf16_traced")
    return C, cycles


def weave_tune(X1, W1, partials, residual, weight, eps, W2, stream_compute, stream_comm, offsets=(), reps=5,
               multiple=0, fused_cu_budget=CU_SHARED, gemm_cu_budget=0, out=None, residual_out=None, Y=None,
               schedule=WEAVE_AUTO):
    """tw_weave_tune. Returns (best_row, us): us[0] the unsplit chain, us[1] the smart row, us[2 + i] offsets[i];
    negative where a candidate was not run. Waits for the device."""
    import torch
    a, keep, out, residual_out = _fused_pack(partials, residual, weight, eps, fused_cu_budget, out, residual_out)
    T, H = residual.shape
    K1 = X1.shape[1]
    N2 = W2.shape[0]
    if Y is None:
        Y = torch.empty((T, N2), dtype=torch.bfloat16, device=residual.device)
    la = LayerArgs(_bf16_ptr(X1, "X1", (T, K1)), _bf16_ptr(W1, "W1", (H, K1)), K1, a,
                   _bf16_ptr(W2, "W2", (N2, H)), N2, _bf16_ptr(Y, "Y", (T, N2)), int(gemm_cu_budget), int(schedule))
    offs = (_i64 * max(1, len(offsets)))(*[int(o) for o in offsets])
    us = (ctypes.c_float * (2 + len(offsets)))()
    best = _i64(-1)
    _check(lib().tw_weave_tune(ctypes.byref(la), int(multiple), offs, len(offsets), int(reps),
                               _stream_handle(stream_compute), _stream_handle(stream_comm), ctypes.byref(best), us),
           "tw_weave_tune")
    return int(best.value), [float(x) for x in us]


class CuMaskedStream:
    """tw_stream_create_cu_masked: a stream confined to n_cus compute units. `.stream` is a
    torch.cuda.ExternalStream over it; call close() once its work is done."""

    def __init__(self, first_cu, n_cus):
        import torch
        h = _vp()
        _check(lib().tw_stream_create_cu_masked(int(first_cu), int(n_cus), ctypes.byref(h)),
               "tw_stream_create_cu_masked")
        self.handle = h.value
        self.stream = torch.cuda.ExternalStream(self.handle)

    def close(self):
        if self.handle:
            self.stream.synchronize()
            _check(lib().tw_stream_destroy(_vp(self.handle)), "tw_stream_destroy")
            self.handle = None
            self.stream = None

    def __enter__(self):
        return self.stream

    def __exit__(self, *exc):
        self.close()
        return False


def split_threshold(K1, H, P, N2, cus=256):
    """tw_split_threshold: the built-in token threshold of one block boundary."""
    return int(lib().tw_split_threshold(int(K1), int(H), int(P), int(N2), int(cus)))


def policy_split_row(T, K1, H, P, N2, cus=256, threshold=0, multiple=64):
    """tw_policy_split_row: the row the per-iteration policy cuts a batch of T tokens at (T: not split)."""
    return int(lib().tw_policy_split_row(int(T), int(K1), int(H), int(P), int(N2), int(cus), int(threshold),
                                         int(multiple)))


def weave_schedule(T, K1, H, P, N2, fused_cu_budget=CU_SHARED, schedule=WEAVE_AUTO, cus=256):
    """tw_weave_schedule: the schedule tw_weave_layer takes for these sizes."""
    return int(lib().tw_weave_schedule(int(T), int(K1), int(H), int(P), int(N2), int(fused_cu_budget), int(schedule),
                                       int(cus)))


def fused_layout(H):
    """tw_fused_layout: (waves_per_row, vectors_per_thread, rows_per_trip, threads_per_workgroup)."""
    v = [ctypes.c_int(-1) for _ in range(4)]
    _check(lib().tw_fused_layout(int(H), *[ctypes.byref(x) for x in v]), "tw_fused_layout")
    return tuple(x.value for x in v)


def should_split(num_tokens, threshold=0):
    """tw_should_split."""
    return bool(lib().tw_should_split(int(num_tokens), int(threshold)))
