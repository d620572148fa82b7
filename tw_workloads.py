"""Seeded synthetic inputs for libtw's tests, smoke check and benchmark.

This module only draws numbers and quantises them to bf16 bit patterns. It
holds none of the method's arithmetic and imports neither the HIP library's
package nor the oracle; both sides are fed from here.

The shapes stand in for the microbenchmark workloads of TokenWeave (arXiv
2505.11329, Table 1 / Table 2 / Fig. 9: hidden size 8192, bf16, 64..64K
tokens) and for the structure of a tensor-parallel block's output: P partial
sums of smaller variance than the accumulated residual stream, with a heavy
tail of outlier channels in the residual for the 70B-class case.

Generator: counter-based, so that element i of stream s under seed k is a pure
function of (k, s, i) whatever the array size or chunking:
    u64  = splitmix64_finalise(key(k, s) + i * golden_gamma)
    unif = (u64 >> 11 [+1]) * 2^-53
    normals by Box-Muller on consecutive pairs of uniforms, in float64,
    then scaled, cast to float32 and rounded to bf16 (nearest, ties to even).
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 21  # elements per work item (even)

# stream ids: one independent sequence per tensor
STREAM_PARTIAL0 = 0        # partial p uses STREAM_PARTIAL0 + p
STREAM_RESIDUAL = 100
STREAM_WEIGHT = 200
STREAM_OUTLIER = 300
STREAM_GEMM_A = 400
STREAM_GEMM_B = 401


def _mix(z):
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _key(seed, stream):
    with np.errstate(over="ignore"):
        k = _mix(np.uint64(seed) * _GAMMA + np.uint64(0x1234567))
        return _mix(k ^ (np.uint64(stream) * _M2 + _GAMMA))


def _uniform_chunk(key, start, count, open_low):
    """count uniforms for counters start..start+count-1; (0,1] if open_low else [0,1)."""
    with np.errstate(over="ignore"):
        idx = np.arange(start, start + count, dtype=np.uint64)
        bits = _mix(key + (idx + np.uint64(1)) * _GAMMA) >> np.uint64(11)
    u = bits.astype(np.float64)
    if open_low:
        u += 1.0
    u *= 2.0 ** -53
    return u


def _normal_chunk(key, start, count):
    """Standard normals for element indices start..start+count-1 (start even)."""
    npairs = (count + 1) // 2
    with np.errstate(over="ignore"):
        j = np.arange(start // 2, start // 2 + npairs, dtype=np.uint64)
        b1 = _mix(key + (np.uint64(2) * j + np.uint64(1)) * _GAMMA) >> np.uint64(11)
        b2 = _mix(key + (np.uint64(2) * j + np.uint64(2)) * _GAMMA) >> np.uint64(11)
    u1 = (b1.astype(np.float64) + 1.0) * 2.0 ** -53      # (0, 1]
    u2 = b2.astype(np.float64) * 2.0 ** -53              # [0, 1)
    r = np.sqrt(-2.0 * np.log(u1))
    th = (2.0 * np.pi) * u2
    out = np.empty(2 * npairs, dtype=np.float64)
    out[0::2] = r * np.cos(th)
    out[1::2] = r * np.sin(th)
    return out[:count]


def f32_to_bf16_bits(a):
    """float32 array -> uint16 bf16 bit patterns, round to nearest even."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = a.view(np.uint32)
    lsb = (b >> np.uint32(16)) & np.uint32(1)
    rounded = (b + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    out = rounded.astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        out[nan] = 0x7FC0
    return out


def bf16_bits_to_f32(a):
    """uint16 bf16 bit patterns -> float32 (exact)."""
    a = np.ascontiguousarray(a, dtype=np.uint16)
    return (a.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _workers():
    return max(1, min(16, (os.cpu_count() or 1)))


def _fill(n, fn):
    """Evaluate fn(start, count) -> uint16[count] over [0, n) in even-sized chunks."""
    out = np.empty(n, dtype=np.uint16)
    starts = list(range(0, n, _CHUNK))

    def work(s):
        c = min(_CHUNK, n - s)
        out[s:s + c] = fn(s, c)

    if len(starts) <= 1:
        for s in starts:
            work(s)
    else:
        with ThreadPoolExecutor(_workers()) as ex:
            list(ex.map(work, starts))
    return out


def normal_bf16(shape, std, seed, stream, outlier_frac=0.0, outlier_scale=1.0):
    """bf16 N(0, std^2); optionally an independent Bernoulli(outlier_frac) subset of
    the entries is multiplied by outlier_scale before rounding."""
    n = int(np.prod(shape))
    key = _key(seed, stream)
    okey = _key(seed, STREAM_OUTLIER + stream)

    def fn(s, c):
        z = _normal_chunk(key, s, c) * std
        if outlier_frac > 0.0:
            hit = _uniform_chunk(okey, s, c, False) < outlier_frac
            z[hit] *= outlier_scale
        return f32_to_bf16_bits(z.astype(np.float32))

    return _fill(n, fn).reshape(shape)


def uniform_bf16(shape, lo, hi, seed, stream):
    """bf16 U(lo, hi)."""
    n = int(np.prod(shape))
    key = _key(seed, stream)

    def fn(s, c):
        u = lo + (hi - lo) * _uniform_chunk(key, s, c, False)
        return f32_to_bf16_bits(u.astype(np.float32))

    return _fill(n, fn).reshape(shape)


# The five workload configurations. N may be a tuple (a sweep).
CONFIGS = {
    # tiny fused step; the oracle runs it in well under a second
    "c1_tiny": dict(N=64, H=512, P=2, partial_std=1.0, residual_std=1.0,
                    outlier_frac=0.0, outlier_scale=1.0, eps=1e-6, seed=0),
    # 8B-class shape, TP=2
    "c2_8b_tp2": dict(N=2048, H=4096, P=2, partial_std=0.5, residual_std=1.0,
                      outlier_frac=0.0, outlier_scale=1.0, eps=1e-5, seed=0,
                      cu_budgets=(8, 16, 32, 256)),
    # 70B-class: one GPU's 1/8 share of an 8192-token batch, TP=8
    "c3_70b_shard_tp8": dict(N=1024, H=8192, P=8, partial_std=0.25, residual_std=1.0,
                             outlier_frac=0.01, outlier_scale=50.0, eps=1e-5, seed=0),
    # token-split sweep, TP=4, value distributions of c2
    "c4_split_sweep_tp4": dict(N=(256, 1024, 4096, 16384), H=8192, P=4, partial_std=0.5,
                               residual_std=1.0, outlier_frac=0.0, outlier_scale=1.0,
                               eps=1e-5, seed=0, split_multiple=128,
                               cu_budgets=(16, 32, 64)),
    # overlap demo: fused on half A next to a GEMM on half B
    "c5_overlap_tp8": dict(N=4096, H=8192, P=8, partial_std=0.25, residual_std=1.0,
                           outlier_frac=0.01, outlier_scale=50.0, eps=1e-5, seed=0,
                           gemm=dict(M=2048, K=8192, N=3584, std=0.02)),
}


def make_fused_inputs(cfg, N=None, seed=None, H=None, P=None):
    """Inputs of one fused step for a CONFIGS entry (or any dict with its keys).

    Returns dict(partials=[P arrays uint16 [N,H]], residual=uint16 [N,H],
    weight=uint16 [H], eps=float, N, H, P)."""
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    N = cfg["N"] if N is None else N
    H = cfg["H"] if H is None else H
    P = cfg["P"] if P is None else P
    seed = cfg["seed"] if seed is None else seed
    if isinstance(N, tuple):
        raise ValueError("pick one N of the sweep")
    partials = [normal_bf16((N, H), cfg["partial_std"], seed, STREAM_PARTIAL0 + p)
                for p in range(P)]
    residual = normal_bf16((N, H), cfg["residual_std"], seed, STREAM_RESIDUAL,
                           cfg["outlier_frac"], cfg["outlier_scale"])
    weight = uniform_bf16((H,), 0.5, 1.5, seed, STREAM_WEIGHT)
    return dict(partials=partials, residual=residual, weight=weight,
                eps=float(cfg["eps"]), N=N, H=H, P=P)


def make_gemm_inputs(M, K, N, std, seed, b_layout):
    """A bf16 [M,K]; B bf16 holding B(k,n) ~ N(0,std^2), stored [K,N] ('kn') or
    [N,K] ('nk'). The value of B(k,n) does not depend on the storage order."""
    A = normal_bf16((M, K), std, seed, STREAM_GEMM_A)
    Bkn = normal_bf16((K, N), std, seed, STREAM_GEMM_B)
    if b_layout == "kn":
        B = Bkn
    elif b_layout == "nk":
        B = np.ascontiguousarray(Bkn.T)
    else:
        raise ValueError("b_layout must be 'kn' or 'nk'")
    return dict(A=A, B=B, M=M, K=K, N=N, b_layout=b_layout)
