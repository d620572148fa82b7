"""Pins for the fp64 oracle: it is checked against things other than itself.

Each pin is a function pin_*(impl) that raises AssertionError when `impl`
(a callable (partials, residual, weight, eps) -> (out_f64, res_f64) on uint16
bf16 bit patterns) does not compute the fused reduce + residual-add + RMSNorm of
TokenWeave (arXiv 2505.11329), Appendix A Listing 1. The oracle must pass every
pin; every member of a list of deliberately wrong implementations (mistakes
planted on the CPU: a dropped term, a wrong sign, eps outside the root, H-1,
a transposed index ...) must fail at least one, which shows the pins bite.
"""
import itertools
import math
import os
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
import tw_workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf(a):
    """float array (values exact in bf16 or not) -> bf16 bits via the generator's codec."""
    return W.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def dec(a):
    return W.bf16_bits_to_f32(a).astype(np.float64)


def small_inputs(N, H, P, seed, std=1.0):
    cfg = dict(N=N, H=H, P=P, partial_std=std, residual_std=1.0, outlier_frac=0.0,
               outlier_scale=1.0, eps=1e-5, seed=seed)
    return W.make_fused_inputs(cfg)


# --------------------------------------------------------------------------
# pins
# --------------------------------------------------------------------------

def pin_worked_example(impl):
    """Hand-derived 3-4-5 example (tests/golden/worked_example_h4.txt)."""
    rows = {}
    with open(os.path.join(GOLDEN, "worked_example_h4.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            rows[k] = v
    f64 = lambda k: np.array([float(x) for x in rows[k]])
    parts = [bf(f64("partial0"))[None, :], bf(f64("partial1"))[None, :]]
    out, res = impl(parts, bf(f64("residual"))[None, :], bf(f64("weight")), float(rows["eps"][0]))
    np.testing.assert_allclose(res[0], f64("expect_res"), rtol=0, atol=0)
    np.testing.assert_allclose(out[0], f64("expect_out"), rtol=1e-15, atol=0)
    want_bits = np.array([int(x, 16) for x in rows["expect_out_bf16_bits"]], dtype=np.uint16)
    assert (oracle.f64_to_bf16(out[0]) == want_bits).all()
    want_bits = np.array([int(x, 16) for x in rows["expect_res_bf16_bits"]], dtype=np.uint16)
    assert (oracle.f64_to_bf16(res[0]) == want_bits).all()


def pin_plain_rmsnorm_library(impl):
    """P=1 with a zero residual is plain RMSNorm: compare with torch's CPU
    rms_norm in float64 (Section 4.2: the op being fused is RMSNorm with the
    residual add fused in)."""
    d = small_inputs(7, 96, 1, seed=11)
    zero = np.zeros_like(d["residual"])
    for eps in (1e-6, 0.25):
        out, res = impl(d["partials"], zero, d["weight"], eps)
        x = torch.from_numpy(dec(d["partials"][0]))
        w = torch.from_numpy(dec(d["weight"]))
        want = torch.nn.functional.rms_norm(x, (96,), weight=w, eps=float(np.float32(eps)))
        np.testing.assert_allclose(out, want.numpy(), rtol=1e-13, atol=0)
        np.testing.assert_array_equal(res, x.numpy())


def pin_unit_weight_rms(impl):
    """With weight == 1 each output row has RMS sqrt(ms / (ms + eps)), ms the mean
    square of the new residual row."""
    d = small_inputs(9, 64, 3, seed=5)
    ones = bf(np.ones(64))
    for eps in (1e-5, 3.0):
        out, res = impl(d["partials"], d["residual"], ones, eps)
        ms = (res ** 2).mean(axis=1)
        got = np.sqrt((out ** 2).mean(axis=1))
        want = np.sqrt(ms / (ms + float(np.float32(eps))))
        np.testing.assert_allclose(got, want, rtol=1e-13)
    out, _ = impl(d["partials"], d["residual"], ones, 1e-6)
    assert np.all(np.abs(np.sqrt((out ** 2).mean(axis=1)) - 1.0) < 1e-5)


def pin_exact_rational(impl):
    """Brute force with exact rationals on tiny inputs, H not a power of two so
    that H vs H-1 and eps placement show; 50-digit square root."""
    getcontext().prec = 50
    for (N, H, P, seed, eps) in [(3, 5, 2, 1, 0.5), (2, 12, 3, 2, 1e-5), (1, 7, 1, 3, 0.0),
                                 (4, 3, 4, 4, 2.0)]:
        d = small_inputs(N, H, P, seed)
        out, res = impl(d["partials"], d["residual"], d["weight"], eps)
        epsq = Fraction(float(np.float32(eps)))
        for r in range(N):
            xs = []
            for c in range(H):
                x = Fraction(float(dec(d["residual"])[r, c]))
                for p in range(P):
                    x += Fraction(float(dec(d["partials"][p])[r, c]))
                xs.append(x)
            ms = sum(x * x for x in xs) / H + epsq
            root = (Decimal(ms.numerator) / Decimal(ms.denominator)).sqrt()
            for c in range(H):
                assert Fraction(float(res[r, c])) == xs[c]          # sums are exact in fp64
                wq = Fraction(float(dec(d["weight"])[c]))
                num = xs[c] * wq
                want = float(Decimal(num.numerator) / Decimal(num.denominator) / root)
                assert out[r, c] == pytest.approx(want, rel=4e-16 * 4, abs=0)


def pin_permutation(impl):
    """The P partials enter through a sum: any order gives the same fp64 result
    (sums of <= 17 bf16 values are exact in fp64). Also the residual is just one
    more addend, so swapping it with a partial changes nothing."""
    d = small_inputs(4, 40, 4, seed=9)
    out0, res0 = impl(d["partials"], d["residual"], d["weight"], 1e-5)
    for perm in itertools.permutations(range(4)):
        out, res = impl([d["partials"][i] for i in perm], d["residual"], d["weight"], 1e-5)
        assert np.array_equal(out, out0) and np.array_equal(res, res0)
    parts = list(d["partials"])
    parts[2], swapped = d["residual"], parts[2]
    out, res = impl(parts, swapped, d["weight"], 1e-5)
    assert np.array_equal(out, out0) and np.array_equal(res, res0)
    d8 = small_inputs(3, 24, 8, seed=10)
    out0, res0 = impl(d8["partials"], d8["residual"], d8["weight"], 1e-5)
    rng = np.random.default_rng(0)
    for _ in range(5):
        perm = rng.permutation(8)
        out, res = impl([d8["partials"][i] for i in perm], d8["residual"], d8["weight"], 1e-5)
        assert np.array_equal(out, out0) and np.array_equal(res, res0)


def pin_row_split(impl):
    """Rows are independent (token-level op, Section 4.2): rows [0,k) and [k,N)
    computed separately equal the whole batch, bit for bit."""
    d = small_inputs(10, 32, 2, seed=21)
    out0, res0 = impl(d["partials"], d["residual"], d["weight"], 1e-5)
    for k in (0, 1, 5, 9, 10):
        sl = [slice(0, k), slice(k, 10)]
        outs, ress = [], []
        for s in sl:
            if s.stop - s.start == 0:
                continue
            o, r = impl([p[s] for p in d["partials"]], d["residual"][s], d["weight"], 1e-5)
            outs.append(o)
            ress.append(r)
        assert np.array_equal(np.concatenate(outs), out0)
        assert np.array_equal(np.concatenate(ress), res0)
    # and a permutation of the rows permutes the outputs
    perm = np.random.default_rng(1).permutation(10)
    o, r = impl([p[perm] for p in d["partials"]], d["residual"][perm], d["weight"], 1e-5)
    assert np.array_equal(o, out0[perm]) and np.array_equal(r, res0[perm])


def pin_power_of_two_scaling(impl):
    """With eps = 0, scaling every partial and the residual by 2^j scales the new
    residual exactly and leaves the normalised output unchanged."""
    d = small_inputs(5, 48, 3, seed=31)
    out0, res0 = impl(d["partials"], d["residual"], d["weight"], 0.0)
    for j in (-3, 4):
        sc = lambda a: bf(dec(a) * 2.0 ** j)
        out, res = impl([sc(p) for p in d["partials"]], sc(d["residual"]), d["weight"], 0.0)
        assert np.array_equal(res, res0 * 2.0 ** j)
        np.testing.assert_allclose(out, out0, rtol=4e-16, atol=0)


def pin_weight_is_per_column(impl):
    """out is linear in weight[c], column by column: doubling one weight entry
    doubles exactly that output column and nothing else."""
    d = small_inputs(6, 16, 2, seed=41)
    out0, _ = impl(d["partials"], d["residual"], d["weight"], 1e-5)
    w = dec(d["weight"]).copy()
    w[3] *= 2.0
    out, _ = impl(d["partials"], d["residual"], bf(w), 1e-5)
    want = out0.copy()
    want[:, 3] *= 2.0
    assert np.array_equal(out, want)


def pin_large_eps_limit(impl):
    """eps >> ms: out -> x * w / sqrt(eps) (eps is inside the root, added to the
    MEAN square)."""
    d = small_inputs(3, 24, 2, seed=51)
    eps = 2.0 ** 40
    out, res = impl(d["partials"], d["residual"], d["weight"], eps)
    want = res * dec(d["weight"])[None, :] / 2.0 ** 20
    np.testing.assert_allclose(out, want, rtol=1e-10)


PINS = [pin_worked_example, pin_plain_rmsnorm_library, pin_unit_weight_rms, pin_exact_rational,
        pin_permutation, pin_row_split, pin_power_of_two_scaling, pin_weight_is_per_column,
        pin_large_eps_limit]


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_oracle_passes_pin(pin):
    pin(oracle.fused)


# --------------------------------------------------------------------------
# planted mistakes: a numpy fp64 implementation with switchable defects. It is
# NOT used as a reference anywhere; it only shows that every defect is caught.
# --------------------------------------------------------------------------

def _mutant(defect):
    def impl(partials, residual, weight, eps):
        eps = float(np.float32(eps))
        parts = [dec(p) for p in partials]
        r = dec(residual)
        w = dec(weight)
        H = r.shape[1]
        use = parts[:-1] if defect == "drop_last_partial" and len(parts) > 1 else parts
        acc = np.zeros_like(r)
        for p in use:
            acc = acc + p
        if defect == "partial0_twice":
            acc = acc + parts[0] - parts[-1]
        x = acc if defect == "drop_residual" else (acc - r if defect == "residual_sign" else acc + r)
        xn = acc if defect == "sumsq_before_residual" else x
        if defect == "column_mean" and x.shape[0] == x.shape[1]:
            ms = (xn ** 2).mean(axis=0)[:, None]
        else:
            ms = (xn ** 2).sum(axis=1, keepdims=True) / (H - 1 if defect == "h_minus_1" and H > 1 else H)
        if defect == "eps_outside_root":
            s = 1.0 / (np.sqrt(ms) + eps)
        elif defect == "eps_on_sum":
            s = 1.0 / np.sqrt((ms * H + eps) / H)
        elif defect == "no_root":
            s = 1.0 / (ms + eps)
        elif defect == "mean_abs":
            s = 1.0 / np.sqrt(np.abs(xn).mean(axis=1, keepdims=True) ** 2 + eps)
        else:
            s = 1.0 / np.sqrt(ms + eps)
        if defect == "no_weight":
            out = x * s
        elif defect == "weight_reversed":
            out = x * s * w[::-1][None, :]
        elif defect == "weight_plus_one":
            out = x * s * (1.0 + w)[None, :]
        else:
            out = x * s * w[None, :]
        res = acc if defect == "res_out_without_residual" else x
        if defect == "res_out_normalised":
            res = out
        return out, res
    return impl


DEFECTS = ["drop_last_partial", "partial0_twice", "drop_residual", "residual_sign",
           "sumsq_before_residual", "h_minus_1", "eps_outside_root", "eps_on_sum", "no_root",
           "mean_abs", "no_weight", "weight_reversed", "weight_plus_one",
           "res_out_without_residual", "res_out_normalised"]


def test_defect_free_mutant_passes_all_pins():
    for pin in PINS:
        pin(_mutant(None))


@pytest.mark.parametrize("defect", DEFECTS)
def test_pins_catch_planted_mistake(defect):
    caught = []
    for pin in PINS:
        try:
            pin(_mutant(defect))
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, "no pin notices the planted mistake %r" % defect


# --------------------------------------------------------------------------
# the other oracle entry points
# --------------------------------------------------------------------------

def test_threaded_oracle_equals_single_thread():
    d = small_inputs(37, 72, 3, seed=61)
    a = oracle.fused(d["partials"], d["residual"], d["weight"], 1e-5)
    for nt in (1, 2, 5, 64):
        b = oracle.fused_mt(d["partials"], d["residual"], d["weight"], 1e-5, nt)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_empty_batch():
    d = small_inputs(0, 16, 2, seed=1)
    out, res = oracle.fused(d["partials"], d["residual"], d["weight"], 1e-5)
    assert out.shape == (0, 16) and res.shape == (0, 16)


# ---- the second reading of x (Listing 1 read literally), pinned on its own ----

def _golden_rows(name):
    rows = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            rows[k] = v
    return rows


def pin_rx_worked_example(impl):
    """Hand-derived example in which rounding x moves both the sum of squares and
    the output (tests/golden/rounded_x_example_h2.txt)."""
    rows = _golden_rows("rounded_x_example_h2.txt")
    f64 = lambda k: np.array([float(x) for x in rows[k]])
    parts = [bf(f64("partial0"))[None, :], bf(f64("partial1"))[None, :]]
    out, res = impl(parts, bf(f64("residual"))[None, :], bf(f64("weight")), float(rows["eps"][0]))
    np.testing.assert_array_equal(res[0], f64("expect_res"))
    np.testing.assert_allclose(out[0], f64("expect_out_rounded_x"), rtol=4e-16, atol=0)


def pin_rx_is_the_definition_on_the_stored_row(impl):
    """Rounding x and then normalising is the fused definition applied to the row
    that was stored: one partial equal to bf16(x), a zero residual."""
    d = small_inputs(11, 72, 3, seed=23)
    for eps in (1e-5, 0.5):
        out, res = impl(d["partials"], d["residual"], d["weight"], eps)
        _, x = oracle.fused(d["partials"], d["residual"], d["weight"], eps)
        np.testing.assert_array_equal(res, x)             # the stream itself is reported unrounded
        stored = oracle.f64_to_bf16(x)
        want, _ = oracle.fused([stored], np.zeros_like(stored), d["weight"], eps)
        np.testing.assert_array_equal(out, want)


def pin_rx_equals_unrounded_when_x_is_exact(impl):
    """Small integers: every x is exact in bf16, so the two readings coincide."""
    rng = np.random.default_rng(17)
    N, H, P = 5, 24, 3
    ints = lambda lo, hi, shape: bf(rng.integers(lo, hi + 1, shape).astype(np.float32))
    parts = [ints(-20, 20, (N, H)) for _ in range(P)]
    resid = ints(-40, 40, (N, H))
    w = bf(rng.choice([0.5, 1.0, 2.0], H))
    a = impl(parts, resid, w, 1e-5)
    b = oracle.fused(parts, resid, w, 1e-5)
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1], b[1])


RX_PINS = [pin_rx_worked_example, pin_rx_is_the_definition_on_the_stored_row,
           pin_rx_equals_unrounded_when_x_is_exact]


@pytest.mark.parametrize("pin", RX_PINS, ids=lambda f: f.__name__)
def test_rounded_x_oracle_passes_pin(pin):
    pin(oracle.fused_rounded_x)


def test_unrounded_reading_on_the_same_example():
    """The golden file also states what the fused definition proper gives on it."""
    rows = _golden_rows("rounded_x_example_h2.txt")
    f64 = lambda k: np.array([float(x) for x in rows[k]])
    parts = [bf(f64("partial0"))[None, :], bf(f64("partial1"))[None, :]]
    out, res = oracle.fused(parts, bf(f64("residual"))[None, :], bf(f64("weight")), 0.0)
    np.testing.assert_array_equal(res[0], f64("expect_res"))
    np.testing.assert_allclose(out[0], f64("expect_out_unrounded_x"), rtol=4e-16, atol=0)


def _rx_mutant(defect):
    """numpy fp64 restatement of the second reading with switchable mistakes; it
    is no reference, it only shows that the pins above notice each of them."""
    def impl(partials, residual, weight, eps):
        eps = float(np.float32(eps))
        x = dec(residual) + sum(dec(p) for p in partials)
        xr = oracle.bf16_to_f64(oracle.f64_to_bf16(x))
        x_for_ss = x if defect == "sum_of_squares_unrounded" else xr
        x_for_out = x if defect == "scaling_unrounded" else xr
        if defect == "truncates":
            bits = oracle.f64_to_bf16(x)
            down = oracle.bf16_to_f64(np.where(np.abs(oracle.bf16_to_f64(bits)) > np.abs(x), bits - 1, bits))
            x_for_ss = x_for_out = down
        s = 1.0 / np.sqrt((x_for_ss ** 2).mean(axis=1, keepdims=True) + eps)
        res = xr if defect == "reports_rounded_stream" else x
        return x_for_out * s * dec(weight)[None, :], res
    return impl


def test_defect_free_rounded_x_mutant_passes():
    for pin in RX_PINS:
        pin(_rx_mutant(None))


@pytest.mark.parametrize("defect", ["sum_of_squares_unrounded", "scaling_unrounded", "truncates",
                                    "reports_rounded_stream"])
def test_rounded_x_pins_catch_planted_mistake(defect):
    caught = []
    for pin in RX_PINS:
        try:
            pin(_rx_mutant(defect))
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, "no pin notices the planted mistake %r" % defect


@pytest.mark.parametrize("name,N", [("c1_tiny", 64), ("c2_8b_tp2", 48), ("c3_70b_shard_tp8", 24),
                                    ("c4_split_sweep_tp4", 24)])
def test_two_readings_of_x_agree_within_half_tolerance(name, N):
    """Listing 1 read literally takes the sum of squares on the bf16 vector it
    stores; the device path (fp32 accumulation) takes it on the unrounded sum.
    The choice must not decide a parity verdict. A bf16 rounding moves a value by
    at most 2^-8 relative (8 significand bits), i.e. 0.39 %, against a tolerance
    of 1 % + 1e-3: the two readings stay within half of the parity tolerance of
    each other."""
    d = W.make_fused_inputs(name, N=N)
    a, _ = oracle.fused(d["partials"], d["residual"], d["weight"], d["eps"])
    b, _ = oracle.fused_rounded_x(d["partials"], d["residual"], d["weight"], d["eps"])
    tol = 1e-2 * np.abs(a) + 1e-3
    assert np.all(np.abs(a - b) <= 0.5 * tol)
    assert not np.array_equal(a, b)


def test_non_finite_inputs_stay_in_their_row():
    d = small_inputs(4, 16, 2, seed=71)
    out0, res0 = oracle.fused(d["partials"], d["residual"], d["weight"], 1e-5)
    p0 = d["partials"][0].copy()
    p0[1, 3] = 0x7F80  # +Inf
    p0[2, 5] = 0x7FC0  # NaN
    out, res = oracle.fused([p0, d["partials"][1]], d["residual"], d["weight"], 1e-5)
    assert np.array_equal(out[[0, 3]], out0[[0, 3]]) and np.array_equal(res[[0, 3]], res0[[0, 3]])
    assert np.isinf(res[1, 3]) and np.isnan(res[2, 5])
    assert np.isnan(out[2]).all()
    assert np.isnan(out[1, 3])                     # Inf * rsqrt(Inf) = Inf * 0
    assert np.all(out[1, np.arange(16) != 3] == 0)  # finite * 0


# ---- bf16 codec of the oracle, against the format's definition and torch ----

def test_bf16_decode_matches_format():
    bits = np.array([0x0000, 0x8000, 0x3F80, 0xBF80, 0x4000, 0x3F81, 0x0001, 0x0080, 0x7F7F, 0x7F80],
                    dtype=np.uint16)
    want = [0.0, -0.0, 1.0, -1.0, 2.0, 1.0 + 2.0 ** -7, 2.0 ** -133, 2.0 ** -126,
            (2 - 2.0 ** -7) * 2.0 ** 127, math.inf]
    got = oracle.bf16_to_f64(bits)
    assert list(got) == want
    assert math.copysign(1, got[1]) == -1
    assert np.isnan(oracle.bf16_to_f64(np.array([0x7FC0], dtype=np.uint16))[0])
    allbits = np.arange(65536, dtype=np.uint16)
    t = torch.from_numpy(allbits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(oracle.bf16_to_f64(allbits), t)


def test_bf16_encode_ties_and_single_rounding():
    cases = [
        (1.0 + 2.0 ** -8, 0x3F80),                 # tie, 1.0 is even
        (1.0 + 2.0 ** -7 + 2.0 ** -8, 0x3F82),     # tie, rounds up to even
        (1.0 + 2.0 ** -8 + 2.0 ** -40, 0x3F81),    # above the tie by less than a float32 ulp
        (1.0 + 2.0 ** -8 - 2.0 ** -40, 0x3F80),
        (-(1.0 + 2.0 ** -8 + 2.0 ** -40), 0xBF81),
        (0.0, 0x0000), (-0.0, 0x8000),
        ((2 - 2.0 ** -7) * 2.0 ** 127, 0x7F7F),
        ((2 - 2.0 ** -8) * 2.0 ** 127, 0x7F80),    # halfway to 2^128 -> even = overflow
        ((2 - 2.0 ** -8) * 2.0 ** 127 * (1 - 2.0 ** -30), 0x7F7F),
        (1e300, 0x7F80), (-1e300, 0xFF80),
        (2.0 ** -133, 0x0001), (2.0 ** -134, 0x0000), (2.0 ** -134 * 1.0001, 0x0001),
        (1.5 * 2.0 ** -133, 0x0002),               # tie between 1 and 2 quanta -> even
        (2.0 ** -126 * (1 - 2.0 ** -9), 0x0080),   # top of the subnormals rounds up into normals
        (math.inf, 0x7F80), (-math.inf, 0xFF80),
    ]
    vals = np.array([c[0] for c in cases])
    got = oracle.f64_to_bf16(vals)
    for (v, w), g in zip(cases, got):
        assert g == w, (v, hex(g), hex(w))
    assert oracle.f64_to_bf16(np.array([math.nan]))[0] & 0x7FFF > 0x7F80


def test_bf16_encode_matches_torch_on_float32_inputs():
    rng = np.random.default_rng(3)
    bits = rng.integers(0, 2 ** 32, size=200000, dtype=np.uint64).astype(np.uint32)
    f = bits.view(np.float32)
    f = f[np.isfinite(f)]
    want = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.f64_to_bf16(f.astype(np.float64))
    np.testing.assert_array_equal(got, want)
    # encode(decode(b)) == b for every non-NaN pattern
    allbits = np.arange(65536, dtype=np.uint16)
    ok = (allbits & 0x7FFF) <= 0x7F80
    rt = oracle.f64_to_bf16(oracle.bf16_to_f64(allbits[ok]))
    np.testing.assert_array_equal(rt, allbits[ok])


def test_generator_codec_agrees_with_oracle_codec():
    """Two independently written bf16 encoders (numpy bit trick in the generator,
    fp64 arithmetic in the oracle) agree on float32 inputs."""
    rng = np.random.default_rng(4)
    f = rng.standard_normal(100000).astype(np.float32) * np.float32(3.0)
    np.testing.assert_array_equal(W.f32_to_bf16_bits(f), oracle.f64_to_bf16(f.astype(np.float64)))


# ---- GEMM stand-in: textbook product, pinned to numpy's matmul ----

@pytest.mark.parametrize("layout", ["kn", "nk"])
def test_gemm_oracle_matches_numpy_matmul(layout):
    g = W.make_gemm_inputs(33, 70, 29, 0.5, seed=7, b_layout=layout)
    C = oracle.gemm(g["A"], g["B"], layout)
    A = dec(g["A"])
    B = dec(g["B"]) if layout == "kn" else dec(g["B"]).T
    np.testing.assert_allclose(C, A @ B, rtol=1e-12, atol=1e-13)
    # one-hot operands pick out single entries: catches a transposed operand
    E = np.zeros((33, 70), dtype=np.float32)
    E[2, 5] = 1.0
    Cs = oracle.gemm(bf(E), g["B"], layout)
    assert np.array_equal(Cs[2], B[5]) and np.count_nonzero(Cs[np.arange(33) != 2]) == 0
    ms = np.array([0, 32, 7, 7])
    ns = np.array([0, 28, 3, 20])
    np.testing.assert_array_equal(oracle.gemm_samples(g["A"], g["B"], layout, ms, ns), C[ms, ns])


def test_gemm_layouts_describe_the_same_matrix():
    a = W.make_gemm_inputs(8, 16, 24, 0.5, seed=1, b_layout="kn")
    b = W.make_gemm_inputs(8, 16, 24, 0.5, seed=1, b_layout="nk")
    assert np.array_equal(a["B"], b["B"].T)
    assert np.array_equal(oracle.gemm(a["A"], a["B"], "kn"), oracle.gemm(b["A"], b["B"], "nk"))


# ---- the unfused three-pass pipeline (ablation oracle) --------------------------

def _read_golden(name):
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *rest = line.split()
            vals[k] = rest
    return vals


def test_unfused_worked_example():
    g = _read_golden("unfused_example_h2.txt")
    H, P = int(g["H"][0]), int(g["P"][0])
    enc = lambda k: W.f32_to_bf16_bits(np.array([float(v) for v in g[k]], dtype=np.float32)).reshape(1, H)
    parts = [enc("partial%d" % p) for p in range(P)]
    for p in range(P):      # the inputs of the example are exact in bf16
        assert np.array_equal(oracle.bf16_to_f64(parts[p])[0], [float(v) for v in g["partial%d" % p]])
    out, res = oracle.unfused(parts, enc("residual"), enc("weight").reshape(H), float(g["eps"][0]))
    assert np.array_equal(res[0], [float(v) for v in g["expect_res"]])
    assert np.allclose(out[0], [float(v) for v in g["expect_out"]], rtol=1e-15, atol=0)
    # and the one-pass definition differs on it, as the file says
    _, res_f = oracle.fused(parts, enc("residual"), enc("weight").reshape(H), float(g["eps"][0]))
    assert np.array_equal(res_f[0], [float(v) for v in g["fused_res"]])


def test_unfused_equals_fused_when_no_rounding_happens():
    """Small integers: every sum is an integer below 256, exact in bf16, so both
    intermediate roundings are no-ops and the two definitions coincide."""
    rng = np.random.default_rng(5)
    N, H, P = 6, 40, 4
    ints = lambda lo, hi, shape: W.f32_to_bf16_bits(rng.integers(lo, hi + 1, shape).astype(np.float32))
    parts = [ints(-20, 20, (N, H)) for _ in range(P)]
    resid = ints(-40, 40, (N, H))
    w = W.f32_to_bf16_bits(rng.choice([0.5, 1.0, 2.0], H).astype(np.float32))
    a = oracle.unfused(parts, resid, w, 1e-5)
    b = oracle.fused(parts, resid, w, 1e-5)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_unfused_single_partial_isolates_the_stage_three_rounding():
    """P = 1: the all-reduce has nothing to round, x equals the fused x, the
    sum of squares is the same, and the output differs exactly by the factor
    bf16(x)/x that re-reading the stored residual stream introduces."""
    d = W.make_fused_inputs("c1_tiny", N=16, seed=3, P=1)
    a_out, a_res = oracle.unfused(d["partials"], d["residual"], d["weight"], d["eps"])
    b_out, b_res = oracle.fused(d["partials"], d["residual"], d["weight"], d["eps"])
    assert np.array_equal(a_res, b_res)
    stored = oracle.bf16_to_f64(oracle.f64_to_bf16(b_res))
    nz = b_res != 0
    assert np.allclose(a_out[nz], b_out[nz] * (stored[nz] / b_res[nz]), rtol=1e-14, atol=0)
    assert np.all(a_out[~nz] == 0)


@pytest.mark.parametrize("name", ["c1_tiny", "c3_70b_shard_tp8"])
def test_unfused_stays_within_one_rounding_of_the_partial_sum(name):
    """x differs from the one-pass x by the single rounding of the partial sum:
    at most half a bf16 ulp, i.e. at most 2^-8 relative to that sum (an ulp is
    2^-7 of the binade's lower end)."""
    d = W.make_fused_inputs(name, N=32)
    _, a_res = oracle.unfused(d["partials"], d["residual"], d["weight"], d["eps"])
    _, b_res = oracle.fused(d["partials"], d["residual"], d["weight"], d["eps"])
    psum = sum(oracle.bf16_to_f64(p) for p in d["partials"])
    assert np.all(np.abs(a_res - b_res) <= 2.0 ** -8 * np.abs(psum))
    assert np.any(a_res != b_res)       # and the rounding does happen on real data
    # stage 1 is the exact sum rounded once: x - residual is that rounding, bit for bit
    t = a_res - oracle.bf16_to_f64(d["residual"])
    assert np.array_equal(oracle.f64_to_bf16(t), oracle.f64_to_bf16(psum))
    assert np.array_equal(oracle.bf16_to_f64(oracle.f64_to_bf16(t)), t)


def test_unfused_sum_readings_worked_example():
    """One element on which the exact sum and the binary32 rank-order sum round to
    different bf16 neighbours (tests/golden/unfused_sum_readings_h1.txt)."""
    g = _read_golden("unfused_sum_readings_h1.txt")
    P = int(g["P"][0])
    enc = lambda k: W.f32_to_bf16_bits(np.array([float(v) for v in g[k]], dtype=np.float32)).reshape(1, 1)
    parts = [enc("partial%d" % p) for p in range(P)]
    for p in range(P):
        assert oracle.bf16_to_f64(parts[p])[0, 0] == float(g["partial%d" % p][0])
    args = (parts, enc("residual"), enc("weight").reshape(1), float(g["eps"][0]))
    out, res = oracle.unfused(*args)
    assert res[0, 0] == float(g["expect_res_exact_sum"][0]) and out[0, 0] == float(g["expect_out"][0])
    out, res = oracle.unfused_f32sum(*args)
    assert res[0, 0] == float(g["expect_res_f32_sum"][0]) and out[0, 0] == float(g["expect_out"][0])
    # the exact reading does not depend on the rank order
    rev = (parts[::-1],) + args[1:]
    assert oracle.unfused(*rev)[1][0, 0] == float(g["expect_res_exact_sum"][0])


@pytest.mark.parametrize("name,P", [("c1_tiny", 2), ("c3_70b_shard_tp8", 8), ("c3_70b_shard_tp8", 16)])
def test_unfused_sum_readings_differ_only_across_a_tie(name, P):
    """The binary32 rank-order sum is within P * 2^-24 (relative to the sum of
    magnitudes) of the exact sum, so the two readings give the same bf16 t unless
    a rounding boundary lies between the two sums, and then t moves by exactly one
    bf16 step. With P <= 2 the binary32 sum of two bf16 values of these
    magnitudes is exact and the readings coincide."""
    d = W.make_fused_inputs(name, N=64, P=P)
    a_out, a_res = oracle.unfused(d["partials"], d["residual"], d["weight"], d["eps"])
    b_out, b_res = oracle.unfused_f32sum(d["partials"], d["residual"], d["weight"], d["eps"])
    resid = oracle.bf16_to_f64(d["residual"])
    ta, tb = oracle.f64_to_bf16(a_res - resid), oracle.f64_to_bf16(b_res - resid)
    steps = np.abs(ta.astype(np.int64) - tb.astype(np.int64))
    assert steps.max() <= 1                       # neighbouring bf16 bit patterns (same sign)
    diff = steps == 1
    if P <= 2:
        assert not diff.any()
    else:
        assert diff.mean() < 1e-3                 # rare
    # where they differ, the exact sum sits within the binary32 error of the midpoint of the two
    psum = sum(oracle.bf16_to_f64(p) for p in d["partials"])
    pabs = sum(np.abs(oracle.bf16_to_f64(p)) for p in d["partials"])
    mid = 0.5 * (oracle.bf16_to_f64(ta) + oracle.bf16_to_f64(tb))
    assert np.all(np.abs(psum - mid)[diff] <= P * 2.0 ** -24 * pabs[diff])
    # and the outputs of the two readings stay far inside the parity tolerance of each other
    assert np.all(np.abs(a_out - b_out) <= 0.5 * (1e-2 * np.abs(a_out) + 1e-3))


def test_unfused_f32sum_equals_exact_reading_when_sums_are_exact():
    rng = np.random.default_rng(9)
    N, H, P = 4, 32, 5
    ints = lambda lo, hi, shape: W.f32_to_bf16_bits(rng.integers(lo, hi + 1, shape).astype(np.float32))
    parts = [ints(-20, 20, (N, H)) for _ in range(P)]
    resid = ints(-40, 40, (N, H))
    w = W.f32_to_bf16_bits(rng.choice([0.5, 1.0, 2.0], H).astype(np.float32))
    a = oracle.unfused(parts, resid, w, 1e-5)
    b = oracle.unfused_f32sum(parts, resid, w, 1e-5)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
