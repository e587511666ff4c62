"""Pins the CPU oracle to things other than itself.

Each check is something the paper or the mathematics fixes: hand-worked rows
(tests/golden), the rounding-error bound of Eq. 2 (Sec. 3.1: |error| <= s/2, no
clipping under the min-max range), symmetries of the quantizer, brute-force
integer sums, numpy's own float16 conversion and int64 matmul, the balancing
identity of Eq. 3 (Sec. 4.2), and exact special cases of the epilogue.
"""
import os

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(seed, M, K, scale=1.0):
    g = np.random.default_rng(seed)
    return (g.standard_normal((M, K)) * scale).astype(np.float16)


# ---- fp16 conversions against numpy's --------------------------------------

def test_half_to_float_all_bit_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_to_float(int(b)) for b in bits], np.float32)
    same = (ref.view(np.uint32) == got.view(np.uint32)) | (np.isnan(ref) & np.isnan(got))
    assert same.all()


def test_float_to_half_against_numpy(oracle):
    g = np.random.default_rng(7)
    vals = [g.standard_normal(4000).astype(np.float32) * np.float32(s)
            for s in (1e-8, 1e-6, 6e-5, 1e-3, 1.0, 300.0, 3e4, 7e4)]
    # every midpoint between two neighbouring finite halves (ties) and its fp32 neighbours
    h = np.arange(0, 0x7BFF, dtype=np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    mid = ((lo + hi) / 2).astype(np.float32)
    assert (mid.astype(np.float64) == (lo + hi) / 2).all()  # midpoints are exact in fp32
    vals += [mid, np.nextafter(mid, np.float32(np.inf)), np.nextafter(mid, np.float32(-np.inf)), -mid]
    vals.append(np.array([0.0, -0.0, 65504.0, 65519.996, 65520.0, 65536.0, 1e9, -1e9,
                          np.inf, -np.inf, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001,
                          2.0 ** -14, 2.0 ** -14 * (1 - 2.0 ** -12)], np.float32))
    v = np.concatenate(vals)
    with np.errstate(over="ignore"):
        ref = v.astype(np.float16).view(np.uint16)
    got = np.array([oracle.float_to_half(x) for x in v], np.uint16)
    assert (ref == got).all(), np.flatnonzero(ref != got)[:10]


def test_float_to_half_nan(oracle):
    b = oracle.float_to_half(float("nan"))
    assert (b & 0x7C00) == 0x7C00 and (b & 0x3FF) != 0


# ---- the quantizer: hand examples --------------------------------------------

def _golden_rows():
    out = []
    with open(os.path.join(GOLDEN, "quantizer_hand_examples.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            xs, qs, sc = [p.strip() for p in line.split("|")]
            num, den = sc.split("/")
            out.append((np.array(xs.split(), np.float64), np.array(qs.split(), np.int64),
                        np.float32(np.float32(num) / np.float32(den))))
    return out


def test_golden_file_has_rows():
    assert len(_golden_rows()) >= 6


@pytest.mark.parametrize("case", range(6))
def test_quantizer_hand_examples(oracle, case):
    x, q, scale = _golden_rows()[case]
    x16 = x.astype(np.float16)
    assert (x16.astype(np.float64) == x).all()  # the fixture values are exact in fp16
    xq, xs = oracle.quantize_per_token(x16[None, :])
    assert xq[0].tolist() == q.tolist()
    assert xs[0] == scale


def test_weight_quantizer_hand_example(oracle):
    # qmax = 7: absmax 3.5 -> factor 2: 3.5 -> 7, 0.25 -> 0.5 (tie -> 0), 0.75 -> 1.5 (tie -> 2),
    # -1.25 -> -2.5 (tie -> -2), -3.5 -> -7
    w = np.array([[3.5, 0.25, 0.75, -1.25, -3.5, 0.0]], np.float32)
    wq, ws = oracle.quantize_weight(w, None, 4)
    assert wq[0].tolist() == [7, 0, 2, -2, -7, 0]
    assert ws[0] == np.float32(3.5) / np.float32(7)
    wq8, ws8 = oracle.quantize_weight(np.array([[254.0, -1.0, 3.0, -127.0]], np.float32), None, 8)
    assert wq8[0].tolist() == [127, 0, 2, -64]  # -0.5 -> -0 ; 1.5 -> 2 ; -63.5 -> -64
    assert ws8[0] == np.float32(2.0)


# ---- the quantizer: closed forms and symmetries ---------------------------------

@pytest.mark.parametrize("seed,K,scale", [(1, 1152, 1.0), (2, 64, 40.0), (3, 333, 1e-3), (4, 4608, 5.0)])
def test_rounding_error_at_most_half_a_step_and_extreme_code_present(oracle, seed, K, scale):
    x = _rows(seed, 37, K, scale)
    g = np.random.default_rng(seed + 100)
    cm = np.exp(g.uniform(np.log(0.25), np.log(4.0), K)).astype(np.float32)
    for chan_mul in (None, cm):
        xq, xs = oracle.quantize_per_token(x, chan_mul)
        t = x.astype(np.float32) if chan_mul is None else x.astype(np.float32) * chan_mul[None, :]
        t = t.astype(np.float64)  # the fp32 product, exactly
        s = xs.astype(np.float64)[:, None]
        # Eq. 2: rounding error within [-s/2, s/2] (slack: fp32 rounding of the reciprocal)
        assert (np.abs(xq.astype(np.float64) * s - t) <= 0.5 * s * (1 + 2.0 ** -15)).all()
        # min-max range: nothing clipped, the extreme code sits where |t| is largest
        amax = np.abs(t).max(axis=1)
        assert np.array_equal(xs, (amax.astype(np.float32) / np.float32(127)))
        pos = np.abs(t).argmax(axis=1)
        assert (np.abs(xq[np.arange(len(pos)), pos]) == 127).all()
        assert np.abs(xq.astype(np.int32)).max() <= 127
        # sign agrees with the value wherever the code is not zero
        nz = xq != 0
        assert (np.sign(xq[nz]) == np.sign(t[nz])).all()


def test_power_of_two_scaling_negation_permutation(oracle):
    x = _rows(11, 29, 1152, 3.0)
    xq, xs = oracle.quantize_per_token(x)
    xq2, xs2 = oracle.quantize_per_token((x.astype(np.float32) * 2).astype(np.float16))
    assert np.array_equal(xq, xq2) and np.array_equal(xs2, xs * np.float32(2))
    xqn, xsn = oracle.quantize_per_token(-x)
    assert np.array_equal(xqn, -xq) and np.array_equal(xsn, xs)
    perm = np.random.default_rng(5).permutation(x.shape[1])
    xqp, xsp = oracle.quantize_per_token(np.ascontiguousarray(x[:, perm]))
    assert np.array_equal(xqp, xq[:, perm]) and np.array_equal(xsp, xs)
    # a uniform power-of-two balancing factor only rescales the step
    cm = np.full(x.shape[1], 2.0 ** -3, np.float32)
    xqc, xsc = oracle.quantize_per_token(x, cm)
    assert np.array_equal(xqc, xq) and np.array_equal(xsc, xs * np.float32(2.0 ** -3))
    # chan_mul of ones is the same as none
    xq1, xs1 = oracle.quantize_per_token(x, np.ones(x.shape[1], np.float32))
    assert np.array_equal(xq1, xq) and np.array_equal(xs1, xs)


def test_chan_mul_is_applied_per_channel(oracle):
    # a single channel scaled up by chan_mul must take over the absmax
    x = np.ones((1, 16), np.float16)
    cm = np.ones(16, np.float32)
    cm[5] = 4.0
    xq, xs = oracle.quantize_per_token(x, cm)
    exp = np.full(16, 32, np.int8)  # 1 * 127/4 = 31.75 -> 32
    exp[5] = 127
    assert xq[0].tolist() == exp.tolist() and xs[0] == np.float32(4.0) / np.float32(127)


def test_zero_token_and_tokens_are_independent(oracle):
    x = _rows(12, 8, 256)
    x[3] = 0
    xq, xs = oracle.quantize_per_token(x)
    assert xs[3] == 0 and not xq[3].any() and np.isfinite(xs).all()
    for m in range(8):  # each token only depends on itself
        q1, s1 = oracle.quantize_per_token(x[m:m + 1])
        assert np.array_equal(q1[0], xq[m]) and s1[0] == xs[m]


def test_fp16_subnormals_and_large_values(oracle):
    x = np.array([[6e-8, -6e-8, 1.2e-7, 0], [65504, -65504, 1, 32752]], np.float16)
    xq, xs = oracle.quantize_per_token(x)
    assert xq[0].tolist() == [64, -64, 127, 0]        # 0.5 * 127 = 63.5 -> 64 (tie to even)
    assert xq[1].tolist() == [127, -127, 0, 64]       # 32752/65504 * 127 = 63.5 -> 64
    assert np.isfinite(xs).all() and xs[0] > 0


@settings(max_examples=60, deadline=None)
@given(st.integers(1, 40), st.integers(0, 2 ** 31 - 1))
def test_quantizer_matches_float32_numpy_statement(oracle, K, seed):
    # the same rule stated with numpy float32 operations (np.rint rounds halves to even)
    g = np.random.default_rng(seed)
    x = (g.standard_normal((3, K)) * 10.0 ** g.integers(-3, 3)).astype(np.float16)
    cm = np.exp(g.uniform(-1.4, 1.4, K)).astype(np.float32)
    t = x.astype(np.float32) * cm[None, :]
    amax = np.abs(t).max(axis=1)
    with np.errstate(divide="ignore", invalid="ignore"):
        inv = np.where(amax > 0, np.float32(127) / amax, np.float32(0)).astype(np.float32)
        scale = np.where(amax > 0, amax / np.float32(127), np.float32(0)).astype(np.float32)
    q = np.clip(np.rint(t * inv[:, None]), -127, 127).astype(np.int8)
    xq, xs = oracle.quantize_per_token(x, cm)
    assert np.array_equal(xq, q) and np.array_equal(xs, scale)


# ---- weights ---------------------------------------------------------------------

@pytest.mark.parametrize("bits,qmax", [(8, 127), (4, 7)])
def test_weight_quantizer_bounds(oracle, bits, qmax):
    g = np.random.default_rng(21)
    w = g.normal(0, 0.02, (48, 320)).astype(np.float32)
    w[7] = 0
    s = np.exp(g.uniform(np.log(0.25), np.log(4.0), 320)).astype(np.float32)
    wq, ws = oracle.quantize_weight(w, s, bits)
    t = (w * s[None, :]).astype(np.float64)  # fp32 product, widened exactly
    sc = ws.astype(np.float64)[:, None]
    assert (np.abs(wq * sc - t) <= 0.5 * sc * (1 + 2.0 ** -15)).all()
    assert np.abs(wq.astype(np.int32)).max() == qmax
    rows = np.arange(48) != 7
    assert (np.abs(wq[rows]).max(axis=1) == qmax).all()
    assert ws[7] == 0 and not wq[7].any()
    # folding s before the call is the same as passing it (Eq. 3: diag(s) W)
    wq2, ws2 = oracle.quantize_weight((w * s[None, :]).astype(np.float32), None, bits)
    assert np.array_equal(wq, wq2) and np.array_equal(ws, ws2)


def test_int4_pack_unpack_exhaustive(oracle):
    vals = np.arange(-8, 8, dtype=np.int8)
    lo, hi = np.meshgrid(vals, vals, indexing="ij")
    pairs = np.stack([lo.ravel(), hi.ravel()], axis=1).astype(np.int8)  # all 256 nibble pairs
    packed = oracle.pack_int4(pairs)
    assert packed.shape == (256, 1)
    exp = (pairs[:, 0].astype(np.int32) & 0xF) | ((pairs[:, 1].astype(np.int32) & 0xF) << 4)
    assert np.array_equal(packed[:, 0], exp.astype(np.uint8))
    assert len(set(packed[:, 0].tolist())) == 256  # a bijection onto the byte values
    assert np.array_equal(oracle.unpack_int4(packed), pairs)
    # all 256 byte values decode to two's-complement nibbles
    allb = np.arange(256, dtype=np.uint16).astype(np.uint8)[:, None]
    un = oracle.unpack_int4(allb)
    for b in range(256):
        l, h = b & 0xF, b >> 4
        assert un[b, 0] == (l - 16 if l >= 8 else l) and un[b, 1] == (h - 16 if h >= 8 else h)
    # byte order along K: element 2j in the low nibble of byte j
    row = np.array([[1, 2, 3, 4, -1, -2]], np.int8)
    assert oracle.pack_int4(row)[0].tolist() == [0x21, 0x43, 0xEF]
    with pytest.raises(oracle.OracleError):
        oracle.pack_int4(np.array([[9, 0]], np.int8))


# ---- integer contraction --------------------------------------------------------------

@settings(max_examples=40, deadline=None)
@given(st.integers(1, 6), st.integers(1, 6), st.integers(1, 48), st.integers(0, 2 ** 31 - 1))
def test_gemm_brute_force_tiny(oracle, M, N, K, seed):
    g = np.random.default_rng(seed)
    xq = g.integers(-128, 128, (M, K), dtype=np.int8)
    wq = g.integers(-128, 128, (N, K), dtype=np.int8)
    acc = oracle.gemm_i8(xq, wq)
    for m in range(M):
        for n in range(N):
            assert int(acc[m, n]) == sum(int(xq[m, k]) * int(wq[n, k]) for k in range(K))


def test_gemm_against_numpy_int64_and_special_cases(oracle):
    g = np.random.default_rng(31)
    xq = g.integers(-127, 128, (70, 1152), dtype=np.int8)
    wq = g.integers(-127, 128, (90, 1152), dtype=np.int8)
    acc = oracle.gemm_i8(xq, wq)
    assert acc.dtype == np.int32
    assert np.array_equal(acc.astype(np.int64), xq.astype(np.int64) @ wq.astype(np.int64).T)
    # W = identity picks the activations; the operands are not interchangeable (asymmetric shapes)
    eye = np.eye(64, dtype=np.int8)
    xs = g.integers(-127, 128, (5, 64), dtype=np.int8)
    assert np.array_equal(oracle.gemm_i8(xs, eye), xs.astype(np.int32))
    assert np.array_equal(oracle.gemm_i8(xs, np.ones((3, 64), np.int8)),
                          np.repeat(xs.astype(np.int32).sum(axis=1)[:, None], 3, axis=1))
    # far beyond 2^24: a float accumulator would lose this
    big = oracle.gemm_i8(np.full((2, 4608), 127, np.int8), np.full((3, 4608), -127, np.int8))
    assert (big == -74322432).all()


def test_gemm_overflow_is_reported(oracle):
    K = 133153  # K * 127 * 127 > 2^31 - 1
    with pytest.raises(oracle.OracleError):
        oracle.gemm_i8(np.full((1, K), 127, np.int8), np.full((1, K), 127, np.int8))
    K = 133144  # largest K whose worst case still fits
    assert int(oracle.gemm_i8(np.full((1, K), 127, np.int8), np.full((1, K), 127, np.int8))[0, 0]) == K * 16129


def test_w4_gemm_reduces_to_int8_gemm(oracle):
    g = np.random.default_rng(41)
    wq = g.integers(-7, 8, (24, 128), dtype=np.int8)
    xq = g.integers(-127, 128, (9, 128), dtype=np.int8)
    assert np.array_equal(oracle.gemm_i8(xq, oracle.unpack_int4(oracle.pack_int4(wq))),
                          xq.astype(np.int64) @ wq.astype(np.int64).T)


# ---- epilogue ---------------------------------------------------------------------------

def test_dequant_exact_cases(oracle):
    g = np.random.default_rng(51)
    acc = g.integers(-2047, 2048, (6, 10)).astype(np.int32)  # integers below 2^11 are exact in fp16
    y = oracle.dequant(acc, np.ones(6, np.float32), np.ones(10, np.float32))
    assert np.array_equal(y.astype(np.int32), acc)
    # powers of two commute with rounding; bias 0.5 on small integers stays exact
    xs = np.float32(2.0) ** g.integers(-3, 3, 6).astype(np.float32)
    ws = np.float32(2.0) ** g.integers(-3, 3, 10).astype(np.float32)
    small = g.integers(-60, 60, (6, 10)).astype(np.int32)
    bias = np.full(10, 0.5, np.float16)
    y = oracle.dequant(small, xs, ws, bias)
    exp = small.astype(np.float64) * xs[:, None].astype(np.float64) * ws[None, :].astype(np.float64) + 0.5
    assert np.array_equal(y.astype(np.float64), exp.astype(np.float16).astype(np.float64))
    # which scale belongs to which axis
    a = np.ones((2, 3), np.int32)
    y = oracle.dequant(a, np.array([1, 2], np.float32), np.array([1, 4, 16], np.float32))
    assert y.astype(np.float32).tolist() == [[1, 4, 16], [2, 8, 32]]
    # zero token scale -> the row is the bias
    b = np.array([0.25, -1.5, 3.0], np.float16)
    y = oracle.dequant(np.full((1, 3), 12345, np.int32), np.zeros(1, np.float32), np.ones(3, np.float32), b)
    assert np.array_equal(y[0], b)


def test_dequant_close_to_float64_evaluation(oracle):
    g = np.random.default_rng(52)
    acc = g.integers(-70_000_000, 70_000_000, (40, 50)).astype(np.int32)
    xs = np.exp(g.uniform(-9, -2, 40)).astype(np.float32)
    ws = np.exp(g.uniform(-12, -6, 50)).astype(np.float32)
    bias = g.normal(0, 0.01, 50).astype(np.float16)
    y = oracle.dequant(acc, xs, ws, bias).astype(np.float64)
    ref = acc.astype(np.float64) * xs[:, None] * ws[None, :] + bias.astype(np.float64)[None, :]
    # half an fp16 ulp of the result plus a few fp32 ulps of the terms
    ulp16 = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 2.0 ** -14))) - 10), 2.0 ** -24)
    tol = 0.5 * ulp16 + 4 * 2.0 ** -24 * (np.abs(ref) + np.abs(bias.astype(np.float64))[None, :])
    assert (np.abs(y - ref) <= tol).all()


# ---- balancing (Eq. 3) and the whole layer ---------------------------------------------------

def test_balancing_identity_in_float64():
    g = np.random.default_rng(61)
    X = g.standard_normal((20, 96))
    W = g.normal(0, 0.02, (30, 96))
    s = np.exp(g.uniform(np.log(0.25), np.log(4.0), 96))
    y0 = X @ W.T
    y1 = (X / s[None, :]) @ (W * s[None, :]).T
    assert np.abs(y1 - y0).max() <= 1e-12 * np.abs(y0).max()


def test_power_of_two_mask_leaves_the_layer_bit_identical(oracle):
    g = np.random.default_rng(62)
    x = _rows(63, 33, 256, 2.0)
    w = g.normal(0, 0.02, (40, 256)).astype(np.float32)
    bias = g.normal(0, 0.01, 40).astype(np.float16)
    wq0, ws0 = oracle.quantize_weight(w, None, 8)
    base = oracle.linear(x, None, wq0, 8, ws0, bias)
    s = np.full(256, 4.0, np.float32)
    wq1, ws1 = oracle.quantize_weight(w, s, 8)
    bal = oracle.linear(x, (np.float32(1) / s), wq1, 8, ws1, bias)
    assert np.array_equal(wq0, wq1) and np.array_equal(base["xq"], bal["xq"])
    assert np.array_equal(base["acc"], bal["acc"]) and np.array_equal(base["y"], bal["y"])


def test_linear_is_the_composition_of_its_steps(oracle):
    g = np.random.default_rng(71)
    x = _rows(72, 50, 384, 1.5)
    x[17] = 0
    w = g.normal(0, 0.02, (72, 384)).astype(np.float32)
    bias = g.normal(0, 0.01, 72).astype(np.float16)
    s = np.exp(g.uniform(np.log(0.25), np.log(4.0), 384)).astype(np.float32)
    cm = np.float32(1) / s
    for bits in (8, 4):
        wq, ws = oracle.quantize_weight(w, s, bits)
        wdev = wq if bits == 8 else oracle.pack_int4(wq)
        out = oracle.linear(x, cm, wdev, bits, ws, bias)
        xq, xs = oracle.quantize_per_token(x, cm)
        acc = oracle.gemm_i8(xq, wq)
        y = oracle.dequant(acc, xs, ws, bias)
        assert np.array_equal(out["xq"], xq) and np.array_equal(out["x_scale"], xs)
        assert np.array_equal(out["acc"], acc) and np.array_equal(out["y"], y)
        assert np.array_equal(out["y"][17], bias)  # a token of zeros yields the bias, no NaN
        assert np.isfinite(out["y"].astype(np.float32)).all()


@pytest.mark.parametrize("bits", [8, 4])
def test_layer_error_within_the_rounding_error_bound(oracle, bits):
    # Each factor is off by at most half a step (Eq. 2), so
    # |y_q - y| <= sum_k (|x| s_w/2 + |w| s_x/2 + s_x s_w/4) (+ output rounding)
    g = np.random.default_rng(81)
    x = _rows(82, 24, 512, 1.0)
    w = g.normal(0, 0.02, (36, 512)).astype(np.float32)
    s = np.exp(g.uniform(np.log(0.25), np.log(4.0), 512)).astype(np.float32)
    cm = (np.float32(1) / s).astype(np.float32)
    wq, ws = oracle.quantize_weight(w, s, bits)
    out = oracle.linear(x, cm, wq if bits == 8 else oracle.pack_int4(wq), bits, ws, None)
    xh = x.astype(np.float64) * cm.astype(np.float64)[None, :]
    wh = w.astype(np.float64) * s.astype(np.float64)[None, :]
    ref = xh @ wh.T
    sx = out["x_scale"].astype(np.float64)[:, None]
    sw = ws.astype(np.float64)[None, :]
    bound = (np.abs(xh).sum(axis=1)[:, None] * sw / 2 + np.abs(wh).sum(axis=1)[None, :] * sx / 2
             + 512 * sx * sw / 4)
    err = np.abs(out["y"].astype(np.float64) - ref)
    assert (err <= bound * (1 + 1e-3) + 2.0 ** -11 * np.abs(ref) + 2.0 ** -24).all()
    # typical error: rounding errors behave like independent uniform noise of variance step^2/12
    pred = ((xh ** 2).sum(axis=1)[:, None] * sw ** 2 / 12 + (wh ** 2).sum(axis=1)[None, :] * sx ** 2 / 12
            + 512 * (sx * sw) ** 2 / 144)
    ratio = (err ** 2).sum() / pred.sum()
    assert 0.5 < ratio < 2.0, ratio
